"""Pins for the padded ("vanilla") ablation's oracle: the paper's statement that attention
masks keep padding tokens out of the computation (Sec. 3.1) means the real rows of the padded
method equal the unpadded method's rows; Table 1 fixes the padding bookkeeping."""
import os

import numpy as np
import pytest
import torch

import oracle
from workloads import HEAD_MAJOR, TOKEN_MAJOR, bits, make_batch, make_config, pad_batch
from test_oracle_attention import run_oracle
from test_oracle_accept_append import read_table1


def run_padded_oracle(p):
    return oracle.padded_verify_attention(
        bits(p.q_pad), bits(p.k_new_pad), bits(p.v_new_pad), bits(p.k_cache), bits(p.v_cache),
        p.row_stride, p.head_stride, p.cap, p.key_mask.cpu().numpy(), p.k_valid.cpu().numpy(),
        p.k_max, p.l_pad, p.H, p.D, p.scale, p.dtype)


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
@pytest.mark.parametrize("interleave", [True, False])
def test_padded_real_rows_equal_unpadded_rows(layout, interleave):
    for b in (make_config(1, layout=layout),
              make_batch([0, 9, 33, 2], [3, 1, 7, 2], H=2, D=16, dtype=torch.bfloat16, seed=80,
                         capacity=48, layout=layout)):
        p = pad_batch(b, interleave=interleave, extra_pad=5)
        want = run_oracle(b)
        got = run_padded_oracle(p)
        assert got.shape[0] == b.B * p.k_max
        assert np.isfinite(got).all()
        # masked keys contribute exact zeros and the real keys keep their order: bit-identical
        assert np.array_equal(got[p.real_rows.numpy()], want)


def test_padding_changes_nothing_when_its_values_change():
    b = make_batch([6, 20], [2, 5], H=2, D=16, seed=81, capacity=32)
    p1, p2 = pad_batch(b, seed=1), pad_batch(b, seed=1)
    junk = p2.key_mask.bool().logical_not()           # [B, cap] padding keys
    view = p2.k_cache.view(p2.rows, p2.H, p2.D)
    view[junk.reshape(-1)] = 3.0
    r = p1.real_rows.numpy()
    assert np.array_equal(run_padded_oracle(p1)[r], run_padded_oracle(p2)[r])


def test_padded_append_follows_table1():
    """Table 1: accepted {4,1} then {2,6}: every sample grows by the batch maximum; the
    padding written is {0,3} then {4,0} rows; the aligned length grows by 4 then 6."""
    table = read_table1()
    H, D, k_max, cap = 1, 8, 6, 64
    l_pad = 8
    rng = np.random.default_rng(2)
    kc = np.zeros(2 * cap * H * D, dtype=np.uint16)
    vc = np.zeros_like(kc)
    mask = np.zeros((2, cap), dtype=np.uint8)
    mask[:, :l_pad] = 1
    real = [l_pad, l_pad]
    for step in (1, 2):
        rows = sorted([r for r in table if r[0] == step], key=lambda r: r[1])
        accept = [r[4] for r in rows]
        tau_max = max(accept)
        kn = rng.integers(1, 30000, 2 * k_max * H * D).astype(np.uint16)
        vn = rng.integers(1, 30000, 2 * k_max * H * D).astype(np.uint16)
        oracle.padded_kv_append(kc, vc, H * D, D, cap, mask, kn, vn, accept, k_max, l_pad, tau_max, H, D)
        for i in range(2):
            new = mask[i, l_pad:l_pad + tau_max]
            assert new.tolist() == [1] * accept[i] + [0] * (tau_max - accept[i])
            assert int((new == 0).sum()) == rows[i][5]            # the table's padding column
            got = kc.reshape(2 * cap, H * D)[i * cap + l_pad:i * cap + l_pad + tau_max]
            assert np.array_equal(got, kn.reshape(2 * k_max, H * D)[i * k_max:i * k_max + tau_max])
            real[i] += accept[i]
        l_pad += tau_max
    assert l_pad == 8 + 4 + 6 and real == [8 + 4 + 2, 8 + 1 + 6]
    assert mask.sum(axis=1).tolist() == real
    assert (mask[:, l_pad:] == 0).all() and (kc.reshape(2 * cap, -1)[l_pad:cap] == 0).all()
