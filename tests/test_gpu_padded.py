"""GPU parity of the padded ("vanilla", Sec. 3.1) ablation kernels against their oracle, and
against the unpadded path: real rows must agree, padding must not leak."""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
from workloads import HEAD_MAJOR, TOKEN_MAJOR, bits, make_batch, make_config, pad_batch
from helpers import hip_attention, oracle_attention, to_device

pytestmark = pytest.mark.gpu


def hip_padded_attention(p, out_dtype=None):
    import paper_2405_07542_amd as ems
    out = torch.full_like(p.q_pad, float("nan"), dtype=out_dtype or p.dtype)
    ws = torch.empty(ems.ems_attention_workspace_bytes(p.B, p.B * p.k_max, p.H, p.D, p.l_pad),
                     dtype=torch.uint8, device=p.q_pad.device)
    ems.ems_padded_verify_attention(
        p.q_pad, p.k_new_pad, p.v_new_pad,
        ems.kv_cache(p.k_cache, p.v_cache, p.row_stride, p.head_stride, p.rows), p.cap, p.key_mask,
        p.k_valid, out, k_max=p.k_max, l_pad=p.l_pad, scale=p.scale, workspace=ws)
    torch.cuda.synchronize()
    return out


def padded_to_device(p):
    kw = {f.name: (getattr(p, f.name).cuda() if isinstance(getattr(p, f.name), torch.Tensor)
                   else getattr(p, f.name)) for f in dataclasses.fields(p)}
    return type(p)(**kw)


CASES = [
    dict(kv_len=[17, 40], k=[3, 5], H=2, D=64, dtype=torch.float16),
    dict(kv_len=[0, 1, 31, 32, 33, 100, 257], k=[1, 16, 3, 7, 2, 11, 5], H=4, D=128, dtype=torch.bfloat16),
    dict(kv_len=[700, 64, 1500], k=[2, 9, 4], H=3, D=128, dtype=torch.float16),
]


@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_padded_attention_matches_its_oracle_and_the_unpadded_path(case, layout):
    c = CASES[case]
    b = make_batch(c["kv_len"], c["k"], H=c["H"], D=c["D"], dtype=c["dtype"], seed=90 + case,
                   capacity=max(c["kv_len"]) + 32, layout=layout)
    p = pad_batch(b, interleave=True, extra_pad=case * 7)
    print("padded case", case, layout, "k_max", p.k_max, "l_pad", p.l_pad, "cap", p.cap, flush=True)
    want_pad = oracle.padded_verify_attention(
        bits(p.q_pad), bits(p.k_new_pad), bits(p.v_new_pad), bits(p.k_cache), bits(p.v_cache),
        p.row_stride, p.head_stride, p.cap, p.key_mask.numpy(), p.k_valid.numpy(), p.k_max, p.l_pad,
        p.H, p.D, p.scale, p.dtype)
    got_pad = hip_padded_attention(padded_to_device(p), out_dtype=torch.float32).double().cpu().numpy()
    real = p.real_rows.numpy()
    assert np.isfinite(got_pad[real]).all()
    assert np.abs(got_pad[real] - want_pad[real]).max() <= 2e-3
    # the unpadded path on the unpadded data gives the same rows (Sec. 3.1: masks keep padding out)
    got_unpad = hip_attention(to_device(b), out_dtype=torch.float32).double().cpu().numpy()
    want_unpad = oracle_attention(b)
    assert np.array_equal(want_pad[real], want_unpad)
    assert np.abs(got_unpad - want_unpad).max() <= 2e-3
    assert np.abs(got_unpad - got_pad[real]).max() <= 4e-3


def test_padded_ranges_of_nothing_but_padding_through_the_in_workgroup_merge():
    """Left-padded caches of very different lengths, large enough for the library to merge the
    partials of a workgroup's waves in LDS: whole waves see only padding keys (running max
    -inf, sum 0), as the first, a middle or the last part of a pair."""
    kv_len = [6000, 100, 3000, 0, 50, 2000, 10, 4000]
    k = [2, 5, 1, 3, 4, 2, 1, 6]
    b = make_batch(kv_len, k, H=8, D=64, dtype=torch.bfloat16, seed=97, capacity=6100)
    p = pad_batch(b, interleave=False, extra_pad=200)
    assert b.B * b.H * ((p.l_pad + 31) // 32 + 1) >= 12 * 1024      # the size from which the merge is on
    want_pad = oracle.padded_verify_attention(
        bits(p.q_pad), bits(p.k_new_pad), bits(p.v_new_pad), bits(p.k_cache), bits(p.v_cache),
        p.row_stride, p.head_stride, p.cap, p.key_mask.numpy(), p.k_valid.numpy(), p.k_max, p.l_pad,
        p.H, p.D, p.scale, p.dtype)
    got_pad = hip_padded_attention(padded_to_device(p), out_dtype=torch.float32).double().cpu().numpy()
    real = p.real_rows.numpy()
    assert np.isfinite(got_pad[real]).all()
    assert np.abs(got_pad[real] - want_pad[real]).max() <= 2e-3


def test_padded_append_matches_its_oracle():
    import paper_2405_07542_amd as ems
    n_layers = 3
    kv_len, k = [20, 5, 33], [6, 2, 4]
    accepted = [4, 1, 2]
    tau_max = max(accepted)
    layers = [pad_batch(make_batch(kv_len, k, H=2, D=64, seed=95 + l, capacity=64), seed=l) for l in range(n_layers)]
    # all layers share one key mask (padding positions are a property of the batch, not the layer)
    mask0 = layers[0].key_mask.clone()
    dev = [padded_to_device(p) for p in layers]
    g_mask = mask0.cuda()
    acc = torch.tensor(accepted, dtype=torch.int32, device="cuda")
    p0 = layers[0]
    ems.ems_padded_kv_append([p.k_new_pad for p in dev], [p.v_new_pad for p in dev],
                             [ems.kv_cache(p.k_cache, p.v_cache, p.row_stride, p.head_stride, p.rows) for p in dev],
                             p0.cap, g_mask, acc, k_max=p0.k_max, l_pad=p0.l_pad, tau_max=tau_max)
    torch.cuda.synchronize()
    for p_cpu, p in zip(layers, dev):
        okc, ovc = bits(p_cpu.k_cache).copy(), bits(p_cpu.v_cache).copy()
        omask = mask0.numpy().copy()
        oracle.padded_kv_append(okc, ovc, p_cpu.row_stride, p_cpu.head_stride, p_cpu.cap, omask,
                                bits(p_cpu.k_new_pad), bits(p_cpu.v_new_pad), accepted, p_cpu.k_max,
                                p_cpu.l_pad, tau_max, p_cpu.H, p_cpu.D)
        assert np.array_equal(bits(p.k_cache), okc) and np.array_equal(bits(p.v_cache), ovc)
        assert np.array_equal(g_mask.cpu().numpy(), omask)


def test_padded_config4_real_rows_on_sampled_outputs():
    """Full-size config 4 in the padded layout (the launch the bench times): real rows of a
    few sampled samples against the unpadded oracle restricted to those samples."""
    b = make_config(4, with_logits=False)
    p = pad_batch(b)
    got = hip_padded_attention(padded_to_device(p)).double().cpu().numpy()
    cu = b.cu_seqlens.numpy()
    for i in (0, 31, 63):
        sub = make_sub_batch(b, i)
        want = oracle_attention(sub)
        rows = np.arange(cu[i], cu[i + 1]) - cu[i] + i * p.k_max
        assert np.abs(got[rows] - want).max() <= 2e-3


def make_sub_batch(b, i):
    """Sample i of batch b as a one-sample batch that shares b's arena."""
    cu = b.cu_seqlens
    sl = slice(int(cu[i]), int(cu[i + 1]))
    return dataclasses.replace(
        b, B=1, T=sl.stop - sl.start, cu_seqlens=torch.tensor([0, sl.stop - sl.start], dtype=torch.int32),
        kv_start=b.kv_start[i:i + 1], kv_len=b.kv_len[i:i + 1], q=b.q[sl], k_new=b.k_new[sl],
        v_new=b.v_new[sl], max_k=sl.stop - sl.start, max_kv_len=int(b.kv_len[i]))
