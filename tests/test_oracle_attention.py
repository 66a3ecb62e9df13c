"""Pins for the attention oracle: none of them re-types its formula.

* dense padded per-sample brute force (numpy matmul + dense additive mask)
* torch's CPU attention in the two special cases that reduce to it
* autoregressive equivalence (Appendix A: verifying several tokens at once gives
  what one-token-at-a-time decoding gives)
* closed forms and invariants
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import (HEAD_MAJOR, TOKEN_MAJOR, arena_view, bits, from_bits, make_batch,
                       make_config)


def run_oracle(b, k_cache=None, v_cache=None):
    return oracle.verify_attention(
        bits(b.q), bits(b.k_new), bits(b.v_new),
        bits(b.k_cache if k_cache is None else k_cache),
        bits(b.v_cache if v_cache is None else v_cache),
        b.row_stride, b.head_stride, b.cu_seqlens.numpy(), b.kv_start.numpy(),
        b.kv_len.numpy(), b.H, b.D, b.scale, b.dtype)


def padded_brute_force(b):
    """Vanilla-style computation, one sample at a time: pad every sample to the
    batch-wide maximum key count, dense additive mask, softmax, matmul."""
    cu = b.cu_seqlens.numpy()
    ks = b.kv_start.numpy()
    kl = b.kv_len.numpy()
    K = arena_view(b.k_cache, b.layout, b.rows, b.H, b.D).double().numpy()
    V = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D).double().numpy()
    q, kn, vn = b.q.double().numpy(), b.k_new.double().numpy(), b.v_new.double().numpy()
    kmax = int(max(cu[1:] - cu[:-1]))
    Nmax = int(max(kl)) + kmax
    out = np.zeros((b.T, b.H, b.D))
    for i in range(b.B):
        k = int(cu[i + 1] - cu[i])
        L = int(kl[i])
        keys = np.zeros((Nmax, b.H, b.D))
        vals = np.zeros((Nmax, b.H, b.D))
        # left-pad the cache so that the new tokens of all samples line up at the end
        pad = Nmax - kmax - L
        keys[pad:pad + L] = K[ks[i]:ks[i] + L]
        vals[pad:pad + L] = V[ks[i]:ks[i] + L]
        keys[pad + L:pad + L + k] = kn[cu[i]:cu[i + 1]]
        vals[pad + L:pad + L + k] = vn[cu[i]:cu[i + 1]]
        qp = np.zeros((kmax, b.H, b.D))
        qp[:k] = q[cu[i]:cu[i + 1]]
        col = np.arange(Nmax)[None, :]
        row = np.arange(kmax)[:, None]
        visible = (col >= pad) & (col <= pad + L + row)
        add = np.where(visible, 0.0, -np.inf)
        for h in range(b.H):
            s = np.float64(np.float32(b.scale)) * (qp[:, h] @ keys[:, h].T) + add
            s = s - s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=1, keepdims=True)
            out[cu[i]:cu[i + 1], h] = (p @ vals[:, h])[:k]
    return out


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_tiny_config_equals_padded_brute_force(layout):
    b = make_config(1, layout=layout)
    got = run_oracle(b)
    want = padded_brute_force(b)
    assert got.shape == (8, 2, 64)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_random_tiny_shapes_equal_padded_brute_force(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 5))
    kv_len = rng.integers(0, 37, B).tolist()
    k = rng.integers(1, 8, B).tolist()
    H = int(rng.integers(1, 4))
    D = int(rng.choice([8, 16, 64]))
    order = rng.permutation(B)          # regions need not be in sample order
    sizes = [kv_len[i] + k[i] + 3 for i in range(B)]
    pos = 0
    starts = [0] * B
    for i in order:
        starts[i] = pos
        pos += sizes[i]
    dtype = torch.float16 if seed % 2 == 0 else torch.bfloat16
    layout = TOKEN_MAJOR if seed % 3 else HEAD_MAJOR
    b = make_batch(kv_len, k, H=H, D=D, dtype=dtype, seed=100 + seed, kv_start=starts, rows=pos,
                   layout=layout)
    np.testing.assert_allclose(run_oracle(b), padded_brute_force(b), rtol=0, atol=1e-12)


def test_single_query_rows_equal_torch_decode_attention():
    """k_i = 1 everywhere: ordinary one-token decode attention over L_i + 1 keys."""
    kv_len, k = [5, 33, 12], [1, 1, 1]
    b = make_batch(kv_len, k, H=3, D=16, seed=7)
    got = run_oracle(b)
    K = arena_view(b.k_cache, b.layout, b.rows, b.H, b.D).double()
    V = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D).double()
    for i, L in enumerate(kv_len):
        s = int(b.kv_start[i])
        keys = torch.cat([K[s:s + L], b.k_new[i:i + 1].double()]).permute(1, 0, 2)[None]
        vals = torch.cat([V[s:s + L], b.v_new[i:i + 1].double()]).permute(1, 0, 2)[None]
        qq = b.q[i:i + 1].double().permute(1, 0, 2)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(qq, keys, vals, scale=b.scale)
        np.testing.assert_allclose(got[i], ref[0, :, 0].numpy(), rtol=0, atol=1e-12)


def test_empty_caches_equal_torch_causal_attention():
    """kv_len = 0: textbook causal self-attention over the k_i new rows."""
    k = [4, 1, 7]
    b = make_batch([0, 0, 0], k, H=2, D=32, seed=8, capacity=8)
    got = run_oracle(b)
    cu = b.cu_seqlens.numpy()
    for i in range(3):
        sl = slice(cu[i], cu[i + 1])
        qq = b.q[sl].double().permute(1, 0, 2)[None]
        kk = b.k_new[sl].double().permute(1, 0, 2)[None]
        vv = b.v_new[sl].double().permute(1, 0, 2)[None]
        ref = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=True,
                                                               scale=b.scale)
        np.testing.assert_allclose(got[sl], ref[0].permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


def test_autoregressive_equivalence():
    """Row j of a k-row verification equals the j-th of k one-row steps, each
    followed by appending that row's K/V to the cache."""
    kv_len, k = [9, 20], [4, 6]
    b = make_batch(kv_len, k, H=2, D=16, seed=9, capacity=40)
    multi = run_oracle(b)
    cu = b.cu_seqlens.numpy()
    kc, vc = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    lens = np.array(kv_len, dtype=np.int32)
    single = np.zeros_like(multi)
    for j in range(max(k)):
        live = [i for i in range(b.B) if j < k[i]]
        rows = [cu[i] + j for i in live]
        step_cu = np.arange(len(live) + 1, dtype=np.int32)
        qj, kj, vj = bits(b.q)[rows], bits(b.k_new)[rows], bits(b.v_new)[rows]
        o = oracle.verify_attention(qj, kj, vj, kc, vc, b.row_stride, b.head_stride, step_cu,
                                    b.kv_start.numpy()[live], lens[live], b.H, b.D, b.scale,
                                    b.dtype)
        single[rows] = o
        new_len = oracle.kv_append(kc, vc, b.row_stride, b.head_stride, kj, vj, step_cu,
                                   np.ones(len(live), dtype=np.int32),
                                   b.kv_start.numpy()[live], lens[live], b.H, b.D)
        lens[live] = new_len
    np.testing.assert_allclose(multi, single, rtol=0, atol=1e-13)
    assert lens.tolist() == [13, 26]


def test_equal_keys_give_mean_of_visible_values():
    kv_len, k = [6, 3], [3, 2]
    b = make_batch(kv_len, k, H=2, D=8, seed=10, capacity=16)
    one_k = from_bits(np.full(b.k_cache.numel(), 0x3C00, dtype=np.uint16), torch.float16)  # 1.0
    k_new = torch.ones_like(b.k_new)
    got = oracle.verify_attention(bits(b.q), bits(k_new), bits(b.v_new), bits(one_k),
                                  bits(b.v_cache), b.row_stride, b.head_stride,
                                  b.cu_seqlens.numpy(), b.kv_start.numpy(), b.kv_len.numpy(),
                                  b.H, b.D, b.scale, b.dtype)
    V = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D).double().numpy()
    cu = b.cu_seqlens.numpy()
    for i in range(b.B):
        s, L = int(b.kv_start[i]), kv_len[i]
        for j in range(k[i]):
            vis = np.concatenate([V[s:s + L], b.v_new[cu[i]:cu[i] + j + 1].double().numpy()])
            np.testing.assert_allclose(got[cu[i] + j], vis.mean(axis=0), rtol=0, atol=1e-13)


def test_dominant_key_selects_its_value_row():
    b = make_batch([10], [2], H=1, D=8, seed=11, capacity=16, scale=1.0)
    K = arena_view(b.k_cache, b.layout, b.rows, b.H, b.D)
    K[:10] = 0
    K[4, 0] = 64.0
    b.k_new[:] = 0
    b.q[:] = 1.0                       # score of key 4 = 512, all others 0
    got = run_oracle(b)
    V = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D).double().numpy()
    for r in range(2):
        np.testing.assert_allclose(got[r, 0], V[4, 0], rtol=0, atol=1e-12)


def test_outputs_are_convex_combinations_of_visible_values():
    b = make_config(1)
    got = run_oracle(b)
    V = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D).double().numpy()
    cu = b.cu_seqlens.numpy()
    for i in range(b.B):
        s, L = int(b.kv_start[i]), int(b.kv_len[i])
        for j in range(cu[i + 1] - cu[i]):
            vis = np.concatenate([V[s:s + L], b.v_new[cu[i]:cu[i] + j + 1].double().numpy()])
            o = got[cu[i] + j]
            assert (o <= vis.max(axis=0) + 1e-12).all() and (o >= vis.min(axis=0) - 1e-12).all()


def test_later_new_tokens_and_other_samples_do_not_matter():
    """Causality inside a sample, isolation between samples, and sentinel rows."""
    kv_len, k = [7, 11, 5], [3, 4, 2]
    b = make_batch(kv_len, k, H=2, D=16, seed=12, capacity=20)
    base = run_oracle(b)
    assert np.isfinite(base).all()     # rows beyond kv_len hold NaN: none was read
    cu = b.cu_seqlens.numpy()
    # change sample 1's cache and new rows: samples 0 and 2 unchanged bit for bit
    b2 = make_batch(kv_len, k, H=2, D=16, seed=12, capacity=20)
    K2 = arena_view(b2.k_cache, b2.layout, b2.rows, b2.H, b2.D)
    K2[20:31] = K2[20:31] * 0.5 + 1
    b2.v_new[cu[1]:cu[2]] += 1
    out2 = run_oracle(b2)
    assert np.array_equal(out2[cu[0]:cu[1]], base[cu[0]:cu[1]])
    assert np.array_equal(out2[cu[2]:cu[3]], base[cu[2]:cu[3]])
    assert not np.array_equal(out2[cu[1]:cu[2]], base[cu[1]:cu[2]])
    # change the LAST new row of sample 0: its earlier rows are unchanged
    b3 = make_batch(kv_len, k, H=2, D=16, seed=12, capacity=20)
    b3.k_new[cu[1] - 1] += 2
    b3.v_new[cu[1] - 1] -= 1
    out3 = run_oracle(b3)
    assert np.array_equal(out3[:cu[1] - 1], base[:cu[1] - 1])
    assert not np.array_equal(out3[cu[1] - 1], base[cu[1] - 1])


def test_relocation_and_batch_permutation_leave_outputs_identical():
    kv_len, k = [7, 11, 5], [3, 4, 2]
    H, D = 2, 16
    a = make_batch(kv_len, k, H=H, D=D, seed=13, capacity=20)
    base = run_oracle(a)
    cu = a.cu_seqlens.numpy()
    perm = [2, 0, 1]
    new_start = {0: 50, 1: 3, 2: 25}
    rows = 80
    Ka = arena_view(a.k_cache, a.layout, a.rows, H, D)
    Va = arena_view(a.v_cache, a.layout, a.rows, H, D)
    for layout in (TOKEN_MAJOR, HEAD_MAJOR):
        p = make_batch([kv_len[i] for i in perm], [k[i] for i in perm], H=H, D=D, seed=99,
                       kv_start=[new_start[i] for i in perm], rows=rows, layout=layout)
        Kp = arena_view(p.k_cache, layout, rows, H, D)
        Vp = arena_view(p.v_cache, layout, rows, H, D)
        pcu = p.cu_seqlens.numpy()
        for slot, i in enumerate(perm):
            s_old = int(a.kv_start[i])
            Kp[new_start[i]:new_start[i] + kv_len[i]] = Ka[s_old:s_old + kv_len[i]]
            Vp[new_start[i]:new_start[i] + kv_len[i]] = Va[s_old:s_old + kv_len[i]]
            for name in ("q", "k_new", "v_new"):
                getattr(p, name)[pcu[slot]:pcu[slot + 1]] = getattr(a, name)[cu[i]:cu[i + 1]]
        out = run_oracle(p)
        for slot, i in enumerate(perm):
            assert np.array_equal(out[pcu[slot]:pcu[slot + 1]], base[cu[i]:cu[i + 1]])


def test_zero_query_sample_contributes_nothing():
    b = make_batch([6, 9, 4], [2, 0, 3], H=1, D=8, seed=14, capacity=16)
    got = run_oracle(b)
    assert got.shape[0] == 5
    np.testing.assert_allclose(got, padded_brute_force(b), rtol=0, atol=1e-12)


def test_scale_is_applied_as_the_float_it_was_passed_as():
    b = make_batch([12], [2], H=1, D=64, seed=15, scale=0.1)
    got = run_oracle(b)
    want = padded_brute_force(b)       # uses float64(float32(0.1))
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)
