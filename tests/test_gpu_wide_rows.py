"""GPU parity with more than 16 rows per sample (up to 64): the attention calls then run the staged
kernel (head dims 80 and 128: tiles staged through LDS by requesting waves, four computing waves
of 16 rows each per stream) or the one-wave wide kernel (head dim 64, very large batches), which
holds 32 rows per (sample, head) pair and makes two pairs of a sample with more.  Causal and tree
masks, write-through, accept and append, against the oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_07542_amd as ems
from workloads import HEAD_MAJOR, TOKEN_MAJOR, bits, grow_trees, make_batch
from helpers import hip_accept, oracle_accept, oracle_attention, to_device
from test_gpu_parity import check_attention, run_accept_and_append
from test_gpu_tree import check_accept_and_append, check_tree_attention

pytestmark = pytest.mark.gpu

KV = [0, 1, 31, 32, 33, 64, 100, 257, 5, 700, 12]
K = [64, 17, 33, 48, 1, 32, 63, 16, 49, 20, 0]


@pytest.mark.parametrize("dtype,D,layout", [(torch.float16, 128, TOKEN_MAJOR), (torch.bfloat16, 64, HEAD_MAJOR),
                                            (torch.bfloat16, 80, TOKEN_MAJOR), (torch.float16, 64, TOKEN_MAJOR)])
def test_causal_rows_beyond_sixteen(dtype, D, layout):
    b = make_batch(KV, K, H=3, D=D, dtype=dtype, seed=80, capacity=800, layout=layout, vocab_for_ids=9,
                   match_p=0.9)
    assert b.max_k == 64
    check_attention(b, out_dtype=torch.float32, label="wide f32 out")
    check_attention(b, label="wide 16-bit out")
    run_accept_and_append(b)


def test_wide_pairs_merged_from_partials():
    # few long pairs: every pair's tiles are spread over many waves
    b = make_batch([5000, 3000], [40, 64], H=1, D=128, dtype=torch.bfloat16, seed=81)
    check_attention(b, out_dtype=torch.float32, label="wide, merged")


def test_sixteen_rows_or_fewer_through_the_wide_kernel():
    """max_k only selects the kernel: with k_i <= 16 everywhere, max_k = 64 (the wide kernel, one
    block of rows in use) must meet the oracle as the max_k = 16 launch does."""
    b_cpu = make_batch([900, 1200, 31, 0], [7, 3, 16, 11], H=4, D=128, dtype=torch.bfloat16, seed=82)
    b = to_device(b_cpu)
    want = oracle_attention(b_cpu)
    for max_k in (16, 64):
        out = torch.full((b.T, b.H, b.D), float("nan"), dtype=torch.float32, device="cuda")
        ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len), dtype=torch.uint8,
                         device="cuda")
        ems.ems_verify_attention(b.q, b.k_new, b.v_new,
                                 ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows),
                                 b.cu_seqlens, b.kv_start, b.kv_len, out, max_k=max_k, max_kv_len=b.max_kv_len,
                                 scale=b.scale, workspace=ws)
        torch.cuda.synchronize()
        assert np.abs(out.double().cpu().numpy() - want).max() <= 2e-3, max_k


@pytest.mark.parametrize("shape", ["random", "wide", "star", "chain"])
@pytest.mark.parametrize("dtype,D,layout", [(torch.float16, 128, TOKEN_MAJOR), (torch.bfloat16, 80, HEAD_MAJOR)])
def test_trees_of_up_to_64_rows(shape, dtype, D, layout):
    b = make_batch(KV, K, H=3, D=D, dtype=dtype, seed=83, capacity=800, layout=layout, vocab_for_ids=9)
    t = grow_trees(b, 84, match_p=0.85, shape=shape, duplicate_p=0.2)
    check_tree_attention(t, out_dtype=torch.float32)
    check_tree_attention(t)
    check_accept_and_append(t, use_logits=False, n_layers=2)


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_write_through_with_wide_rows(layout):
    b_cpu = make_batch(KV, K, H=3, D=128, dtype=torch.float16, seed=85, capacity=800, layout=layout)
    b = to_device(b_cpu)
    kc, vc = b.k_cache.clone(), b.v_cache.clone()
    out = torch.full((b.T, b.H, b.D), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len), dtype=torch.uint8, device="cuda")
    ems.ems_verify_attention_write_through(b.q, b.k_new, b.v_new,
                                           ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows),
                                           b.cu_seqlens, b.kv_start, b.kv_len, out, max_k=b.max_k,
                                           max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
    torch.cuda.synchronize()
    assert np.abs(out.double().cpu().numpy() - oracle_attention(b_cpu)).max() <= 2e-3
    okc, ovc = bits(b_cpu.k_cache).copy(), bits(b_cpu.v_cache).copy()
    oracle.kv_write_through(okc, ovc, b_cpu.row_stride, b_cpu.head_stride, bits(b_cpu.k_new), bits(b_cpu.v_new),
                            b_cpu.cu_seqlens.numpy(), b_cpu.kv_start.numpy(), b_cpu.kv_len.numpy(), b_cpu.H, b_cpu.D)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(vc), ovc)


def test_limits_of_the_other_variants():
    b = to_device(make_batch([10, 20], [17, 3], H=2, D=64, seed=86, capacity=64))
    out = torch.empty_like(b.q)
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len), dtype=torch.uint8, device="cuda")
    cache = ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows)
    ems.ems_set_attention_variant(ems.EMS_ATTN_VALU)
    try:
        with pytest.raises(ems.EmsError) as e:
            ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                     max_k=17, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
        assert e.value.status == ems.EMS_ERR_UNSUPPORTED
    finally:
        ems.ems_set_attention_variant(ems.EMS_ATTN_MFMA)
    with pytest.raises(ems.EmsError) as e:
        ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                 max_k=65, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
    assert e.value.status == ems.EMS_ERR_UNSUPPORTED


def test_staged_attention_is_deterministic():
    """The requesting and the computing waves of the staged kernel meet through counters, in an
    order that differs from run to run; what each wave adds up, and in which order partials are
    merged, does not: the output bits are the same every time."""
    from helpers import hip_attention
    b = to_device(make_batch([900, 1200, 31, 2000], [40, 64, 17, 33], H=8, D=128, dtype=torch.bfloat16, seed=48))
    first = hip_attention(b, out_dtype=torch.float32)
    for _ in range(4):
        assert torch.equal(hip_attention(b, out_dtype=torch.float32).view(torch.int32), first.view(torch.int32))


@pytest.mark.parametrize("B,dtype,D,layout", [(8192, torch.bfloat16, 128, TOKEN_MAJOR), (8192, torch.float16, 80, HEAD_MAJOR),
                                               (7000, torch.float16, 128, HEAD_MAJOR), (5000, torch.bfloat16, 128, TOKEN_MAJOR)])
def test_very_large_batches_through_the_wide_kernel(B, dtype, D, layout):
    """Thousands of samples, a few of them with more than 16 rows.  The staged kernel runs while LDS
    has room for its tile rings beside the tile prefix sums (B = 5000 and 7000: 128 KiB + 4 B per
    sample); beyond that (B = 8192) the library falls back to the one-wave kernel with two pairs of
    32 rows per head, which these cases are here to cover: causal, tree and write-through."""
    rng = np.random.default_rng(159 + B)
    kv = rng.integers(0, 41, B).tolist()
    k = rng.integers(0, 4, B).tolist()
    for i in rng.choice(B, 40, replace=False):
        k[i] = int(rng.integers(17, 65))
    k[0], k[-1] = 64, 33
    b = make_batch(kv, k, H=1, D=D, dtype=dtype, seed=160, capacity=112, layout=layout, vocab_for_ids=9,
                   match_p=0.8)
    assert b.max_k == 64
    check_attention(b, out_dtype=torch.float32, label="wide, B=%d" % B)
    run_accept_and_append(b)
    t = grow_trees(b, 161, match_p=0.8, shape="random")
    check_tree_attention(t, out_dtype=torch.float32)
    dev = to_device(b)
    kc, vc = dev.k_cache.clone(), dev.v_cache.clone()
    out = torch.full((b.T, b.H, b.D), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len), dtype=torch.uint8, device="cuda")
    ems.ems_verify_attention_write_through(dev.q, dev.k_new, dev.v_new,
                                           ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows),
                                           dev.cu_seqlens, dev.kv_start, dev.kv_len, out, max_k=b.max_k,
                                           max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
    torch.cuda.synchronize()
    assert np.abs(out.double().cpu().numpy() - oracle_attention(b)).max() <= 2e-3
    okc, ovc = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    oracle.kv_write_through(okc, ovc, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new),
                            b.cu_seqlens.numpy(), b.kv_start.numpy(), b.kv_len.numpy(), b.H, b.D)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(vc), ovc)
