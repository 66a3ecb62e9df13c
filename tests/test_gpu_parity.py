"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the
same seeded inputs.  Bit-exact for ids, counts, offsets and cache bytes; attention
output within max-abs 2e-3 (see helpers.attention_tolerance)."""
import numpy as np
import pytest
import torch

import oracle
from workloads import (HEAD_MAJOR, TOKEN_MAJOR, arena_view, bits, make_batch, make_config)
from helpers import (attention_tolerance, hip_accept, hip_attention, oracle_accept,
                     oracle_attention, to_device)

pytestmark = pytest.mark.gpu


def check_attention(b_cpu, out_dtype=None, label="", plain_bar=False, want=None):
    """plain_bar: assert the stated max-abs 2e-3 as it is, also for a bf16 output (the widened
    bound of helpers.attention_tolerance is for bf16 outputs of short caches only, where the
    rounding of the result itself exceeds the bar)."""
    print("attention case:", label or b_cpu.name, "B", b_cpu.B, "H", b_cpu.H, "D", b_cpu.D,
          b_cpu.dtype, b_cpu.layout, "out", out_dtype, flush=True)
    b = to_device(b_cpu)
    got = hip_attention(b, out_dtype=out_dtype).double().cpu().numpy()
    want = oracle_attention(b_cpu) if want is None else want
    assert np.isfinite(got).all(), "non-finite output (a sentinel row was read, or a row was not written)"
    err = np.abs(got - want)
    tol = np.full(want.shape, 2e-3) if plain_bar else attention_tolerance(b_cpu, want, out_dtype or b_cpu.dtype)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert (err <= tol).all(), "max err %.3e at %s (tol %.3e)" % (err[worst], worst, tol[worst])
    return float(err.max())


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_tiny_config_attention(layout):
    check_attention(make_config(1, layout=layout))
    check_attention(make_config(1, layout=layout), out_dtype=torch.float32)


RAGGED_KV = [0, 1, 31, 32, 33, 64, 100, 257, 5]
RAGGED_K = [1, 16, 3, 7, 2, 11, 1, 5, 16]


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
@pytest.mark.parametrize("D", [128, 64])
def test_ragged_lengths_span_tiles_and_tails(dtype, layout, D):
    b = make_batch(RAGGED_KV, RAGGED_K, H=4, D=D, dtype=dtype, seed=40, capacity=300, layout=layout)
    check_attention(b, out_dtype=torch.float32, label="ragged f32 out")
    check_attention(b, label="ragged 16-bit out")


def test_one_pair_shared_by_many_waves():
    """B=1, H=1 with a long cache: the pair's tiles are cut over many waves, so the
    output comes entirely from the partial-merge kernel."""
    b = make_batch([6000], [9], H=1, D=128, dtype=torch.float16, seed=41)
    check_attention(b, out_dtype=torch.float32)
    b = make_batch([3000, 10, 2500], [16, 1, 4], H=2, D=64, dtype=torch.bfloat16, seed=42,
                   layout=HEAD_MAJOR)
    check_attention(b, out_dtype=torch.float32)


def test_one_very_long_cache_merged_from_a_thousand_partials():
    """One (sample, head) pair of 300 000 cached rows: every wave of the launch holds a slice of
    it, so its rows are merged from ~1000 partials; byte offsets inside the sample reach 150 MB."""
    b = make_batch([300000], [5], H=1, D=128, dtype=torch.bfloat16, seed=77)
    check_attention(b, out_dtype=torch.float32, label="L=300000")
    # the same with a looser length bound, from which the library merges the partials of each
    # workgroup's four waves in LDS and writes 256 partials instead of 1024
    want = oracle_attention(b)
    got = hip_attention(to_device(b), out_dtype=torch.float32, max_kv_len=400000).double().cpu().numpy()
    assert np.abs(got - want).max() <= 2e-3


def test_degenerate_batches():
    # empty caches everywhere; finished samples (k_i = 0) in between; maximum rows per sample
    check_attention(make_batch([0, 0, 0], [4, 1, 16], H=2, D=128, seed=43, capacity=32))
    check_attention(make_batch([40, 9, 70, 3], [2, 0, 0, 16], H=3, D=64, seed=44, capacity=100))
    # T = 0 is a legal no-op
    import paper_2405_07542_amd as ems
    b = to_device(make_batch([5, 6], [0, 0], H=2, D=64, seed=45, capacity=16))
    out = torch.empty((0, 2, 64), dtype=torch.float16, device="cuda")
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    ems.ems_verify_attention(b.q, b.k_new, b.v_new,
                             ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows),
                             b.cu_seqlens, b.kv_start, b.kv_len, out, max_k=0, max_kv_len=6,
                             scale=b.scale, workspace=ws)
    torch.cuda.synchronize()


def test_regions_in_any_order_and_loose_upper_bounds():
    kv_len, k = [70, 33, 120], [5, 9, 2]
    b_cpu = make_batch(kv_len, k, H=4, D=128, seed=46, kv_start=[400, 0, 150], rows=600)
    b = to_device(b_cpu)
    want = oracle_attention(b_cpu)
    got = hip_attention(b, out_dtype=torch.float32, max_kv_len=4096).double().cpu().numpy()
    assert np.abs(got - want).max() <= 2e-3
    import paper_2405_07542_amd as ems
    ems.ems_validate_inputs(b.cu_seqlens, b.kv_start, b.kv_len, T=b.T, max_k=16, max_kv_len=4096,
                            rows=b.rows)
    bad = b.kv_start.clone()
    bad[1] = 390                         # sample 1 now overlaps sample 0's region
    with pytest.raises(ems.EmsError) as e:
        ems.ems_validate_inputs(b.cu_seqlens, bad, b.kv_len, T=b.T, max_k=16, max_kv_len=4096,
                                rows=b.rows)
    assert e.value.status == ems.EMS_ERR_INVALID_ARG and "overlap" in str(e.value)


def test_attention_is_deterministic():
    b = to_device(make_batch([900, 1200, 31], [7, 3, 16], H=8, D=128, dtype=torch.bfloat16, seed=47))
    a1 = hip_attention(b)
    a2 = hip_attention(b)
    assert torch.equal(a1.view(torch.int16), a2.view(torch.int16))


@pytest.mark.parametrize("n,layout", [(2, TOKEN_MAJOR), (2, HEAD_MAJOR), (3, TOKEN_MAJOR),
                                      (4, TOKEN_MAJOR), (4, HEAD_MAJOR)])
def test_baseline_configs_full_size(n, layout):
    """Configs 2-4 at full size, every output element against the oracle at the stated bar
    itself -- max-abs 2e-3, with the fp32 output and with the 16-bit output (config 4's is
    bf16: its caches hold >= 1024 rows, so |out| stays far below the 0.5 from which bf16's own
    rounding would exceed the bar) -- plus acceptance on the full [T, 50272] logits and the
    append into the arena."""
    b_cpu = make_config(n, layout=layout)
    want = oracle_attention(b_cpu)
    err32 = check_attention(b_cpu, out_dtype=torch.float32, plain_bar=True, want=want)
    err16 = check_attention(b_cpu, plain_bar=True, want=want)
    print("config", n, layout, "max abs err: fp32 out %.3e, 16-bit out %.3e (bar 2e-3)" % (err32, err16), flush=True)
    run_accept_and_append(b_cpu)


def run_accept_and_append(b_cpu, n_layers=1):
    import paper_2405_07542_amd as ems
    b = to_device(b_cpu)
    tgt, acc, acc_cu, toks = hip_accept(b, use_logits=b.logits is not None)
    x, o_acc, o_cu, o_toks = oracle_accept(b_cpu)
    assert np.array_equal(tgt.cpu().numpy(), x)
    assert np.array_equal(x, b_cpu.target_ids.numpy()) or b_cpu.logits is None
    assert np.array_equal(acc.cpu().numpy(), o_acc)
    assert np.array_equal(acc_cu.cpu().numpy(), o_cu)
    assert np.array_equal(toks.cpu().numpy()[:o_cu[-1]], o_toks)
    k = np.diff(b_cpu.cu_seqlens.numpy())
    assert ((o_acc >= np.minimum(k, 1)) & (o_acc <= k)).all()
    # append on the GPU and in the oracle, compare whole arenas bit for bit
    kc, vc = b.k_cache.clone(), b.v_cache.clone()
    new_len = torch.empty_like(b.kv_len)
    ems.ems_kv_append([b.k_new], [b.v_new],
                      [ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows)],
                      b.cu_seqlens, acc, b.kv_start, b.kv_len, new_len)
    torch.cuda.synchronize()
    okc, ovc = bits(b_cpu.k_cache).copy(), bits(b_cpu.v_cache).copy()
    o_len = oracle.kv_append(okc, ovc, b_cpu.row_stride, b_cpu.head_stride, bits(b_cpu.k_new),
                             bits(b_cpu.v_new), b_cpu.cu_seqlens.numpy(), o_acc,
                             b_cpu.kv_start.numpy(), b_cpu.kv_len.numpy(), b_cpu.H, b_cpu.D)
    assert np.array_equal(new_len.cpu().numpy(), o_len)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(vc), ovc)
    return b, kc, vc, new_len


def test_tiny_config_accept_and_append():
    run_accept_and_append(make_config(1))
    run_accept_and_append(make_config(1, layout=HEAD_MAJOR))


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("V", [50272, 32000, 4099, 7, 128256, 262144])
def test_argmax_on_unplanted_logits_with_natural_ties(dtype, V):
    """Plain N(0,1) rows: at 16-bit precision the maximum is often attained twice."""
    g = torch.Generator().manual_seed(50 + V)
    T = 37
    b_cpu = make_batch([3] * 5, [9, 1, 12, 7, 8], H=1, D=64, dtype=dtype, seed=51, V=V)
    b_cpu.logits = torch.randn(T, V, generator=g).to(dtype)
    b_cpu.logits[3] = -b_cpu.logits[3].abs() - 1          # an all-negative row
    b_cpu.logits[4, :] = 0.0                              # +-0 only: index 0 wins
    b_cpu.logits[4, 1::2] = -0.0
    b_cpu.logits[5, V - 1] = 30.0                         # maximum in the last column
    x = oracle.argmax(bits(b_cpu.logits), dtype)
    b_cpu.input_ids[1:] = torch.from_numpy(x[:-1].astype(np.int32))   # long accepted runs
    b = to_device(b_cpu)
    tgt, acc, acc_cu, toks = hip_accept(b)
    _, o_acc, o_cu, o_toks = oracle_accept(b_cpu)
    assert np.array_equal(tgt.cpu().numpy(), x)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and o_acc.max() > 1
    assert np.array_equal(acc_cu.cpu().numpy(), o_cu)
    assert np.array_equal(toks.cpu().numpy()[:o_cu[-1]], o_toks)


def test_accept_at_the_largest_row_count():
    """T = 65535 packed rows (the most a call accepts) in 8192 samples, logits over a small
    vocabulary, bf16."""
    rng = np.random.default_rng(95)
    B = 8192
    k = np.full(B, 8, dtype=np.int64)
    k[-1] = 65535 - 8 * (B - 1)                     # 7 rows: T = 65535 exactly
    b_cpu = make_batch([1] * B, k.tolist(), H=1, D=64, dtype=torch.bfloat16, seed=96, V=24, match_p=0.8)
    assert b_cpu.T == 65535
    b = to_device(b_cpu)
    tgt, acc, acc_cu, toks = hip_accept(b)
    x, o_acc, o_cu, o_toks = oracle_accept(b_cpu)
    assert np.array_equal(tgt.cpu().numpy(), x)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(acc_cu.cpu().numpy(), o_cu)
    assert np.array_equal(toks.cpu().numpy()[:o_cu[-1]], o_toks)


def test_accept_without_logits_many_samples_and_empty_ones():
    rng = np.random.default_rng(52)
    B = 3000                                              # more samples than threads in the scan block
    k = rng.integers(0, 17, B).tolist()
    k[0] = 0
    k[-1] = 0
    b_cpu = make_batch([1] * B, k, H=1, D=64, seed=53, match_p=0.8, vocab_for_ids=11)
    b = to_device(b_cpu)
    tgt, acc, acc_cu, toks = hip_accept(b, use_logits=False)
    _, o_acc, o_cu, o_toks = oracle_accept(b_cpu, use_logits=False)
    assert np.array_equal(acc.cpu().numpy(), o_acc)
    assert np.array_equal(acc_cu.cpu().numpy(), o_cu)
    assert np.array_equal(toks.cpu().numpy()[:o_cu[-1]], o_toks)
    assert (toks.cpu().numpy()[o_cu[-1]:] == -7).all()   # nothing written past the total
    # long draft runs (k_i > 64) exercise the chunked ballot
    b2 = make_batch([1, 1, 1], [200, 65, 64], H=1, D=64, seed=54, match_p=0.995, vocab_for_ids=9)
    _, acc2, cu2, _ = hip_accept(to_device(b2), use_logits=False)
    _, o2, ocu2, _ = oracle_accept(b2, use_logits=False)
    assert np.array_equal(acc2.cpu().numpy(), o2) and np.array_equal(cu2.cpu().numpy(), ocu2)
    assert o2.max() > 64


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_append_many_layers_in_place_lengths(layout):
    """34 layers (two launches), kv_len_out aliasing kv_len, sentinel rows untouched."""
    import paper_2405_07542_amd as ems
    n_layers = 34
    kv_len, k = [7, 0, 12, 3, 20], [4, 3, 1, 5, 0]
    accepted = [2, 3, 1, 0, 0]
    layers = [make_batch(kv_len, k, H=3, D=64, dtype=torch.bfloat16, seed=60 + l, capacity=32,
                         layout=layout) for l in range(n_layers)]
    dev = [to_device(b) for b in layers]
    acc = torch.tensor(accepted, dtype=torch.int32, device="cuda")
    lens = dev[0].kv_len.clone()
    ems.ems_kv_append([b.k_new for b in dev], [b.v_new for b in dev],
                      [ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows) for b in dev],
                      dev[0].cu_seqlens, acc, dev[0].kv_start, lens, lens)
    torch.cuda.synchronize()
    assert lens.cpu().tolist() == [9, 3, 13, 3, 20]
    for b_cpu, b in zip(layers, dev):
        okc, ovc = bits(b_cpu.k_cache).copy(), bits(b_cpu.v_cache).copy()
        oracle.kv_append(okc, ovc, b_cpu.row_stride, b_cpu.head_stride, bits(b_cpu.k_new),
                         bits(b_cpu.v_new), b_cpu.cu_seqlens.numpy(), accepted,
                         b_cpu.kv_start.numpy(), b_cpu.kv_len.numpy(), b_cpu.H, b_cpu.D)
        assert np.array_equal(bits(b.k_cache), okc) and np.array_equal(bits(b.v_cache), ovc)


def test_verify_loop_of_several_steps():
    """attention -> accept -> append, five times; the GPU's own caches and lengths
    feed its next step and must track the oracle's exactly."""
    import paper_2405_07542_amd as ems
    rng = np.random.default_rng(70)
    B, H, D, cap = 6, 4, 128, 160
    lens0 = rng.integers(0, 90, B).tolist()
    first = make_batch(lens0, [1] * B, H=H, D=D, seed=71, capacity=cap)
    g_kc, g_vc = first.k_cache.cuda(), first.v_cache.cuda()
    o_kc, o_vc = bits(first.k_cache).copy(), bits(first.v_cache).copy()
    g_len = first.kv_len.cuda()
    o_len = first.kv_len.numpy().copy()
    for step in range(5):
        k = rng.integers(1, 9, B).tolist()
        s_cpu = make_batch(o_len.tolist(), k, H=H, D=D, seed=100 + step, capacity=cap,
                           vocab_for_ids=50, match_p=0.7)
        s = to_device(s_cpu)
        got = hip_attention(s, out_dtype=torch.float32, k_cache=g_kc, v_cache=g_vc, kv_len=g_len,
                            max_kv_len=cap).double().cpu().numpy()
        want = oracle.verify_attention(bits(s_cpu.q), bits(s_cpu.k_new), bits(s_cpu.v_new), o_kc, o_vc,
                                       s_cpu.row_stride, s_cpu.head_stride, s_cpu.cu_seqlens.numpy(),
                                       s_cpu.kv_start.numpy(), o_len, H, D, s_cpu.scale, s_cpu.dtype)
        assert np.abs(got - want).max() <= 2e-3, "step %d" % step
        _, acc, _, _ = hip_accept(s, use_logits=False)
        _, o_acc, _, _ = oracle_accept(s_cpu, use_logits=False)
        assert np.array_equal(acc.cpu().numpy(), o_acc)
        ems.ems_kv_append([s.k_new], [s.v_new],
                          [ems.kv_cache(g_kc, g_vc, s.row_stride, s.head_stride, s.rows)],
                          s.cu_seqlens, acc, s.kv_start, g_len, g_len)
        o_len = oracle.kv_append(o_kc, o_vc, s_cpu.row_stride, s_cpu.head_stride, bits(s_cpu.k_new),
                                 bits(s_cpu.v_new), s_cpu.cu_seqlens.numpy(), o_acc,
                                 s_cpu.kv_start.numpy(), o_len, H, D)
        torch.cuda.synchronize()
        assert np.array_equal(g_len.cpu().numpy(), o_len)
        assert np.array_equal(bits(g_kc), o_kc) and np.array_equal(bits(g_vc), o_vc)


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
@pytest.mark.parametrize("dtype,D", [(torch.float16, 128), (torch.bfloat16, 64), (torch.bfloat16, 80)])
def test_write_through_variant(layout, dtype, D):
    """Paper order: the attention call also stores every new row's K/V at the sample's own
    location; then only the lengths advance.  Output as for the plain call; cache bit-equal to
    the oracle's write-through; untouched rows keep their sentinel."""
    import paper_2405_07542_amd as ems
    b_cpu = make_batch(RAGGED_KV, RAGGED_K, H=4, D=D, dtype=dtype, seed=48, capacity=300, layout=layout)
    b = to_device(b_cpu)
    kc, vc = b.k_cache.clone(), b.v_cache.clone()
    out = torch.full((b.T, b.H, b.D), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len), dtype=torch.uint8, device="cuda")
    ems.ems_verify_attention_write_through(b.q, b.k_new, b.v_new,
                                           ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows),
                                           b.cu_seqlens, b.kv_start, b.kv_len, out, max_k=b.max_k,
                                           max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
    _, acc, _, _ = hip_accept(b, use_logits=False)
    lens = b.kv_len.clone()
    ems.ems_kv_advance(lens, acc, lens)
    torch.cuda.synchronize()
    want = oracle_attention(b_cpu)
    assert np.abs(out.double().cpu().numpy() - want).max() <= 2e-3
    okc, ovc = bits(b_cpu.k_cache).copy(), bits(b_cpu.v_cache).copy()
    oracle.kv_write_through(okc, ovc, b_cpu.row_stride, b_cpu.head_stride, bits(b_cpu.k_new),
                            bits(b_cpu.v_new), b_cpu.cu_seqlens.numpy(), b_cpu.kv_start.numpy(),
                            b_cpu.kv_len.numpy(), b_cpu.H, b_cpu.D)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(vc), ovc)
    _, o_acc, _, _ = oracle_accept(b_cpu, use_logits=False)
    assert np.array_equal(lens.cpu().numpy(), b_cpu.kv_len.numpy() + o_acc)


def test_opt_13b_head_count():
    """OPT-13b geometry (40 heads of 128): nothing in the path depends on H being a power of two."""
    b = make_batch([300, 1, 77], [4, 9, 1], H=40, D=128, dtype=torch.float16, seed=49)
    check_attention(b, out_dtype=torch.float32, label="H=40")
    run_accept_and_append(b)


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_head_dim_80(dtype, layout):
    """OPT-2.7b geometry (32 heads of 80): a head dim that is not a power of two.  Ragged
    lengths over several tiles with tails, pairs merged from partials, the last row of the
    last head at the very end of the arena, then accept and append on the same batch."""
    b = make_batch(RAGGED_KV, RAGGED_K, H=4, D=80, dtype=dtype, seed=56, capacity=300, layout=layout)
    check_attention(b, out_dtype=torch.float32, label="D=80 ragged f32 out")
    check_attention(b, label="D=80 ragged 16-bit out")
    big = make_batch([1500, 40, 2047], [7, 16, 1], H=32, D=80, dtype=dtype, seed=57, capacity=2048,
                     kv_start=[0, 2048, 4096 + 0], rows=4096 + 2048, layout=layout)
    check_attention(big, label="D=80 OPT-2.7b shape, arena filled to its last row")
    run_accept_and_append(make_batch([300, 1, 77], [4, 9, 1], H=32, D=80, dtype=dtype, seed=58, layout=layout))


def test_argmax_rows_of_minus_infinity():
    """A row (or a slice of it) that holds only -inf has every element equal: index 0 wins."""
    V = 50272
    b_cpu = make_batch([2, 2], [3, 2], H=1, D=64, dtype=torch.float16, seed=55, V=V)
    b_cpu.logits[1, :] = float("-inf")
    b_cpu.logits[2, :] = float("-inf")
    b_cpu.logits[2, 40000] = -5.0                       # one finite value in a late slice
    b = to_device(b_cpu)
    tgt, _, _, _ = hip_accept(b)
    want = oracle.argmax(bits(b_cpu.logits), torch.float16)
    assert want[1] == 0 and want[2] == 40000
    assert np.array_equal(tgt.cpu().numpy(), want)


def test_maximum_batch_size():
    """B = 8192, the most samples a call accepts: 32 KiB of tile prefix sums in LDS, one merge
    block per (sample, head); many samples bring no rows at all."""
    rng = np.random.default_rng(59)
    B = 8192
    kv = rng.integers(0, 41, B).tolist()
    k = rng.integers(0, 4, B).tolist()
    k[0], k[-1] = 3, 2
    b = make_batch(kv, k, H=1, D=64, dtype=torch.float16, seed=60, capacity=48)
    check_attention(b, out_dtype=torch.float32, label="B=8192")
    run_accept_and_append(b)


@pytest.mark.parametrize("B,k_max", [(2, 5), (64, 11), (3000, 16), (8192, 3), (5, 200)])
def test_pack_tokens(B, k_max):
    """Alg. 1 on the device against the oracle's: running sum of the counts, packed ids, nothing
    written past the total; the result feeds ems_validate_inputs' checks of cu_seqlens."""
    import paper_2405_07542_amd as ems
    rng = np.random.default_rng(91 + B)
    lens = rng.integers(0, k_max + 1, B).astype(np.int32)
    padded = rng.integers(0, 50272, (B, k_max)).astype(np.int32)
    cat, nums, total = oracle.concatenate_tokens(padded, lens)
    cu = torch.full((B + 1,), -7, dtype=torch.int32, device="cuda")
    packed = torch.full((B * k_max,), -7, dtype=torch.int32, device="cuda")
    ems.ems_pack_tokens(torch.from_numpy(padded).cuda(), torch.from_numpy(lens).cuda(), cu, packed)
    torch.cuda.synchronize()
    assert np.array_equal(cu.cpu().numpy(), np.concatenate([[0], np.cumsum(nums)]))
    assert np.array_equal(packed.cpu().numpy()[:total], cat)
    assert (packed.cpu().numpy()[total:] == -7).all()


def test_paper_order_with_every_row_as_its_own_work_item():
    """The paper's own formulation (Sec. 3.2 with the launch shape of Appendix D): the K/V of all
    new tokens is written at the samples' locations first, then every packed token attends, on
    its own, to its sample's cache up to and including itself.  Presenting every packed row as
    a one-row sample whose cache ends just before it must reproduce the oracle's outputs."""
    import paper_2405_07542_amd as ems
    b_cpu = make_batch(RAGGED_KV, RAGGED_K, H=4, D=128, dtype=torch.float16, seed=78, capacity=300)
    b = to_device(b_cpu)
    kc, vc = b.k_cache.clone(), b.v_cache.clone()
    cache = ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows)
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.T, b.T, b.H, b.D, b.max_kv_len + b.max_k),
                     dtype=torch.uint8, device="cuda")
    out = torch.empty((b.T, b.H, b.D), dtype=torch.float32, device="cuda")
    ems.ems_verify_attention_write_through(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len,
                                           out, max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale,
                                           workspace=ws)
    k = np.diff(b_cpu.cu_seqlens.numpy())
    sample = np.repeat(np.arange(b.B), k)
    pos = np.arange(b.T) - b_cpu.cu_seqlens.numpy()[:-1][sample]
    cu = torch.arange(b.T + 1, dtype=torch.int32, device="cuda")
    ks = torch.from_numpy(b_cpu.kv_start.numpy()[sample].astype(np.int32)).cuda()
    kl = torch.from_numpy((b_cpu.kv_len.numpy()[sample] + pos).astype(np.int32)).cuda()
    out.fill_(float("nan"))
    ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, cu, ks, kl, out, max_k=1,
                             max_kv_len=b.max_kv_len + b.max_k, scale=b.scale, workspace=ws)
    torch.cuda.synchronize()
    want = oracle_attention(b_cpu)
    assert np.abs(out.double().cpu().numpy() - want).max() <= 2e-3


@pytest.mark.parametrize("V", [50272, 4099, 6])
def test_accept_from_fp32_logits(V):
    """fp32 logits (EMS_F32): arg-max by 16-byte loads of four floats, or element by element when V
    is not a multiple of four; natural ties, an all -inf row, +-0."""
    import paper_2405_07542_amd as ems
    b_cpu = make_batch([3, 4, 5], [6, 1, 9], H=1, D=64, dtype=torch.float16, seed=93, vocab_for_ids=V)
    rng = np.random.default_rng(94 + V)
    lg = np.round(rng.standard_normal((b_cpu.T, V)).astype(np.float32) * 4) / 4     # coarse grid: many ties
    lg[2, :] = -np.inf
    lg[3, :] = -0.0
    lg[3, V - 1] = 0.0
    want = oracle.argmax_f32(lg)
    assert np.array_equal(want, np.argmax(lg, axis=1))
    b = to_device(b_cpu)
    logits = torch.from_numpy(lg).cuda()
    target = torch.full((b.T,), -7, dtype=torch.int32, device="cuda")
    accepted = torch.empty(b.B, dtype=torch.int32, device="cuda")
    accepted_cu = torch.empty(b.B + 1, dtype=torch.int32, device="cuda")
    ws = torch.empty(ems.ems_accept_workspace_bytes(b.T, V), dtype=torch.uint8, device="cuda")
    ems.ems_greedy_accept(logits, target, b.input_ids, b.cu_seqlens, accepted, accepted_cu, None, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(target.cpu().numpy(), want)
    o_acc, o_cu, _ = oracle.greedy_accept(want, b_cpu.input_ids.numpy(), b_cpu.cu_seqlens.numpy())
    assert np.array_equal(accepted.cpu().numpy(), o_acc) and np.array_equal(accepted_cu.cpu().numpy(), o_cu)
