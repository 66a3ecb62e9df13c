"""GPU parity on a seeded sweep of random valid shapes: batch size, head count, head dim, dtype,
cache layout, ragged cached lengths (empty caches, exact tile multiples, tails), rows per
sample (0..16, and 0..64 in the cases that exercise the wide kernel), regions placed in shuffled
order with gaps.  Every case runs the whole step
(attention, accept from given ids, append) and its tree-structured twin against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_07542_amd as ems
from workloads import HEAD_MAJOR, TOKEN_MAJOR, bits, grow_trees, make_batch
from helpers import attention_tolerance, hip_attention, oracle_attention, to_device
from test_gpu_parity import check_attention, run_accept_and_append
from test_gpu_tree import check_accept_and_append, check_tree_attention, oracle_tree_attention

pytestmark = pytest.mark.gpu


def random_case(seed, k_hi=16):
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.choice([1, 2, 3, 5, 9, 17, 40]))
    H = int(rng.choice([1, 2, 3, 5, 8, 12]))
    D = int(rng.choice([64, 80, 128]))
    dtype = [torch.float16, torch.bfloat16][int(rng.integers(0, 2))]
    layout = [TOKEN_MAJOR, HEAD_MAJOR][int(rng.integers(0, 2))]
    pool = [0, 1, 2, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129]
    kv = [int(rng.choice(pool)) if rng.random() < 0.5 else int(rng.integers(0, 700)) for _ in range(B)]
    k = [int(rng.integers(0, k_hi + 1)) for _ in range(B)]
    if sum(k) == 0:
        k[0] = 1
    # regions in shuffled order, each with room for the sample's new rows and a random gap after it
    order = rng.permutation(B)
    starts, pos = [0] * B, int(rng.integers(0, 5))
    for i in order:
        starts[i] = pos
        pos += kv[i] + k[i] + int(rng.integers(0, 40))
    b = make_batch(kv, k, H=H, D=D, dtype=dtype, seed=2000 + seed, kv_start=starts, rows=pos + 1,
                   layout=layout, vocab_for_ids=17, match_p=0.75)
    return b


@pytest.mark.parametrize("seed", list(range(24)) + [(s, 64) for s in range(100, 112)])
def test_random_shape(seed):
    """(seed) draws up to 16 rows per sample; (seed, 64) up to 64, i.e. the wide kernel."""
    k_hi = 16
    if isinstance(seed, tuple):
        seed, k_hi = seed
    b = random_case(seed, k_hi)
    print("case", seed, "B", b.B, "H", b.H, "D", b.D, b.dtype, b.layout, "kv", b.kv_len.tolist(),
          "k", np.diff(b.cu_seqlens.numpy()).tolist(), "start", b.kv_start.tolist(), flush=True)
    dev = to_device(b)
    ems.ems_validate_inputs(dev.cu_seqlens, dev.kv_start, dev.kv_len, T=b.T, max_k=k_hi,
                            max_kv_len=max(1, b.max_kv_len), rows=b.rows)
    check_attention(b, out_dtype=torch.float32, label="random %d f32" % seed)
    check_attention(b, label="random %d" % seed)
    run_accept_and_append(b)
    t = grow_trees(b, 3000 + seed, match_p=0.75, shape=["random", "wide", "star"][seed % 3])
    check_tree_attention(t, out_dtype=torch.float32)
    check_accept_and_append(t, use_logits=False, n_layers=2)


@pytest.mark.parametrize("seed", list(range(200, 216)) + [(s, 64) for s in range(300, 312)])
def test_random_shape_with_a_loose_length_bound(seed):
    """max_kv_len is only a bound; a loose one makes the library size the launch for far more
    tiles than there are (1024 waves, most of them with one tile or none) and switches on the
    in-workgroup merge of partials that it keeps off for short walks: every pair is then cut
    over many waves and workgroups.  The outputs must not change beyond rounding."""
    k_hi = 16
    if isinstance(seed, tuple):         # up to 64 rows per sample: the wide kernel, two pairs per head
        seed, k_hi = seed
    b = random_case(seed, k_hi)
    loose = 32 * (-(-14000 // (b.B * b.H)) + 1)
    print("case", seed, "B", b.B, "H", b.H, "D", b.D, b.dtype, b.layout, "kv", b.kv_len.tolist(),
          "k", np.diff(b.cu_seqlens.numpy()).tolist(), "bound", loose, flush=True)
    assert loose > b.max_kv_len
    want = oracle_attention(b)
    got = hip_attention(to_device(b), out_dtype=torch.float32, max_kv_len=loose).double().cpu().numpy()
    assert np.isfinite(got).all()
    err = np.abs(got - want)
    assert (err <= attention_tolerance(b, want, torch.float32)).all(), err.max()

    # the write-through variant and the tree call take the same route
    dev = to_device(b)
    kc, vc = dev.k_cache.clone(), dev.v_cache.clone()
    out = torch.full((b.T, b.H, b.D), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, loose), dtype=torch.uint8, device="cuda")
    ems.ems_verify_attention_write_through(dev.q, dev.k_new, dev.v_new,
                                           ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows),
                                           dev.cu_seqlens, dev.kv_start, dev.kv_len, out, max_k=b.max_k,
                                           max_kv_len=loose, scale=b.scale, workspace=ws)
    torch.cuda.synchronize()
    assert (np.abs(out.double().cpu().numpy() - want) <= attention_tolerance(b, want, torch.float32)).all()
    okc, ovc = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    oracle.kv_write_through(okc, ovc, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new),
                            b.cu_seqlens.numpy(), b.kv_start.numpy(), b.kv_len.numpy(), b.H, b.D)
    assert np.array_equal(bits(kc), okc) and np.array_equal(bits(vc), ovc)

    t = grow_trees(b, 5000 + seed, match_p=0.75, shape=["random", "wide", "star"][seed % 3])
    td = to_device(t)
    out = torch.full((t.T, t.H, t.D), float("nan"), dtype=torch.float32, device="cuda")
    ems.ems_tree_verify_attention(td.q, td.k_new, td.v_new,
                                  ems.kv_cache(td.k_cache, td.v_cache, t.row_stride, t.head_stride, t.rows),
                                  td.cu_seqlens, td.parent, td.kv_start, td.kv_len, out, max_k=t.max_k,
                                  max_kv_len=loose, scale=t.scale, workspace=ws)
    torch.cuda.synchronize()
    want_tree = oracle_tree_attention(t)
    assert (np.abs(out.double().cpu().numpy() - want_tree) <= attention_tolerance(t, want_tree, torch.float32)).all()
