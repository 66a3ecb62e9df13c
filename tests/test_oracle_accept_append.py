"""Pins for the acceptance, prefix-sum, arg-max, append and index-restoring oracles."""
import os

import numpy as np
import pytest
import torch

import oracle
from workloads import HEAD_MAJOR, TOKEN_MAJOR, arena_view, bits, from_bits, make_batch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_case_analysis.txt")


def read_table1():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append([int(x) for x in line.split()])
    return rows


def ids_for(predict, accept, rng, vocab=1000):
    """Token lists for one sample: `predict` drafts of which the first accept-1 agree
    with the target and draft number `accept` (if there is one) does not."""
    k = predict + 1
    x = rng.integers(0, vocab, k)
    ids = np.zeros(k, dtype=np.int64)
    ids[0] = rng.integers(0, vocab)
    for j in range(predict):
        ids[j + 1] = x[j] if j < accept - 1 else (x[j] + 1 + rng.integers(0, vocab - 1)) % vocab
    return x, ids


def test_table1_replay():
    """Table 1 / Sec. 3.1 case analysis / Sec. 3.2: predicted {5,2} then {2,5} drafts,
    accepted {4,1} then {2,6}; vanilla padding counts; cache locations advance by the
    accepted counts only."""
    rng = np.random.default_rng(1)
    table = read_table1()
    kv_len = np.array([10, 20], dtype=np.int32)
    for step in (1, 2):
        rows = sorted([r for r in table if r[0] == step], key=lambda r: r[1])
        predict = [r[2] for r in rows]
        accept = [r[4] for r in rows]
        xs, idss = zip(*[ids_for(p, a, rng) for p, a in zip(predict, accept)])
        cu = np.concatenate([[0], np.cumsum([p + 1 for p in predict])]).astype(np.int32)
        acc, acc_cu, out = oracle.greedy_accept(np.concatenate(xs), np.concatenate(idss), cu)
        assert acc.tolist() == accept
        assert acc_cu.tolist() == [0, accept[0], accept[0] + accept[1]]
        assert out.tolist() == list(xs[0][:accept[0]]) + list(xs[1][:accept[1]])
        # what the vanilla method would have to pad (the table's Padding columns)
        assert [max(predict) - p for p in predict] == [r[3] for r in rows]
        assert [int(acc.max() - a) for a in acc] == [r[5] for r in rows]
        assert all(1 <= a <= p + 1 for a, p in zip(acc, predict))
        kv_len = kv_len + acc
    assert kv_len.tolist() == [10 + 4 + 2, 20 + 1 + 6]


def first_mismatch_definition(x, d):
    """The acceptance-length equation read directly: tau is the first j in 1..k+1
    with x_{j-1} != d_{j-1}, where d_k does not exist and therefore never matches."""
    k = len(d)
    for j in range(1, k + 2):
        if j == k + 1 or x[j - 1] != d[j - 1]:
            return j
    raise AssertionError


@pytest.mark.parametrize("seed", range(5))
def test_accept_equals_first_mismatch_definition(seed):
    rng = np.random.default_rng(seed)
    B = 40
    k = rng.integers(0, 9, B)            # includes k_i = 0 (finished sample) and 1 (no drafts)
    cu = np.concatenate([[0], np.cumsum(k)]).astype(np.int32)
    T = int(cu[-1])
    x = rng.integers(0, 3, T)            # tiny vocabulary: long accepted runs are common
    ids = rng.integers(0, 3, T)
    acc, acc_cu, out = oracle.greedy_accept(x, ids, cu)
    want_out = []
    for i in range(B):
        if k[i] == 0:
            assert acc[i] == 0
            continue
        sl = slice(cu[i], cu[i + 1])
        tau = first_mismatch_definition(x[sl], ids[sl][1:])
        assert acc[i] == tau and 1 <= tau <= k[i]
        want_out += x[sl][:tau].tolist()
    assert acc_cu[0] == 0 and np.array_equal(np.diff(acc_cu), acc)
    assert out.tolist() == want_out


def test_accept_special_cases():
    cu = np.array([0, 4, 8, 9, 13], dtype=np.int32)
    x = np.array([5, 6, 7, 8, 5, 6, 7, 8, 3, 1, 1, 1, 1])
    ids = np.array([9, 5, 6, 7, 9, 0, 6, 7, 3, 1, 1, 0, 1])
    acc, acc_cu, out = oracle.greedy_accept(x, ids, cu)
    # all drafts right -> k_i; first draft wrong -> 1 (later agreements do not count);
    # no drafts -> 1; a wrong draft in the middle stops the run
    assert acc.tolist() == [4, 1, 1, 2]
    assert acc_cu.tolist() == [0, 4, 5, 6, 8]
    assert out.tolist() == [5, 6, 7, 8, 5, 3, 1, 1]


def test_accepted_length_statistics_match_geometric_model():
    """Appendix B: with per-draft accuracy p the accepted length is geometric,
    P(tau = t) = p^(t-1) (1-p), truncated at k_i; E tau -> 1/(1-p) for long drafts;
    the batch maximum follows P(tau_max <= t) = (1 - p^t)^b."""
    p, B, kk = 0.7, 4000, 40
    b = make_batch([1] * B, [kk] * B, H=1, D=8, seed=3, match_p=p, vocab_for_ids=50272)
    acc, _, _ = oracle.greedy_accept(b.target_ids.numpy(), b.input_ids.numpy(),
                                     b.cu_seqlens.numpy())
    assert abs(acc.mean() - 1 / (1 - p)) < 0.15
    for t in (1, 2, 3, 5):
        assert abs((acc == t).mean() - p ** (t - 1) * (1 - p)) < 0.025
    bsz = 8
    tmax = acc[: (B // bsz) * bsz].reshape(-1, bsz).max(axis=1)
    for t in (3, 5, 8):
        assert abs((tmax <= t).mean() - (1 - p ** t) ** bsz) < 0.06


def test_argmax_lowest_index_wins_ties():
    for dtype, one, two in ((torch.float16, 0x3C00, 0x4000), (torch.bfloat16, 0x3F80, 0x4000)):
        lg = np.full((4, 37), one, dtype=np.uint16)
        lg[0, [9, 20]] = two                 # duplicate maximum at 9 < 20
        lg[1, 36] = two                      # maximum in the last column
        lg[2, :] = 0x8000                    # all -0 ...
        lg[2, 5] = 0x0000                    # ... and one +0: equal, index 0 wins
        lg[3, 0] = two
        assert oracle.argmax(lg, dtype).tolist() == [9, 36, 0, 0]
        # draft = lower index is accepted, draft = higher index of the tie is not
        x = oracle.argmax(lg[:1], dtype)
        cu = np.array([0, 2], dtype=np.int32)
        assert oracle.greedy_accept([x[0], 0], [1, 9], cu)[0].tolist() == [2]
        assert oracle.greedy_accept([x[0], 0], [1, 20], cu)[0].tolist() == [1]


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_argmax_equals_numpy_on_random_rows(dtype):
    g = torch.Generator().manual_seed(5)
    lg = torch.randn(12, 5003, generator=g).to(dtype)
    want = np.argmax(lg.double().numpy(), axis=1)     # numpy returns the first maximum
    assert oracle.argmax(bits(lg), dtype).tolist() == want.tolist()
    # negative values only (sign handling)
    neg = (-lg.abs() - 1).to(dtype)
    assert oracle.argmax(bits(neg), dtype).tolist() == np.argmax(neg.double().numpy(), 1).tolist()


def test_generator_plants_the_row_maximum_where_it_says():
    b = make_batch([4, 4, 4], [5, 3, 6], H=1, D=8, seed=22, V=1999, dtype=torch.bfloat16)
    assert oracle.argmax(bits(b.logits), b.dtype).tolist() == b.target_ids.tolist()
    vals = b.logits.double().numpy()
    assert ((vals == vals.max(axis=1, keepdims=True)).sum(axis=1) > 1).any()   # real ties exist


def test_widening_is_exact_for_every_bit_pattern():
    """The oracle reads fp16/bf16 through its own bit-level widening; check it against
    torch's conversion for all 65536 patterns by arg-maxing two-column rows."""
    allbits = np.arange(65536, dtype=np.uint16)
    for dtype in (torch.float16, torch.bfloat16):
        vals = from_bits(allbits, dtype).double().numpy()
        finite = np.isfinite(vals)
        order = np.argsort(vals[finite], kind="stable")
        srt = allbits[finite][order]
        pairs = np.stack([srt[:-1], srt[1:]], axis=1)            # ascending neighbours
        got = oracle.argmax(pairs, dtype)
        sv = vals[finite][order]
        want = (sv[1:] > sv[:-1]).astype(np.int32)               # equal (+-0) -> index 0
        assert np.array_equal(got, want)


@pytest.mark.parametrize("counts", [[5, 2], [6, 3], [1, 1, 1], [0, 4, 0, 2]])
def test_restore_index_matches_cu_seqlens_lookup(counts):
    """Alg. 1 packs the per-sample token lists; Alg. 2 walks token_nums_per_sample to
    recover (sample, position).  Both must agree with a search in the running sum.
    [5, 2] is the example of Fig. 3 (7 packed rows)."""
    lists = [[100 * i + j for j in range(n)] for i, n in enumerate(counts)]
    concatenated, token_nums, total = [], [0] * len(lists), 0      # Alg. 1
    for i, toks in enumerate(lists):
        total += len(toks)
        token_nums[i] = len(toks)
        concatenated.extend(toks)
    assert total == sum(counts)
    cu = np.concatenate([[0], np.cumsum(token_nums)])
    for r in range(total):
        i, pos = oracle.restore_index(token_nums, r)
        assert concatenated[r] == lists[i][pos]
        assert i == int(np.searchsorted(cu, r, side="right") - 1) and pos == r - cu[i]
    with pytest.raises(IndexError):
        oracle.restore_index(token_nums, total)


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_append_writes_exactly_the_accepted_rows(layout, dtype):
    kv_len, k = [7, 0, 12, 3], [4, 3, 1, 5]
    accepted = [2, 3, 1, 0]
    b = make_batch(kv_len, k, H=3, D=8, dtype=dtype, seed=30, capacity=24, layout=layout)
    kc, vc = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    k0, v0 = kc.copy(), vc.copy()
    new_len = oracle.kv_append(kc, vc, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new),
                               b.cu_seqlens.numpy(), accepted, b.kv_start.numpy(),
                               b.kv_len.numpy(), b.H, b.D)
    assert new_len.tolist() == [9, 3, 13, 3]
    cu = b.cu_seqlens.numpy()
    for arena, before, new in ((kc, k0, b.k_new), (vc, v0, b.v_new)):
        after3 = arena_view(from_bits(arena, dtype), layout, b.rows, b.H, b.D)
        before3 = arena_view(from_bits(before, dtype), layout, b.rows, b.H, b.D)
        untouched = np.ones(b.rows, dtype=bool)
        for i in range(b.B):
            s, L = int(b.kv_start[i]), kv_len[i]
            for j in range(accepted[i]):
                assert np.array_equal(bits(after3[s + L + j]), bits(new[cu[i] + j]))
                untouched[s + L + j] = False
        # every other row -- old cache rows and NaN sentinel rows alike -- is bit-identical
        assert np.array_equal(bits(after3[untouched]), bits(before3[untouched]))
        assert int((~untouched).sum()) == sum(accepted)


def test_multi_step_cache_is_the_concatenation_of_accepted_rows():
    """After several verification steps each cache is contiguous, of length
    kv_len + sum(accepted), and holds the accepted rows in order."""
    rng = np.random.default_rng(4)
    B, H, D, steps = 3, 2, 8, 6
    b = make_batch([5, 9, 2], [1, 1, 1], H=H, D=D, seed=31, capacity=64)
    kc, vc = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    lens = b.kv_len.numpy().copy()
    history = [[] for _ in range(B)]
    for step in range(steps):
        k = rng.integers(1, 7, B)
        cu = np.concatenate([[0], np.cumsum(k)]).astype(np.int32)
        nb = make_batch(lens.tolist(), k.tolist(), H=H, D=D, seed=500 + step, capacity=64)
        acc = np.array([rng.integers(1, kk + 1) for kk in k], dtype=np.int32)
        lens = oracle.kv_append(kc, vc, b.row_stride, b.head_stride, bits(nb.k_new),
                                bits(nb.v_new), cu, acc, b.kv_start.numpy(), lens, H, D)
        for i in range(B):
            history[i].append(bits(nb.k_new)[cu[i]:cu[i] + acc[i]])
    view = kc.reshape(b.rows, H, D)
    for i in range(B):
        s, L0 = int(b.kv_start[i]), int(b.kv_len[i])
        want = np.concatenate(history[i])
        assert lens[i] == L0 + len(want)
        assert np.array_equal(view[s + L0:s + lens[i]], want)
        assert (view[s + lens[i]:s + 64] == 0x7E00).all()       # the rest is still sentinel


def test_widening_gives_exact_values():
    """One key, no cache: softmax weight is exactly 1, so the output is the widened V row.
    Feeding every finite bit pattern as V pins the oracle's fp16/bf16 decoding."""
    allbits = np.arange(65536, dtype=np.uint16)
    for dtype in (torch.float16, torch.bfloat16):
        vals = from_bits(allbits, dtype).double().numpy()
        fin = allbits[np.isfinite(vals)]
        D = len(fin)
        zeros = np.zeros(D, dtype=np.uint16)
        out = oracle.verify_attention(zeros, zeros, fin, zeros[:0], zeros[:0], D, D,
                                      [0, 1], [0], [0], 1, D, 1.0, dtype)
        assert np.array_equal(out.reshape(-1), vals[np.isfinite(vals)])


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_write_through_then_advance_equals_append_on_the_live_rows(layout):
    """Sec. 3.2 in the paper's own order: write every new row at the sample's location, then
    advance the location by the accepted count.  On rows [0, kv_len+accepted) this must give
    what appending only the accepted rows gives; rejected drafts sit beyond the new length;
    nothing else in the arena changes."""
    kv_len, k = [7, 0, 12, 3], [4, 3, 1, 5]
    accepted = [2, 3, 1, 1]
    b = make_batch(kv_len, k, H=3, D=8, dtype=torch.float16, seed=33, capacity=24, layout=layout)
    a_k, a_v = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    new_len = oracle.kv_append(a_k, a_v, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new),
                               b.cu_seqlens.numpy(), accepted, b.kv_start.numpy(), b.kv_len.numpy(),
                               b.H, b.D)
    w_k, w_v = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    oracle.kv_write_through(w_k, w_v, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new),
                            b.cu_seqlens.numpy(), b.kv_start.numpy(), b.kv_len.numpy(), b.H, b.D)
    cu = b.cu_seqlens.numpy()
    for arena_w, arena_a, new in ((w_k, a_k, b.k_new), (w_v, a_v, b.v_new)):
        W = arena_view(from_bits(arena_w, b.dtype), layout, b.rows, b.H, b.D)
        A = arena_view(from_bits(arena_a, b.dtype), layout, b.rows, b.H, b.D)
        for i in range(b.B):
            s, L = int(b.kv_start[i]), kv_len[i]
            assert np.array_equal(bits(W[s:s + new_len[i]]), bits(A[s:s + new_len[i]]))
            assert np.array_equal(bits(W[s + L:s + L + k[i]]), bits(new[cu[i]:cu[i + 1]]))
            assert (bits(W[s + L + k[i]:s + 24]) == 0x7E00).all()


def test_concatenation_of_input_tokens_alg_1():
    """Alg. 1 against plain Python list concatenation, the example of Fig. 3 (samples with 5 and
    2 tokens give 7 packed rows), and Alg. 2 as its inverse on every packed row."""
    rng = np.random.default_rng(90)
    for B, k_max in ((2, 5), (7, 9), (33, 16), (1, 1)):
        lens = rng.integers(0, k_max + 1, B).astype(np.int32)
        if (B, k_max) == (2, 5):
            lens = np.array([5, 2], dtype=np.int32)
        padded = rng.integers(0, 1000, (B, k_max)).astype(np.int32)
        cat, nums, total = oracle.concatenate_tokens(padded, lens)
        want = sum((padded[i, :lens[i]].tolist() for i in range(B)), [])
        assert cat.tolist() == want and total == len(want) and np.array_equal(nums, lens)
        if (B, k_max) == (2, 5):
            assert total == 7
        for r in range(total):
            i, pos = oracle.restore_index(nums, r)
            assert cat[r] == padded[i, pos]


def test_argmax_of_fp32_logits():
    rng = np.random.default_rng(92)
    lg = rng.standard_normal((40, 1003)).astype(np.float32)
    lg[3, 17] = lg[3, 900] = 9.0                 # a tie: the lower index wins
    lg[5, :] = -np.inf
    lg[6, 0] = 0.0; lg[6, 1:] = -0.0             # +0 and -0 are equal: index 0
    lg[7, 1002] = 50.0                           # last column
    want = np.argmax(lg, axis=1)                 # numpy returns the first maximum
    got = oracle.argmax_f32(lg)
    assert np.array_equal(got, want) and got[3] == 17 and got[5] == 0 and got[6] == 0 and got[7] == 1002
