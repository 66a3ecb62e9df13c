"""Pins for the oracle of tree-structured verification (the paper's Limitations, item 4,
names tree decoding as the next thing to combine with the multi-sample method and gives no
algorithm; these pins tie the oracle to definitions that are written independently of it):

* a chain is ordinary speculative decoding: all three functions reduce to the already
  pinned causal ones, bit for bit;
* path equivalence: a tree row's attention output is what causal attention gives on the
  sequence of rows from the root to it -- the reason tree verification is lossless;
* a dense brute force whose mask comes from the transitive closure of the parent relation
  as a boolean matrix (no parent walking);
* acceptance from a per-node validity rule (no walk from the root), hand-built cases,
  and the chain extracted from the accepted path replayed through plain greedy acceptance;
* gathered append against a numpy gather on sentinel-filled arenas.
"""
import numpy as np
import pytest
import torch

import oracle
from workloads import (HEAD_MAJOR, TOKEN_MAJOR, arena_view, bits, grow_trees, make_batch)


def tree_attention(b):
    return oracle.tree_verify_attention(
        bits(b.q), bits(b.k_new), bits(b.v_new), bits(b.k_cache), bits(b.v_cache),
        b.row_stride, b.head_stride, b.cu_seqlens.numpy(), b.parent.numpy(), b.kv_start.numpy(),
        b.kv_len.numpy(), b.H, b.D, b.scale, b.dtype)


def causal_attention(b, q=None, k_new=None, v_new=None, cu=None):
    return oracle.verify_attention(
        bits(b.q if q is None else q), bits(b.k_new if k_new is None else k_new),
        bits(b.v_new if v_new is None else v_new), bits(b.k_cache), bits(b.v_cache),
        b.row_stride, b.head_stride, b.cu_seqlens.numpy() if cu is None else cu,
        b.kv_start.numpy(), b.kv_len.numpy(), b.H, b.D, b.scale, b.dtype)


def small_tree_batch(seed, shape="random", layout=TOKEN_MAJOR, dtype=torch.float16):
    b = make_batch([7, 0, 33, 12], [6, 9, 1, 16], H=2, D=64, dtype=dtype, seed=seed, capacity=64,
                   layout=layout, vocab_for_ids=40)
    return grow_trees(b, seed + 1000, shape=shape)


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_chain_is_ordinary_verification(layout):
    b = small_tree_batch(1, shape="chain", layout=layout)
    assert np.array_equal(tree_attention(b), causal_attention(b))
    x, ids, cu = b.target_ids.numpy(), b.input_ids.numpy(), b.cu_seqlens.numpy()
    acc, acc_cu, toks, rows = oracle.tree_accept(x, ids, b.parent.numpy(), cu)
    acc2, acc_cu2, toks2 = oracle.greedy_accept(x, ids, cu)
    assert np.array_equal(acc, acc2) and np.array_equal(acc_cu, acc_cu2) and np.array_equal(toks, toks2)
    assert np.array_equal(rows, np.concatenate([cu[i] + np.arange(acc[i]) for i in range(b.B)]))
    k1, v1 = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    k2, v2 = k1.copy(), v1.copy()
    l1 = oracle.kv_append_rows(k1, v1, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new), rows,
                               acc_cu, b.kv_start.numpy(), b.kv_len.numpy(), b.H, b.D)
    l2 = oracle.kv_append(k2, v2, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new), cu, acc2,
                          b.kv_start.numpy(), b.kv_len.numpy(), b.H, b.D)
    assert np.array_equal(l1, l2) and np.array_equal(k1, k2) and np.array_equal(v1, v2)


@pytest.mark.parametrize("shape", ["random", "wide", "star"])
@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_every_row_equals_causal_attention_along_its_path(shape, dtype):
    b = small_tree_batch(2, shape=shape, dtype=dtype)
    got = tree_attention(b)
    cu, par = b.cu_seqlens.numpy(), b.parent.numpy()
    for i in range(b.B):
        for j in range(cu[i + 1] - cu[i]):
            path = [j]
            while par[cu[i] + path[-1]] >= 0:
                path.append(int(par[cu[i] + path[-1]]))
            path = path[::-1]                             # root ... j
            sel = torch.tensor([cu[i] + u for u in path])
            # a batch that holds only sample i with the path as its (causal) new rows
            cu1 = np.zeros(b.B + 1, dtype=np.int32)
            cu1[i + 1:] = len(path)
            out = causal_attention(b, q=b.q[sel], k_new=b.k_new[sel], v_new=b.v_new[sel], cu=cu1)
            assert np.abs(out[-1] - got[cu[i] + j]).max() < 1e-12


def closure_brute_force(b):
    """Dense per-sample attention; the new-row mask is the reflexive transitive closure of
    the child->parent relation computed by boolean matrix powers."""
    cu, par, ks, kl = (b.cu_seqlens.numpy(), b.parent.numpy(), b.kv_start.numpy(), b.kv_len.numpy())
    K = arena_view(b.k_cache, b.layout, b.rows, b.H, b.D).double().numpy()
    V = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D).double().numpy()
    q, kn, vn = b.q.double().numpy(), b.k_new.double().numpy(), b.v_new.double().numpy()
    out = np.zeros((b.T, b.H, b.D))
    for i in range(b.B):
        k, L = int(cu[i + 1] - cu[i]), int(kl[i])
        if k == 0:
            continue
        P = np.zeros((k, k), dtype=np.int64)
        for j in range(1, k):
            P[j, par[cu[i] + j]] = 1
        reach = np.eye(k, dtype=np.int64)
        step = np.eye(k, dtype=np.int64)
        for _ in range(k):
            step = (step @ P > 0).astype(np.int64)
            reach |= step
        visible = np.concatenate([np.ones((k, L), dtype=bool), reach > 0], axis=1)
        keys = np.concatenate([K[ks[i]:ks[i] + L], kn[cu[i]:cu[i + 1]]])
        vals = np.concatenate([V[ks[i]:ks[i] + L], vn[cu[i]:cu[i + 1]]])
        for h in range(b.H):
            s = np.float64(np.float32(b.scale)) * (q[cu[i]:cu[i + 1], h] @ keys[:, h].T)
            s = np.where(visible, s, -np.inf)
            p = np.exp(s - s.max(axis=1, keepdims=True))
            out[cu[i]:cu[i + 1], h] = (p / p.sum(axis=1, keepdims=True)) @ vals[:, h]
    return out


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
@pytest.mark.parametrize("shape", ["random", "wide"])
def test_dense_brute_force_with_closure_mask(layout, shape):
    b = small_tree_batch(3, shape=shape, layout=layout)
    assert np.abs(tree_attention(b) - closure_brute_force(b)).max() < 1e-12


def test_a_sibling_is_never_visible():
    """Two children of the root with very different values: each child's output lies in the
    hull of {cache, root, itself}; moving the sibling's V far away changes nothing."""
    b = small_tree_batch(4, shape="star")
    ref = tree_attention(b)
    cu = b.cu_seqlens.numpy()
    v2 = b.v_new.clone()
    v2[cu[0] + 2] += 1000.0                       # row 2 of sample 0: a sibling of rows 1, 3, 4, 5
    import dataclasses
    moved = tree_attention(dataclasses.replace(b, v_new=v2))
    rows = [cu[0] + j for j in (0, 1, 3, 4, 5)]
    assert np.array_equal(moved[rows], ref[rows])
    assert np.abs(moved[cu[0] + 2] - ref[cu[0] + 2]).max() > 1.0


def validity_rule_accept(x, ids, par, cu):
    """Acceptance without a walk: a row is on the accepted path iff its parent is, its token
    equals the target's token after the parent, and no earlier sibling carries that token."""
    acc, rows_out, toks = [], [], []
    for i in range(len(cu) - 1):
        c0, k = int(cu[i]), int(cu[i + 1] - cu[i])
        valid = [False] * k
        for j in range(k):
            if j == 0:
                valid[j] = True
                continue
            u = int(par[c0 + j])
            first = not any(par[c0 + c] == u and ids[c0 + c] == ids[c0 + j] for c in range(j))
            valid[j] = valid[u] and ids[c0 + j] == x[c0 + u] and first
        on = [j for j in range(k) if valid[j]]
        acc.append(len(on))
        rows_out += [c0 + j for j in on]
        toks += [int(x[c0 + j]) for j in on]
    return np.array(acc), np.array(rows_out), np.array(toks)


@pytest.mark.parametrize("shape", ["random", "wide", "star", "chain"])
@pytest.mark.parametrize("seed", [5, 6, 7])
def test_accept_matches_the_validity_rule_and_replays_as_a_chain(shape, seed):
    b = make_batch([3] * 12, [16, 11, 1, 0, 7, 16, 2, 5, 9, 16, 3, 13], H=1, D=64, seed=seed, capacity=24,
                   vocab_for_ids=12)
    b = grow_trees(b, seed + 50, match_p=0.8, shape=shape, duplicate_p=0.3)
    x, ids, par, cu = (b.target_ids.numpy(), b.input_ids.numpy(), b.parent.numpy(), b.cu_seqlens.numpy())
    acc, acc_cu, toks, rows = oracle.tree_accept(x, ids, par, cu)
    w_acc, w_rows, w_toks = validity_rule_accept(x, ids, par, cu)
    assert np.array_equal(acc, w_acc) and np.array_equal(rows, w_rows) and np.array_equal(toks, w_toks)
    assert np.array_equal(acc_cu, np.concatenate([[0], np.cumsum(acc)]))
    k = np.diff(cu)
    assert ((acc >= np.minimum(k, 1)) & (acc <= k)).all()
    if shape == "star":
        assert (acc <= 2).all()
    # the accepted path, replayed as an ordinary draft sequence, is accepted whole; with one
    # more (non-matching) draft appended it is accepted up to exactly that draft
    for i in range(b.B):
        path = rows[acc_cu[i]:acc_cu[i + 1]]
        if len(path) == 0:
            continue
        seq_ids = np.concatenate([ids[path], [x[path[-1]] + 1]]).astype(np.int32)
        seq_x = np.concatenate([x[path], [0]]).astype(np.int32)
        a, _, t = oracle.greedy_accept(seq_x, seq_ids, np.array([0, len(path) + 1], dtype=np.int32))
        assert a[0] == len(path) and np.array_equal(t, toks[acc_cu[i]:acc_cu[i + 1]])


def test_hand_built_tree():
    #            0
    #          / | \
    #         1  2  3        tokens 7, 9, 9      target after 0: 9  -> row 2 (lowest index with 9)
    #            |  |
    #            4  5        tokens 5, 5         target after 2: 5  -> row 4;  after 4: 8, no child
    par = np.array([-1, 0, 0, 0, 2, 3], dtype=np.int32)
    ids = np.array([1, 7, 9, 9, 5, 5], dtype=np.int32)
    x = np.array([9, 0, 5, 5, 8, 0], dtype=np.int32)
    cu = np.array([0, 6], dtype=np.int32)
    acc, acc_cu, toks, rows = oracle.tree_accept(x, ids, par, cu)
    assert acc.tolist() == [3] and rows.tolist() == [0, 2, 4] and toks.tolist() == [9, 5, 8]
    # the root's target matches nobody: only the root is accepted
    acc, _, toks, rows = oracle.tree_accept(np.array([4, 0, 5, 5, 8, 0], dtype=np.int32), ids, par, cu)
    assert acc.tolist() == [1] and rows.tolist() == [0] and toks.tolist() == [4]


def test_parent_array_must_be_a_topologically_ordered_tree():
    b = small_tree_batch(8)
    import dataclasses
    for bad_row, bad_val in ((0, 0), (1, 1), (2, 5), (3, -1)):
        p = b.parent.clone()
        p[bad_row] = bad_val
        with pytest.raises(ValueError):
            tree_attention(dataclasses.replace(b, parent=p))


@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_gathered_append_on_sentinel_arena(layout):
    b = small_tree_batch(9, layout=layout)
    x, ids, par, cu = (b.target_ids.numpy(), b.input_ids.numpy(), b.parent.numpy(), b.cu_seqlens.numpy())
    acc, acc_cu, _, rows = oracle.tree_accept(x, ids, par, cu)
    kc, vc = bits(b.k_cache).copy(), bits(b.v_cache).copy()
    new_len = oracle.kv_append_rows(kc, vc, b.row_stride, b.head_stride, bits(b.k_new), bits(b.v_new),
                                    rows, acc_cu, b.kv_start.numpy(), b.kv_len.numpy(), b.H, b.D)
    assert np.array_equal(new_len, b.kv_len.numpy() + acc)
    from workloads import from_bits
    K0 = arena_view(b.k_cache, layout, b.rows, b.H, b.D).view(torch.int16).numpy().copy()
    V0 = arena_view(b.v_cache, layout, b.rows, b.H, b.D).view(torch.int16).numpy().copy()
    kn, vn = b.k_new.view(torch.int16).numpy(), b.v_new.view(torch.int16).numpy()
    for i in range(b.B):
        dst = int(b.kv_start[i]) + int(b.kv_len[i])
        src = rows[acc_cu[i]:acc_cu[i + 1]]
        K0[dst:dst + len(src)] = kn[src]
        V0[dst:dst + len(src)] = vn[src]
    K1 = arena_view(from_bits(kc, b.dtype).view(b.k_cache.shape), layout, b.rows, b.H, b.D).view(torch.int16).numpy()
    V1 = arena_view(from_bits(vc, b.dtype).view(b.v_cache.shape), layout, b.rows, b.H, b.D).view(torch.int16).numpy()
    assert np.array_equal(K1, K0) and np.array_equal(V1, V0)
