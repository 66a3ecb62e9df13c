"""GPU parity of tree-structured verification (ems_tree_verify_attention, ems_tree_accept,
ems_kv_append_rows) against the oracle's tree functions on the same seeded inputs: attention
within the stated tolerance, every id, count, offset, row index and cache byte exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_07542_amd as ems
from workloads import HEAD_MAJOR, TOKEN_MAJOR, bits, grow_trees, make_batch, make_config
from helpers import attention_tolerance, to_device

pytestmark = pytest.mark.gpu


def hip_tree_attention(b, out_dtype=None):
    out = torch.full((b.T, b.H, b.D), float("nan"), dtype=out_dtype or b.dtype, device=b.q.device)
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len),
                     dtype=torch.uint8, device=b.q.device)
    ems.ems_tree_verify_attention(b.q, b.k_new, b.v_new,
                                  ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows),
                                  b.cu_seqlens, b.parent, b.kv_start, b.kv_len, out, max_k=b.max_k,
                                  max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
    torch.cuda.synchronize()
    return out


def oracle_tree_attention(b):
    return oracle.tree_verify_attention(
        bits(b.q), bits(b.k_new), bits(b.v_new), bits(b.k_cache), bits(b.v_cache), b.row_stride,
        b.head_stride, b.cu_seqlens.numpy(), b.parent.numpy(), b.kv_start.numpy(), b.kv_len.numpy(),
        b.H, b.D, b.scale, b.dtype)


def check_tree_attention(b_cpu, out_dtype=None):
    print("tree attention case:", b_cpu.name, "B", b_cpu.B, "H", b_cpu.H, "D", b_cpu.D, b_cpu.dtype,
          b_cpu.layout, "out", out_dtype, flush=True)
    got = hip_tree_attention(to_device(b_cpu), out_dtype).double().cpu().numpy()
    want = oracle_tree_attention(b_cpu)
    assert np.isfinite(got).all()
    err = np.abs(got - want)
    tol = attention_tolerance(b_cpu, want, out_dtype or b_cpu.dtype)
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert (err <= tol).all(), "max err %.3e at %s (tol %.3e)" % (err[worst], worst, tol[worst])


KV = [0, 1, 31, 32, 33, 64, 100, 257, 5, 900]
K = [1, 16, 3, 7, 2, 11, 1, 5, 16, 0]


@pytest.mark.parametrize("shape", ["random", "wide", "star", "chain"])
@pytest.mark.parametrize("dtype,D,layout", [(torch.float16, 128, TOKEN_MAJOR), (torch.bfloat16, 64, HEAD_MAJOR),
                                            (torch.bfloat16, 80, TOKEN_MAJOR)])
def test_tree_attention_ragged(shape, dtype, D, layout):
    b = make_batch(KV, K, H=4, D=D, dtype=dtype, seed=60, capacity=1000, layout=layout, vocab_for_ids=30)
    b = grow_trees(b, 61, shape=shape)
    check_tree_attention(b, out_dtype=torch.float32)
    check_tree_attention(b)


def test_chain_tree_is_bit_identical_to_the_causal_call():
    from helpers import hip_attention
    b_cpu = grow_trees(make_batch(KV, K, H=4, D=128, dtype=torch.bfloat16, seed=62, capacity=1000), 63,
                       shape="chain")
    b = to_device(b_cpu)
    assert torch.equal(hip_tree_attention(b).view(torch.int16), hip_attention(b).view(torch.int16))


def test_tree_attention_config_4_full_size():
    b = grow_trees(make_config(4), 64, shape="random")
    check_tree_attention(b)


def hip_tree_accept(b, use_logits):
    dev = b.q.device
    accepted = torch.full((b.B,), -7, dtype=torch.int32, device=dev)
    accepted_cu = torch.full((b.B + 1,), -7, dtype=torch.int32, device=dev)
    out_tokens = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device=dev)
    rows = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device=dev)
    if use_logits:
        target = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device=dev)
        ws = torch.empty(max(8, ems.ems_accept_workspace_bytes(b.T, b.V)), dtype=torch.uint8, device=dev)
        logits = b.logits
    else:
        target, ws, logits = b.target_ids.clone(), None, None
    ems.ems_tree_accept(logits, target, b.input_ids, b.parent, b.cu_seqlens, accepted, accepted_cu,
                        out_tokens, rows, workspace=ws)
    torch.cuda.synchronize()
    return target[:b.T], accepted, accepted_cu, out_tokens, rows


def check_accept_and_append(b_cpu, use_logits, n_layers=1, in_place=False):
    b = to_device(b_cpu)
    tgt, acc, acc_cu, toks, rows = hip_tree_accept(b, use_logits)
    x = oracle.argmax(bits(b_cpu.logits), b_cpu.dtype) if use_logits else b_cpu.target_ids.numpy()
    o_acc, o_cu, o_toks, o_rows = oracle.tree_accept(x, b_cpu.input_ids.numpy(), b_cpu.parent.numpy(),
                                                     b_cpu.cu_seqlens.numpy())
    n = int(o_cu[-1])
    assert np.array_equal(tgt.cpu().numpy(), x)
    assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(acc_cu.cpu().numpy(), o_cu)
    assert np.array_equal(toks.cpu().numpy()[:n], o_toks) and np.array_equal(rows.cpu().numpy()[:n], o_rows)
    assert (toks.cpu().numpy()[n:] == -7).all() and (rows.cpu().numpy()[n:] == -7).all()
    # gathered append, every layer with the same new rows but its own arena copy
    kcs = [b.k_cache.clone() for _ in range(n_layers)]
    vcs = [b.v_cache.clone() for _ in range(n_layers)]
    lens = b.kv_len.clone()
    new_len = lens if in_place else torch.empty_like(lens)
    ems.ems_kv_append_rows([b.k_new] * n_layers, [b.v_new] * n_layers,
                           [ems.kv_cache(kcs[l], vcs[l], b.row_stride, b.head_stride, b.rows) for l in range(n_layers)],
                           rows, acc_cu, b.kv_start, lens, new_len)
    torch.cuda.synchronize()
    okc, ovc = bits(b_cpu.k_cache).copy(), bits(b_cpu.v_cache).copy()
    o_len = oracle.kv_append_rows(okc, ovc, b_cpu.row_stride, b_cpu.head_stride, bits(b_cpu.k_new),
                                  bits(b_cpu.v_new), o_rows, o_cu, b_cpu.kv_start.numpy(),
                                  b_cpu.kv_len.numpy(), b_cpu.H, b_cpu.D)
    assert np.array_equal(new_len.cpu().numpy(), o_len)
    for l in range(n_layers):
        assert np.array_equal(bits(kcs[l]), okc) and np.array_equal(bits(vcs[l]), ovc)
    return o_acc


@pytest.mark.parametrize("shape", ["random", "wide", "star", "chain"])
@pytest.mark.parametrize("layout", [TOKEN_MAJOR, HEAD_MAJOR])
def test_tree_accept_and_gathered_append(shape, layout):
    b = make_batch(KV, K, H=4, D=64, dtype=torch.float16, seed=65, capacity=1000, layout=layout,
                   vocab_for_ids=12)
    b = grow_trees(b, 66, match_p=0.8, shape=shape, duplicate_p=0.3)
    acc = check_accept_and_append(b, use_logits=False, n_layers=3)
    assert acc.max() >= 2          # the inputs do exercise paths beyond the root
    check_accept_and_append(b, use_logits=False, in_place=True)


def test_tree_accept_from_logits_many_samples():
    rng = np.random.default_rng(67)
    B = 300
    k = rng.integers(0, 17, B).tolist()
    b = make_batch([2] * B, k, H=1, D=64, dtype=torch.bfloat16, seed=68, capacity=24, V=4099)
    b = grow_trees(b, 69, match_p=0.75, shape="random")
    check_accept_and_append(b, use_logits=True)


def test_tree_step_config_4_full_size():
    b = grow_trees(make_config(4), 70, match_p=0.7, shape="wide")
    acc = check_accept_and_append(b, use_logits=True)
    print("config 4 as trees: mean accepted %.2f of mean %.2f rows" % (acc.mean(), np.diff(b.cu_seqlens.numpy()).mean()))


def test_tree_entry_points_reject_bad_arguments():
    b = to_device(grow_trees(make_batch([5, 6], [3, 2], H=2, D=64, seed=71, capacity=16), 72))
    ems.ems_validate_tree(b.cu_seqlens, b.parent)
    for row, value in ((0, 0), (1, 1), (3, 2), (4, -1)):        # rows 0-2 = sample 0, rows 3-4 = sample 1
        bad = b.parent.clone()
        bad[row] = value
        with pytest.raises(ems.EmsError) as e:
            ems.ems_validate_tree(b.cu_seqlens, bad)
        assert e.value.status == ems.EMS_ERR_INVALID_ARG and "parent" in str(e.value)
    out = torch.empty_like(b.q)
    ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len), dtype=torch.uint8, device="cuda")
    cache = ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows)
    with pytest.raises(TypeError, match="parent must be a tensor"):      # the binding refuses it ...
        ems.ems_tree_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, None, b.kv_start, b.kv_len, out,
                                      max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
    import ctypes                                                        # ... and so does the C layer itself
    assert ems.lib().ems_tree_verify_attention(
        b.q.data_ptr(), b.k_new.data_ptr(), b.v_new.data_ptr(), ctypes.byref(cache), b.cu_seqlens.data_ptr(), None,
        b.kv_start.data_ptr(), b.kv_len.data_ptr(), out.data_ptr(), ems.EMS_F16, b.B, b.T, b.H, b.D, b.max_k,
        b.max_kv_len, b.scale, ems.EMS_F16, ws.data_ptr(), ws.numel(), None) == ems.EMS_ERR_INVALID_ARG
    ems.ems_set_attention_variant(ems.EMS_ATTN_VALU)
    try:
        with pytest.raises(ems.EmsError) as e:
            ems.ems_tree_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.parent, b.kv_start,
                                          b.kv_len, out, max_k=b.max_k, max_kv_len=b.max_kv_len,
                                          scale=b.scale, workspace=ws)
        assert e.value.status == ems.EMS_ERR_UNSUPPORTED
    finally:
        ems.ems_set_attention_variant(ems.EMS_ATTN_MFMA)
