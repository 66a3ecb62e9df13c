"""GPU parity of ems_greedy_accept_append (acceptance and append as one call): against the fp64-free
integer oracle (arg-max, acceptance lengths, running sum, emitted tokens, appended cache rows: all
bit for bit) and against the two separate calls on the same inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2405_07542_amd as ems
from workloads import HEAD_MAJOR, TOKEN_MAJOR, bits, make_batch, make_config
from helpers import oracle_accept, to_device

pytestmark = pytest.mark.gpu


def fused(b, caches, news, use_logits=True, in_place=False):
    """Runs the one-call form on device batch b; caches / news: per layer (k_cache, v_cache) clones and
    (k_new, v_new).  Returns every output."""
    dev = b.q.device
    accepted = torch.full((b.B,), -7, dtype=torch.int32, device=dev)
    accepted_cu = torch.full((b.B + 1,), -7, dtype=torch.int32, device=dev)
    out_tokens = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device=dev)
    logits = b.logits if use_logits else None
    if logits is not None:
        target = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device=dev)
        ws = torch.empty(max(8, ems.ems_accept_workspace_bytes(b.T, b.V)), dtype=torch.uint8, device=dev)
    else:
        target = b.target_ids.clone()
        ws = None
    kv_len = b.kv_len.clone()
    new_len = kv_len if in_place else torch.full_like(kv_len, -7)
    ems.ems_greedy_accept_append(logits, target, b.input_ids, b.cu_seqlens, accepted, accepted_cu, out_tokens,
                                 [kn for kn, _ in news], [vn for _, vn in news],
                                 [ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows) for kc, vc in caches],
                                 b.kv_start, kv_len, new_len, workspace=ws)
    torch.cuda.synchronize()
    return target[:b.T], accepted, accepted_cu, out_tokens, new_len


def check(b_cpu, n_layers=1, use_logits=True, in_place=False):
    b = to_device(b_cpu)
    g = torch.Generator().manual_seed(4242)
    # layer 0 is the batch's own K/V; further layers get other new rows and the same cache contents
    news_cpu = [(b_cpu.k_new, b_cpu.v_new)]
    for _ in range(n_layers - 1):
        news_cpu.append((torch.randn(b_cpu.k_new.shape, generator=g).to(b_cpu.dtype),
                         torch.randn(b_cpu.v_new.shape, generator=g).to(b_cpu.dtype)))
    news = [(kn.cuda(), vn.cuda()) for kn, vn in news_cpu]
    caches = [(b.k_cache.clone(), b.v_cache.clone()) for _ in range(n_layers)]
    tgt, acc, acc_cu, toks, new_len = fused(b, caches, news, use_logits=use_logits and b_cpu.logits is not None,
                                            in_place=in_place)
    # the oracle
    x, o_acc, o_cu, o_toks = oracle_accept(b_cpu, use_logits=use_logits)
    assert np.array_equal(tgt.cpu().numpy(), x)
    assert np.array_equal(acc.cpu().numpy(), o_acc)
    assert np.array_equal(acc_cu.cpu().numpy(), o_cu)
    assert np.array_equal(toks.cpu().numpy()[:o_cu[-1]], o_toks)
    for l in range(n_layers):
        okc, ovc = bits(b_cpu.k_cache).copy(), bits(b_cpu.v_cache).copy()
        o_len = oracle.kv_append(okc, ovc, b_cpu.row_stride, b_cpu.head_stride, bits(news_cpu[l][0]),
                                 bits(news_cpu[l][1]), b_cpu.cu_seqlens.numpy(), o_acc,
                                 b_cpu.kv_start.numpy(), b_cpu.kv_len.numpy(), b_cpu.H, b_cpu.D)
        assert np.array_equal(new_len.cpu().numpy(), o_len)
        assert np.array_equal(bits(caches[l][0]), okc) and np.array_equal(bits(caches[l][1]), ovc), "layer %d" % l
    # the two separate calls give the same bits
    acc2 = torch.full_like(acc, -7)
    cu2 = torch.full_like(acc_cu, -7)
    toks2 = torch.full_like(toks, -7)
    logits = b.logits if (use_logits and b_cpu.logits is not None) else None
    tgt2 = torch.full((max(b.T, 1),), -7, dtype=torch.int32, device="cuda") if logits is not None else b.target_ids.clone()
    ws = torch.empty(max(8, ems.ems_accept_workspace_bytes(b.T, b.V)), dtype=torch.uint8, device="cuda") if logits is not None else None
    ems.ems_greedy_accept(logits, tgt2, b.input_ids, b.cu_seqlens, acc2, cu2, toks2, workspace=ws)
    caches2 = [(b.k_cache.clone(), b.v_cache.clone()) for _ in range(n_layers)]
    len2 = torch.full_like(b.kv_len, -7)
    ems.ems_kv_append([kn for kn, _ in news], [vn for _, vn in news],
                      [ems.kv_cache(kc, vc, b.row_stride, b.head_stride, b.rows) for kc, vc in caches2],
                      b.cu_seqlens, acc2, b.kv_start, b.kv_len, len2)
    torch.cuda.synchronize()
    assert torch.equal(tgt2[:b.T], tgt) and torch.equal(acc2, acc) and torch.equal(cu2, acc_cu)
    assert torch.equal(toks2[:int(o_cu[-1])], toks[:int(o_cu[-1])]) and torch.equal(len2, new_len)
    for l in range(n_layers):
        assert np.array_equal(bits(caches2[l][0]), bits(caches[l][0])) and np.array_equal(bits(caches2[l][1]), bits(caches[l][1]))


def test_tiny_config_both_layouts():
    check(make_config(1))
    check(make_config(1, layout=HEAD_MAJOR))
    check(make_config(1), use_logits=False)


@pytest.mark.parametrize("dtype,D,layout,n_layers", [(torch.float16, 128, TOKEN_MAJOR, 1), (torch.bfloat16, 80, HEAD_MAJOR, 3),
                                                      (torch.bfloat16, 64, TOKEN_MAJOR, 2)])
def test_ragged_batch_with_empty_samples_and_long_runs(dtype, D, layout, n_layers):
    kv = [0, 1, 31, 32, 33, 64, 100, 257, 5, 700, 12, 3, 3]
    k = [64, 17, 0, 48, 1, 32, 63, 16, 0, 20, 2, 1, 9]
    b = make_batch(kv, k, H=3, D=D, dtype=dtype, seed=610, capacity=800, layout=layout, V=4099, match_p=0.95)
    assert b.logits is not None
    check(b, n_layers=n_layers)
    check(b, n_layers=n_layers, use_logits=False)


def test_more_than_sixty_four_rows_in_a_sample():
    """Acceptance has no limit on the rows of a sample (attention has): 130 and 200 rows, nearly all
    drafts right, so the leading run crosses the 64-row passes of the counting workgroup."""
    b = make_batch([5, 9, 2, 7], [130, 1, 200, 64], H=1, D=64, dtype=torch.float16, seed=611, capacity=256,
                   vocab_for_ids=50, match_p=0.995)
    _, o_acc, _, _ = oracle_accept(b, use_logits=False)
    assert o_acc.max() > 64
    check(b, use_logits=False)
    b.input_ids[1:130] = b.target_ids[0:129]        # every draft of sample 0 right: all 130 accepted
    _, o_acc, _, _ = oracle_accept(b, use_logits=False)
    assert o_acc[0] == 130
    check(b, use_logits=False)


def test_lengths_in_place_and_many_layers_take_the_two_call_path():
    b = make_batch([40, 3, 90], [5, 2, 7], H=2, D=64, dtype=torch.bfloat16, seed=612, capacity=128, V=777)
    check(b, n_layers=2, in_place=True)
    check(b, n_layers=33)


def test_full_size_config_4():
    check(make_config(4))
    check(make_config(3, layout=HEAD_MAJOR))
