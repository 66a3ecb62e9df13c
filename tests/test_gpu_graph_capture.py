"""The three calls of a verification step allocate nothing and never synchronise, so a step
can be captured into a HIP graph and replayed.  Every replay (with eager work and
synchronisations in between) must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

import paper_2405_07542_amd as ems
from workloads import make_config
from helpers import to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("config,k_range", [(2, None), (3, None), (3, (17, 32))],
                         ids=["config2", "config3-merge-in-lds", "config3-wide-kernel"])
def test_a_captured_step_replays_bit_identically(config, k_range):
    """config 2: short walks, every partial through the workspace; config 3: the in-workgroup
    merge of partials (a barrier and LDS hand-over inside the kernel); 17..32 rows per sample:
    the wide kernel, which asks for more than 64 KiB of LDS (raised at the eager warm-up call)."""
    b = to_device(make_config(config, k_range=k_range))
    dev = b.q.device
    cache_k, cache_v = b.k_cache.clone(), b.v_cache.clone()
    cache = ems.kv_cache(cache_k, cache_v, b.row_stride, b.head_stride, b.rows)
    ws_attn = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len),
                          dtype=torch.uint8, device=dev)
    ws_acc = torch.empty(ems.ems_accept_workspace_bytes(b.T, b.V), dtype=torch.uint8, device=dev)
    out = torch.zeros((b.T, b.H, b.D), dtype=b.dtype, device=dev)
    target = torch.zeros(b.T, dtype=torch.int32, device=dev)
    accepted = torch.zeros(b.B, dtype=torch.int32, device=dev)
    accepted_cu = torch.zeros(b.B + 1, dtype=torch.int32, device=dev)
    out_tokens = torch.zeros(b.T, dtype=torch.int32, device=dev)
    new_len = torch.zeros(b.B, dtype=torch.int32, device=dev)

    def step():
        ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                 max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws_attn)
        ems.ems_greedy_accept(b.logits, target, b.input_ids, b.cu_seqlens, accepted, accepted_cu, out_tokens,
                              workspace=ws_acc)
        ems.ems_kv_append([b.k_new], [b.v_new], [cache], b.cu_seqlens, accepted, b.kv_start, b.kv_len, new_len)

    outputs = (out, target, accepted, accepted_cu, out_tokens, new_len, cache_k, cache_v)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in outputs]

    def clear():
        for t in (out, target, accepted, accepted_cu, out_tokens, new_len):
            t.zero_()
        cache_k.copy_(b.k_cache)
        cache_v.copy_(b.v_cache)

    step()
    eager = snapshot()
    assert int(eager[3][-1]) >= b.B                      # something was accepted and appended

    clear()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                           # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(3):
        clear()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for name, g, e in zip(("out", "target", "accepted", "accepted_cu", "out_tokens", "new_len", "k", "v"),
                              got, eager):
            assert torch.equal(g.view(torch.int16) if g.dtype.is_floating_point else g,
                               e.view(torch.int16) if e.dtype.is_floating_point else e), (replay, name)
        # eager work of the program itself between replays
        step()
        torch.cuda.synchronize()
