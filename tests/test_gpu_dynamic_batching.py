"""Dynamic batching (the paper's Sec. 4.4 / Limitations: replace a finished sample by a new one
instead of waiting for the whole batch): slots retire (k_i = 0 for a step) and are refilled
with a new sample that gets a fresh region of the arena (new kv_start, new cached length).
The library needs nothing new for it -- per-sample start locations are the method -- so this
checks, against the oracle carried along, that ragged verification keeps working while the
set of samples, their regions and their length mix drift from step to step."""
import numpy as np
import pytest
import torch

import oracle
from workloads import arena_view, bits, make_batch
from helpers import hip_accept, hip_attention, oracle_accept, to_device

pytestmark = pytest.mark.gpu


def test_slots_retire_and_are_refilled_in_fresh_regions():
    import paper_2405_07542_amd as ems
    rng = np.random.default_rng(200)
    B, H, D, rows = 6, 4, 128, 2400
    dtype = torch.float16
    region = 200                                   # rows handed out per new sample
    next_free = 0
    starts = np.zeros(B, dtype=np.int32)
    lens = np.zeros(B, dtype=np.int32)
    alive = np.zeros(B, dtype=bool)
    budget = np.zeros(B, dtype=np.int32)           # tokens still to generate per slot

    seed_batch = make_batch([1], [1], H=H, D=D, dtype=dtype, seed=201, rows=rows)
    g_k = seed_batch.k_cache.cuda()                # arena full of NaN sentinels (+ one unused row)
    g_v = seed_batch.v_cache.cuda()
    o_k, o_v = bits(seed_batch.k_cache).copy(), bits(seed_batch.v_cache).copy()
    rs, hs = seed_batch.row_stride, seed_batch.head_stride

    def admit(slot, step):
        """A new sample enters `slot`: fresh region, its prompt's K/V written as a prefill would."""
        nonlocal next_free
        L = int(rng.integers(5, 120))
        starts[slot], lens[slot], alive[slot] = next_free, L, True
        budget[slot] = int(rng.integers(4, 25))
        next_free += region
        assert next_free <= rows
        fill = make_batch([L], [1], H=H, D=D, dtype=dtype, seed=300 + 10 * step + slot, rows=L + 1)
        for dst_g, dst_o, src in ((g_k, o_k, fill.k_cache), (g_v, o_v, fill.v_cache)):
            rows_src = arena_view(src, fill.layout, L + 1, H, D)[:L]
            arena_view(dst_g, seed_batch.layout, rows, H, D)[starts[slot]:starts[slot] + L] = rows_src.cuda()
            dst_o.reshape(rows, H, D)[starts[slot]:starts[slot] + L] = bits(rows_src)

    for slot in range(B):
        admit(slot, -1)
    retired_total = 0
    for step in range(14):
        # finished slots sit out one step with k_i = 0, then get a new sample
        k = [int(rng.integers(1, 9)) if alive[s] else 0 for s in range(B)]
        print("step", step, "k", k, "lens", lens.tolist(), "starts", starts.tolist(), flush=True)
        b_cpu = make_batch(lens.tolist(), k, H=H, D=D, dtype=dtype, seed=400 + step, kv_start=starts.tolist(),
                           rows=rows, vocab_for_ids=50, match_p=0.7)
        b = to_device(b_cpu)
        ems.ems_validate_inputs(b.cu_seqlens, b.kv_start, b.kv_len, T=b.T, max_k=16, max_kv_len=region,
                                rows=rows)
        got = hip_attention(b, out_dtype=torch.float32, k_cache=g_k, v_cache=g_v, max_kv_len=region)
        want = oracle.verify_attention(bits(b_cpu.q), bits(b_cpu.k_new), bits(b_cpu.v_new), o_k, o_v, rs, hs,
                                       b_cpu.cu_seqlens.numpy(), starts, lens, H, D, b_cpu.scale, dtype)
        assert np.isfinite(got.cpu().numpy()).all()
        assert np.abs(got.double().cpu().numpy() - want).max() <= 2e-3, "step %d" % step
        _, acc, acc_cu, _ = hip_accept(b, use_logits=False)
        _, o_acc, o_cu, _ = oracle_accept(b_cpu, use_logits=False)
        assert np.array_equal(acc.cpu().numpy(), o_acc) and np.array_equal(acc_cu.cpu().numpy(), o_cu)
        assert all((a == 0) == (kk == 0) for a, kk in zip(o_acc, k))
        g_len = b.kv_len.clone()
        ems.ems_kv_append([b.k_new], [b.v_new], [ems.kv_cache(g_k, g_v, rs, hs, rows)], b.cu_seqlens, acc,
                          b.kv_start, g_len, g_len)
        lens[:] = oracle.kv_append(o_k, o_v, rs, hs, bits(b_cpu.k_new), bits(b_cpu.v_new),
                                   b_cpu.cu_seqlens.numpy(), o_acc, starts, lens, H, D)
        torch.cuda.synchronize()
        assert np.array_equal(g_len.cpu().numpy(), lens)
        assert np.array_equal(bits(g_k), o_k) and np.array_equal(bits(g_v), o_v)
        for s in range(B):
            if alive[s]:
                budget[s] -= o_acc[s]
                if budget[s] <= 0:
                    alive[s] = False               # retires: next step it brings no rows
                    retired_total += 1
            elif next_free + region <= rows:
                admit(s, step)                     # the slot is refilled in a fresh region
    assert retired_total >= 4 and next_free > B * region
