"""Side modes of bench.py (each replaces the headline run and prints its own JSON object):
the dynamic-batching workload, the sweep over rows per sample at 512 cached tokens (the shape
of the paper's Fig. 5), the paper's own launch shape (Appendix D: one work item per head and
packed token) against the shared-K/V call, the matrix-core vs vector-ALU sweep, and the plain
device copy that calibrates rocprofv3's FETCH_SIZE / WRITE_SIZE.  Run through
`python bench.py --<mode>`; inputs are seeded and synthetic as in bench.py."""
import time

from bench import attention_algorithmic_bytes


def copy_calibration(mib):
    import torch
    src = torch.ones(mib << 20, dtype=torch.uint8, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    return {"copy_calibration_bytes": src.numel(), "launches": 5}


def dynamic_batching_bench(args, B=64, H=32, D=128, n_steps=120, region=4096):
    """Dynamic batching (the paper's Sec. 4.4 proposal, not implemented there): every slot of the
    batch serves a stream of samples; when its sample finishes, the slot brings no rows for one
    step (k_i = 0) and then starts a new sample in a FRESH region of the arena with a new cached
    length.  Per-sample start locations make this free: nothing is moved or padded.  The
    lengths advance on the device; retirements follow a fixed seeded schedule, so the host
    never reads anything back.  Reports the throughput of the drifting batch next to that of
    the same loop with no retirements."""
    import numpy as np
    import torch
    import paper_2405_07542_amd as ems
    from workloads import make_batch
    dev = "cuda:0"
    dtype = torch.bfloat16

    def run(retire):
        rng = np.random.default_rng(77)
        lifetimes = rng.integers(8, 40, size=(B, 64))          # steps each successive sample of a slot lives
        prompt = rng.integers(256, 2049, size=(B, 64))         # its cached length when it enters
        n_regions = B * (2 + n_steps // 8) if retire else B
        rows = n_regions * region
        base = make_batch([1], [1], H=H, D=D, dtype=dtype, seed=78, rows=8, device=dev)
        # the arena's content does not matter for timing; it must only be finite
        k_arena = torch.randn(rows * H * D // 2, device=dev, dtype=torch.float32).view(torch.int16).view(dtype)
        k_arena = torch.nan_to_num(k_arena, nan=0.0, posinf=1.0, neginf=-1.0).clamp_(-4, 4)
        v_arena = k_arena.roll(12345)
        cache = ems.kv_cache(k_arena, v_arena, H * D, D, rows)
        kv_start = torch.arange(B, dtype=torch.int32, device=dev) * region
        kv_len = torch.tensor(prompt[:, 0], dtype=torch.int32, device=dev)
        next_region, gen_idx = B, np.zeros(B, dtype=np.int64)
        left = lifetimes[:, 0].copy()
        plan = []                                               # per step: device tensors + host-planned updates
        for step in range(n_steps):
            k = [int(rng.integers(1, 12)) if left[s] > 0 else 0 for s in range(B)]
            T = sum(k)
            cu = torch.tensor(np.concatenate([[0], np.cumsum(k)]), dtype=torch.int32, device=dev)
            q = torch.randn((T, H, D), device=dev, dtype=torch.float32).to(dtype)
            ids = torch.randint(0, 50272, (T,), device=dev, dtype=torch.int32)
            tgt = ids.roll(-1).clone()
            tgt[torch.rand(T, device=dev) > 0.7] += 1           # drafts agree with probability 0.7
            refill = []
            for s in range(B):
                if left[s] > 0:
                    left[s] -= 1
                    if not retire:
                        left[s] = 1
                elif retire:                                     # the slot sat out this step: new sample next step
                    gen_idx[s] += 1
                    refill.append((s, next_region * region, int(prompt[s, gen_idx[s] % 64])))
                    left[s] = lifetimes[s, gen_idx[s] % 64]
                    next_region += 1
            assert next_region <= n_regions
            upd = None
            if refill:
                idx = torch.tensor([r[0] for r in refill], device=dev)
                upd = (idx, torch.tensor([r[1] for r in refill], dtype=torch.int32, device=dev),
                       torch.tensor([r[2] for r in refill], dtype=torch.int32, device=dev))
            plan.append((T, cu, q, q.roll(1, 0), q.roll(2, 0), ids, tgt, upd, max(k)))
        ws = torch.empty(ems.ems_attention_workspace_bytes(B, 16 * B, H, D, region), dtype=torch.uint8, device=dev)
        out = torch.empty((16 * B, H, D), dtype=dtype, device=dev)
        accepted = torch.empty(B, dtype=torch.int32, device=dev)
        accepted_cu = torch.empty(B + 1, dtype=torch.int32, device=dev)
        total_acc = torch.zeros((), dtype=torch.int64, device=dev)
        start0, len0 = kv_start.clone(), kv_len.clone()

        def loop(count):
            kv_start.copy_(start0)
            kv_len.copy_(len0)
            for T, cu, q, kn, vn, ids, tgt, upd, max_k in plan:
                ems.ems_verify_attention(q, kn, vn, cache, cu, kv_start, kv_len, out[:T], max_k=16,
                                         max_kv_len=region - 16, scale=D ** -0.5, workspace=ws)
                ems.ems_greedy_accept(None, tgt, ids, cu, accepted, accepted_cu, None)
                ems.ems_kv_append([kn], [vn], [cache], cu, accepted, kv_start, kv_len, kv_len)
                if count:
                    total_acc.add_(accepted_cu[-1])
                if upd is not None:                              # admit the new samples (device-side writes)
                    kv_start[upd[0]] = upd[1]
                    kv_len[upd[0]] = upd[2]
        loop(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        loop(True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        rows_total = sum(p[0] for p in plan)
        return {"ms_per_step": round(dt * 1e3 / n_steps, 4), "verified_tokens_per_s": round(int(total_acc) / dt, 1),
                "query_tokens_per_s": round(rows_total / dt, 1), "regions_used": int(next_region),
                "mean_live_samples": round(float(np.mean([sum(1 for x in np.diff(p[1].cpu().numpy()) if x > 0)
                                                         for p in plan])), 1)}

    return {"mode": "dynamic batching, 1 layer, B=%d slots, %d steps, bf16, rows per live sample U[1,11]" % (B, n_steps),
            "static_batch": run(False), "dynamic_batch": run(True)}


def sweep_k():
    """Attention-call time as the number of rows per sample grows, 512 cached tokens per sample
    (the paper's Fig. 5 measures the whole model this way: 16.6 ms at 1 token vs 22.6 ms at 5
    tokens per sample, B=16, one A100).  Here only the attention path is timed."""
    import torch
    import paper_2405_07542_amd as ems
    from workloads import make_batch
    dev = "cuda:0"
    rows = []
    for B in (4, 16):
        for k in range(1, 9):
            sets = []
            for v in range(4):
                b = make_batch([512] * B, [k] * B, H=32, D=128, dtype=torch.float16, seed=900 + 10 * k + v,
                               capacity=1024, device=dev)
                ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len),
                                 dtype=torch.uint8, device=dev)
                sets.append((b, ws, torch.empty_like(b.q),
                             ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows)))

            def call(s):
                b, ws, out, cache = s
                ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                         max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
            for i in range(8):
                call(sets[i % 4])
            torch.cuda.synchronize()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 200
            ev0.record()
            for i in range(reps):
                call(sets[i % 4])
            ev1.record()
            torch.cuda.synchronize()
            rows.append({"B": B, "rows_per_sample": k, "attention_call_us": round(ev0.elapsed_time(ev1) / reps * 1e3, 2)})
    return {"sweep": "attention call time vs rows per sample, kv_len=512, H=32, D=128, fp16", "results": rows}


def per_token_rows_as_samples(b):
    """Index arrays that present every packed row of `b` as a sample of its own (k = 1) whose cache is
    its real sample's cache plus the new rows before it -- which must already have been written
    through to rows kv_len + j.  This is the paper's formulation (Sec. 3.2 with the grid of Appendix
    D): K/V of all new tokens stored first, then one work item per (head, token)."""
    import torch
    k = (b.cu_seqlens[1:] - b.cu_seqlens[:-1]).long()
    sample = torch.repeat_interleave(torch.arange(b.B, device=k.device), k)
    pos = torch.arange(b.T, device=k.device) - b.cu_seqlens[:-1].long()[sample]
    cu = torch.arange(b.T + 1, dtype=torch.int32, device=k.device)
    kv_start = b.kv_start[sample].to(torch.int32)
    kv_len = (b.kv_len.long()[sample] + pos).to(torch.int32)
    return cu, kv_start.contiguous(), kv_len.contiguous()


def per_token_grid(args, reps=60):
    import torch
    import paper_2405_07542_amd as ems
    from workloads import make_config
    dev = "cuda:0"
    sets = []
    for v in range(3):
        b = make_config(4, device=dev, layout=args.layout, with_logits=False, variant=v)
        cache = ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows)
        ws = torch.empty(ems.ems_attention_workspace_bytes(b.T, b.T, b.H, b.D, b.max_kv_len + b.max_k),
                         dtype=torch.uint8, device=dev)
        out = torch.empty_like(b.q)
        # paper order: the new rows' K/V enter the cache first (one write-through call), then ...
        ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                 max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws,
                                 write_through=True)
        shared_out = out.clone()
        sets.append((b, cache, ws, out, per_token_rows_as_samples(b), shared_out))
    torch.cuda.synchronize()

    def shared(s):
        b, cache, ws, out, _, _ = s
        ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                 max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)

    def per_token(s):
        b, cache, ws, out, (cu, ks, kl), _ = s
        ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, cu, ks, kl, out, max_k=1,
                                 max_kv_len=b.max_kv_len + b.max_k, scale=b.scale, workspace=ws)

    res = {}
    for name, fn in (("shared_kv", shared), ("per_token", per_token)):
        for i in range(6):
            fn(sets[i % 3])
        torch.cuda.synchronize()
        ems.ems_profile_enable(reps)
        for i in range(reps):
            fn(sets[i % 3])
        torch.cuda.synchronize()
        ms, n = ems.ems_profile_read()
        ems.ems_profile_enable(0)
        res[name + "_kernel_us"] = round(ms / n * 1e3, 1)
    # the two formulations agree on every output row (same tolerance as against the oracle)
    worst = 0.0
    for s in sets:
        per_token(s)
        torch.cuda.synchronize()
        worst = max(worst, float((s[3].float() - s[5].float()).abs().max()))
    b = sets[0][0]
    rows = float(sum(s[0].T for s in sets)) / len(sets)
    res.update({"mode": "paper's launch shape (one work item per head and packed token) vs shared K/V, config 4 attention",
                "layout": args.layout, "packed_rows": rows, "max_abs_difference_of_outputs": worst,
                "slowdown": round(res["per_token_kernel_us"] / res["shared_kv_kernel_us"], 2)})
    return res


def sweep_variants(B=64, L=2048, ks=(1, 2, 4, 6, 8, 12, 16, 32, 64)):
    """The two formulations of the attention kernel on one HBM-bound shape (config 4's batch and
    mean cache length, every sample with the same k): kernel time from HIP events around the main
    kernel, and the algorithmic bandwidth it amounts to.  The matrix-core path costs the same for
    any k <= 16, ~10 % more for 17..32 (the wider kernel) and ~1.6x for 33..64 (still one stream of the
    cache, but the wave is then bound by its own arithmetic);
    the vector-ALU path pays per row."""
    import torch
    import paper_2405_07542_amd as ems
    from workloads import make_batch
    dev = "cuda:0"
    out_rows = []
    for k in ks:
        sets = []
        for v in range(3):
            b = make_batch([L] * B, [k] * B, H=32, D=128, dtype=torch.bfloat16, seed=700 + 10 * k + v,
                           capacity=L + 16, device=dev)
            ws = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len),
                             dtype=torch.uint8, device=dev)
            sets.append((b, ws, torch.empty_like(b.q),
                         ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows)))
        alg = attention_algorithmic_bytes(sets[0][0], 2)
        row = {"rows_per_sample": k, "algorithmic_bytes": alg}
        for name, variant in (("mfma", ems.EMS_ATTN_MFMA), ("valu", ems.EMS_ATTN_VALU)):
            if variant == ems.EMS_ATTN_VALU and k > 16:      # beyond 16 rows only the matrix-core kernels exist
                continue
            ems.ems_set_attention_variant(variant)

            def call(s):
                b, ws, out, cache = s
                ems.ems_verify_attention(b.q, b.k_new, b.v_new, cache, b.cu_seqlens, b.kv_start, b.kv_len, out,
                                         max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale, workspace=ws)
            for i in range(6):
                call(sets[i % 3])
            torch.cuda.synchronize()
            reps = 60
            ems.ems_profile_enable(reps)
            for i in range(reps):
                call(sets[i % 3])
            torch.cuda.synchronize()
            ms, n = ems.ems_profile_read()
            ems.ems_profile_enable(0)
            us = ms / n * 1e3
            row[name + "_kernel_us"] = round(us, 2)
            row[name + "_gbs"] = round(alg / (us * 1e-6) / 1e9, 1)
        ems.ems_set_attention_variant(ems.EMS_ATTN_MFMA)
        out_rows.append(row)
        del sets
        torch.cuda.empty_cache()
    return {"sweep": "attention kernel time, matrix-core vs vector-ALU formulation, B=%d, kv_len=%d, H=32, D=128, bf16"
                     % (B, L), "results": out_rows}
