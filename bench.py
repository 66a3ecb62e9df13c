#!/usr/bin/env python3
"""Benchmark of the ragged verification step (EMS-SD hot path) on one MI355X.

A step = one pass of the whole path over one synthetic batch that is already
resident in HBM:  ems_verify_attention (one OPT-6.7b-shaped layer) ->
ems_greedy_accept (arg-max over [T, 50272] logits, acceptance, prefix sum) ->
ems_kv_append (accepted rows into the per-sample caches).

Prints ONE JSON line: verified tokens/s (sum of accepted tokens / step time), the
roofline figures of the dominant kernel (the main attention kernel, timed with HIP
events recorded around it on its own stream inside the timed region) and the
oracle's throughput on the host cores as a CPU baseline.

    python bench.py [--steps K] [--warmup W] [--config 2|3|4|5] [--layout token_major|head_major]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=4, help="BASELINE config number (2..5)")
    ap.add_argument("--layout", default="token_major", choices=["token_major", "head_major"])
    ap.add_argument("--sets", type=int, default=0,
                    help="independent buffer sets rotated between steps so that no step finds its K/V in the "
                         "last-level cache; 0 (default) = as many as make the rotated K/V at least 2 GiB, "
                         "between 3 and 16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-logits", action="store_true", help="skip the [T,V] arg-max (ids given)")
    ap.add_argument("--breakdown", action="store_true", help="also time each call on its own")
    ap.add_argument("--no-ablation", action="store_true", help="skip the padded (vanilla) ablation")
    ap.add_argument("--write-through", action="store_true",
                    help="paper-order variant: attention also stores the new rows' K/V, append only advances lengths")
    ap.add_argument("--attention-variant", default="mfma", choices=["mfma", "valu"],
                    help="arithmetic units of the attention kernel's contractions: matrix cores (default) "
                         "or the vector ALU (a measurement aid; see ems_set_attention_variant)")
    ap.add_argument("--tree-rows", type=int, default=0, metavar="N",
                    help="with --tree: every sample brings U{N/2..N} rows (tree nodes) instead of the "
                         "config's 1..11 (N <= 64; above 16 the attention call runs the wide kernel)")
    ap.add_argument("--tree", default=None, choices=["random", "wide", "star", "chain"],
                    help="tree-structured verification: the same config with every sample's new rows arranged "
                         "as a token tree of this shape (ems_tree_verify_attention / ems_tree_accept / "
                         "ems_kv_append_rows instead of the three causal calls)")
    ap.add_argument("--layers", type=int, default=32, help="config 5 only: layers of the verify loop")
    ap.add_argument("--loop-steps", type=int, default=20, help="config 5 only: successive verify steps")
    ap.add_argument("--dynamic-batching", action="store_true",
                    help="instead of the bench: a 1-layer verify loop in which finished samples are replaced "
                         "by new ones in fresh cache regions (the paper's proposed dynamic batching), B=64")
    ap.add_argument("--sweep-k", action="store_true",
                    help="instead of the bench: attention time vs rows per sample at 512 cached tokens "
                         "(the shape of the paper's Fig. 5), B in {4, 16}, k = 1..8")
    ap.add_argument("--per-token-grid", action="store_true",
                    help="instead of the bench: the paper's own launch shape (Appendix D: one work item per head and "
                         "packed token, every token streaming its sample's whole cache) emulated on config 4 by "
                         "writing the new rows through and calling the same kernel with every packed row as a "
                         "sample of its own; reports the attention time next to the shared-K/V call")
    ap.add_argument("--sweep-variants", action="store_true",
                    help="instead of the bench: attention kernel time of the matrix-core and the vector-ALU "
                         "formulation vs rows per sample, B=64, 2048 cached tokens each, bf16")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="instead of the bench: run a plain device copy of MIB MiB five times "
                         "(the known-size kernel that scales rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def device_memory_figures():
    """What the runtime reports for the card's memory (clock in kHz, bus width in bits), as
    context beside the published 8 TB/s that `peak` uses; None where it reports nothing."""
    import torch
    import paper_2405_07542_amd as ems
    props = torch.cuda.get_device_properties(0)
    clock_khz, width_bits = ems.ems_device_memory_figures()
    return {"name": props.name, "memory_clock_khz": clock_khz, "memory_bus_width_bits": width_bits,
            "total_memory_gib": round(props.total_memory / 2**30, 1)}


def measured_read_ceiling(buf, reps=10):
    """GB/s of the library's read-only streaming kernel over `buf` (a K arena: far larger
    than the caches), HIP events on the current stream."""
    import torch
    import paper_2405_07542_amd as ems
    sink = torch.zeros(1, dtype=torch.int32, device=buf.device)
    flat = buf.view(-1)
    for _ in range(3):
        ems.ems_stream_read_probe(flat, sink)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(reps):
        ems.ems_stream_read_probe(flat, sink)
    ev1.record()
    torch.cuda.synchronize()
    nbytes = flat.numel() * flat.element_size()
    return round(nbytes / (ev0.elapsed_time(ev1) / reps * 1e-3) / 1e9, 1)


def attention_algorithmic_bytes(b, out_elem_bytes):
    """What the method itself must move per layer: each cached K/V row once, the new
    K/V rows, Q and O once, and the index arrays."""
    e = 2
    kv_len = b.kv_len.cpu().tolist()
    k = (b.cu_seqlens[1:] - b.cu_seqlens[:-1]).cpu().tolist()
    hd = b.H * b.D
    total = 0
    for L, kk in zip(kv_len, k):
        if kk == 0:
            continue
        total += 2 * L * hd * e + 2 * kk * hd * e + kk * hd * e + kk * hd * out_elem_bytes
    return total + (3 * b.B + 1) * 4


def read_traffic(workload_key):
    """HBM bytes per launch of the main attention kernel from a committed rocprofv3 --pmc
    summary (FETCH_SIZE + WRITE_SIZE, calibrated against a copy kernel), if one exists."""
    path = os.path.join(ROOT, "profiles", "verify_attention_traffic.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 2 and parts[0] == workload_key:
            try:
                return float(parts[1])
            except ValueError:
                return None
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (--gpus 1); the path would shard by sample or by "
              "head with no exchange between GPUs, so the figure for N GPUs is N times this one", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2405_07542_amd as ems
    from workloads import make_config, CONFIG_NAMES

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    ems.lib()     # fail loudly if the HIP library is missing
    ems.ems_set_attention_variant(ems.EMS_ATTN_VALU if args.attention_variant == "valu" else ems.EMS_ATTN_MFMA)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": src.numel(), "launches": 5}))
        return
    n = args.config
    with_logits = not args.no_logits
    if args.tree and (args.write_through or args.attention_variant == "valu" or n == 5):
        sys.exit("--tree runs the matrix-core kernel with the gathered append on configs 2-4 only")
    if args.tree_rows and (not args.tree or not 1 <= args.tree_rows <= 64):
        sys.exit("--tree-rows N goes with --tree and 1 <= N <= 64")
    if args.per_token_grid:
        print(json.dumps(per_token_grid(args)), flush=True)
        return
    if args.sweep_variants:
        print(json.dumps(sweep_variants()), flush=True)
        return
    if args.sweep_k:
        print(json.dumps(sweep_k()), flush=True)
        return
    if args.dynamic_batching:
        print(json.dumps(dynamic_batching_bench(args)), flush=True)
        return
    if n == 5:
        print(json.dumps(verify_loop_bench(args, with_logits)), flush=True)
        return

    sets = []
    n_sets = args.sets
    v = 0
    while n_sets == 0 or v < n_sets:
        b = make_config(n, device=dev, layout=args.layout, with_logits=with_logits, variant=v,
                        k_range=(max(1, args.tree_rows // 2), args.tree_rows) if args.tree_rows else None)
        if n_sets == 0:      # sized from the first draw: 256 MB of Infinity Cache must not hold a whole rotation
            n_sets = int(min(16, max(3, -(-(2 << 30) // max(1, attention_algorithmic_bytes(b, 2))))))
        if args.tree:
            from workloads import grow_trees
            b = grow_trees(b, 4242 + v, match_p=0.7, shape=args.tree)
        ws_attn = torch.empty(ems.ems_attention_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len),
                              dtype=torch.uint8, device=dev)
        ws_acc = torch.empty(max(8, ems.ems_accept_workspace_bytes(b.T, b.V)), dtype=torch.uint8, device=dev)
        st = dict(
            b=b, ws_attn=ws_attn, ws_acc=ws_acc,
            cache=ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows),
            out=torch.empty((b.T, b.H, b.D), dtype=b.dtype, device=dev),
            target=torch.empty(b.T, dtype=torch.int32, device=dev) if with_logits else b.target_ids.clone(),
            accepted=torch.empty(b.B, dtype=torch.int32, device=dev),
            accepted_cu=torch.empty(b.B + 1, dtype=torch.int32, device=dev),
            out_tokens=torch.empty(b.T, dtype=torch.int32, device=dev),
            accepted_rows=torch.empty(b.T, dtype=torch.int32, device=dev),
            # the lengths are NOT advanced between timed steps, so every step does the same work
            new_len=torch.empty(b.B, dtype=torch.int32, device=dev))
        sets.append(st)
        v += 1
    torch.cuda.synchronize()

    def attention(st):
        b = st["b"]
        if args.tree:
            ems.ems_tree_verify_attention(b.q, b.k_new, b.v_new, st["cache"], b.cu_seqlens, b.parent, b.kv_start,
                                          b.kv_len, st["out"], max_k=b.max_k, max_kv_len=b.max_kv_len,
                                          scale=b.scale, workspace=st["ws_attn"])
            return
        ems.ems_verify_attention(b.q, b.k_new, b.v_new, st["cache"], b.cu_seqlens, b.kv_start, b.kv_len,
                                 st["out"], max_k=b.max_k, max_kv_len=b.max_kv_len, scale=b.scale,
                                 workspace=st["ws_attn"], write_through=args.write_through)

    def accept(st):
        b = st["b"]
        if args.tree:
            ems.ems_tree_accept(b.logits if with_logits else None, st["target"], b.input_ids, b.parent,
                                b.cu_seqlens, st["accepted"], st["accepted_cu"], st["out_tokens"],
                                st["accepted_rows"], workspace=st["ws_acc"])
            return
        ems.ems_greedy_accept(b.logits if with_logits else None, st["target"], b.input_ids, b.cu_seqlens,
                              st["accepted"], st["accepted_cu"], st["out_tokens"], workspace=st["ws_acc"])

    def append(st):
        b = st["b"]
        if args.tree:
            ems.ems_kv_append_rows([b.k_new], [b.v_new], [st["cache"]], st["accepted_rows"], st["accepted_cu"],
                                   b.kv_start, b.kv_len, st["new_len"])
            return
        if args.write_through:
            ems.ems_kv_advance(b.kv_len, st["accepted"], st["new_len"])
            return
        ems.ems_kv_append([b.k_new], [b.v_new], [st["cache"]], b.cu_seqlens, st["accepted"], b.kv_start,
                          b.kv_len, st["new_len"])

    def step(st):
        attention(st)
        accept(st)
        append(st)

    # Set-up, untimed: every buffer set is run once, so that its accepted counts (the numerator
    # of `value`) exist however few steps are timed, and so that no set is touched for the first
    # time inside the timed region (the first pass over a fresh 2 GiB arena costs ~90 us more);
    # then the read ceiling that the roofline object quotes as context.
    for st in sets:
        step(st)
    torch.cuda.synchronize()
    ceiling = measured_read_ceiling(sets[0]["b"].k_cache)

    for w in range(args.warmup):
        step(sets[w % len(sets)])
    torch.cuda.synchronize()

    ems.ems_profile_enable(args.steps)
    t0 = time.perf_counter()
    for s in range(args.steps):
        step(sets[s % len(sets)])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    attn_ms_total, attn_launches = ems.ems_profile_read()
    ems.ems_profile_enable(0)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    accepted_per_step = float(np.mean([int(st["accepted_cu"][-1]) for st in sets]))
    rows_per_step = float(np.mean([st["b"].T for st in sets]))
    value = accepted_per_step / (ms_per_step * 1e-3)

    out_bytes = 2
    alg_bytes = float(np.mean([attention_algorithmic_bytes(st["b"], out_bytes) for st in sets]))
    attn_ms = attn_ms_total / max(1, attn_launches)
    achieved = alg_bytes / (attn_ms * 1e-3) / 1e9
    workload_key = "config%d_%s" % (n, args.layout) + ("_tree_rows%d" % args.tree_rows if args.tree_rows else "")
    wide = max(st["b"].max_k for st in sets) > 16
    roofline = {
        "bound": "hbm", "kernel": "verify_attention_wide_kernel" if wide else "verify_attention_kernel",
        "achieved": round(achieved, 1),
        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": read_traffic(workload_key),
        "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": round(attn_ms, 5),
        "launches_timed": attn_launches,
        # context, not the peak: a plain read-only streaming kernel over one K arena, same run
        "measured_read_ceiling": ceiling, "frac_of_measured_ceiling": round(achieved / ceiling, 4),
        "device_reported": device_memory_figures(),
    }

    result = {
        "metric": "verified tokens/s (attention + greedy accept + KV append, 1 layer)",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if sets[0]["b"].dtype == torch.bfloat16 else "f16", "data": "synthetic",
        "config": {"workload": "BASELINE config %d: %s" % (n, CONFIG_NAMES[n]), "layout": args.layout,
                   "B": sets[0]["b"].B, "H": sets[0]["b"].H, "D": sets[0]["b"].D,
                   "query_rows_per_step": rows_per_step, "accepted_per_step": accepted_per_step,
                   "logits": with_logits, "buffer_sets": len(sets),
                   "variant": "write-through + advance" if args.write_through else "verify + append",
                   "attention_variant": args.attention_variant, "tree": args.tree,
                   "tree_rows": args.tree_rows or None},
        "query_tokens_per_s": round(rows_per_step / (ms_per_step * 1e-3), 1),
        "roofline": roofline,
    }

    if args.breakdown:
        def time_call(fn, reps=100):
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for r in range(5):
                fn(sets[r % len(sets)])
            torch.cuda.synchronize()
            ev0.record()
            for r in range(reps):
                fn(sets[r % len(sets)])
            ev1.record()
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) / reps
        result["breakdown_ms"] = {"attention_call": round(time_call(attention), 5),
                                  "accept_call": round(time_call(accept), 5),
                                  "append_call": round(time_call(append), 5)}

    if not args.no_ablation and not args.tree:      # the padded ablation is the causal method's
        result["padded_ablation"] = padded_ablation(sets, args, with_logits, alg_bytes, ms_per_step)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(sets[0]["b"], with_logits)
    print(json.dumps(result), flush=True)


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


def verify_loop_bench(args, with_logits):
    """BASELINE config 5: a 32-layer OPT-6.7b-shaped verify loop, B=128, 20 successive steps;
    each step = attention per layer + accept + append into all layers' caches; the lengths
    advance on the device.  `--steps` repetitions of the whole loop are timed (caches are
    reset to their initial lengths between repetitions: appended rows are simply overwritten)."""
    import numpy as np
    import torch
    import paper_2405_07542_amd as ems
    from paper_2405_07542_amd.verify_loop import VerifyLoopRunner
    from workloads import make_verify_loop
    dev = "cuda:0"
    loop = make_verify_loop(n_layers=args.layers, n_steps=args.loop_steps, device=dev, layout=args.layout,
                            V=50272 if with_logits else 0)
    kv_len = loop.kv_len0.clone()
    runner = VerifyLoopRunner(k_caches=loop.k_caches, v_caches=loop.v_caches, row_stride=loop.row_stride,
                              head_stride=loop.head_stride, rows=loop.rows, kv_start=loop.kv_start,
                              kv_len=kv_len, H=loop.H, D=loop.D, V=loop.V, dtype=loop.dtype,
                              scale=loop.scale, max_k=loop.max_k, max_kv_len=loop.max_kv_len,
                              max_rows=max(st.T for st in loop.steps))
    acc_total = torch.zeros((), dtype=torch.int64, device=dev)

    def run_loop(count):
        kv_len.copy_(loop.kv_len0)
        for st in loop.steps:
            runner.step(st.q, st.k_new, st.v_new, st.cu_seqlens, st.logits, st.input_ids,
                        None if with_logits else st.target_ids)
            if count:
                acc_total.add_(runner.accepted_cu[-1])

    reps = max(1, min(args.steps, 3))
    run_loop(False)                                     # warm-up repetition
    torch.cuda.synchronize()
    lens_after = kv_len.clone()
    ems.ems_profile_enable(reps * args.loop_steps * args.layers)
    t0 = time.perf_counter()
    for _ in range(reps):
        run_loop(True)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    attn_ms_total, launches = ems.ems_profile_read()
    ems.ems_profile_enable(0)
    n_steps = reps * args.loop_steps
    ms_per_step = (t1 - t0) * 1e3 / n_steps
    accepted = int(acc_total) / reps
    rows = sum(st.T for st in loop.steps)
    hd = loop.H * loop.D
    # algorithmic bytes of all attention launches of one loop (lengths grow step by step)
    lens = loop.kv_len0.cpu().numpy().astype(np.int64)
    grown = lens_after.cpu().numpy().astype(np.int64) - lens
    alg = 0.0
    frac = np.linspace(0.0, 1.0, args.loop_steps, endpoint=False)
    for s, st in enumerate(loop.steps):
        L = lens + np.round(grown * frac[s])            # lengths at step s (linear in the step, +-1 row)
        alg += (2 * L.sum() * hd * 2 + 4 * st.T * hd * 2 + (3 * loop.B + 1) * 4) * args.layers
    attn_ms = attn_ms_total / max(1, launches)
    achieved = alg / (args.loop_steps * args.layers) / (attn_ms * 1e-3) / 1e9
    return {
        "metric": "verified tokens/s (32-layer verify loop: attention per layer + greedy accept + KV append)",
        "value": round(accepted / (ms_per_step * args.loop_steps * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": n_steps, "warmup": args.loop_steps, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "BASELINE config 5: %d-layer verify loop, B=128, %d successive steps" %
                   (args.layers, args.loop_steps), "layout": args.layout, "layers": args.layers,
                   "accepted_per_loop": accepted, "query_rows_per_loop": rows, "logits": with_logits,
                   "cache_GB": round(2 * args.layers * loop.rows * hd * 2 / 1e9, 1)},
        "query_tokens_per_s": round(rows / (ms_per_step * args.loop_steps * 1e-3), 1),
        "roofline": {"bound": "hbm", "kernel": "verify_attention_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None, "algorithmic_bytes_per_launch": alg / (args.loop_steps * args.layers),
                     "kernel_ms": round(attn_ms, 5), "launches_timed": launches},
    }


def padded_ablation(sets, args, with_logits, unpadded_alg_bytes, unpadded_ms):
    """The vanilla method of Sec. 3.1 on the same data, same library: inputs padded to k_max
    rows, caches aligned to the longest sample with padding keys masked, tau_max rows appended
    for every sample.  Timed like the main loop (fewer steps)."""
    import numpy as np
    import torch
    import paper_2405_07542_amd as ems
    from workloads import pad_batch
    dev = sets[0]["b"].q.device
    psets = []
    for st in sets:
        b = st["b"]
        p = pad_batch(b)
        Tp = b.B * p.k_max
        ids = torch.full((Tp,), -1, dtype=torch.int32, device=dev)     # padding ids never match
        ids[p.real_rows] = b.input_ids
        tgt = torch.zeros(Tp, dtype=torch.int32, device=dev)
        tgt[p.real_rows] = st["target"]
        logits = None
        if with_logits:
            logits = torch.randn((Tp, b.V), device=dev, dtype=torch.float32).to(b.dtype)
            logits[p.real_rows] = b.logits
        psets.append(dict(
            p=p, ids=ids, tgt=tgt, logits=logits,
            cu=torch.arange(0, Tp + 1, p.k_max, dtype=torch.int32, device=dev),
            cache=ems.kv_cache(p.k_cache, p.v_cache, p.row_stride, p.head_stride, p.rows),
            out=torch.empty_like(p.q_pad),
            ws=torch.empty(ems.ems_attention_workspace_bytes(p.B, Tp, p.H, p.D, p.l_pad), dtype=torch.uint8, device=dev),
            ws_acc=torch.empty(max(8, ems.ems_accept_workspace_bytes(Tp, b.V)), dtype=torch.uint8, device=dev),
            accepted=torch.empty(b.B, dtype=torch.int32, device=dev),
            accepted_cu=torch.empty(b.B + 1, dtype=torch.int32, device=dev),
            out_tokens=torch.empty(Tp, dtype=torch.int32, device=dev),
            tau_max=int(st["accepted"].max())))
    torch.cuda.synchronize()

    def step(ps):
        p = ps["p"]
        ems.ems_padded_verify_attention(p.q_pad, p.k_new_pad, p.v_new_pad, ps["cache"], p.cap, p.key_mask,
                                        p.k_valid, ps["out"], k_max=p.k_max, l_pad=p.l_pad, scale=p.scale,
                                        workspace=ps["ws"])
        ems.ems_greedy_accept(ps["logits"], ps["tgt"], ps["ids"], ps["cu"], ps["accepted"],
                              ps["accepted_cu"], ps["out_tokens"], workspace=ps["ws_acc"])
        ems.ems_padded_kv_append([p.k_new_pad], [p.v_new_pad], [ps["cache"]], p.cap, p.key_mask,
                                 ps["accepted"], k_max=p.k_max, l_pad=p.l_pad, tau_max=ps["tau_max"])

    steps = max(10, args.steps // 3)
    for w in range(5):
        step(psets[w % len(psets)])
    torch.cuda.synchronize()
    ems.ems_profile_enable(steps)
    t0 = time.perf_counter()
    for s in range(steps):
        step(psets[s % len(psets)])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    attn_ms_total, launches = ems.ems_profile_read()
    ems.ems_profile_enable(0)
    ms = (t1 - t0) * 1e3 / steps
    attn_ms = attn_ms_total / max(1, launches)
    # the padded path must accept exactly what the unpadded path accepted
    same = all(torch.equal(ps["accepted"], st["accepted"]) for ps, st in zip(psets, sets))
    p = psets[0]["p"]
    hd = p.H * p.D
    moved = float(np.mean([2 * ps["p"].B * ps["p"].l_pad * hd * 2 + 4 * ps["p"].B * ps["p"].k_max * hd * 2
                           + ps["p"].B * ps["p"].l_pad for ps in psets]))
    real_keys = float(np.mean([int(st["b"].kv_len.sum()) for st in sets]))
    pad_keys = float(np.mean([ps["p"].B * ps["p"].l_pad for ps in psets]))
    real_rows = float(np.mean([st["b"].T for st in sets]))
    return {
        "ms_per_step": round(ms, 5), "attention_kernel_ms": round(attn_ms, 5), "steps": steps,
        "moved_GBps": round(moved / (attn_ms * 1e-3) / 1e9, 1),
        "useful_GBps": round(unpadded_alg_bytes / (attn_ms * 1e-3) / 1e9, 1),
        "kv_padding_ratio": round((pad_keys - real_keys) / pad_keys, 4),
        "input_padding_ratio": round(1.0 - real_rows / (p.B * p.k_max), 4),
        "accepted_equal_to_unpadded": bool(same),
        "unpadded_speedup_step": round(ms / unpadded_ms, 3),
    }


def cpu_baseline(b, with_logits, budget_s=15.0):
    """The oracle, as it stands, on the host cores, over the first samples of the batch."""
    import numpy as np
    import oracle
    from workloads import bits
    cu = b.cu_seqlens.cpu().numpy()
    ks = b.kv_start.cpu().numpy()
    kl = b.kv_len.cpu().numpy()
    # token-major view of the sampled caches only (the arena may be tens of GB)
    def run(ns):
        rows = int(cu[ns])
        if rows == 0:
            return 0.0, 0
        from workloads import arena_view
        Kv = arena_view(b.k_cache, b.layout, b.rows, b.H, b.D)
        Vv = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D)
        cap = int(max(kl[:ns])) + 16
        kc = np.zeros((ns * cap, b.H, b.D), dtype=np.uint16)
        vc = np.zeros((ns * cap, b.H, b.D), dtype=np.uint16)
        for i in range(ns):
            kc[i * cap:i * cap + kl[i]] = bits(Kv[ks[i]:ks[i] + kl[i]])
            vc[i * cap:i * cap + kl[i]] = bits(Vv[ks[i]:ks[i] + kl[i]])
        starts = (np.arange(ns) * cap).astype(np.int32)
        q, kn, vn = bits(b.q[:rows]), bits(b.k_new[:rows]), bits(b.v_new[:rows])
        lg = bits(b.logits[:rows]) if with_logits else None
        ids = b.input_ids[:rows].cpu().numpy()
        tgt = b.target_ids[:rows].cpu().numpy()
        t0 = time.perf_counter()
        oracle.verify_attention(q, kn, vn, kc.reshape(-1), vc.reshape(-1), b.H * b.D, b.D, cu[:ns + 1],
                                starts, kl[:ns], b.H, b.D, b.scale, b.dtype)
        x = oracle.argmax(lg, b.dtype) if with_logits else tgt
        acc, _, _ = oracle.greedy_accept(x, ids, cu[:ns + 1])
        oracle.kv_append(kc.reshape(-1), vc.reshape(-1), b.H * b.D, b.D, kn, vn, cu[:ns + 1], acc, starts,
                         kl[:ns], b.H, b.D)
        return time.perf_counter() - t0, int(acc.sum())

    probe = max(1, min(2, b.B))
    t_probe, _ = run(probe)
    ns = int(max(probe, min(b.B, budget_s / max(t_probe / probe, 1e-6))))
    t, accepted = run(ns)
    reps = 1
    while t < 1.5 and reps < 8:          # ~10-30 s of CPU work over all threads, for a steady figure
        t2, a2 = run(ns)
        t, accepted, reps = t + t2, accepted + a2, reps + 1
    cores = oracle.num_threads()
    # the same on one thread, over an eighth of the samples (context for the figure above)
    oracle.set_num_threads(1)
    try:
        n1 = max(1, ns // 8)
        t1, a1 = run(n1)
    finally:
        oracle.set_num_threads(cores)
    return {"value": round(accepted / t, 2), "unit": "tokens/s", "cores": cores,
            "kind": "oracle", "seconds": round(t, 3),
            "sample": "first %d of %d samples of the same batch, all heads, one layer: fp64 oracle "
                      "attention + arg-max + accept + append, %d time%s over" % (ns, b.B, reps, "" if reps == 1 else "s"),
            "one_thread": {"value": round(a1 / t1, 2), "seconds": round(t1, 3), "sample": "first %d samples" % n1}}


if __name__ == "__main__":
    main()
