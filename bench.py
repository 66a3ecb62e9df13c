#!/usr/bin/env python3
"""Benchmark of the ragged verification step (EMS-SD hot path) on one MI355X.

A step = one pass of the whole path over one synthetic batch that is already
resident in HBM:  ems_verify_attention (one OPT-6.7b-shaped layer) ->
ems_greedy_accept (arg-max over [T, 50272] logits, acceptance, prefix sum) ->
ems_kv_append (accepted rows into the per-sample caches).

Prints ONE JSON line: verified tokens/s (sum of accepted tokens / step time) at BASELINE
config 4 (B=64, bf16, the configuration the target is quoted on), the roofline figures of
the dominant kernel (the main attention kernel, timed with HIP events recorded around it on
its own stream inside the timed region), the padded ablation on the same data, the oracle's
throughput on the host cores as a CPU baseline, `parity` (what the timed run left in buffer
set 0 against the oracle: max-abs error of the attention output, equality of ids, counts,
offsets and appended cache rows) and `all_configs` (brief runs of configs 2, 3 and 5, so
that B = 8, 32, 64 and 128 are all in the line).

    python bench.py [--steps K] [--warmup W] [--config 2|3|4|5] [--layout head_major|token_major]

The cache arenas are head-major ([H, R, D]) unless --layout says otherwise: both layouts are the
library's (a strided view), head-major is the one it reads 1-3 % faster.

Side modes (sweeps, the paper's launch shape, dynamic batching) live in bench_modes.py.
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
    ap.add_argument("--layout", default="head_major", choices=["token_major", "head_major"],
                    help="cache arena [H, R, D] (default: a 32-key tile of one head is 8 KiB contiguous) or [R, H, D]")
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
    ap.add_argument("--separate-accept-append", action="store_true",
                    help="acceptance and append as two calls (three launches) instead of ems_greedy_accept_append")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="config 4 only: skip the brief runs of configs 2, 3 and 5 that fill `all_configs`")
    ap.add_argument("--source-digest", action="store_true",
                    help="print the digest of the attention kernels' sources (stored with counter summaries) and exit")
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


KERNEL_SOURCES = ("attention_tiles.h", "ems_device.h", "ems_kernels.h", "verify_attention.hip",
                  "verify_attention_wide.hip", "verify_attention_staged.hip")


def kernel_source_digest():
    """sha256 (first 16 hex digits) over the sources of the attention kernels, in a fixed order.
    A stored counter figure carries the digest of the sources it was measured with; when the
    sources have changed since, the figure is not quoted (see read_traffic)."""
    import hashlib
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2405_07542_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def read_traffic(workload_key):
    """(HBM bytes per launch of the main attention kernel, where the figure comes from) from the
    committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE, each scaled by what the same
    counter reads for a plain copy of known size).  The summary states the digest of the kernel
    sources it was measured with; if the sources differ now, the figure is stale and None is
    returned in its place."""
    rel = os.path.join("profiles", "verify_attention_traffic.txt")
    path = os.path.join(ROOT, rel)
    source = {"file": rel, "commit": None, "kernel_source_digest": None, "current_digest": kernel_source_digest(),
              "stale": None}
    if not os.path.exists(path):
        return None, None
    value = None
    for line in open(path):
        parts = line.split()
        if len(parts) >= 3 and parts[0] == "#" and parts[1] in ("commit", "kernel_source_digest"):
            source[parts[1]] = parts[2]
        elif len(parts) >= 2 and parts[0] == workload_key:
            try:
                value = float(parts[1])
            except ValueError:
                value = None
    source["stale"] = source["kernel_source_digest"] != source["current_digest"]
    if value is None:
        return None, None
    return (None if source["stale"] else value), source


def build_sets(n, args, with_logits, dev):
    """Independent buffer sets of config n, rotated between steps so that no step finds its K/V
    in the last-level cache."""
    import torch
    import paper_2405_07542_amd as ems
    from workloads import make_config
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
        ws_attn = torch.empty(ems.ems_workspace_bytes(b.B, b.T, b.H, b.D, b.max_kv_len),
                              dtype=torch.uint8, device=dev)
        ws_acc = torch.empty(max(8, ems.ems_accept_workspace_bytes(b.T, b.V)), dtype=torch.uint8, device=dev)
        sets.append(dict(
            b=b, ws_attn=ws_attn, ws_acc=ws_acc,
            cache=ems.kv_cache(b.k_cache, b.v_cache, b.row_stride, b.head_stride, b.rows),
            out=torch.empty((b.T, b.H, b.D), dtype=b.dtype, device=dev),
            target=torch.empty(b.T, dtype=torch.int32, device=dev) if with_logits else b.target_ids.clone(),
            accepted=torch.empty(b.B, dtype=torch.int32, device=dev),
            accepted_cu=torch.empty(b.B + 1, dtype=torch.int32, device=dev),
            out_tokens=torch.empty(b.T, dtype=torch.int32, device=dev),
            accepted_rows=torch.empty(b.T, dtype=torch.int32, device=dev),
            # the lengths are NOT advanced between timed steps, so every step does the same work
            new_len=torch.empty(b.B, dtype=torch.int32, device=dev)))
        v += 1
    torch.cuda.synchronize()
    return sets


def step_functions(args, with_logits):
    import paper_2405_07542_amd as ems

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

    def accept_append(st):
        b = st["b"]
        ems.ems_greedy_accept_append(b.logits if with_logits else None, st["target"], b.input_ids, b.cu_seqlens,
                                     st["accepted"], st["accepted_cu"], st["out_tokens"], [b.k_new], [b.v_new],
                                     [st["cache"]], b.kv_start, b.kv_len, st["new_len"], workspace=st["ws_acc"])

    def step(st):
        attention(st)
        if args.tree or args.write_through or args.separate_accept_append:
            accept(st)
            append(st)
        else:
            accept_append(st)       # the same two steps, the counts and the copy in one launch

    return attention, accept, append, step


def time_one_layer_config(n, args, with_logits, steps, warmup, dev, with_ceiling):
    """Times `steps` steps of config n (2, 3 or 4: one layer).  Returns (figures, sets)."""
    import numpy as np
    import torch
    import paper_2405_07542_amd as ems
    sets = build_sets(n, args, with_logits, dev)
    attention, accept, append, step = step_functions(args, with_logits)

    # Set-up, untimed: every buffer set is run once, so that its accepted counts (the numerator
    # of `value`) exist however few steps are timed, and so that no set is touched for the first
    # time inside the timed region (the first pass over a fresh 2 GiB arena costs ~90 us more);
    # then the read ceiling that the roofline object quotes as context.
    for st in sets:
        step(st)
    torch.cuda.synchronize()
    ceiling = measured_read_ceiling(sets[0]["b"].k_cache) if with_ceiling else None

    for w in range(warmup):
        step(sets[w % len(sets)])
    torch.cuda.synchronize()

    ems.ems_profile_enable(steps)
    t0 = time.perf_counter()
    for s in range(steps):
        step(sets[s % len(sets)])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    attn_ms_total, call_ms_total, attn_launches = ems.ems_profile_read_calls()
    ems.ems_profile_enable(0)

    ms_per_step = (t1 - t0) * 1e3 / steps
    accepted_per_step = float(np.mean([int(st["accepted_cu"][-1]) for st in sets]))
    rows_per_step = float(np.mean([st["b"].T for st in sets]))
    alg_bytes = float(np.mean([attention_algorithmic_bytes(st["b"], 2) for st in sets]))
    attn_ms = attn_ms_total / max(1, attn_launches)
    call_ms = call_ms_total / max(1, attn_launches)
    achieved = alg_bytes / (attn_ms * 1e-3) / 1e9
    achieved_call = alg_bytes / (call_ms * 1e-3) / 1e9
    wide = max(st["b"].max_k for st in sets) > 16
    roofline = {
        "bound": "hbm", "kernel": "verify_attention_wide_kernel" if wide else "verify_attention_kernel",
        # achieved / frac: algorithmic bytes of the attention call over the duration of its main
        # kernel (HIP events right around that kernel); *_call: over the whole call, i.e. with
        # the partial-merge kernel that writes the outputs of pairs shared between workgroups
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "achieved_call": round(achieved_call, 1), "frac_call": round(achieved_call / HBM_PEAK_GBS, 4),
        "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": round(attn_ms, 5), "call_ms": round(call_ms, 5),
        "launches_timed": attn_launches,
    }
    figures = {"ms_per_step": ms_per_step, "value": accepted_per_step / (ms_per_step * 1e-3),
               "query_tokens_per_s": rows_per_step / (ms_per_step * 1e-3), "accepted_per_step": accepted_per_step,
               "rows_per_step": rows_per_step, "alg_bytes": alg_bytes, "roofline": roofline, "ceiling": ceiling,
               "steps": steps, "warmup": warmup}
    return figures, (sets, attention, accept, append)


LOGITS_NOTE = ("[T, 50272] N(0,1) with the row maximum planted (8.0 at the target id, repeated at a higher "
               "index on 25 % of the rows to force ties); cost is data-independent")


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (--gpus 1); the path would shard by sample or by "
              "head with no exchange between GPUs, so the figure for N GPUs is N times this one", file=sys.stderr)
        sys.exit(2)
    if args.source_digest:
        print(kernel_source_digest())
        return
    import torch
    import paper_2405_07542_amd as ems
    from workloads import CONFIG_NAMES

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    ems.lib()     # fail loudly if the HIP library is missing
    ems.ems_set_attention_variant(ems.EMS_ATTN_VALU if args.attention_variant == "valu" else ems.EMS_ATTN_MFMA)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    n = args.config
    with_logits = not args.no_logits
    if args.tree and (args.write_through or args.attention_variant == "valu" or n == 5):
        sys.exit("--tree runs the matrix-core kernel with the gathered append on configs 2-4 only")
    if args.tree_rows and (not args.tree or not 1 <= args.tree_rows <= 64):
        sys.exit("--tree-rows N goes with --tree and 1 <= N <= 64")
    side_mode = (args.copy_calibration > 0 or args.per_token_grid or args.sweep_variants or args.sweep_k
                 or args.dynamic_batching)
    if side_mode:
        import bench_modes
        if args.copy_calibration > 0:
            res = bench_modes.copy_calibration(args.copy_calibration)
        elif args.per_token_grid:
            res = bench_modes.per_token_grid(args)
        elif args.sweep_variants:
            res = bench_modes.sweep_variants()
        elif args.sweep_k:
            res = bench_modes.sweep_k()
        else:
            res = bench_modes.dynamic_batching_bench(args)
        print(json.dumps(res), flush=True)
        return
    if n == 5:
        print(json.dumps(verify_loop_bench(args, with_logits)), flush=True)
        return

    fig, (sets, attention, accept, append) = time_one_layer_config(n, args, with_logits, args.steps, args.warmup,
                                                                   dev, with_ceiling=True)
    ms_per_step = fig["ms_per_step"]
    roofline = fig["roofline"]
    workload_key = "config%d_%s" % (n, args.layout) + ("_tree_rows%d" % args.tree_rows if args.tree_rows else "")
    traffic, traffic_source = read_traffic(workload_key)
    roofline.update({
        "traffic": traffic, "traffic_source": traffic_source,
        # context, not the peak: a plain read-only streaming kernel over one K arena, same run
        "measured_read_ceiling": fig["ceiling"],
        "frac_of_measured_ceiling": round(roofline["achieved"] / fig["ceiling"], 4),
        "device_reported": device_memory_figures(),
    })
    b0 = sets[0]["b"]
    result = {
        "metric": "verified tokens/s (attention + greedy accept + KV append, 1 layer)",
        "value": round(fig["value"], 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if b0.dtype == torch.bfloat16 else "f16", "data": "synthetic",
        "config": {"workload": "BASELINE config %d: %s" % (n, CONFIG_NAMES[n]), "layout": args.layout,
                   "B": b0.B, "H": b0.H, "D": b0.D,
                   "query_rows_per_step": fig["rows_per_step"], "accepted_per_step": fig["accepted_per_step"],
                   "logits": LOGITS_NOTE if with_logits else None, "buffer_sets": len(sets),
                   "variant": "write-through + advance" if args.write_through else "verify + append",
                   "accept_and_append": "two calls" if (args.tree or args.write_through or args.separate_accept_append)
                   else "one call (ems_greedy_accept_append)",
                   "attention_variant": args.attention_variant, "tree": args.tree,
                   "tree_rows": args.tree_rows or None},
        "query_tokens_per_s": round(fig["query_tokens_per_s"], 1),
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
        result["padded_ablation"] = padded_ablation(sets, args, with_logits, fig["alg_bytes"], ms_per_step)
    if not args.no_cpu_baseline:
        result["cpu_baseline"], result["parity"] = cpu_baseline(sets[0], with_logits, tree=bool(args.tree),
                                                                write_through=args.write_through)
    del sets, attention, accept, append
    torch.cuda.empty_cache()

    # The metric is quoted for B = 8 .. 128: the other three one-GPU configurations, each timed
    # briefly in the same run (config 5: one repetition of the 32-layer, 20-step loop).
    if not args.no_all_configs and n == 4 and not (args.tree or args.write_through or args.attention_variant == "valu"):
        others = []
        for m, steps, warmup in ((2, 400, 40), (3, 150, 15)):
            f, keep = time_one_layer_config(m, args, with_logits, steps, warmup, dev, with_ceiling=False)
            mb = keep[0][0]["b"]
            others.append({"config": m, "workload": CONFIG_NAMES[m], "B": mb.B,
                           "dtype": "bf16" if mb.dtype == torch.bfloat16 else "f16", "steps": steps,
                           "ms_per_step": round(f["ms_per_step"], 5), "value": round(f["value"], 1),
                           "query_tokens_per_s": round(f["query_tokens_per_s"], 1), "roofline": f["roofline"]})
            del keep, f
            torch.cuda.empty_cache()
        loop_args = argparse.Namespace(**vars(args))
        loop_args.steps = 1
        r5 = verify_loop_bench(loop_args, with_logits)
        others.append({"config": 5, "workload": r5["config"]["workload"], "B": 128, "dtype": r5["dtype"],
                       "steps": r5["steps"], "ms_per_step": r5["ms_per_step"], "value": r5["value"],
                       "query_tokens_per_s": r5["query_tokens_per_s"],
                       "note": "a step here is one 32-layer verify step (32 attention calls + accept + append)",
                       "roofline": {k: r5["roofline"][k] for k in ("bound", "kernel", "achieved", "peak", "unit", "frac",
                                                                  "achieved_call", "frac_call",
                                                                  "algorithmic_bytes_per_launch", "kernel_ms",
                                                                  "call_ms", "launches_timed")}})
        result["all_configs"] = others
    print(json.dumps(result), flush=True)


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
    attn_ms_total, call_ms_total, launches = ems.ems_profile_read_calls()
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
    call_ms = call_ms_total / max(1, launches)
    achieved = alg / (args.loop_steps * args.layers) / (attn_ms * 1e-3) / 1e9
    achieved_call = alg / (args.loop_steps * args.layers) / (call_ms * 1e-3) / 1e9
    return {
        "metric": "verified tokens/s (32-layer verify loop: attention per layer + greedy accept + KV append)",
        "value": round(accepted / (ms_per_step * args.loop_steps * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": n_steps, "warmup": args.loop_steps, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "BASELINE config 5: %d-layer verify loop, B=128, %d successive steps" %
                   (args.layers, args.loop_steps), "layout": args.layout, "layers": args.layers,
                   "accepted_per_loop": accepted, "query_rows_per_loop": rows,
                   "logits": LOGITS_NOTE if with_logits else None,
                   "cache_GB": round(2 * args.layers * loop.rows * hd * 2 / 1e9, 1)},
        "query_tokens_per_s": round(rows / (ms_per_step * args.loop_steps * 1e-3), 1),
        "roofline": {"bound": "hbm", "kernel": "verify_attention_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "achieved_call": round(achieved_call, 1), "frac_call": round(achieved_call / HBM_PEAK_GBS, 4),
                     "traffic": None, "algorithmic_bytes_per_launch": alg / (args.loop_steps * args.layers),
                     "kernel_ms": round(attn_ms, 5), "call_ms": round(call_ms, 5), "launches_timed": launches},
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
            ws=torch.empty(ems.ems_workspace_bytes(p.B, Tp, p.H, p.D, p.l_pad), dtype=torch.uint8, device=dev),
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


def cpu_baseline(st, with_logits, budget_s=15.0, tree=False, write_through=False):
    """The oracle, as it stands, on the host cores, over the first samples of buffer set `st`'s
    batch -- timed as the CPU baseline, and compared with what the HIP path left in that same
    buffer set (its last timed step): returns (cpu_baseline, parity)."""
    import numpy as np
    import torch
    import oracle
    from workloads import arena_view, bits
    b = st["b"]
    cu = b.cu_seqlens.cpu().numpy()
    ks = b.kv_start.cpu().numpy()
    kl = b.kv_len.cpu().numpy()
    Kv = arena_view(b.k_cache, b.layout, b.rows, b.H, b.D)
    Vv = arena_view(b.v_cache, b.layout, b.rows, b.H, b.D)

    # token-major copies of the sampled caches only (the arena may be tens of GB)
    def run(ns):
        rows = int(cu[ns])
        if rows == 0:
            return 0.0, 0, None
        cap = int(max(kl[:ns])) + int(max(np.diff(cu[:ns + 1]))) + 1
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
        out = oracle.verify_attention(q, kn, vn, kc.reshape(-1), vc.reshape(-1), b.H * b.D, b.D, cu[:ns + 1],
                                      starts, kl[:ns], b.H, b.D, b.scale, b.dtype)
        x = oracle.argmax(lg, b.dtype) if with_logits else tgt
        acc, acc_cu, toks = oracle.greedy_accept(x, ids, cu[:ns + 1])
        new_len = oracle.kv_append(kc.reshape(-1), vc.reshape(-1), b.H * b.D, b.D, kn, vn, cu[:ns + 1], acc,
                                   starts, kl[:ns], b.H, b.D)
        dt = time.perf_counter() - t0
        return dt, int(acc.sum()), dict(out=out, x=x, acc=acc, acc_cu=acc_cu, toks=toks, new_len=new_len, kc=kc,
                                        vc=vc, cap=cap, rows=rows)

    probe = max(1, min(2, b.B))
    t_probe, _, _ = run(probe)
    ns = int(max(probe, min(b.B, budget_s / max(t_probe / probe, 1e-6))))
    t, accepted, ref = run(ns)
    reps = 1
    while t < 1.5 and reps < 8:          # ~10-30 s of CPU work over all threads, for a steady figure
        t2, a2, _ = run(ns)
        t, accepted, reps = t + t2, accepted + a2, reps + 1
    cores = oracle.num_threads()
    # the same on one thread, over an eighth of the samples (context for the figure above)
    oracle.set_num_threads(1)
    try:
        n1 = max(1, ns // 8)
        t1, a1, _ = run(n1)
    finally:
        oracle.set_num_threads(cores)
    baseline = {"value": round(accepted / t, 2), "unit": "tokens/s", "cores": cores,
                "kind": "oracle", "seconds": round(t, 3),
                "sample": "first %d of %d samples of the same batch, all heads, one layer: fp64 oracle "
                          "attention + arg-max + accept + append, %d time%s over" % (ns, b.B, reps, "" if reps == 1 else "s"),
                "one_thread": {"value": round(a1 / t1, 2), "seconds": round(t1, 3), "sample": "first %d samples" % n1}}

    # Parity of the run that was just timed: what the HIP path left in this buffer set against
    # the oracle on the same inputs (causal verify + append only: the tree and write-through
    # variants have their own oracle functions and are compared in the tests).
    parity = None
    if ref is not None and not tree and not write_through:
        rows = ref["rows"]
        got = st["out"][:rows].double().cpu().numpy()
        err = float(np.abs(got - ref["out"]).max())
        n_acc = int(ref["acc_cu"][ns])
        cache_equal = bool(np.array_equal(st["new_len"][:ns].cpu().numpy(), ref["new_len"]))
        for i in range(ns):                      # the rows the append wrote, in the arena itself
            a, cap = int(ref["acc"][i]), ref["cap"]
            lo = int(ks[i] + kl[i])
            cache_equal &= bool(np.array_equal(bits(Kv[lo:lo + a]), ref["kc"][i * cap + kl[i]:i * cap + kl[i] + a]))
            cache_equal &= bool(np.array_equal(bits(Vv[lo:lo + a]), ref["vc"][i * cap + kl[i]:i * cap + kl[i] + a]))
        parity = {
            "against": "fp64 oracle, same inputs, buffer set 0, first %d of %d samples, %d rows, every element" % (ns, b.B, rows),
            "attention_max_abs_err": err, "bar": 2e-3, "attention_within_bar": bool(err <= 2e-3),
            "out_dtype": "bf16" if st["out"].dtype == torch.bfloat16 else "f16",
            "target_ids_equal": bool(np.array_equal(st["target"][:rows].cpu().numpy(), ref["x"])),
            "accepted_equal": bool(np.array_equal(st["accepted"][:ns].cpu().numpy(), ref["acc"])),
            "accepted_cu_equal": bool(np.array_equal(st["accepted_cu"][:ns + 1].cpu().numpy(), ref["acc_cu"])),
            "out_tokens_equal": bool(np.array_equal(st["out_tokens"][:n_acc].cpu().numpy(), ref["toks"])),
            "cache_equal": cache_equal,
        }
    return baseline, parity


if __name__ == "__main__":
    main()
