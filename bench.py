#!/usr/bin/env python3
"""Benchmark of prefix-shared decode attention on one MI355X.

A step is one pass of the whole hot path (partial attention over the scheduled
tasks + per-query reduction) over one synthetic batch whose Q/K/V already sit
in HBM.  The step is timed cold: consecutive steps rotate over enough copies of
the K/V pools that nothing of a pool survives in L2 / Infinity Cache until its
next use, which is what a multi-layer decode loop sees.

Prints ONE JSON line.  ``value`` is GB/s of unique KV bytes (every node counted
once) over the whole step of the headline workload (cfg5c, the largest
configuration that fits one GPU); ``roofline`` prices the partial-attention
kernel alone against the 8 TB/s HBM peak and against a plain streaming-read
kernel measured in the same run; ``cpu_baseline`` is the fp64 oracle timed on
this machine's host cores on a bounded sample.  ``per_config`` carries, for every
configuration, its own ``roofline`` and ``cpu_baseline`` objects, the planner
variants (the solver of Sec. 5.1 as printed and the library's two extensions
of it, one at a time and together), the flat (no-sharing) baseline of the same
library and the tree/flat speedup.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0        # dense bf16 / fp16 matrix peak of the chip
COLD_FOOTPRINT_BYTES = 3 << 30        # rotate pool copies until this much K/V is cycled through
MIN_WARM_SECONDS = 0.25


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg5c", help="headline configuration")
    ap.add_argument("--configs", default="cfg1,cfg2,cfg3,cfg4,cfg5a,cfg5b,cfg5c",
                    help="configurations reported in per_config ('' = headline only)")
    ap.add_argument("--layout", default="htd", choices=["thd", "htd", "hktd"],
                    help="page layout: htd = [page][kv_head][token][d] (a page-head is one 4 KB run), thd = [page][token][kv_head][d], "
                         "hktd = one pool [page][kv_head][K|V][token][d] (K and V of a page-head are one 8 KB run)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-flat", action="store_true")
    ap.add_argument("--num-slots", type=int, default=0)
    ap.add_argument("--split-align", type=int, default=0)
    ap.add_argument("--max-rows", type=int, default=0)
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample (headline)")
    ap.add_argument("--cpu-seconds-other", type=float, default=3.0,
                    help="target CPU time of the oracle sample of the other configurations")
    ap.add_argument("--no-stream-calibration", action="store_true",
                    help="skip the plain streaming-read kernel (roofline.frac_of_measured_stream is then null)")
    ap.add_argument("--sweep", default="", help="run one of the paper-shaped synthetic sweeps instead of the "
                    "configurations: seqlen, batch, depth, ratio, shape, ablation, granularity")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy 3 times (reference for scaling FETCH_SIZE / "
                         "WRITE_SIZE counters when the run is profiled)")
    return ap.parse_args()


class Rotating:
    """``copies`` clones of the K/V pools of a workload, all resident in HBM."""

    def __init__(self, w, copies):
        import torch
        if getattr(w, "kv_pool", None) is not None:        # K and V are views of one pool: clone that
            pools = [w.kv_pool] + [w.kv_pool.clone() for _ in range(copies - 1)]
            self.k = [p[:, :, 0] for p in pools]
            self.v = [p[:, :, 1] for p in pools]
        else:
            self.k = [w.k_pool] + [w.k_pool.clone() for _ in range(copies - 1)]
            self.v = [w.v_pool] + [w.v_pool.clone() for _ in range(copies - 1)]
        self.n = copies
        torch.cuda.synchronize()

    def pools(self, i):
        return self.k[i % self.n], self.v[i % self.n]


def time_plan(pa, w, rot, steps, warmup, phases=True):
    """Whole-step time over exactly ``steps`` steps plus per-phase kernel times from HIP events."""
    import torch
    out = torch.empty_like(w.q)
    stream = torch.cuda.current_stream()
    for i in range(warmup):
        k, v = rot.pools(i)
        pa.decode(w.q, k, v, out)
    torch.cuda.synchronize()
    # the card clocks down while the host builds a workload or a plan: keep it busy for a quarter of a
    # second more (untimed), or the first variant measured on a new workload reads 2-3 % slow
    t_busy = time.perf_counter()
    i = warmup
    while time.perf_counter() - t_busy < MIN_WARM_SECONDS:
        for _ in range(8):
            k, v = rot.pools(i)
            pa.decode(w.q, k, v, out)
            i += 1
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(steps):
        k, v = rot.pools(warmup + i)
        pa.decode(w.q, k, v, out)
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    step_ms = e0.elapsed_time(e1) / steps

    if not phases:
        return {"step_ms": step_ms, "wall_ms": wall_ms}, out
    # second pass over the same steps: events around each phase, on the stream the kernels run on
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for i in range(steps):
        k, v = rot.pools(warmup + i)
        ev[i][0].record(stream)
        pa.partial_attention(w.q, k, v)
        ev[i][1].record(stream)
        pa.partial_reduction(out)
        ev[i][2].record(stream)
    torch.cuda.synchronize()
    pac = sorted(e[0].elapsed_time(e[1]) for e in ev)
    por = sorted(e[1].elapsed_time(e[2]) for e in ev)
    return {"step_ms": step_ms, "wall_ms": wall_ms,
            "pac_ms_avg": sum(pac) / steps, "pac_ms_min": pac[0], "pac_ms_med": pac[steps // 2],
            "por_ms_avg": sum(por) / steps}, out


def run_config(name, args, steps, warmup, want_flat):
    import torch
    import paper_2505_17694_amd as C
    from workloads import make_config, forest_stats

    w = make_config(name, device="cuda:0", layout=args.layout)
    st = forest_stats(w.forest)
    unique_bytes = st["unique_tokens"] * w.head.bytes_per_token
    flat_bytes = st["flat_tokens"] * w.head.bytes_per_token
    pool_bytes = 2 * w.k_pool.numel() * 2
    copies = max(1, min(int(math.ceil(COLD_FOOTPRINT_BYTES / max(pool_bytes, 1))), 64))
    free, _ = torch.cuda.mem_get_info()
    copies = max(1, min(copies, int(free * 0.8 // max(pool_bytes, 1)) + 1))
    rot = Rotating(w, copies)
    res = {"workload": name, "unique_kv_bytes": unique_bytes, "flat_kv_bytes": flat_bytes,
           "mean_sharing": round(st["mean_sharing"], 3), "pool_copies": copies,
           "requests": st["num_requests"], "nodes": st["num_nodes"]}
    outs = {}
    # "tree": the prefix-shared plan with both planner extensions (what the library is measured on);
    # "flat": the no-sharing baseline of the same library
    for key, share, ext in ([("tree", 1, 3), ("flat", 0, 0)] if want_flat else [("tree", 1, 3)]):
        t0 = time.perf_counter()
        pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", share=share, extensions=ext,
                                num_slots=args.num_slots, split_align=args.split_align,
                                max_rows=args.max_rows)
        plan_ms = (time.perf_counter() - t0) * 1e3
        view = pa.export()
        t, out = time_plan(pa, w, rot, steps, warmup)
        outs[share] = out.clone()
        res[key] = {
            "us_per_step": round(t["step_ms"] * 1e3, 2),
            "pac_us": round(t["pac_ms_avg"] * 1e3, 2), "pac_us_min": round(t["pac_ms_min"] * 1e3, 2),
            "por_us": round(t["por_ms_avg"] * 1e3, 2),
            "unique_kv_GBps": round(unique_bytes / (t["step_ms"] * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(unique_bytes / (t["step_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "read_GBps": round((unique_bytes if share else flat_bytes) / (t["step_ms"] * 1e-3) / 1e9, 1),
            "plan_ms": round(plan_ms, 2), "tasks": len(view["tasks"]), "part_rows": view["part_rows"],
            "est_makespan": view["makespan"], "cost_l": view["cost_l"],
        }
        res[key]["_raw"] = t
        if share:
            # carrying the plan over to the next step's lengths (host work + metadata upload) against
            # planning again: what a serving loop pays per step between two plannings
            t0 = time.perf_counter()
            pa.refresh(w.forest.node_len)
            res[key]["refresh_ms"] = round((time.perf_counter() - t0) * 1e3, 3)
        pa.close()
    if want_flat:
        # the solver of Sec. 5.1 as printed (Eq. 5 bound, node-by-node grid search), then each of the
        # library's two extensions of it alone: what each addition is worth on this workload
        for key, ext in (("tree_sec5_as_printed", 0), ("tree_slack_only", 1), ("tree_diagonal_only", 2)):
            pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", share=1, extensions=ext,
                                    num_slots=args.num_slots, split_align=args.split_align, max_rows=args.max_rows)
            view = pa.export()
            t, _ = time_plan(pa, w, rot, steps, warmup)
            res[key] = {"us_per_step": round(t["step_ms"] * 1e3, 2), "pac_us": round(t["pac_ms_avg"] * 1e3, 2),
                        "tasks": len(view["tasks"]), "est_makespan": view["makespan"]}
            pa.close()
        # the same prefix-shared tasks taken from a run-time queue instead of the static slot lists
        pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", share=1, schedule=1, extensions=3,
                                num_slots=args.num_slots, split_align=args.split_align, max_rows=args.max_rows)
        view = pa.export()
        t, _ = time_plan(pa, w, rot, steps, warmup)
        res["tree_queued"] = {"us_per_step": round(t["step_ms"] * 1e3, 2), "pac_us": round(t["pac_ms_avg"] * 1e3, 2),
                              "entries": len(view["queue_off"]) - 1, "slots": view["num_slots"]}
        pa.close()
        # one launch: the workgroup that delivers a request's last partial result reduces it (fused = 1)
        pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", share=1, fused=1, extensions=3,
                                num_slots=args.num_slots, split_align=args.split_align, max_rows=args.max_rows)
        t, _ = time_plan(pa, w, rot, steps, warmup, phases=False)
        res["tree_single_launch"] = {"us_per_step": round(t["step_ms"] * 1e3, 2)}
        pa.close()
        # the library's own choices: the plan with the lowest estimated makespan among its candidates
        # (share = 2), static schedule or run-time queue by the number of queue entries (schedule = 2),
        # one launch or two by the estimated makespan (fused = 2)
        t0 = time.perf_counter()
        pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", share=2, schedule=2, fused=2, extensions=3,
                                num_slots=args.num_slots, split_align=args.split_align, max_rows=args.max_rows)
        plan_ms = (time.perf_counter() - t0) * 1e3
        view = pa.export()
        t, _ = time_plan(pa, w, rot, steps, warmup)
        res["best_plan"] = {"us_per_step": round(t["step_ms"] * 1e3, 2), "pac_us": round(t["pac_ms_avg"] * 1e3, 2),
                            "picked": {"share": view["share"], "max_rows": view["max_rows"],
                                       "schedule": view["schedule"], "fused": view["fused"]},
                            "plan_ms": round(plan_ms, 2), "est_makespan": view["makespan"]}
        pa.close()
        res["speedup_vs_flat"] = round(res["flat"]["us_per_step"] / res["tree"]["us_per_step"], 3)
        res["tree_vs_flat_max_abs_diff"] = float((outs[1].float() - outs[0].float()).abs().max())
    return res, w, outs[1]


def roofline_of(name, res, w, args, stream_gbps):
    """Roofline objects of the partial-attention kernel for one configuration.

    Algorithmic bytes per launch = unique KV bytes (512 B per token and KV head, every node once);
    duration = the kernel's average over the timed launches, HIP events on the launch stream.
    """
    raw = res["tree"]["_raw"]
    unique = res["unique_kv_bytes"]
    achieved = unique / (raw["pac_ms_avg"] * 1e-3) / 1e9
    # HBM bytes per launch as counted by rocprofv3 (--pmc FETCH_SIZE / WRITE_SIZE, scaled by a known
    # copy): a committed measurement of the same command, not taken live
    traffic = None
    try:
        with open(os.path.join(ROOT, "profiles", "pac_kernel_traffic.json")) as f:
            t = json.load(f).get(name)
        if t and args.layout == "htd" and not (args.num_slots or args.split_align or args.max_rows):
            traffic = t["fetch_bytes"] + t["write_bytes"]
    except OSError:
        pass
    roof = {"bound": "hbm", "kernel": "pac_kernel (partial attention)",
            "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
            "algorithmic_bytes_per_launch": unique,
            "avg_launch_us": round(raw["pac_ms_avg"] * 1e3, 2),
            "measured_stream_read_GBps": stream_gbps,
            "frac_of_measured_stream": round(achieved / stream_gbps, 4) if stream_gbps else None}
    out = {"roofline": roof}
    # algorithmic flops: 4 * head_dim per (query row, token) pair = 4 d * sum over requests of context * h_q
    f = w.forest
    ctx = sum(int(f.node_len[n]) for r in range(f.num_requests) for n in f.path(r))
    flops = 4.0 * w.head.head_dim * ctx * w.head.num_q_heads
    tf = flops / (raw["pac_ms_avg"] * 1e-3) / 1e12
    out["roofline_mfma"] = {"bound": "mfma", "kernel": "pac_kernel (partial attention)", "achieved": round(tf, 1),
                            "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                            "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                            "algorithmic_flops_per_launch": flops}
    return out


def stream_calibration():
    """Read rate of a plain streaming kernel on this machine: 8 GiB, 16-byte loads, 4 KB chunks per workgroup."""
    import torch
    import paper_2505_17694_amd as C
    nbytes = 8 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    buf.view(torch.int32).random_(0, 1 << 30)
    sink = torch.zeros(1 << 16, dtype=torch.int32, device="cuda:0")
    stream = torch.cuda.current_stream()
    res = {}
    for label, pattern, nt in (("linear", 0, 0), ("linear_nontemporal", 0, 1),
                               ("scattered_4KB", 1, 0), ("scattered_4KB_nontemporal", 1, 1)):
        best = None
        for groups in (2048, 4096, 8192):
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                st = C.codec_stream_read_probe(buf.data_ptr(), nbytes, pattern, nt, groups, sink.data_ptr(),
                                               stream.cuda_stream)
                e1.record(stream)
                if st != C.CODEC_OK:
                    raise C.CodecError(st, "codec_stream_read_probe")
                torch.cuda.synchronize()
                gbps = nbytes / (e0.elapsed_time(e1) * 1e-3) / 1e9
                best = gbps if best is None else max(best, gbps)
        res[label] = round(best, 1)
    del buf, sink
    torch.cuda.empty_cache()
    return res


NO_DIVISION = 1 << 20          # split_align above every node length: no node is divided


def run_sweep(args):
    """Paper-shaped synthetic sweeps (Sec. 7): tree vs flat per point; the ablation grid; fixed slice counts."""
    import torch
    import paper_2505_17694_amd as C
    from workloads import make_workload, forest_stats
    from workloads.sweeps import sweep_points, sweep_head, SWEEP_SEED

    head = sweep_head()
    if args.sweep == "granularity":
        points = sweep_points("ablation") + [p for p in sweep_points("batch") if p[0] == "requests=32"]
        variants = [("adaptive", {})] + [(f"fixed={n}", {"fixed_slices": n}) for n in (1, 2, 4, 8, 16, 32, 64)]
    elif args.sweep == "ablation":
        points = sweep_points("ablation")
        variants = [("none", {"share": 0, "split_align": NO_DIVISION}),
                    ("tree_only", {"share": 1, "split_align": NO_DIVISION}),
                    ("division_only", {"share": 0}), ("all", {"share": 1})]
    else:
        points = sweep_points(args.sweep)
        variants = [("tree", {"share": 1}), ("flat", {"share": 0}), ("best_plan", {"share": 2, "schedule": 2})]
    steps = max(5, min(args.steps, 20))
    out_points = []
    for label, forest in points:
        w = make_workload(label, forest, head, SWEEP_SEED, device="cuda:0", layout=args.layout)
        st = forest_stats(forest)
        unique_bytes = st["unique_tokens"] * head.bytes_per_token
        pool_bytes = 2 * w.k_pool.numel() * 2
        copies = max(1, min(int(math.ceil(COLD_FOOTPRINT_BYTES / max(pool_bytes, 1))), 64))
        free, _ = torch.cuda.mem_get_info()
        copies = max(1, min(copies, int(free * 0.8 // max(pool_bytes, 1)) + 1))
        rot = Rotating(w, copies)
        pt = {"point": label, "requests": st["num_requests"], "nodes": st["num_nodes"],
              "unique_kv_bytes": unique_bytes, "mean_sharing": round(st["mean_sharing"], 3)}
        for key, kw in variants:
            opts = {"share": 1, "num_slots": args.num_slots, "split_align": args.split_align, "max_rows": args.max_rows,
                    "extensions": 3}
            opts.update(kw)
            pa = C.PlannedAttention(w.forest, w.paged, w.head, device="cuda:0", **opts)
            view = pa.export()
            t, _ = time_plan(pa, w, rot, steps, args.warmup)
            pt[key] = {"us_per_step": round(t["step_ms"] * 1e3, 2),
                       "unique_kv_GBps": round(unique_bytes / (t["step_ms"] * 1e-3) / 1e9, 1),
                       "tasks": len(view["tasks"]), "est_makespan": view["makespan"]}
            if opts["share"] == 2:
                pt[key]["picked"] = {"share": view["share"], "max_rows": view["max_rows"], "schedule": view["schedule"]}
            pa.close()
        base = {"ablation": "none", "granularity": "fixed=1"}.get(args.sweep, "flat")
        best = {"ablation": "all", "granularity": "adaptive"}.get(args.sweep, "tree")
        pt["speedup"] = round(pt[base]["us_per_step"] / pt[best]["us_per_step"], 3)
        if args.sweep == "granularity":
            fixed_best = min(v["us_per_step"] for k, v in pt.items() if isinstance(v, dict) and k.startswith("fixed="))
            pt["adaptive_vs_best_fixed"] = round(fixed_best / pt["adaptive"]["us_per_step"], 3)
        print(f"[sweep {args.sweep}] {label}: " + ", ".join(
            f"{k} {v['us_per_step']} us" for k, v in pt.items() if isinstance(v, dict)) + f", speedup {pt['speedup']}x",
              file=sys.stderr, flush=True)
        out_points.append(pt)
        del rot, w
        torch.cuda.empty_cache()
    speedups = [p["speedup"] for p in out_points]
    geo = math.exp(sum(math.log(x) for x in speedups) / len(speedups))
    line = {"metric": f"sweep_{args.sweep}_speedup_geomean", "value": round(geo, 3), "unit": "x",
            "n_gpus": 1, "steps": steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"sweep:{args.sweep}", "q_heads": head.num_q_heads, "kv_heads": head.num_kv_heads,
                       "head_dim": head.head_dim, "page_size": head.page_size, "kv_layout": args.layout},
            "points": out_points}
    print(json.dumps(line))


def cpu_baseline(w, gpu_out, seconds):
    """The fp64 oracle, as it stands, on a bounded sample of (request, head) pairs of the workload."""
    import numpy as np
    from oracle import attention as A

    f, h = w.forest, w.head
    B, H = f.num_requests, h.num_q_heads
    ctx = np.array([sum(int(f.node_len[n]) for n in f.path(r)) for r in range(B)], dtype=np.int64)
    total_tokens = int(ctx.sum()) * H                    # (request, head, token) triples of one step
    rng = np.random.Generator(np.random.PCG64(4242))
    order = rng.permutation(B * H)
    threads = A.max_threads()
    # the host copies of the inputs are made once, outside the timed region
    qb, kb, vb = w.q_bits(), w.k_bits(), w.v_bits()
    p = w.paged

    def run(pairs):
        t0 = time.perf_counter()
        out, _ = A.decode_attention(f.parent, f.node_len, f.req_node, p.node_page_off, p.page_ids,
                                    p.page_size, H, h.num_kv_heads, h.head_dim, h.dtype, h.scale,
                                    qb, kb, vb, p.page_stride, p.token_stride, p.head_stride, sel=pairs)
        return time.perf_counter() - t0, out

    probe = [(int(i // H), int(i % H)) for i in order[:2 * threads]]
    t_probe, _ = run(probe)
    per_token = t_probe / max(1, sum(int(ctx[r]) for r, _ in probe))
    n = int(min(B * H, max(2 * threads, seconds / max(per_token * ctx.mean(), 1e-9))))
    pairs = [(int(i // H), int(i % H)) for i in order[:n]]
    t, out = run(pairs)
    sample_tokens = sum(int(ctx[r]) for r, _ in pairs)
    t_full = t * total_tokens / sample_tokens
    got = gpu_out.double().cpu().numpy()
    err = float(np.max(np.abs(np.stack([got[r, hq] for r, hq in pairs]) - out)))
    unique_bytes = w.unique_kv_bytes
    return {"value": round(unique_bytes / t_full / 1e9, 4), "unit": "GB/s", "cores": threads,
            "kind": "oracle",
            "sample": f"{n} of {B * H} (request, head) pairs of {w.name} ({sample_tokens} of {total_tokens} "
                      f"(request, head, token) triples) in {t:.2f} s; scaled to one full step = {t_full:.2f} s",
            "seconds_per_step": round(t_full, 3), "gpu_vs_oracle_max_abs_err_on_sample": err}


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on ONE GPU; --gpus {args.gpus} is not supported "
              "(no collectives, no sharding: the path would shard over KV heads, each head on its own GPU, "
              "with no exchange inside attention)", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    if args.sweep:
        run_sweep(args)
        return

    stream = None
    if not args.no_stream_calibration:
        stream = stream_calibration()
        print(f"[bench] streaming-read kernel, 8 GiB: {stream} GB/s", file=sys.stderr, flush=True)
    # the reference rate for the attention kernel: the scattered 4 KB walk (a paged pool's pattern) with
    # the hint the kernel itself uses for slices that are read once
    stream_gbps = stream["scattered_4KB_nontemporal"] if stream else None

    names = [c for c in args.configs.split(",") if c]
    if args.workload not in names:
        names.append(args.workload)
    per_config = {}
    headline = None
    for name in names:
        is_head = name == args.workload
        steps = args.steps if is_head else max(10, min(args.steps, 30))
        res, w, out = run_config(name, args, steps, args.warmup, not args.no_flat)
        print(f"[bench] {name}: tree {res['tree']['us_per_step']} us/step "
              f"({res['tree']['unique_kv_GBps']} GB/s unique KV)"
              + (f", flat {res['flat']['us_per_step']} us, speedup {res['speedup_vs_flat']}x" if "flat" in res else ""),
              file=sys.stderr, flush=True)
        res.update(roofline_of(name, res, w, args, stream_gbps))
        if name != "cfg5a" and not (is_head and name == "cfg5c"):
            res.pop("roofline_mfma")                    # the matrix roof matters where query sets are large
        if not args.no_cpu_baseline:
            res["cpu_baseline"] = cpu_baseline(w, out, args.cpu_seconds if is_head else args.cpu_seconds_other)
        raw = res["tree"]["_raw"]
        for k in ("tree", "flat"):
            if k in res:
                res[k].pop("_raw", None)
        if is_head:
            headline = (res, w.head, raw)
        del w, out
        torch.cuda.empty_cache()
        per_config[name] = res

    if args.copy_calibration:
        # reads 1 GiB and writes 1 GiB; shows up in a profile as an elementwise kernel with "MulFunctor"
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.5, out=dst)
        torch.cuda.synchronize()
        del src, dst

    res, head, raw = headline
    line = {
        "metric": "decode_attention_unique_kv_bandwidth",
        "value": res["tree"]["unique_kv_GBps"],
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(raw["step_ms"], 5),
        "us_per_step": res["tree"]["us_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if head.dtype == 1 else "fp16",
        "data": "synthetic",
        "config": {"workload": args.workload, "q_heads": head.num_q_heads, "kv_heads": head.num_kv_heads,
                   "head_dim": head.head_dim, "page_size": head.page_size, "kv_layout": args.layout,
                   "requests": res["requests"], "nodes": res["nodes"], "unique_kv_bytes": res["unique_kv_bytes"],
                   "plan": "prefix-shared, static schedule, planner extensions slack+diagonal",
                   "cold_cache": f"rotation over {res['pool_copies']} K/V pool copies"},
        "speedup_vs_flat": res.get("speedup_vs_flat"),
        "roofline": res["roofline"],
        "cpu_baseline": res.get("cpu_baseline"),
        "stream_read_calibration_GBps": stream,
        "per_config": per_config,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
