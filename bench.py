#!/usr/bin/env python3
"""Benchmark of the incremental-update hot path on one MI355X.

One "step" = one ink_apply_updates call: a batch of B edge updates pushed through the whole
path (graph store, events, grouping, aggregation, combination, compare-and-emit) for every
layer.  Inputs are seeded and synthetic (R-MAT graph, N(0,1) features, Xavier weights); the
update batches are resident in HBM before the timed region starts.

Prints ONE JSON line: metric/value (edge updates per second), latency percentiles, the roofline
block for the dominant kernel class (neighbour-gather aggregation, HBM-bound) and the CPU
oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per aggregation launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two runs
# of this script, summaries under profiles/): all aggregation kernels of one update batch, fetch
# counter scaled by 2.0 and write counter by 1.0 (what a plain 1 GiB copy kernel reads back in the
# same runs), divided by the aggregation launches of the batch (one per layer).
MEASURED_TRAFFIC_PER_LAUNCH = {
    2: {"bytes": 7.16e9, "source": "profiles/all_kernels_cfg2_gcn.md"},
    3: {"bytes": 8.82e8, "source": "profiles/all_kernels_cfg3_sage_max.md"},
}


def agg_algorithmic_bytes(layer_stats, agg_width, n_del, select):
    """Bytes the aggregation kernels of one step must move (per layer, summed).

    events: 4 B payload each; every non-delete event reads one source row (4 d B);
    targets: the cached row is read and, when alpha changed, rewritten.  A cached row is alpha
    alone for the sum-type aggregators (4 d B) and alpha + holder + runner-up value + runner-up
    id for max / min (16 d B; the runner-up pair, 8 d B, is rewritten for every target);
    recomputes: per neighbour one id (4 B) and one message row (4 d B).
    A dense layer is a recompute of every node."""
    total = 0
    row = 16 if select else 4
    for L, d in zip(layer_stats, agg_width):
        if L["dense"]:
            total += L["n_regather_nb"] * (4 + 4 * d) + L["n_targets"] * row * d
            continue
        ev = L["n_events"]
        total += ev * 4 + max(ev - n_del, 0) * 4 * d
        total += L["n_targets"] * row * d + L["n_alpha_changed"] * row * d
        if select:
            total += (L["n_targets"] - L["n_alpha_changed"]) * 8 * d
        total += L["n_regather_nb"] * (4 + 4 * d)
    return total


def cpu_baseline(cfg, model, ink, keys, X, target_s=12.0):
    """Oracle full inference on the current snapshot, timed on a sample of destination rows."""
    import oracle
    n = cfg.n_nodes
    rp, col = oracle.csr_from_keys(n, keys)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    k = len(model["layers"])
    rows = max(256, n // 4096)
    hs = [X] + [ink.get_layer(l, 0) for l in range(1, k)]       # realistic layer inputs for timing
    while True:
        rows = min(rows, n)
        sub_rp = rp[: rows + 1]
        sub_col = col[: sub_rp[-1]]
        t0 = time.perf_counter()
        for l in range(k):
            a, _ = oracle.aggregate(sub_rp, sub_col, hs[l], model["agg"])
            oracle.transform(model, l, a, hs[l][:rows], "f64")
        dt = time.perf_counter() - t0
        if dt >= target_s / 3 or rows == n:
            break
        rows = int(rows * min(8.0, max(2.0, target_s / max(dt, 1e-3) * 0.6)))
    t_full = dt * (n / rows)
    return dict(value=cfg.batch / t_full, unit="edge updates/s", cores=cores, kind="oracle",
                sample="full %d-layer inference of destination rows [0,%d) of %d (%.1f s), scaled by N/rows; "
                       "one full inference per batch => %.1f s per batch" % (k, rows, n, dt, t_full),
                seconds_per_full_inference=t_full)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--scale-div", type=int, default=1)
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--method", choices=["incremental", "affected"], default="incremental",
                    help="affected: time the affected-area recompute baseline (Sec. 4.1) instead")
    ap.add_argument("--sweep", action="store_true",
                    help="after the timed steps, run 20 seeded batches at each batch size 1..100k and report p50/p99")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy so that a profiler's byte counters can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import synth
    from paper_2309_11071_amd import Ink
    from paper_2309_11071_amd.binding import make_updates
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.get_config(args.config, args.scale_div)
    if args.batch:
        from dataclasses import replace
        cfg = replace(cfg, batch=args.batch)
    t0 = time.perf_counter()
    src, dst = synth.make_graph(cfg)
    rp, col = synth.in_csr_from_edges(cfg.n_nodes, src, dst, assume_sorted=True)
    X = synth.make_features(cfg)
    model = synth.make_model(cfg)
    t_gen = time.perf_counter() - t0
    print("[bench] %s: N=%d E=%d generated in %.1f s" % (cfg.name, cfg.n_nodes, src.size, t_gen), file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    ink = Ink(rp, col, X, model, profile=True, batch_device=True)
    t_create = time.perf_counter() - t0
    ink.full_infer()                  # first call also sizes the library's work buffers
    t0 = time.perf_counter()
    ink.full_infer()                  # steady state: this one is reported
    t_full = time.perf_counter() - t0
    full_stats = ink.stats()
    print("[bench] create %.1f s, full inference %.3f s" % (t_create, t_full), file=sys.stderr, flush=True)
    sampler = synth.BatchSampler(cfg, src, dst)
    del rp, col
    batches = []
    for _ in range(args.warmup + args.steps):
        op, bs, bd = sampler.next_batch()
        u = make_updates(op, bs, bd)
        batches.append(torch.from_numpy(u.view(np.uint8).copy()).cuda())
    torch.cuda.synchronize()
    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        torch.mul(a, 1.0, out=b)        # plain elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
    # practical HBM ceiling next to the nominal one: a plain device copy (1 GiB read + 1 GiB written)
    copy_gbs = None
    try:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        torch.mul(a, 1.0, out=b)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            torch.mul(a, 1.0, out=b)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 5 * 2 * a.numel() * 4 / 1e9 / (e0.elapsed_time(e1) / 1e3)
        del a, b
    except RuntimeError:
        pass
    aff = args.method == "affected"
    for i in range(args.warmup):
        ink.apply_updates_device(batches[i].data_ptr(), cfg.batch, affected=aff)
    lat, agg_ms, agg_launches, agg_bytes, changed = [], 0.0, 0, 0, 0
    per_class = {}
    layer_tot = None
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        t1 = time.perf_counter()
        r = ink.apply_updates_device(batches[i].data_ptr(), cfg.batch, affected=aff)
        lat.append(time.perf_counter() - t1)
        st = ink.stats()                      # host-side struct copy, no GPU work
        agg_ms += st["ms"]["agg"]
        agg_launches += sum(1 for L in st["layers"] if L["n_events"] > 0)
        agg_bytes += agg_algorithmic_bytes(st["layers"], ink.agg_widths, r["n_applied_del"],
                                           cfg.agg in ("max", "min"))
        changed += r["n_changed"]
        for k_, v in st["ms"].items():
            per_class[k_] = per_class.get(k_, 0.0) + v
        if layer_tot is None:
            layer_tot = [dict(L) for L in st["layers"]]
        else:
            for a, b in zip(layer_tot, st["layers"]):
                for k_ in a:
                    a[k_] += b[k_]
    torch.cuda.synchronize()
    total = time.perf_counter() - t_start
    lat_ms = np.array(lat) * 1e3
    value = cfg.batch * args.steps / total
    achieved = (agg_bytes / 1e9) / (agg_ms / 1e3) if agg_ms > 0 else 0.0
    out = {
        "metric": "edge updates/sec",
        "value": value,
        "unit": "edge updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": total / args.steps * 1e3,
        "p50_ms": float(np.percentile(lat_ms, 50)),
        "p99_ms": float(np.percentile(lat_ms, 99)),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "method": args.method,
        "config": {"workload": cfg.name, "model": cfg.model, "aggregator": cfg.agg, "nodes": cfg.n_nodes,
                   "edges": int(src.size), "dims": list(cfg.dims), "batch": cfg.batch,
                   "hub_biased_deletes": cfg.hub_biased_deletes},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": (MEASURED_TRAFFIC_PER_LAUNCH.get(args.config, {}).get("bytes")
                                 if args.scale_div == 1 and not args.batch else None),
                     "traffic_source": MEASURED_TRAFFIC_PER_LAUNCH.get(args.config, {}).get("source"),
                     "algorithmic_bytes_per_launch": agg_bytes / max(agg_launches, 1),
                     "kernel": "aggregation (k_agg_events / k_agg_full / k_big_*), all layers",
                     "avg_launch_ms": agg_ms / max(agg_launches, 1),
                     "measured_copy_GBs": copy_gbs,
                     "algorithmic_bytes_per_step": agg_bytes / args.steps,
                     "note": "achieved = algorithmic bytes over time; rows gathered many times per launch are "
                             "served by L2 / MALL (compare traffic), so the rate can exceed the HBM peak"},
        "gpu_ms_per_step_by_class": {k_: v / args.steps for k_, v in per_class.items()},
        "per_step_layer_counts": [{k_: v / args.steps for k_, v in L.items()} for L in (layer_tot or [])],
        "changed_nodes_per_step": changed / args.steps,
        "full_inference_s": t_full,
        "full_inference_agg_ms": full_stats["ms"]["agg"],
        # the recompute kernels at their largest shape: every edge gathers one id and one message row,
        # every node writes its cached row (alpha; for max / min also holder, runner-up value and id)
        "full_inference_roofline": (lambda b, ms: {"bound": "hbm", "achieved": b / 1e9 / (ms / 1e3), "peak": HBM_PEAK_GBS,
                                                   "unit": "GB/s", "frac": b / 1e9 / (ms / 1e3) / HBM_PEAK_GBS,
                                                   "algorithmic_bytes": b,
                                                   "note": "algorithmic bytes over time: message tables that fit "
                                                           "L2 / MALL are re-read from cache, so this can exceed the HBM peak"})(
            sum(int(src.size) * (4 + 4 * d) + cfg.n_nodes * (16 if cfg.agg in ("max", "min") else 4) * d
                for d in ink.agg_widths), max(full_stats["ms"]["agg"], 1e-6)),
    }
    if args.sweep:
        sweep = []
        ink.set_profiling(False)
        for B in (1, 10, 100, 1000, 10000, 100000):
            bl = []
            for _ in range(20):
                u = make_updates(*sampler.next_batch(B))
                bl.append(torch.from_numpy(u.view(np.uint8).copy()).cuda())
            torch.cuda.synchronize()
            lt = []
            for t in bl:
                t1 = time.perf_counter()
                ink.apply_updates_device(t.data_ptr(), B, affected=aff)
                lt.append((time.perf_counter() - t1) * 1e3)
            lt = np.array(lt)
            sweep.append({"batch": B, "p50_ms": float(np.percentile(lt, 50)), "p99_ms": float(np.percentile(lt, 99)),
                          "edges_per_s": float(B * len(lt) / (lt.sum() / 1e3))})
            print("[bench] sweep B=%d p50 %.3f ms p99 %.3f ms" % (B, sweep[-1]["p50_ms"], sweep[-1]["p99_ms"]),
                  file=sys.stderr, flush=True)
        out["sweep"] = sweep
        ink.set_profiling(True)
    if not args.no_cpu_baseline:
        cs, cd = sampler.current_edges()
        keys = synth.edge_keys(cs, cd)
        out["cpu_baseline"] = cpu_baseline(cfg, model, ink, keys, X)
    print(json.dumps(out))
    ink.close()


if __name__ == "__main__":
    main()
