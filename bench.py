#!/usr/bin/env python3
"""Benchmark of the incremental-update hot path on one MI355X.

One "step" = one ink_apply_updates call: a batch of B edge updates pushed through the whole
path (graph store, events, grouping, aggregation, combination, compare-and-emit) for every
layer.  Inputs are seeded and synthetic (R-MAT graph, N(0,1) features, Xavier weights).  The
default workload is the largest single-GPU configuration: the 3-layer GraphSAGE-max model on the
20 M-node / 400 M-edge graph with batches of 10 000 updates, followed by the batch-size sweep
1 ... 100 000 on the same graph.

Prints ONE JSON line:
  value / ms_per_step   edge updates per second with the update batches resident in HBM
  host_batches          the same steps with the batch handed over in host memory (H2D included)
  roofline              ONE kernel, the one with the largest share of the step: bytes the method
                        must move for that launch (per-layer counters of the library) over its
                        HIP-event time on the library's stream, against the 8 TB/s HBM peak
  transform             the dense combination: useful fp32 flops over its time, against the MFMA peak
  sweep                 p50 / p99 latency and throughput per batch size
  cpu_baseline          the CPU oracle's full inference, timed on a bounded row sample
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3
SWEEP_SIZES = (1, 10, 100, 1000, 10000, 100000)
KERNEL_NAMES = {"agg_events": "k_agg_events (incremental aggregation over grouped events)",
                "agg_exposed": "k_agg_full over the exposed rows (one wave per row)",
                "agg_long": "k_big_partial / k_big_final (long rows, chunked)",
                "agg_full": "k_agg_full / k_sum_full (recompute of every row)"}


def kernel_bytes(kern, L, d, select, sources, inline_exposed=False):
    """Bytes one launch of an aggregation kernel must move, from the layer's counters.

    The accounting per layer is: every event record read once (4 B, plus 8 B per target for its id
    and segment start); the new row of every DISTINCT changed source once (4 d B each: a row that many
    events name is charged once, however often the cache serves it); the aggregated row and, for
    max / min, the holder row of every target read and written (2 * 4 d, times 2 for max / min);
    a recomputed row reads, per neighbour, one id and one message row (4 + 4 d B).
    Returns (bytes by that accounting, bytes as designed).  As designed adds what this
    implementation moves on top: one source row per non-delete event (mostly cache hits) and the
    two runner-up tables of max / min (another 2 * 2 * 4 d per target).  inline_exposed: the event
    kernel itself recomputed the exposed rows of moderate length (no follow-up launch ran), so their
    neighbour rows count for it."""
    t, e = L["n_targets"], L["n_events"]
    row = 4 * d
    rw = 2 * row * (2 if select else 1)
    nb_long = L["n_regather_nb_long"]
    nb = L["n_regather_nb"]
    if kern == "agg_events":
        alg = e * 4 + t * 8 + sources * row + t * rw + ((nb - nb_long) * (4 + row) if inline_exposed else 0)
        return alg, alg + max(e - sources, 0) * row + (t * rw if select else 0)
    if kern == "agg_long":
        return nb_long * (4 + row), nb_long * (4 + row)
    rows = L["n_exposed"] if kern == "agg_exposed" else L["n_targets"]
    alg = (nb - nb_long) * (4 + row) + (rows * rw if kern == "agg_full" else 0)
    return alg, alg + (rows * rw if select else 0)


def read_traffic(workload, kern):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 counters: kept in the
    profile summary of that kernel and workload (which names the commands that produced it)."""
    path = os.path.join(ROOT, "profiles", "%s_%s.md" % (kern, workload.replace("/", "_")))
    if not os.path.exists(path):
        return None, None
    m = re.search(r"^traffic_bytes_per_launch\s*[:=]\s*([0-9.eE+]+)", open(path).read(), re.M)
    return (float(m.group(1)) if m else None), os.path.relpath(path, ROOT)


def cpu_baseline(cfg, model, ink, keys, X, affected_rows=None, target_s=12.0):
    """Oracle full inference on the current snapshot, timed layer by layer on a sample of destination
    rows and scaled to all rows.  With affected_rows (rows of the theoretical affected area per layer,
    as counted by the library's own affected-area run of one batch) also the cost of the paper's
    "Affected" baseline (Sec. 4.1) on the CPU: each layer's time scaled by its share of rows."""
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
        per_layer = []
        for l in range(k):
            t0 = time.perf_counter()
            a, _ = oracle.aggregate(sub_rp, sub_col, hs[l], model["agg"])
            oracle.transform(model, l, a, hs[l][:rows], "f64")
            per_layer.append(time.perf_counter() - t0)
        dt = sum(per_layer)
        if dt >= target_s / 3 or rows == n:
            break
        rows = int(rows * min(8.0, max(2.0, target_s / max(dt, 1e-3) * 0.6)))
    t_full = dt * (n / rows)
    out = dict(value=cfg.batch / t_full, unit="edge updates/s", cores=cores, kind="oracle",
               sample="full %d-layer inference of destination rows [0,%d) of %d (%.1f s), scaled by N/rows; "
                      "one full inference per batch => %.1f s per batch" % (k, rows, n, dt, t_full),
               seconds_per_full_inference=t_full)
    if affected_rows is not None and model["agg"] != "gcn_sym":
        t_aff = sum(per_layer[l] / rows * affected_rows[l] for l in range(k))
        out["affected"] = dict(value=cfg.batch / max(t_aff, 1e-9), unit="edge updates/s", seconds_per_batch=t_aff,
                               affected_rows_per_layer=[int(x) for x in affected_rows],
                               note="the CPU oracle restricted to the theoretical affected area of one batch (Sec. 4.1 "
                                    "'Affected'): per-layer oracle time per row x rows of the area at that layer")
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--scale-div", type=int, default=1)
    ap.add_argument("--batch", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--method", choices=["incremental", "affected"], default="incremental",
                    help="affected: time the affected-area recompute baseline (Sec. 4.1) instead")
    ap.add_argument("--sweep", dest="sweep", action="store_true", default=None,
                    help="after the timed steps: 3 warm-up + 20 timed seeded batches at each batch size 1..100k "
                         "(default: on for config 5)")
    ap.add_argument("--no-sweep", dest="sweep", action="store_false")
    ap.add_argument("--calibration", action="store_true",
                    help="also launch plain copy and row-gather kernels of known size, so that a profiler's "
                         "byte counters can be scaled (see profiles/)")
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
    sweep = args.sweep if args.sweep is not None else (args.config == 5)
    select = cfg.agg in ("max", "min")
    t0 = time.perf_counter()
    src, dst = synth.make_graph(cfg)
    rp, col = synth.in_csr_from_edges(cfg.n_nodes, src, dst, assume_sorted=True)
    X = synth.make_features(cfg)
    model = synth.make_model(cfg)
    t_gen = time.perf_counter() - t0
    print("[bench] %s: N=%d E=%d generated in %.1f s" % (cfg.name, cfg.n_nodes, src.size, t_gen), file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    ink = Ink(rp, col, X, model, profile=True, batch_device=True, max_batch=max(SWEEP_SIZES) if sweep else cfg.batch)
    t_create = time.perf_counter() - t0
    ink.full_infer()                  # first call also sizes the library's work buffers
    t0 = time.perf_counter()
    ink.full_infer()                  # steady state: this one is reported
    t_full = time.perf_counter() - t0
    full_stats = ink.stats()
    print("[bench] create %.1f s, full inference %.3f s" % (t_create, t_full), file=sys.stderr, flush=True)
    sampler = synth.BatchSampler(cfg, src, dst)
    n_edges = int(src.size)
    del rp, col, src, dst
    aff = args.method == "affected"

    def draw(n_batches, B=None):
        host = [torch.from_numpy(make_updates(*sampler.next_batch(B)).view(np.uint8).copy()).pin_memory()
                for _ in range(n_batches)]
        return host

    # ---- the timed steps: batches resident in HBM before the clock starts
    host_batches = draw(args.warmup + args.steps)
    batches = [h.cuda() for h in host_batches]
    torch.cuda.synchronize()
    if args.calibration:
        calibration_kernels(torch)
    copy_gbs = measured_copy_rate(torch)
    for i in range(args.warmup):
        ink.apply_updates_device(batches[i].data_ptr(), cfg.batch, affected=aff)
    lat, changed = [], 0
    per_class, kern_ms, kern_n, kern_each = {}, {}, {}, {}
    layer_tot, layer_src = None, None
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.warmup, args.warmup + args.steps):
        t1 = time.perf_counter()
        r = ink.apply_updates_device(batches[i].data_ptr(), cfg.batch, affected=aff)
        lat.append(time.perf_counter() - t1)
        st = ink.stats()                      # host-side struct copy, no GPU work
        changed += r["n_changed"]
        for k_, v in st["ms"].items():
            per_class[k_] = per_class.get(k_, 0.0) + v
        for li, L in enumerate(st["layers"]):
            for k_, v in L.pop("ms_kernel").items():
                if v > 0:
                    kern_ms[(li, k_)] = kern_ms.get((li, k_), 0.0) + v
                    kern_n[(li, k_)] = kern_n.get((li, k_), 0) + 1
                    kern_each.setdefault((li, k_), []).append(v)
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

    # ---- the dominant kernel and its roofline
    agg_keys = [k_ for k_ in kern_ms if k_[1].startswith("agg")]
    roof = {"bound": "hbm", "achieved": 0.0, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": 0.0, "traffic": None}
    if agg_keys:
        li, kern = max(agg_keys, key=lambda k_: kern_ms[k_])
        launches = kern_n[(li, kern)]
        L = {k_: v / args.steps for k_, v in layer_tot[li].items()}         # per-step averages of that layer
        d = ink.agg_widths[li]
        inline_exposed = kern == "agg_events" and L["n_exposed"] > 0 and kern_n.get((li, "agg_exposed"), 0) == 0
        alg, designed = kernel_bytes(kern, L, d, select, L["n_sources"], inline_exposed)
        avg_ms = kern_ms[(li, kern)] / launches
        ach = alg / 1e9 / (avg_ms / 1e3)
        traffic, traffic_src = read_traffic(cfg.name, kern)
        roof.update({
            "achieved": ach, "frac": ach / HBM_PEAK_GBS,
            "kernel": "%s, layer %d" % (KERNEL_NAMES[kern], li + 1),
            "launches": launches, "avg_launch_ms": avg_ms,
            "median_launch_ms": float(np.median(kern_each[(li, kern)])),
            "algorithmic_bytes_per_launch": alg,
            "as_designed_bytes_per_launch": designed,
            "as_designed_GBs": designed / 1e9 / (avg_ms / 1e3),
            "traffic": traffic, "traffic_source": traffic_src,
            "measured_copy_GBs": copy_gbs,
            "measured_random_row_gather_GBs": measured_gather_rate(torch, ink.agg_widths[li]),
            "share_of_step": kern_ms[(li, kern)] / args.steps / (total / args.steps * 1e3),
            "units_per_launch": {"targets": L["n_targets"], "events": L["n_events"], "distinct_sources": L["n_sources"],
                                 "row_floats": d, "exposed_rows_recomputed_inside": bool(inline_exposed),
                                 "neighbour_rows_of_those": (L["n_regather_nb"] - L["n_regather_nb_long"]) if inline_exposed else 0},
            "above_hbm_peak": bool(ach > HBM_PEAK_GBS),     # then the launch re-reads rows that L2 / MALL serve: see traffic
            "note": "achieved = bytes the method must move for this launch (each distinct source row once, value and "
                    "holder row of each target read and written) / HIP-event time of this kernel; as_designed adds the "
                    "per-event source-row reads that the caches serve and the two runner-up tables"})
    # every timed kernel, per step
    kernels = [{"layer": li + 1, "kernel": k_, "ms_per_step": v / args.steps} for (li, k_), v in sorted(kern_ms.items())]
    # dense combination against the fp32 MFMA peak
    xf = None
    xf_ms = sum(v for (li, k_), v in kern_ms.items() if k_ == "xform")
    if xf_ms > 0:
        flops = 0.0
        for li, Lm in enumerate(model["layers"]):
            rows = layer_tot[li]["n_transformed"] / args.steps
            if cfg.model == "sage":
                flops += 2.0 * rows * 2 * Lm["in_dim"] * Lm["out_dim"]
            elif cfg.model == "gin":
                flops += 2.0 * rows * (Lm["in_dim"] * Lm["mlp_hidden"] + Lm["mlp_hidden"] * Lm["out_dim"])
            elif li + 1 < len(model["layers"]):
                flops += 2.0 * rows * model["layers"][li + 1]["in_dim"] * model["layers"][li + 1]["out_dim"]
        xf = {"bound": "mfma", "achieved": flops / 1e12 / (xf_ms / args.steps / 1e3), "peak": MFMA_F32_PEAK_TFLOPS,
              "unit": "TFLOP/s", "ms_per_step": xf_ms / args.steps}
        xf["frac"] = xf["achieved"] / MFMA_F32_PEAK_TFLOPS

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
        "config": {"workload": cfg.name, "gnn": cfg.model, "aggregator": cfg.agg, "nodes": cfg.n_nodes,
                   "edges": n_edges, "dims": list(cfg.dims), "batch": cfg.batch,
                   "hub_biased_deletes": cfg.hub_biased_deletes},
        "roofline": roof,
        "transform": xf,
        "kernels_ms_per_step": kernels,
        "gpu_ms_per_step_by_class": {k_: v / args.steps for k_, v in per_class.items()},
        "per_step_layer_counts": [{k_: v / args.steps for k_, v in L.items()} for L in (layer_tot or [])],
        "changed_nodes_per_step": changed / args.steps,
        "full_inference_s": t_full,
        "full_inference_agg_ms": full_stats["ms"]["agg"],
    }
    # the recompute kernels at their largest shape (every edge gathers one id and one message row, every
    # node writes its aggregated row and, for max / min, its holder row)
    fb = sum(n_edges * (4 + 4 * d) + cfg.n_nodes * 4 * d * (2 if select else 1) for d in ink.agg_widths)
    fms = max(full_stats["ms"]["agg"], 1e-6)
    out["full_inference_roofline"] = {"bound": "hbm", "achieved": fb / 1e9 / (fms / 1e3), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                      "frac": fb / 1e9 / (fms / 1e3) / HBM_PEAK_GBS, "algorithmic_bytes": fb,
                                      "note": "all aggregation launches of a full inference; message tables that fit "
                                              "L2 / MALL are re-read from cache"}

    # ---- the same protocol with the batch handed over in host memory: the H2D copy is inside the clock
    ink.set_profiling(False)
    hb = draw(args.steps)
    dev = torch.empty_like(hb[0], device="cuda")
    torch.cuda.synchronize()
    hl = []
    t_start = time.perf_counter()
    for h in hb:
        t1 = time.perf_counter()
        dev.copy_(h, non_blocking=False)
        ink.apply_updates_device(dev.data_ptr(), cfg.batch, affected=aff)
        hl.append(time.perf_counter() - t1)
    torch.cuda.synchronize()
    h_total = time.perf_counter() - t_start
    out["host_batches"] = {"value": cfg.batch * args.steps / h_total, "ms_per_step": h_total / args.steps * 1e3,
                           "p50_ms": float(np.percentile(np.array(hl) * 1e3, 50)),
                           "note": "batch in pinned host memory, copied to the device inside the timed call; profiling off"}

    if sweep:
        res = []
        for B in SWEEP_SIZES:
            bl = [h.cuda() for h in draw(3 + 20, B)]
            torch.cuda.synchronize()
            lt, ev = [], []
            for j, t in enumerate(bl):
                t1 = time.perf_counter()
                ink.apply_updates_device(t.data_ptr(), B, affected=aff)
                if j >= 3:
                    lt.append((time.perf_counter() - t1) * 1e3)
                    ev.append(sum(L["n_events"] for L in ink.stats()["layers"]))
            lt, ev = np.array(lt), np.array(ev, dtype=np.float64)
            slow = int(np.argmax(lt))
            res.append({"batch": B, "p50_ms": float(np.percentile(lt, 50)), "p99_ms": float(np.percentile(lt, 99)),
                        "max_ms": float(lt.max()), "edges_per_s": float(B * len(lt) / (lt.sum() / 1e3)),
                        "events_p50": float(np.median(ev)), "events_of_slowest": float(ev[slow]),
                        "latency_vs_events_corr": float(np.corrcoef(lt, ev)[0, 1]) if ev.std() > 0 and lt.std() > 0 else None})
            print("[bench] sweep B=%d p50 %.3f ms p99 %.3f ms" % (B, res[-1]["p50_ms"], res[-1]["p99_ms"]),
                  file=sys.stderr, flush=True)
        out["sweep"] = res
    ink.set_profiling(True)
    if not args.no_cpu_baseline:
        # one more batch through the affected-area baseline of the library: its targets per layer are the
        # theoretical affected area (the cache ends in the same state as after the incremental call)
        b = draw(1)[0].cuda()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ink.apply_updates_device(b.data_ptr(), cfg.batch, affected=True)
        out["gpu_affected_baseline_ms"] = (time.perf_counter() - t1) * 1e3
        area = [L["n_targets"] for L in ink.stats()["layers"]]
        cs, cd = sampler.current_edges()
        keys = synth.edge_keys(cs, cd)
        out["cpu_baseline"] = cpu_baseline(cfg, model, ink, keys, X, area)
    print(json.dumps(out))
    ink.close()


def measured_copy_rate(torch):
    """Practical HBM ceiling next to the nominal one: a plain device copy (1 GiB read + 1 GiB written)."""
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
        return 5 * 2 * a.numel() * 4 / 1e9 / (e0.elapsed_time(e1) / 1e3)
    except RuntimeError:
        return None


def measured_gather_rate(torch, row_floats):
    """What a plain gather kernel reaches on random rows of the dominant kernel's width (bytes of the
    rows read + written per second): 2^23 random rows out of a 4 GiB table, far larger than L2 and MALL."""
    try:
        rows = (1 << 30) // row_floats
        table = torch.empty(rows * row_floats, dtype=torch.float32, device="cuda").normal_().view(rows, row_floats)
        g = torch.Generator(device="cuda")
        g.manual_seed(11)
        idx = torch.randint(0, rows, (1 << 23,), device="cuda", generator=g)
        out = torch.index_select(table, 0, idx)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(3):
            torch.index_select(table, 0, idx, out=out)
        e1.record()
        torch.cuda.synchronize()
        return 3 * 2 * idx.numel() * row_floats * 4 / 1e9 / (e0.elapsed_time(e1) / 1e3)
    except RuntimeError:
        return None


def calibration_kernels(torch):
    """Kernels of known size for scaling a profiler's byte counters: one streaming copy (1 GiB read,
    1 GiB written) and row gathers of 2^21 random rows of 192 B, 512 B and 1 KiB from a 4 GiB table
    (far larger than L2 and MALL, so every row comes from HBM)."""
    a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    b = torch.empty_like(a)
    torch.cuda.synchronize()
    torch.mul(a, 1.0, out=b)
    torch.cuda.synchronize()
    del a, b
    a = torch.empty(1 << 30, dtype=torch.float32, device="cuda").normal_()
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    for width in (48, 128, 256):
        rows = (1 << 30) // width
        table = a[: rows * width].view(rows, width)
        idx = torch.randint(0, rows, (1 << 21,), device="cuda", generator=g)
        torch.cuda.synchronize()
        out = torch.index_select(table, 0, idx)
        torch.cuda.synchronize()
        del out, idx
    del a


if __name__ == "__main__":
    main()
