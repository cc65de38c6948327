#!/usr/bin/env python3
"""Throughput of the Double Sparsity decode-attention hot path on one MI355X.

A step is one decode step of the attention path over every layer of the
workload: for each layer one ds_sparse_decode call (score -> top-k -> gather ->
softmax.V) on that layer's own label cache and K/V cache, all resident in HBM
before the clock starts.  Distinct caches per layer keep consecutive calls from
re-reading cache-resident data.  Prints one JSON line (see the fields below).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth


def counted_traffic(workload, kernel, library_version):
    """HBM bytes per launch of `kernel` on `workload` as counted by rocprofv3 (FETCH_SIZE plus
    WRITE_SIZE, each scaled by a plain kernel of known size): read from the committed counter
    summary, which names the library version it was taken on.  None when that is not the
    version loaded here (the kernels have changed since), or when the summary has no line for
    this kernel and workload."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")
    found, version_ok = None, False
    try:
        with open(path) as f:
            for line in f:
                tok = line.split()
                if len(tok) == 2 and tok[0] == "library_version":
                    version_ok = int(tok[1]) == library_version
                if len(tok) >= 4 and tok[0] == "traffic_bytes_per_launch" and tok[1] == workload and tok[2] == kernel:
                    found = int(tok[3])
    except OSError:
        pass
    return found if version_ok else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C3", help="C1, C2, C3 (headline), C4a, C4b; C5 = offload pipeline")
    ap.add_argument("--shape", default="",
                    help="B,Hq,Hkv,L,r,k: the named workload with these sizes instead (studies of one part of the path: "
                         "a single unit, almost no rows); d = 128")
    ap.add_argument("--layers", type=int, default=0, help="distinct layer caches to rotate over (0 = workload's)")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every call from Python instead of replaying a HIP graph")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--tune", default="", help="knob=value,... (ds_tune_set)")
    ap.add_argument("--interleaved", action="store_true",
                    help="K|V cache as one [L,2,d] array per head (512-byte gathers), ds_sparse_decode_kv")
    ap.add_argument("--predict", action="store_true",
                    help="C5: select with queries predicted from the previous layer's embedding (W_q GEMV on the select stream)")
    ap.add_argument("--label-bits", type=int, default=16, choices=(16, 4),
                    help="label cache precision: fp16 (the metric's configuration) or the 4-bit cache")
    ap.add_argument("--trace", action="store_true",
                    help="stage stamps of the attention launch: loads the -DDS_TRACE build of the library, runs a few "
                         "layers and prints, per stage, when the workgroups of the last launch reached it")
    ap.add_argument("--label-ablation", action="store_true",
                    help="with / without label cache over the batch x length grid of the paper's ablation table")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU step); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    if args.trace:
        from paper_2408_07092_amd import binding, build as ds_build
        if not os.path.exists(ds_build.LIB_TRACE):
            sys.exit("bench.py --trace: build the stage-stamp library first (python -m paper_2408_07092_amd.build --trace)")
        binding.LIB_PATH = ds_build.LIB_TRACE
    import paper_2408_07092_amd as ds
    from workloads import WORKLOADS, make_calibration_numpy, make_layer_torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = WORKLOADS[args.workload]
    if args.shape:
        B_, Hq_, Hkv_, L_, r_, k_ = (int(x) for x in args.shape.split(","))
        w = w.scaled(name=f"{w.name} as {args.shape}", B=B_, Hq=Hq_, Hkv=Hkv_, L=L_, r=r_, k=k_,
                     note=f"custom shape B{B_} Hq{Hq_} Hkv{Hkv_} L{L_} r{r_} k{k_}")
    for kv in filter(None, args.tune.split(",")):
        kn, val = kv.split("=")
        ds.ds_tune_set(int(kn), int(val))

    if args.label_ablation:
        return bench_label_ablation(args, ds, torch, dev)
    if w.name == "C5":
        return bench_offload(args, w, ds, torch, dev)

    # ---- resident caches: as many distinct layers as the workload has (capped by memory)
    layer_bytes = w.units * w.L * (2 * w.d * 2 + w.r * 2)
    free, _ = torch.cuda.mem_get_info()
    n_layers = args.layers or w.n_layers
    n_layers = max(1, min(n_layers, int(free * 0.8) // layer_bytes))
    shp = ds.shape(w.B, w.Hq, w.Hkv, w.d, w.L, w.L, w.r, w.k)
    mode = ds.DS_CALIB_QK if w.G == 1 else ds.DS_CALIB_Q
    layers = []
    t_gen = time.time()
    for l in range(n_layers):
        qc, kc = make_calibration_numpy(w, layer=l)
        ch = torch.from_numpy(ds.ds_calibrate_channels(qc, kc, w.r, mode)).to(dev)
        t = make_layer_torch(w, dev, layer=l)
        label = torch.empty((w.B, w.Hkv, w.L, w.r), dtype=torch.float16, device=dev)
        ds.ds_build_label(t["K"], ch, label, shp)
        if args.label_bits == 4:
            codes = torch.empty((w.B, w.Hkv, w.L, (w.r + 7) // 8), dtype=torch.int32, device=dev)
            amax = torch.empty((w.B, w.Hkv, w.r), dtype=torch.float32, device=dev)
            ds.ds_build_label_q4(t["K"], ch, codes, amax, shp)
            label = (codes, amax)
        if args.interleaved:
            KV = torch.stack((t["K"], t["V"]), dim=3).contiguous()
            layers.append((t["q"], label, KV, None, ch))
        else:
            layers.append((t["q"], label, t["K"], t["V"], ch))
        del t
    torch.cuda.synchronize()
    t_gen = time.time() - t_gen
    ws = ds.ds_workspace_alloc(shp, dev)
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()   # set-up ran on the default stream, the timed work does not

    def sparse_sweep():
        for (q, label, K, V, ch) in layers:
            if V is None:
                ds.ds_sparse_decode_kv(q, label, K, ch, out, None, ws, shp)
            elif args.label_bits == 4:
                ds.ds_sparse_decode_q4(q, label[0], label[1], K, V, ch, out, None, ws, shp)
            else:
                ds.ds_sparse_decode(q, label, K, V, ch, out, None, ws, shp)

    if args.trace:
        return trace_report(args, w, ds, torch, sparse_sweep)

    def nolabel_sweep():
        for (q, label, K, V, ch) in layers:
            ds.ds_sparse_decode_nolabel(q, K, V, ch, out, None, ws, shp)

    def dense_sweep():
        for (q, label, K, V, ch) in layers:
            ds.ds_dense_decode(q, K, V, out, ws, shp)

    stream = torch.cuda.Stream(device=dev)

    def timed(fn, steps, warmup, use_graph):
        """Returns (ms_per_step by wall clock, ms_per_step by events on the launch stream)."""
        with torch.cuda.stream(stream):
            runner = fn
            if use_graph:
                fn(); stream.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    fn()
                runner = g.replay
            for _ in range(warmup):
                runner()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record(stream)
            for _ in range(steps):
                runner()
            e1.record(stream)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps

    def step_spread(fn, steps, use_graph):
        """Per-step durations (ms) of `steps` further steps, from events between the steps."""
        with torch.cuda.stream(stream):
            runner = fn
            if use_graph:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    fn()
                runner = g.replay
            runner()
            evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            evs[0].record(stream)
            for i in range(steps):
                runner()
                evs[i + 1].record(stream)
            torch.cuda.synchronize()
        return sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(steps))

    use_graph = not args.no_graph
    ms_step, ms_step_ev = timed(sparse_sweep, args.steps, args.warmup, use_graph)
    us_layer = ms_step * 1e3 / n_layers
    spread = step_spread(sparse_sweep, args.steps, use_graph)

    # ---- per-kernel durations of the same K steps (events bracketing every launch, eager)
    ds.ds_profile_reset(); ds.ds_profile_enable(True)
    with torch.cuda.stream(stream):
        for _ in range(args.steps):
            sparse_sweep()
        torch.cuda.synchronize()
    prof = ds.ds_profile_read()
    ds.ds_profile_enable(False); ds.ds_profile_reset()
    kernels_us = {k: round(v[0] * 1e3 / v[1], 3) for k, v in prof.items()}
    alg = w.algorithmic_bytes()                           # label stream + k full K and V rows (Sec. 5.3)
    if args.label_bits == 4:   # 4 bits per label value, eight to a word
        alg = w.units * (w.L * ((w.r + 7) // 8) * 4 + w.k * w.d * 2 * 2)
    dom = "k_refine_attend" if "k_refine_attend" in kernels_us else "k_attend"
    dom_bytes = w.units * w.k * w.d * 2 * 2                   # k full K and V rows per unit
    if dom == "k_refine_attend" and "k_score" not in kernels_us:
        dom_bytes = alg                                       # that launch scored the units itself
    # (units that do not fit the device at once go in several launches per layer, a share each)
    per_layer = max(1, round(prof[dom][1] / (args.steps * n_layers)))
    dom_bytes //= per_layer
    dom_us = kernels_us[dom]
    achieved = dom_bytes / (dom_us * 1e-6) / 1e9

    res = {
        "metric": "sparse decode attention us/layer at L=%d, 1/%d token sparsity (achieved HBM GB/s in extra)" % (w.L, w.L // w.k),
        "value": round(us_layer, 3), "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.note}", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d, "L": w.L,
                   "r": w.r, "k": w.k, "storage": "f16", "layers_per_step": n_layers, "hip_graph": use_graph,
                   "kv_layout": "interleaved [L,2,d]" if args.interleaved else "separate K, V [L,d]",
                   "label_bits": args.label_bits},
        "roofline": {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": None if (args.interleaved or args.label_bits == 4) else counted_traffic(w.name, dom, ds.ds_version()),
                     "algorithmic_bytes_per_launch": dom_bytes, "avg_launch_us": dom_us},
    }
    extra = {
        "algorithmic_bytes_per_layer": alg,
        "achieved_GBps_whole_path": round(alg / (us_layer * 1e-6) / 1e9, 1),
        "hbm_frac_whole_path": round(alg / (us_layer * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "us_per_layer_by_stream_events": round(ms_step_ev * 1e3 / n_layers, 3),
        "us_per_layer_p10_p50_p90": [round(spread[int(q * (len(spread) - 1))] * 1e3 / n_layers, 3) for q in (0.1, 0.5, 0.9)],
        "attention_tokens_per_s": round(w.B / (w.n_layers * us_layer * 1e-6), 1),
        "kernels_avg_us": kernels_us,
        "setup_s": round(t_gen, 1),
    }

    # ---- in-library dense decode on the same caches
    if not args.no_dense and not args.interleaved:
        d_steps = max(2, args.steps // 4)
        d_ms, _ = timed(dense_sweep, d_steps, 1, use_graph)
        d_us = d_ms * 1e3 / n_layers
        extra["dense_us_per_layer"] = round(d_us, 3)
        extra["dense_achieved_GBps"] = round(w.dense_bytes() / (d_us * 1e-6) / 1e9, 1)
        extra["speedup_vs_dense"] = round(d_us / us_layer, 3)

    # ---- the same decode scoring straight from the K rows (what the label cache buys; Sec. 4.2)
    if not args.no_dense and not args.interleaved and args.label_bits == 16:
        n_ms, _ = timed(nolabel_sweep, max(2, args.steps // 4), 1, use_graph)
        extra["nolabel_us_per_layer"] = round(n_ms * 1e3 / n_layers, 3)
        extra["label_cache_speedup"] = round(n_ms * 1e3 / n_layers / us_layer, 3)

    # ---- measured read ceiling of this device: plain 16-byte loads over one layer's K cache at a time
    sink = torch.zeros(1024, dtype=torch.int32, device=dev)

    def probe_sweep():
        for (q, label, K, V, ch) in layers:
            ds.ds_probe_stream_read(K, sink)
    p_ms, _ = timed(probe_sweep, max(2, args.steps // 4), 1, use_graph)
    extra["stream_read_ceiling_GBps"] = round(n_layers * layers[0][2].numel() * 2 / (p_ms * 1e-3) / 1e9, 1)
    if args.interleaved or args.label_bits == 4:
        args.no_cpu = True   # the oracle sample below is the fp16-label, separate-layout path

    # ---- CPU oracle on the host cores, bounded sample
    if not args.no_cpu:
        from oracle import ds_oracle as O
        n_host = min(4, n_layers)            # host copies of a few layers, rotated
        host = []
        for (q, label, K, V, ch) in layers[:n_host]:
            qh, Kh, Vh, chh = q.cpu().numpy(), K.cpu().numpy(), V.cpu().numpy(), ch.cpu().numpy()
            host.append((qh, O.build_label(Kh, chh, w.L), Kh, Vh, chh))
        cores = min(len(os.sched_getaffinity(0)), int(os.environ.get("OMP_NUM_THREADS", "1000000")))  # OpenMP threads the oracle runs on
        reps, t_cpu, ref_out = 0, 0.0, None
        while t_cpu < 10.0 and reps < 2000:
            qh, lab_h, Kh, Vh, chh = host[reps % n_host]
            t0 = time.perf_counter()
            o_out, _ = O.sparse_decode(qh, lab_h, Kh, Vh, chh, w.L, w.k)
            t_cpu += time.perf_counter() - t0
            if reps == 0:
                ref_out = o_out
            reps += 1
        q, label, K, V, ch = layers[0]
        # the sample doubles as an end-of-run sanity check of the timed path
        ds.ds_sparse_decode(q, label, K, V, ch, out, None, ws, shp)
        torch.cuda.synchronize()
        err = float(np.abs(out.cpu().numpy().astype(np.float64) - ref_out).max())
        extra["max_abs_err_vs_oracle_layer0"] = err
        res["cpu_baseline"] = {"value": round(t_cpu / reps * 1e6, 1), "unit": "us/layer", "cores": cores,
                               "kind": "oracle",
                               "sample": f"{reps} layer passes over {n_host} layers of {w.name} (all {w.units} units each), {t_cpu:.1f} s of CPU time"}
    # ---- no bounded wait between workgroups may have run out in any of the launches above
    n_failed, code = ds.ds_workspace_errors(ws, shp)
    if n_failed:
        sys.exit(f"bench.py: {n_failed} unit(s) raised error word {code} (a wait between workgroups ran out): no metric")
    res["extra"] = extra
    print(json.dumps(res))


# Stage numbers that thread 0 of every workgroup of the attention launch stamps (DS_TR in
# csrc/ds_attend.hip), in the order a workgroup passes them.
TRACE_STAGES = [(0, "start"), (11, "chunk scored (keys in LDS)"), (12, "unit histogram complete"),
                (10, "threshold bin known"), (13, "keys counted against the bin"),
                (1, "lists made, candidates handed over"), (2, "arrived at unit counter"),
                (8, "refiner: candidate loads issued"),
                (14, "refiner: first radix pass done"), (15, "refiner: exact threshold known"),
                (9, "refiner: published, histograms cleared"),
                (3, "definite rows attended"), (4, "exact threshold picked up, rest listed"),
                (5, "remaining rows attended"), (6, "partial written, arrived"), (7, "unit merged")]


def trace_report(args, w, ds, torch, sweep):
    """Runs three sweeps with the stage-stamp build and prints, for the last launch, when its
    workgroups reached each stage (us after the first workgroup started; the device's 100 MHz
    wall clock), and how long the stage took in the workgroups that passed it."""
    import ctypes

    import numpy as np
    for _ in range(3):
        sweep()
    torch.cuda.synchronize()
    n_slots = 1 << 14
    buf = np.zeros(n_slots * 16, dtype=np.int64)
    rc = ds.lib().ds_trace_read_attend(ctypes.c_void_p(buf.ctypes.data), ctypes.c_size_t(buf.nbytes))
    assert rc == 0, "ds_trace_read_attend failed"
    tr = buf.reshape(n_slots, 16).astype(np.float64) / 100.0
    live = tr[:, 0] > 0
    # stamps of the last launch: within 500 us of the latest start
    t_last = tr[live, 0].max()
    wg = live & (tr[:, 0] > t_last - 500.0)
    t0 = tr[wg, 0].min()
    print(f"# stage stamps, workload {w.name}, {int(wg.sum())} workgroups in the last launch; us since the first workgroup started")
    print(f"# {'stage':44s} {'n':>5s} {'min':>7s} {'p10':>7s} {'p50':>7s} {'p90':>7s} {'max':>7s}   since previous stage: p50 / max")
    prev = None
    for st, name in TRACE_STAGES:
        ok = wg & (tr[:, st] >= t0)
        if not ok.any():
            continue
        c = tr[ok, st] - t0
        line = (f"  {name:44s} {int(ok.sum()):5d} {c.min():7.2f} {np.percentile(c, 10):7.2f} {np.median(c):7.2f} "
                f"{np.percentile(c, 90):7.2f} {c.max():7.2f}")
        if prev is not None:
            both = ok & (tr[:, prev] >= t0)
            if both.any():
                d = tr[both, st] - tr[both, prev]
                line += f"   {np.median(d):6.2f} / {d.max():6.2f}"
        print(line)
        if int(ok.sum()) > int(wg.sum()) // 2:
            prev = st
    end = max(tr[wg, st].max() for st, _ in TRACE_STAGES) - t0
    print(f"# last stamp of the launch at {end:.2f} us")


def bench_label_ablation(args, ds, torch, dev):
    """The grid of the appendix table "Latency with and without label cache": batch 4 and 32,
    2K to 16K tokens, Llama-2-7B attention shape (32 heads, d = 128), 1/16 channel and token
    sparsity.  One attention layer per call; distinct layer caches are rotated so that no call
    finds its data in a cache.  The paper's milliseconds are another machine's: only the shape of
    the table (label cache faster by a factor) is comparable."""
    from workloads import Workload, make_calibration_numpy, make_layer_torch
    rows = []
    stream = torch.cuda.Stream(device=dev)
    for B in (4, 32):
        for L in (2048, 4096, 8192, 16384):
            w = Workload(f"abl_B{B}_L{L}", B, 32, 32, 128, L, 8, L // 16, 32)
            layer_bytes = w.units * L * (2 * w.d * 2 + w.r * 2)
            n_layers = max(2, min(16, (4 << 30) // layer_bytes))
            shp = ds.shape(w.B, w.Hq, w.Hkv, w.d, L, L, w.r, w.k)
            layers = []
            for l in range(n_layers):
                qc, kc = make_calibration_numpy(w, layer=l)
                ch = torch.from_numpy(ds.ds_calibrate_channels(qc, kc, w.r, ds.DS_CALIB_QK)).to(dev)
                t = make_layer_torch(w, dev, layer=l)
                label = torch.empty((w.B, w.Hkv, L, w.r), dtype=torch.float16, device=dev)
                ds.ds_build_label(t["K"], ch, label, shp)
                layers.append((t["q"], label, t["K"], t["V"], ch))
            ws = ds.ds_workspace_alloc(shp, dev)
            out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device=dev)
            torch.cuda.synchronize()   # set-up ran on the default stream, the timed work does not

            def with_label():
                for (q, label, K, V, ch) in layers:
                    ds.ds_sparse_decode(q, label, K, V, ch, out, None, ws, shp)

            def without_label():
                for (q, label, K, V, ch) in layers:
                    ds.ds_sparse_decode_nolabel(q, K, V, ch, out, None, ws, shp)

            us = []
            for fn in (with_label, without_label):
                with torch.cuda.stream(stream):
                    fn(); stream.synchronize()
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=stream):
                        fn()
                    for _ in range(args.warmup):
                        g.replay()
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    for _ in range(args.steps):
                        g.replay()
                    torch.cuda.synchronize()
                    us.append((time.perf_counter() - t0) * 1e6 / args.steps / n_layers)
            rows.append({"B": B, "L": L, "with_label_us": round(us[0], 2), "without_label_us": round(us[1], 2),
                         "speedup": round(us[1] / us[0], 2), "layer_caches": n_layers})
            del layers, ws, out
            torch.cuda.empty_cache()
    print(json.dumps({"metric": "sparse decode attention us/layer with and without label cache",
                      "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                      "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "label-cache ablation grid: H32/32 d128 r8 k=L/16", "storage": "f16"},
                      "rows": rows}))


def bench_offload(args, w, ds, torch, dev):
    """Config 5: K/V in pinned host memory, label cache on the GPU; per layer select on the GPU,
    fetch the k rows over the host link (double-buffered across layers), attend over them."""
    import numpy as np
    from paper_2408_07092_amd.offload import OffloadDecoder
    from workloads import make_calibration_numpy, make_layer_torch

    n_layers = args.layers or 4
    shp = ds.shape(w.B, w.Hq, w.Hkv, w.d, w.L, w.L, w.r, w.k)
    layers, outs = [], []
    for l in range(n_layers):
        qc, kc = make_calibration_numpy(w, layer=l)
        ch = torch.from_numpy(ds.ds_calibrate_channels(qc, kc, w.r, ds.DS_CALIB_QK)).to(dev)
        t = make_layer_torch(w, dev, layer=l, pin_kv=True)
        label = torch.empty((w.B, w.Hkv, w.L, w.r), dtype=torch.float16, device=dev)
        Kd = t["K"].to(dev)
        ds.ds_build_label(Kd, ch, label, shp)
        torch.cuda.synchronize()
        del Kd
        layers.append((t["q"], label, ch, t["K"], t["V"]))
        outs.append(torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device=dev))
    predict = None
    if args.predict:
        # synthetic stand-ins of the model around the attention: one embedding per layer and the
        # layer's query projection (7B shape: Dm = Hq * d), random; only the shape of the work matters
        Dm = w.Hq * w.d
        g = torch.Generator(device=dev); g.manual_seed(7)
        predict = []
        for l in range(n_layers):
            x = torch.randn((w.B, Dm), generator=g, device=dev, dtype=torch.float32).to(torch.float16)
            Wq = (torch.randn((w.Hq * w.d, Dm), generator=g, device=dev, dtype=torch.float32) / Dm ** 0.5).to(torch.float16)
            predict.append((x, Wq, torch.empty((w.B, w.Hq, w.d), dtype=torch.float16, device=dev)))
    dec = OffloadDecoder(shp, dev)
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        dec.decode(layers, outs, predict)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        dec.decode(layers, outs, predict)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    us_layer = ms_step * 1e3 / n_layers
    # the same stages one after the other on one stream: what the schedule hides
    stage = {"predict": 0.0, "select": 0.0, "fetch": 0.0, "attend": 0.0}
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)]
    for l in range(n_layers):
        q, label, ch, Kp, Vp = layers[l]
        ev[0].record()
        if predict is not None:
            ds.ds_predict_query(*predict[l]); q_sel = predict[l][2]
        else:
            q_sel = q
        ev[1].record()
        ds.ds_select(q_sel, label, ch, dec.idx[0], dec.ws_sel[0], shp)
        ev[2].record()
        ds.ds_gather_rows_host(Kp, Vp, dec.idx[0], dec.rows[0], shp)
        ev[3].record()
        ds.ds_attend_rows(q, dec.rows[0], outs[l], dec.ws_att, shp)
        ev[4].record()
        torch.cuda.synchronize()
        for i, name in enumerate(("predict", "select", "fetch", "attend")):
            stage[name] += ev[i].elapsed_time(ev[i + 1]) * 1e3 / n_layers
    serial = sum(stage.values())
    hidden = (serial - us_layer) / max(serial - max(stage.values()), 1e-9)
    # the alternative transport for the selected rows (Sec. 5.1 leaves it open): index list to the
    # host, rows packed there into a pinned staging buffer, one asynchronous copy to the device
    q, label, ch, Kp, Vp = layers[0]
    ds.ds_select(q, label, ch, dec.idx[0], dec.ws_sel[0], shp)
    torch.cuda.synchronize()
    staging = torch.empty((w.B, w.Hkv, w.k, 2, w.d), dtype=torch.float16).pin_memory()
    pack_us = []
    for _ in range(3):
        t0 = time.perf_counter()
        idx_h = dec.idx[0].cpu().to(torch.int64)                       # waits for the select stream's result
        for b in range(w.B):
            for h in range(w.Hkv):
                torch.index_select(Kp[b, h], 0, idx_h[b, h], out=staging[b, h, :, 0])
                torch.index_select(Vp[b, h], 0, idx_h[b, h], out=staging[b, h, :, 1])
        dec.rows[0].copy_(staging, non_blocking=True)
        torch.cuda.synchronize()
        pack_us.append((time.perf_counter() - t0) * 1e6)
    host_pack_us = min(pack_us)
    ds.ds_gather_rows_host(Kp, Vp, dec.idx[0], dec.rows[1], shp)   # the zero-copy kernel on the same index list
    torch.cuda.synchronize()
    same = bool((dec.rows[0] == dec.rows[1]).all())
    link_bytes = w.units * w.k * w.d * 2 * 2
    # measured host-to-device ceiling: one large pinned -> device copy
    big = layers[0][3].view(-1)[: (1 << 29)]
    dst = torch.empty_like(big, device=dev)
    dst.copy_(big, non_blocking=True); torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        dst.copy_(big, non_blocking=True)
    torch.cuda.synchronize()
    h2d = 3 * big.numel() * 2 / (time.perf_counter() - t0) / 1e9
    link = link_bytes / (us_layer * 1e-6) / 1e9
    res = {
        "metric": "offload sparse decode us/layer at L=%d (K/V in pinned host memory, k=%d rows fetched per unit)" % (w.L, w.k),
        "value": round(us_layer, 2), "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.note}", "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "d": w.d, "L": w.L,
                   "r": w.r, "k": w.k, "storage": "f16", "layers_per_step": n_layers},
        "roofline": {"bound": "host-link", "kernel": "k_gather_host", "achieved": round(link, 1), "peak": round(h2d, 1),
                     "unit": "GB/s", "frac": round(link / h2d, 4), "traffic": None,
                     "note": "peak = measured pinned->device copy rate of this box, not a published figure"},
        "extra": {"link_bytes_per_layer": link_bytes, "hbm_label_bytes_per_layer": w.units * w.L * w.r * 2,
                  "query_prediction": bool(args.predict),
                  "stage_us_per_layer_serial": {k_: round(v, 2) for k_, v in stage.items()},
                  "serial_us_per_layer": round(serial, 2),
                  "host_pack_then_memcpy_us_per_layer": round(host_pack_us, 1),
                  "host_pack_rows_equal_zero_copy_rows": same,
                  "overlap_fraction": round(hidden, 4)},
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
