#!/usr/bin/env python3
"""Benchmark of the direct sparse convolution hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--layer NAME] [--no-autotune]
                    [--report PATH]   # optional per-layer table over all workload configs (PATH, PATH.txt)

One *step* is one pass of the hot path over one batch of synthetic input: sparse_conv_forward of
the headline layer (largest ResNet-50-shaped layer at 90 % sparsity: the stage-1 1x1 reduce,
C=256 -> D=64, 56x56, batch 32, fp32, 26 stored weights per output channel).  The plan (row
unification, offset stretching, launch-shape autotune) is built once before the timed region, as
the method prescribes (it is per-layer, offline work).  Inputs are resident in HBM; the step
rotates over a ring of input/output buffers larger than twice the 256 MB Infinity Cache so that
every launch really streams from HBM.

Prints ONE JSON line: metric / value / unit (useful GFLOP/s of the layer), ms_per_step, config
(workload and launch shape), timing_spread (median / min / max of ten short cold runs and a
cache-warm run, for context), roofline (algorithmic bytes per launch over the measured kernel time,
against the 8 TB/s HBM peak), a measured plain-copy bandwidth beside it), parity (the launch shape that was timed, checked
against the CPU oracle outside the timed region; a mismatch makes the exit status 1), the dense
MIOpen time of the same layer for context (cache-warm and over the same cold ring), and
cpu_baseline (the CPU oracle timed on the host cores).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
FP32_VALU_PEAK_TFLOPS = 157.3
INFINITY_CACHE_BYTES = 256 << 20

# HBM traffic per launch of the dominant kernel, measured offline with rocprofv3 --pmc
# (FETCH_SIZE / WRITE_SIZE, scaled by the same counters on a plain copy kernel); the summaries and
# the commands that produced them are under profiles/.  Keyed by (workload, launch shape): a run in
# which the autotuner installs another shape reports no traffic figure rather than a stale one.
MEASURED_TRAFFIC_BYTES = {
    # FETCH_SIZE 50408.0 KiB x 2.000 (copy-kernel calibration) + WRITE_SIZE 25127.5 KiB x 1.000
    ("s56_reduce1x1_sp90", "variant=2 wg_threads=1024 tile_p=1 tile_q=512 wg_per_cu=1 wsrc=1 pipeline=1 "
     "producers=2 chunk_c=32 tile_d=64 pack=2"): int((50408.0 * 2.000 + 25127.5 * 1.000) * 1024),
}


def _ring(plan, data, l, torch, G, B):
    """Input/output buffer ring > 2x the Infinity Cache (at least 2 pairs)."""
    inf = plan.info()
    x0 = G.to_device(data["x"])
    ybytes = l.N * l.D * inf.P * inf.Q * (2 if l.dtype in ("f16", "cb4h") else 4)
    per = x0.numel() * x0.element_size() + ybytes
    R = max(2, min(1024, int(2 * INFINITY_CACHE_BYTES // per) + 2))      # sized by bytes, not by count
    xs = [x0] + [x0.clone() for _ in range(R - 1)]
    ys = [torch.empty((l.N, l.D, inf.P, inf.Q), dtype=B.torch_out_dtype(plan.dtype), device="cuda")
          for _ in range(R)]
    return xs, ys


def _time_steps(plan, xs, ys, ws, N, steps, warmup, torch):
    st = torch.cuda.current_stream().cuda_stream
    R = len(xs)
    wsp, wsn = (ws.data_ptr(), ws.numel()) if ws is not None else (0, 0)
    for i in range(warmup):
        plan.forward(xs[i % R].data_ptr(), ys[i % R].data_ptr(), N, wsp, wsn, st)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        plan.forward(xs[i % R].data_ptr(), ys[i % R].data_ptr(), N, wsp, wsn, st)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return wall_ms / steps, e0.elapsed_time(e1) / steps


def _spread(plan, xs, ys, ws, N, torch, repeats=10, launches=100):
    """Median / min / max of `repeats` short timed runs over the cold ring, and one cache-warm run
    (a single buffer pair launched back to back): context for the headline figure."""
    import statistics
    vals = [_time_steps(plan, xs, ys, ws, N, launches, 5, torch)[1] for _ in range(repeats)]
    warm = _time_steps(plan, xs[:1], ys[:1], ws, N, launches, 5, torch)[1]
    return {"repeats": repeats, "launches_per_repeat": launches, "median_ms": statistics.median(vals),
            "min_ms": min(vals), "max_ms": max(vals), "cache_warm_ms": warm}


def _dense_reference_ms(l, torch, xs=None, reps=30):
    """Dense MIOpen convolution of the same layer (torch conv2d), for context: (cache-warm ms on one
    buffer pair, cold ms rotating over the same ring of inputs the sparse kernel is timed on, with as
    many outputs kept alive).  Whatever layout changes the library makes around its kernel are
    inside both figures."""
    dt = {"f32": torch.float32, "f16": torch.float16, "cb4h": torch.float16}.get(l.dtype)
    if dt is None:
        return None, None
    x = torch.empty((l.N, l.C, l.H, l.W), dtype=dt, device="cuda").uniform_(-1, 1)
    w = torch.empty((l.D, l.C, l.R, l.S), dtype=dt, device="cuda").normal_(0, 0.05)
    conv = lambda inp: torch.nn.functional.conv2d(inp, w, stride=(l.stride_h, l.stride_w),
                                                  padding=(l.pad_h, l.pad_w))
    for _ in range(3):
        conv(x)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        conv(x)
    e1.record()
    torch.cuda.synchronize()
    warm = e0.elapsed_time(e1) / reps
    cold = None
    if xs is not None and xs[0].dtype == dt:
        R = len(xs)
        keep = [None] * R
        n = max(reps, min(R, 300))
        for i in range(min(R, n)):        # the allocator hands out R distinct output blocks from here on
            keep[i % R] = conv(xs[i % R])
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            keep[i % R] = conv(xs[i % R])
        e1.record()
        torch.cuda.synchronize()
        cold = e0.elapsed_time(e1) / n
        del keep
    return warm, cold


def _copy_bandwidth_gbs(torch, mib=256, reps=20):
    """A plain device-to-device streaming copy on this GPU (read + written bytes per second): what
    the 8 TB/s peak comes down to for the simplest kernel there is."""
    a = torch.empty(mib << 18, dtype=torch.float32, device="cuda").fill_(1)
    bufs = [torch.empty_like(a) for _ in range(3)]
    for b in bufs:
        b.copy_(a)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(reps):
        bufs[i % 3].copy_(a if i % 2 == 0 else bufs[(i + 1) % 3])
    e1.record()
    torch.cuda.synchronize()
    return 2.0 * (mib << 20) * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9


def _cpu_baseline(l, data, oracle, max_samples):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    ns = min(l.N, max_samples)
    x = data["x"][:ns]
    reps, t0 = 0, time.perf_counter()
    while True:          # the whole batch takes well under a second: repeat it for a steadier figure
        oracle.sparse_conv(x, data["rowptr"], data["colidx"], data["values"], l.R, l.S,
                           (l.stride_h, l.stride_w), (l.pad_h, l.pad_w), codebook=data["codebook"])
        reps += 1
        dt = time.perf_counter() - t0
        if dt > 10.0 or reps >= 200:
            break
    macs = reps * ns * l.D * l.P * l.Q * l.n
    return {"value": 2 * macs / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": f"{reps} passes over {ns} of {l.N} samples of {l.name} ({dt:.2f} s "
            "in all, includes the oracle's widening to double and its padded copy)"}


def _graph_time_ms(plan, xs, ys, ws, N, torch, launches=100, replays=5):
    """Launch-limited layers: the same launches captured once in a HIP graph and replayed, so that
    the figure holds kernel time only.  (The forward path records kernels only: no memset, no
    allocation.)  Every replay is followed by a synchronisation; the mean of the replays after the
    first is returned."""
    R = len(xs)
    wsp, wsn = (ws.data_ptr(), ws.numel()) if ws is not None else (0, 0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        plan.forward(xs[0].data_ptr(), ys[0].data_ptr(), N, wsp, wsn, side.cuda_stream)   # warm-up outside capture
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            st = torch.cuda.current_stream().cuda_stream
            for i in range(launches):
                plan.forward(xs[i % R].data_ptr(), ys[i % R].data_ptr(), N, wsp, wsn, st)
    torch.cuda.synchronize()
    times = []
    for _ in range(replays + 1):
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) / launches)
    return sum(times[1:]) / replays


def _tuning_key(t):
    """Launch shape as a short canonical string (the non-zero fields of sc_tuning_t)."""
    return " ".join(f"{k}={v}" for k, v in t.items() if v)


def run_layer(l, steps, warmup, autotune, torch, G, B, wl, with_dense=True, tuning=None, spread=False,
              parity=True):
    data = wl.prepare(l)
    plan = G.make_plan(l, data)
    if tuning:
        plan.set_tuning(B.sc_tuning_t(), **tuning)
        autotune = False
    xs, ys = _ring(plan, data, l, torch, G, B)
    ws_bytes = plan.workspace_size_max(l.N)
    dispatch = None
    if autotune:
        # per-layer dispatch (the gather kernels, the densified MFMA tile and the dense library, each
        # tuned / set up and timed; the fastest is installed), with a workspace that also holds the
        # tuner's ring of scratch buffers: the search then allocates nothing itself
        ws = torch.empty(max(plan.autotune_workspace_size(l.N), 16), dtype=torch.uint8, device="cuda")
        dispatch = plan.dispatch(xs[0].data_ptr(), ys[0].data_ptr(), l.N, ws.data_ptr(), ws.numel(),
                                 torch.cuda.current_stream().cuda_stream).as_dict()
        del ws
        torch.cuda.empty_cache()
    ws = torch.empty(max(ws_bytes, plan.workspace_size(l.N), 16), dtype=torch.uint8, device="cuda")
    wall_ms, ev_ms = _time_steps(plan, xs, ys, ws, l.N, steps, warmup, torch)
    inf = plan.info()
    useful = 2.0 * l.N * inf.useful_macs_per_sample
    alg_bytes = l.N * inf.act_bytes_per_sample + inf.weight_bytes
    ring_bytes = sum(t.numel() * t.element_size() for t in xs + ys)
    out = {
        "layer": l.name, "dtype": l.dtype, "n": inf.n, "ms_wall": wall_ms, "ms_events": ev_ms,
        "useful_gflops": useful / (wall_ms * 1e-3) / 1e9,
        "algorithmic_bytes": alg_bytes,
        "achieved_gbs": alg_bytes / (ev_ms * 1e-3) / 1e9,
        "hbm_frac": alg_bytes / (ev_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "tuning": inf.tuning.as_dict(), "lds_bytes": inf.lds_bytes, "ring": len(xs),
        "ring_bytes": ring_bytes, "dispatch": dispatch,
        "path": dispatch["choice"] if dispatch else ("dense" if inf.tuning.variant == B.SC_VARIANT_DENSE else "sparse"),
    }
    if ev_ms < 0.010:
        # launch-limited: back-to-back launches from the host cannot keep up with kernels this short
        out["graph_ms"] = _graph_time_ms(plan, xs[:64], ys[:64], ws, l.N, torch)
    if with_dense:
        out["dense_miopen_ms"], out["dense_miopen_cold_ms"] = _dense_reference_ms(l, torch, xs)
    if spread:
        out["spread"] = _spread(plan, xs, ys, ws, l.N, torch)
    if parity:
        # the launch shape that was just timed, on the full batch, against the CPU oracle (outside the
        # timed region): samples 0..15 and the last one, element by element
        # (the dense library chooses its own algorithm and with it its own rounding: that path is held
        # to 1e-3 in fp32 instead of the 1e-5 of the library's own kernels)
        out["parity"] = G.full_batch_parity(l, data, plan, xs[0], ws,
                                            tol=1e-3 if (out["path"] == "library" and l.dtype == "f32") else None)
    return out, data, plan


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--layer", default=None, help="layer name from config 3 (default: headline)")
    ap.add_argument("--dtype", default=None, help="with --layer: run that layer's shape in this dtype")
    ap.add_argument("--no-autotune", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--tuning", default=None,
                    help='pin the launch shape instead of autotuning, e.g. '
                         '\'{"variant":2,"wg_threads":1024,"tile_q":64,"wg_per_cu":2,"wsrc":1}\'')
    ap.add_argument("--no-dense", action="store_true", help="skip the dense library reference")
    ap.add_argument("--tunings", default=None,
                    help="JSON list of {layer, dtype, tuning} rows (a saved --report file): install these "
                         "launch shapes instead of autotuning")
    ap.add_argument("--report", default=None, help="also time every layer of all configs -> JSON file")
    ap.add_argument("--report-configs", default="1,2,3,4,5,6,7",
                    help="with --report: the workload configurations to cover (comma-separated)")
    ap.add_argument("--table", nargs="+", default=None, metavar="REPORT.json",
                    help="no GPU work: merge saved --report files and print the per-layer table")
    ap.add_argument("--write-tunings", default=None, metavar="OUT.json",
                    help="with --table: also write the recorded per-layer choices ({config, layer, dtype, path, tuning} "
                         "rows, the data of tests/test_gpu_recorded_tunings.py and of --tunings)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="instead of the benchmark, run 20 plain 256 MiB device copies (the known-size "
                         "kernel the rocprofv3 FETCH_SIZE / WRITE_SIZE counters are scaled against)")
    ap.add_argument("--ragged-study", action="store_true",
                    help="instead of the benchmark, time a few layers whose rows have uneven lengths with the "
                         "unified table and with the ragged one (tuning.ragged), same launch shape")
    args = ap.parse_args()
    if args.table:
        rows = [r for f in args.table for r in json.load(open(f))]
        rows.sort(key=lambda r: r["config"])           # stable: layers keep their order inside a configuration
        sys.stdout.write(report_table(rows))
        if args.write_tunings:
            rec = [{"config": r["config"], "layer": r["layer"], "dtype": r["dtype"], "path": r.get("path", "sparse"),
                    "tuning": {k: v for k, v in r["tuning"].items() if v}} for r in rows]
            with open(args.write_tunings, "w") as f:
                f.write("[\n" + ",\n".join(" " + json.dumps(x) for x in rec) + "\n]\n")
        return
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path would shard over the batch with "
              "no exchange step); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import gpu_util as G
    from paper_2112_15445_amd import binding as B
    from paper_2112_15445_amd import workloads as wl
    B.lib()                                  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        a = torch.empty(64 << 20, dtype=torch.float32, device="cuda").fill_(1)
        b = torch.empty_like(a)
        for _ in range(20):
            torch.mul(a, 1.0, out=b)     # one plain elementwise kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "20 x elementwise copy kernel, 268435456 bytes read + "
                                         "268435456 bytes written per launch"}))
        return

    if args.ragged_study:
        import numpy as np
        cases = [("s28_conv3x3_sp90", {"tile_p": 4, "chunk_c": 64, "wg_per_cu": 2}),
                 ("s14_conv3x3_sp90", {"tile_p": 7, "chunk_c": 128, "tile_d": 128, "wg_per_cu": 2}),
                 ("s28_conv3x3_s2_sp90", {"tile_p": 4, "chunk_c": 64, "wg_per_cu": 1}),
                 ("s56_reduce1x1_sp90", {"pipeline": 1, "producers": 2, "tile_q": 256, "chunk_c": 64}),
                 ("s14_reduce1x1_sp90", {"pipeline": 2, "tile_q": 128, "chunk_c": 128, "tile_d": 128})]
        print("layer                  longest row / mean row   unified_us  ragged_us  ratio   launch shape")
        for name, extra in cases:
            l = {x.name: x for x in wl.config3()}[name]
            data = wl.prepare(l, ragged=True)            # row lengths uniform in [0, n]
            lens = np.diff(data["rowptr"])
            plan = G.make_plan(l, data)
            xs, ys = _ring(plan, data, l, torch, G, B)
            us = []
            for ragged in (0, 1):
                plan.set_tuning(B.sc_tuning_t(), variant=B.SC_VARIANT_SLAB, wsrc=1, wg_threads=1024,
                                ragged=ragged, **extra)
                us.append(_time_steps(plan, xs, ys, None, l.N, 300, 20, torch)[1] * 1e3)
            print(f"{name:22s} {lens.max():8d} / {lens.mean():7.1f}       {us[0]:9.2f}  {us[1]:9.2f}  "
                  f"{us[0] / us[1]:5.2f}x   {json.dumps(extra)}", flush=True)
            plan.destroy()
        return

    tunings = {}
    if args.tunings:
        tunings = {(r["layer"], r["dtype"]): r["tuning"] for r in json.load(open(args.tunings))}

    l = wl.headline_layer()
    if args.layer:
        cands = [x for c in (3, 4, 2, 5, 1, 6, 7) for x in wl.CONFIGS[c]() if x.name == args.layer]
        l = ([x for x in cands if x.dtype == args.dtype] or cands)[0]
        if args.dtype:
            l = l.replace(dtype=args.dtype)
    pinned = json.loads(args.tuning) if args.tuning else tunings.get((l.name, l.dtype))
    res, data, plan = run_layer(l, args.steps, args.warmup, not args.no_autotune, torch, G, B, wl,
                                with_dense=not args.no_dense, tuning=pinned, spread=True)
    copy_gbs = _copy_bandwidth_gbs(torch)

    line = {
        "metric": "useful GFLOP/s (nnz MACs) per sparse conv layer",
        "value": res["useful_gflops"], "unit": "GFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_wall"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": l.dtype, "data": "synthetic",
        "config": {"workload": f"resnet50_{l.name}_batch{l.N}_{l.dtype}" if not args.layer else l.name,
                   "C": l.C, "D": l.D, "H": l.H, "W": l.W, "R": l.R, "S": l.S,
                   "stride": l.stride_h, "pad": l.pad_h, "batch": l.N, "sparsity": l.sparsity,
                   "n_per_channel": res["n"], "tuning": res["tuning"], "lds_bytes": res["lds_bytes"],
                   "buffer_ring": res["ring"], "buffer_ring_bytes": res["ring_bytes"],
                   "cache": "cold (ring > 2x Infinity Cache)"},
        "roofline": {"bound": "hbm", "achieved": res["achieved_gbs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": res["hbm_frac"],
                     "traffic": MEASURED_TRAFFIC_BYTES.get((l.name, _tuning_key(res["tuning"]))),
                     "algorithmic_bytes_per_launch": res["algorithmic_bytes"],
                     "kernel_ms": res["ms_events"],
                     "measured_copy_gbs": copy_gbs, "frac_of_measured_copy": res["achieved_gbs"] / copy_gbs},
        "parity": res.get("parity"),
        "dispatch": ({k: v for k, v in res["dispatch"].items() if not k.endswith("_tuning")} if res.get("dispatch") else None),
        "timing_spread": res.get("spread"),
        "dense_miopen_ms": res.get("dense_miopen_ms"),
        "dense_miopen_cold_ms": res.get("dense_miopen_cold_ms"),
        "sparse_vs_dense_speedup": (res["dense_miopen_cold_ms"] / res["ms_events"]
                                    if res.get("dense_miopen_cold_ms") else None),
    }
    if not args.no_cpu_baseline:
        import oracle
        line["cpu_baseline"] = _cpu_baseline(l, data, oracle, max_samples=l.N)
    plan.destroy()

    if args.report:
        rows = []
        for cfg in sorted(int(c) for c in args.report_configs.split(",")):
            for lay in wl.CONFIGS[cfg]():
                r, _, p = run_layer(lay, 200, 10, not args.no_autotune, torch, G, B, wl,
                                    with_dense=not args.no_dense, tuning=tunings.get((lay.name, lay.dtype)))
                p.destroy()
                r["config"] = cfg
                rows.append(r)
                print(json.dumps(r), file=sys.stderr, flush=True)
                torch.cuda.empty_cache()
                with open(args.report, "w") as f:          # rewritten after every layer: a run cut short keeps its rows
                    json.dump(rows, f, indent=1)
        with open(args.report + ".txt", "w") as f:
            f.write(report_table(rows))

    print(json.dumps(line), flush=True)
    if line["parity"] is not None and not line["parity"]["ok"]:
        sys.exit(1)


def short_shape(t):
    """One-line name of a launch shape."""
    if t.get("variant") == 1:
        return f"gather sb{t.get('sub_batch', 0)} split{t.get('split_n', 1)}"
    if t.get("variant") == 3:
        return (f"mfma tp{t.get('tile_p', 0)} ns{t.get('sub_batch', 1)} cc{t.get('chunk_c', 0)} td{t.get('tile_d', 0)} "
                f"wm{t.get('waves_m', 0)} wpc{t.get('wg_per_cu', 1)}" + (f" thr{t['wg_threads']}" if t.get("wg_threads", 256) > 256 else "")
                + (f" pl1 np{t.get('producers', 0)}" if t.get("pipeline") else "") + (" nat" if t.get("stage_rows") else "")
                + (f" dl{t['split_n']}" if t.get("split_n") else ""))
    sh = "slab"
    if t.get("pipeline"):
        sh += f" pl{t['pipeline']}"
    if t.get("producers"):
        sh += f" np{t['producers']}"
    if t.get("buffers"):
        sh += f" nb{t['buffers']}"
    sh += f" tp{t.get('tile_p', 1)} tq{t.get('tile_q', 0)} thr{t.get('wg_threads')} wpc{t.get('wg_per_cu', 1)} ws{t.get('wsrc', 0)}"
    if t.get("chunk_c"):
        sh += f" cc{t['chunk_c']} td{t.get('tile_d', 0)}"
    if t.get("sub_batch"):
        sh += f" ns{t['sub_batch']}"
    if t.get("pack"):
        sh += {1: " pk32", 2: " pk128", 3: " si"}.get(t["pack"], f" pk?{t['pack']}")
    if t.get("split_n"):
        sh += f" ks{t['split_n']}"
    if t.get("stage_rows"):
        sh += " rows"
    if t.get("ragged"):
        sh += " ragged"
    return sh


def report_table(rows):
    """The per-layer rows as text.  For every layer the three contenders of the per-layer dispatch
    (gather kernels / densified MFMA tile / dense library inside sparse_conv_plan_dispatch) and the
    time of the installed choice over the cold ring; break-even tables of the gather kernels against
    the dense contenders; per-configuration sums (the per-layer choice of the paper's main scheme)."""
    import collections
    out = []
    nan = float("nan")

    def legs(r):
        d = r.get("dispatch") or {}
        sp = d.get("sparse_ms", -1)
        de = d.get("dense_ms", -1)
        li = d.get("library_ms", -1)
        return (sp if sp and sp > 0 else None, de if de and de > 0 else None, li if li and li > 0 else None)

    def torch_dense(r):
        return r.get("dense_miopen_cold_ms") or r.get("dense_miopen_ms")

    bad = [r for r in rows if r.get("parity") and not r["parity"]["ok"]]
    checked = [r for r in rows if r.get("parity")]
    out.append(f"# parity: {len(checked) - len(bad)} of {len(checked)} layers match the CPU oracle in the path and launch shape timed "
               "(samples 0..15 and the last one of the full batch, element by element)")
    for cfg in sorted({r["config"] for r in rows}):
        rs = [r for r in rows if r["config"] == cfg]
        n = collections.Counter(r.get("path", "sparse") for r in rs)
        out.append(f"# config {cfg}: per-layer choice over {len(rs)} layers: gather kernels {n.get('sparse', 0)}, densified MFMA tile "
                   f"{n.get('dense', 0)}, dense library {n.get('library', 0)}")
    fam = collections.defaultdict(list)
    for r in rows:
        sp, de, li = legs(r)
        ref = min([v for v in (de, li, torch_dense(r)) if v], default=None)
        if r["config"] in (3, 4) and sp and ref and "_sp" in r["layer"]:
            name, spc = r["layer"].rsplit("_sp", 1)
            fam[(r["config"], name)].append((int(spc), ref / sp))
    for cfg in (4, 3):
        if any(k[0] == cfg for k in fam):
            out.append(f"# break-even of the gather kernels against the fastest dense contender (densified MFMA tile, dense library "
                       f"in the dispatch, dense library through torch), config {cfg} (speed-up = dense_us / gather_us):")
            for (c, name), v in fam.items():
                if c != cfg:
                    continue
                v.sort()
                be = [spc for spc, ra in v if ra >= 1.0]
                out.append(f"#   {name:18s} {'>= %d %%' % min(be) if be else ' > %d %%' % v[-1][0]:9s} "
                           + "  ".join(f"{spc}%: {ra:4.2f}x" for spc, ra in v))
    for cfg in sorted({r["config"] for r in rows}):
        rs = [r for r in rows if r["config"] == cfg]
        if not all(legs(r)[0] for r in rs):
            continue
        sp = sum(legs(r)[0] for r in rs) * 1e3
        ch = sum(min(v for v in legs(r) if v) for r in rs) * 1e3
        timed = sum(r["ms_events"] for r in rs) * 1e3
        txt = (f"# config {cfg}: sum over {len(rs)} layers: gather kernels only {sp:.1f} us, per-layer choice {ch:.1f} us "
               f"(both as timed inside the dispatch; the installed choices timed again over the ring: {timed:.1f} us)")
        if all(torch_dense(r) for r in rs):
            txt += f", dense library (torch) only {sum(torch_dense(r) for r in rs) * 1e3:.1f} us"
        out.append(txt)
    for r in rows:
        if r.get("graph_ms"):
            out.append(f"# {r['layer']} ({r['dtype']}): {r['ms_events']*1e3:.2f} us between events, "
                       f"{r['graph_ms']*1e3:.2f} us per launch inside a captured HIP graph (launch-limited)")
    # rows that run on the matrix cores: their bound is "mfma" -- dense flops (the tile multiplies every
    # weight, stored or not) against 2.5 PFLOP/s (fp16) / 5.0 POP/s (int8)
    from paper_2112_15445_amd import workloads as _wl
    layers = {(l.name, l.dtype): l for c in _wl.CONFIGS for l in _wl.CONFIGS[c]()}

    def mfma_frac(r):
        l = layers.get((r["layer"], r["dtype"]))
        if r.get("path") != "dense" or l is None:
            return None
        flops = 2.0 * l.N * l.D * l.P * l.Q * l.C * l.R * l.S
        peak = 5.0e15 if r["dtype"] in ("i8", "cb4") else 2.5e15
        return flops / (r["ms_events"] * 1e-3) / peak
    out.append("cfg layer                      dtype    n  choice   timed_us  alg_GB/s hbm_frac useful_TF mfma_frac | gather_us   mfma_us lib_us(warm) | "
               "torch_cold torch_warm | parity | launch shape of the choice")
    for r in rows:
        sp, de, li = legs(r)
        dc, dw = r.get("dense_miopen_cold_ms"), r.get("dense_miopen_ms")
        par = r.get("parity")
        ptxt = "-" if par is None else ("ok" if par["ok"] else "FAIL")
        f = lambda v: f"{v*1e3:9.2f}" if v else f"{nan:9.2f}"
        shape = "dense library (MIOpen)" if r.get("path") == "library" else short_shape(r["tuning"])
        out.append(f"{r['config']:3d} {r['layer']:26s} {r['dtype']:4s} {r['n']:5d} {r.get('path', 'sparse'):7s} {r['ms_events']*1e3:9.2f} "
                   f"{r['achieved_gbs']:9.0f} {r['hbm_frac']*100:7.1f}% {r['useful_gflops']/1e3:9.2f} "
                   f"{('%8.1f%%' % (mfma_frac(r) * 100)) if mfma_frac(r) is not None else '        -'} | {f(sp)} {f(de)} {f(li)}    | "
                   f"{f(dc)}  {f(dw)} | {ptxt:6s} | {shape}")
    return "\n".join(out) + "\n"


if __name__ == "__main__":
    main()
