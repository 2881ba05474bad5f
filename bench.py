#!/usr/bin/env python3
"""Benchmark of the ES-SpMM hot path on one MI355X.

A *step* is one pass of the whole hot path over one synthetic graph: for every
sampling width W of the configuration, es_spmm in bucket and in fastrand mode,
plus the full (unsampled) product -- Algorithm 1 of the paper end to end, and
the exact CSR SpMM it is compared with.  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4]
                    [--main-only] [--no-cpu-baseline]

value         = sum of algorithmic bytes of the step / wall time of the step
algorithmic   = 4(N+1) + 8 nnz_kept + 4 F nnz_kept + 4 F N   bytes per call
                (row pointers, sampled column+value pairs, one row of X per
                kept entry, Y written once)
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

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch of the dominant kernel (mean over the launches of one
# step) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, scaled by a copy
# kernel of known size; filled in from the summaries under profiles/.
MEASURED_TRAFFIC_BYTES = {
    2: 818073543,      # profiles/es_spmm_config2_sweep.md
    3: 7114890775,     # profiles/es_spmm_config3_sweep.md
    4: 31021331251,    # profiles/es_spmm_config4_sweep.md
    (5, 41): 12565809080,   # profiles/es_spmm_config5_F41.md
    (5, 256): 48857946425,  # profiles/es_spmm_config5_F256.md
}

CONFIG_TEXT = {
    2: "configs[1] mid-size citation-like graph: N=170k, power-law degree mean 14, F=128",
    3: "configs[2] dense social-like graph: N=233k, power-law degree mean 490, F=64",
    4: "configs[3] large co-purchase-like graph: N=2.45M, mean degree 50, F=128 (100 padded)",
}


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


def algorithmic_bytes(N: int, nnz_kept: int, F: int) -> int:
    return 4 * (N + 1) + 8 * nnz_kept + 4 * F * nnz_kept + 4 * F * N


class DeviceWorkload:
    def __init__(self, w, dev, X=None, F=None):
        import numpy as np
        import torch
        self.w = w
        self.N, self.nnz = w.N, w.nnz
        self.F = w.F if F is None else F
        self.deg = np.diff(w.rowptr).astype(np.int64)
        self.rowptr = torch.from_numpy(w.rowptr).to(dev)
        self.colidx = torch.from_numpy(w.colidx).to(dev)
        self.vals = torch.from_numpy(w.vals).to(dev)
        self.X = torch.from_numpy(w.X).to(dev) if X is None else X
        self.Y = torch.empty((self.N, self.F), dtype=torch.float32, device=dev)

    def calls(self, Ws):
        out = []
        for W in Ws:
            for mode in ("bucket", "fastrand"):
                out.append((mode, int(W)))
        out.append(("full", 0))
        return out

    def nnz_kept(self, mode, W):
        import numpy as np
        return int(self.nnz if mode == "full" else np.minimum(self.deg, W).sum())

    def launch(self, mode, W, seed=0):
        import paper_2104_10716_amd as es
        es.es_spmm(self.rowptr, self.colidx, self.vals, self.X, self.Y, W, mode, seed, F=self.F)


def time_call(dw, mode, W, reps, flush=None):
    """Median / min ms of one es_spmm call from HIP events on the launch stream."""
    import torch
    ts = []
    for _ in range(reps):
        if flush is not None:
            flush.add_(1.0)
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        dw.launch(mode, W)
        b.record()
        b.synchronize()
        ts.append(a.elapsed_time(b))
    ts.sort()
    return ts[len(ts) // 2], ts[0]


def per_call_table(dw, calls, reps, flush, cold_reps):
    rows = []
    t_full = None
    for mode, W in calls:
        for _ in range(2):
            dw.launch(mode, W)
        med, mn = time_call(dw, mode, W, reps)
        cold = time_call(dw, mode, W, cold_reps, flush)[0] if flush is not None else None
        kept = dw.nnz_kept(mode, W)
        B = algorithmic_bytes(dw.N, kept, dw.F)
        rows.append({"mode": mode, "W": W, "nnz_kept": kept, "ms": round(med, 4), "ms_min": round(mn, 4),
                     "ms_cold": None if cold is None else round(cold, 4),
                     "gflops": round(2.0 * kept * dw.F / (med * 1e6), 1),
                     "eff_GBps": round(B / (med * 1e6), 1),
                     "frac_hbm_peak": round(B / (med * 1e6) / HBM_PEAK_GBPS, 4),
                     "eff_GBps_cold": None if cold is None else round(B / (cold * 1e6), 1)})
        if mode == "full":
            t_full = med
    for r in rows:
        r["speedup_vs_full"] = round(t_full / r["ms"], 2) if t_full else None
    return rows


def cpu_baseline(dw, calls, min_seconds=10.0, max_steps=200):
    """The CPU oracle, as it stands, on whole steps of the same workload,
    repeated until about `min_seconds` of CPU work have been timed."""
    import oracle
    w = dw.w
    step_bytes = sum(algorithmic_bytes(dw.N, dw.nnz_kept(mode, W), dw.F) for mode, W in calls)
    steps = 0
    t0 = time.perf_counter()
    while True:
        for mode, W in calls:
            oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, dw.F, W, mode, 0, want_denom=False)
        steps += 1
        dt = time.perf_counter() - t0
        if dt >= min_seconds or steps >= max_steps:
            break
    out = {"value": round(steps * step_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(),
           "kind": "oracle", "seconds": round(dt, 2),
           "sample": f"{steps} whole steps (every call of the sweep, all rows), fp64 accumulation"}
    all_threads = oracle.threads()
    oracle.set_threads(1)                    # the same oracle on one core, one step
    t0 = time.perf_counter()
    for mode, W in calls:
        oracle.spmm(w.rowptr, w.colidx, w.vals, w.X, dw.F, W, mode, 0, want_denom=False)
    dt1 = time.perf_counter() - t0
    oracle.set_threads(all_threads)
    out["single_core_value"] = round(step_bytes / dt1 / 1e9, 3)
    return out


def cpu_baseline_rows(dw, calls, target_seconds=20.0):
    """For the large graphs: the oracle on a bounded random subset of rows."""
    import numpy as np
    import oracle
    w = dw.w
    Xh = w.X if dw.X.shape == w.X.shape else dw.X.cpu().numpy()
    work = sum(dw.nnz_kept(m, W) for m, W in calls) * dw.F
    frac = min(1.0, target_seconds * 1.0e9 / max(work, 1))     # ~1 G fp64 FMA per second assumed
    nrows = max(1, int(dw.N * frac))
    rows = np.sort(np.random.default_rng(0).choice(dw.N, size=nrows, replace=False)).astype(np.int64)
    t0 = time.perf_counter()
    total_bytes = 0
    for mode, W in calls:
        oracle.spmm(w.rowptr, w.colidx, w.vals, Xh, dw.F, W, mode, 0, rows=rows, want_denom=False)
        kept = int((dw.deg[rows] if mode == "full" else np.minimum(dw.deg[rows], W)).sum())
        total_bytes += algorithmic_bytes(nrows, kept, dw.F)
    dt = time.perf_counter() - t0
    return {"value": round(total_bytes / dt / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"{nrows} random rows of {dw.N} ({100.0 * nrows / dw.N:.1f}%), every call of the sweep"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=(2, 3, 4, 5))
    ap.add_argument("--feature-width", type=int, default=41, choices=(41, 256),
                    help="config 5 only: which SpMM stage of the 2-layer GCN forward to time")
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed sweep of --config (what the rocprofv3 summaries profile)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three 1 GiB device-to-device copies (a kernel of known traffic "
                         "to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings by)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (rows of A shard across GPUs by design, "
              "but no multi-GPU path is built); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2104_10716_amd as es
    from workloads import make_workload
    es.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")

    t0 = time.perf_counter()
    w = make_workload(3 if args.config == 5 else args.config)
    log(f"config {args.config}: N={w.N} nnz={w.nnz} F={w.F} generated in {time.perf_counter() - t0:.1f}s")
    if args.config == 5:
        dw = gcn_stage_workload(w, dev, args.feature_width)
        calls = dw.calls((64,))
        workload_text = (f"configs[4] 2-layer GCN forward on the config-3 graph, SpMM stage at "
                         f"F={args.feature_width} (row stride {args.feature_width})")
    else:
        dw = DeviceWorkload(w, dev)
        calls = dw.calls(w.Ws)
        workload_text = CONFIG_TEXT[args.config]
    step_bytes = sum(algorithmic_bytes(dw.N, dw.nnz_kept(m, W), dw.F) for m, W in calls)
    step_flops = sum(2 * dw.nnz_kept(m, W) * dw.F for m, W in calls)

    def step():
        for mode, W in calls:
            dw.launch(mode, W)

    if args.calibrate_copy:
        src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    ms_per_step = wall * 1e3 / args.steps
    launches = args.steps * len(calls)
    kernel_ms = ev_ms / launches                      # mean launch duration, HIP events
    bytes_per_launch = step_bytes / len(calls)
    achieved = bytes_per_launch / (kernel_ms * 1e6)   # GB/s
    log(f"step: {ms_per_step:.3f} ms wall, {ev_ms / args.steps:.3f} ms by events, "
        f"{step_bytes / 1e9:.3f} GB algorithmic -> {step_bytes / (ms_per_step * 1e6):.0f} GB/s")

    result = {
        "metric": "es_spmm effective HBM bandwidth (algorithmic bytes / time) over the W sweep "
                  "{bucket,fastrand} + full SpMM",
        "value": round(step_bytes / (ms_per_step * 1e6), 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "gflops": round(step_flops / (ms_per_step * 1e6), 1),
        "config": {"workload": workload_text, "N": dw.N, "nnz": dw.nnz, "F": dw.F,
                   "W": sorted({W for _, W in calls if W}), "modes": ["bucket", "fastrand", "full"], "seed": 0,
                   "calls_per_step": len(calls)},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get((5, args.feature_width) if args.config == 5
                                                          else args.config),
                     "kernel": "es_spmm_kernel", "launch_ms": round(kernel_ms, 5),
                     "bytes_per_launch": int(bytes_per_launch)},
    }

    if not args.main_only:
        flush = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev)   # 1 GiB
        flush.zero_()
        result["calls"] = per_call_table(dw, calls, 20, flush, 5)
        result["vendor_csr_spmm_ms"] = vendor_csr_spmm_ms(dw)
        if not args.no_cpu_baseline:
            result["cpu_baseline"] = (cpu_baseline(dw, calls) if args.config == 2
                                      else cpu_baseline_rows(dw, calls))
            log(f"cpu baseline: {result['cpu_baseline']}")
        extra = [tiny_config1(dev)]
        for cfg in (3, 4):
            if cfg == args.config:
                continue
            del dw
            torch.cuda.empty_cache()
            t0 = time.perf_counter()
            w = make_workload(cfg)
            log(f"config {cfg}: N={w.N} nnz={w.nnz} F={w.F} generated in {time.perf_counter() - t0:.1f}s")
            dw = DeviceWorkload(w, dev)
            rows = per_call_table(dw, dw.calls(w.Ws), 10, flush, 3)
            extra.append({"workload": CONFIG_TEXT[cfg], "N": dw.N, "nnz": dw.nnz, "F": dw.F, "calls": rows,
                          "vendor_csr_spmm_ms": vendor_csr_spmm_ms(dw)})
            for r in rows:
                log(f"  cfg{cfg} {r['mode']:8s} W={r['W']:4d}: {r['ms']:.3f} ms  {r['eff_GBps']:.0f} GB/s "
                    f"({100 * r['frac_hbm_peak']:.1f}% of peak)  cold {r['ms_cold']} ms  x{r['speedup_vs_full']} vs full")
            if cfg == 3:
                big = per_call_table(dw, [("bucket", 1792), ("bucket", 2304), ("fastrand", 1792),
                                          ("full", 0)], 5, None, 0)
                extra.append({"workload": "config-3 graph at the widths the paper needs for Bucket on its "
                                          "densest graph (S = 1792, 2304)", "calls": big[:-1]})
                for r in big[:-1]:
                    log(f"  cfg3 {r['mode']:8s} W={r['W']:4d}: {r['ms']:.3f} ms  {r['eff_GBps']:.0f} GB/s  "
                        f"x{r['speedup_vs_full']} vs full")
                extra.append(presampled_ablation(dw, dev))
                extra.append(unweighted_norm_table(dw, dev))
                extra.append(backward_table(dw, dev, ((("fastrand", 16), ("fastrand", 64), ("bucket", 64),
                                                       ("fastrand", 256)))))
                extra.append(gcn_feature_sweep(dw, dev, flush))
        result["extra"] = extra
    elif not args.no_cpu_baseline:
        result["cpu_baseline"] = (cpu_baseline(dw, calls) if args.config == 2
                                  else cpu_baseline_rows(dw, calls))

    print(json.dumps(result), flush=True)
    return 0


def vendor_csr_spmm_ms(dw):
    """Context only: the exact product through torch.sparse.mm on a CSR tensor
    (the vendor sparse library as PyTorch ships and calls it) -- the role
    cuSPARSE plays in the paper's tables.  None if that path is unavailable."""
    import warnings
    import torch
    try:
        with warnings.catch_warnings():
            warnings.simplefilter("ignore")
            A = torch.sparse_csr_tensor(dw.rowptr, dw.colidx, dw.vals, size=(dw.N, dw.N))
            X = dw.X[:, :dw.F].contiguous() if dw.X.shape[1] != dw.F else dw.X
            t = _time_fn(lambda: torch.sparse.mm(A, X), reps=5, warm=2)
        log(f"  vendor CSR SpMM via torch.sparse.mm (context): {t:.3f} ms")
        return round(t, 4)
    except Exception as exc:                                   # noqa: BLE001 - context figure only
        log(f"  vendor CSR SpMM unavailable: {exc}")
        return None


def tiny_config1(dev):
    """configs[0]: ~1 MB moved per call, so a call is launch-bound; report the
    per-call time and the time of the whole sweep replayed as one HIP graph."""
    import torch
    from workloads import make_workload
    w = make_workload(1)
    dw = DeviceWorkload(w, dev)
    calls = dw.calls(w.Ws)
    rows = per_call_table(dw, calls, 50, None, 0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for mode, W in calls:
            dw.launch(mode, W)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for mode, W in calls:
            dw.launch(mode, W)
    t_graph = _time_fn(g.replay, reps=50)
    out = {"workload": "configs[0] tiny GCN aggregation: N=2708, F=16 (launch-bound)", "N": dw.N,
           "nnz": dw.nnz, "F": dw.F, "calls": rows,
           "sweep_as_hip_graph_ms": round(t_graph, 4), "calls_in_graph": len(calls)}
    log(f"  cfg1: per-call {min(r['ms'] for r in rows):.4f}-{max(r['ms'] for r in rows):.4f} ms; "
        f"{len(calls)}-call sweep as one HIP graph {t_graph:.4f} ms")
    return out


def _time_fn(fn, reps=10, warm=2):
    import torch
    for _ in range(warm):
        fn()
    ts = []
    for _ in range(reps):
        a = torch.cuda.Event(enable_timing=True)
        b = torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        b.synchronize()
        ts.append(a.elapsed_time(b))
    ts.sort()
    return ts[len(ts) // 2]


def presampled_ablation(dw, dev):
    """Section 5.6 of the paper: feed a pre-sampled graph to the unsampled
    kernel and compare with the fused kernel on the original graph; here the
    pre-sampling is es_spmm_materialize, which also gives the cost of the
    sampling stage that the paper could not measure from inside its kernel."""
    import torch
    import paper_2104_10716_amd as es
    out = {"workload": "pre-sampled graph ablation (paper Section 5.6) on the config-3 graph, F=64",
           "rows": []}
    for mode in ("bucket", "fastrand"):
        for W in (64, 128, 256):
            t_fused = _time_fn(lambda: dw.launch(mode, W))
            orp, oci, ova = es.es_spmm_materialize(dw.rowptr, dw.colidx, dw.vals, W, mode, 0)
            t_mat = _time_fn(lambda: es.es_spmm_materialize(dw.rowptr, dw.colidx, dw.vals, W, mode, 0,
                                                            orp, oci, ova))
            kept = int(orp[-1].item())
            oci2, ova2 = oci[:kept], ova[:kept]
            t_pre = _time_fn(lambda: es.es_spmm(orp, oci2, ova2, dw.X, dw.Y, 0, "full", F=dw.F))
            row = {"mode": mode, "W": W, "fused_ms": round(t_fused, 4), "materialize_ms": round(t_mat, 4),
                   "full_on_presampled_ms": round(t_pre, 4)}
            out["rows"].append(row)
            log(f"  ablation {mode:8s} W={W:3d}: fused {t_fused:.3f} ms | materialise {t_mat:.3f} ms + "
                f"full SpMM on pre-sampled {t_pre:.3f} ms")
            del orp, oci, ova
    return out


def unweighted_norm_table(dw, dev):
    """Config 3's values are 1/d_i (mean aggregation).  The same product with no
    value array at all: vals = NULL and the 1/n row factor applied in the kernel
    (paper Section 6.1 moves the normalisation into the kernel) -- stage 1 then
    reads only colidx."""
    import torch
    import paper_2104_10716_amd as es
    out = {"workload": f"config-3 graph, F={dw.F}: vals = 1/d_i array vs vals = NULL + in-kernel 1/n", "rows": []}
    Y2 = torch.empty_like(dw.Y)
    for mode, W in (("fastrand", 16), ("fastrand", 64), ("bucket", 64), ("full", 0)):
        t_vals = _time_fn(lambda: dw.launch(mode, W))
        t_norm = _time_fn(lambda: es.es_spmm_norm(dw.rowptr, dw.colidx, None, dw.X, Y2, W, mode, 0,
                                                  "inv_degree", F=dw.F))
        dw.launch(mode, W)
        torch.cuda.synchronize()
        err = float((dw.Y - Y2).abs().max() / dw.Y.abs().max())
        out["rows"].append({"mode": mode, "W": W, "with_vals_ms": round(t_vals, 4),
                            "null_vals_inv_degree_ms": round(t_norm, 4), "max_rel_diff": err})
        log(f"  unweighted {mode:8s} W={W:3d}: vals array {t_vals:.3f} ms | NULL + 1/n in kernel {t_norm:.3f} ms "
            f"(max rel diff {err:.1e})")
    return out


def backward_table(dw, dev, cases):
    """The transposed product dX = sample_W(A)^T dY two ways, beside the forward
    call of the same (mode, W): es_spmm_backward (fp32 atomic scatter) and the
    pull form (es_spmm_materialize_transposed once, then a full product on the
    transposed structure, which can be reused while (W, mode, seed) stay)."""
    import torch
    import paper_2104_10716_amd as es
    dX = torch.empty_like(dw.Y)
    out = {"workload": f"transposed product (backward) on the same graph, F={dw.F}", "rows": []}
    for mode, W in cases:
        kept = dw.nnz_kept(mode, W)
        t_fwd = _time_fn(lambda: dw.launch(mode, W))
        t_bwd = _time_fn(lambda: es.es_spmm_backward(dw.rowptr, dw.colidx, dw.vals, dw.X, dX, W, mode, 0,
                                                     F=dw.F))
        bufs = es.es_spmm_materialize_transposed(dw.rowptr, dw.colidx, dw.vals, W, mode, 0)
        t_build = _time_fn(lambda: es.es_spmm_materialize_transposed(dw.rowptr, dw.colidx, dw.vals, W, mode,
                                                                     0, "none", *bufs))
        ptr, _, idx, val = bufs
        idx, val = idx[:kept], val[:kept]
        t_pull = _time_fn(lambda: es.es_spmm(ptr, idx, val, dw.X, dX, 0, "full", F=dw.F))
        out["rows"].append({"mode": mode, "W": W, "forward_ms": round(t_fwd, 4),
                            "backward_atomic_ms": round(t_bwd, 4), "transpose_build_ms": round(t_build, 4),
                            "backward_pull_ms": round(t_pull, 4)})
        log(f"  backward {mode:8s} W={W:3d}: atomic scatter {t_bwd:.3f} ms | transposed build {t_build:.3f} ms "
            f"+ pull {t_pull:.3f} ms | forward {t_fwd:.3f} ms")
        del bufs, ptr, idx, val
    return out


def gcn_stage_workload(w3, dev, F):
    """DeviceWorkload for one SpMM stage of configs[4]: X = X0 W1 (F=256) or
    X = relu(ES-SpMM(A, X0 W1)) W2 (F=41; first stage run with FastRand, W=64)."""
    import torch
    from workloads import gcn_operands
    X0h, W1h, W2h = gcn_operands(w3.N)
    Z1 = torch.from_numpy(X0h).to(dev) @ torch.from_numpy(W1h).to(dev)
    d1 = DeviceWorkload(w3, dev, X=Z1, F=256)
    if F == 256:
        return d1
    d1.launch("fastrand", 64)
    Z2 = torch.relu(d1.Y) @ torch.from_numpy(W2h).to(dev)
    return DeviceWorkload(w3, dev, X=Z2.contiguous(), F=41)


def gcn_feature_sweep(dw3, dev, flush):
    """configs[4]: the SpMM stages of a 2-layer GCN forward on the config-3
    graph, H1 = relu(A (X0 W1)) at F = 256 and out = A (H1 W2) at F = 41; the
    dense products are torch GEMMs and are not timed."""
    import torch
    from workloads import gcn_operands
    X0h, W1h, W2h = gcn_operands(dw3.N)
    X0 = torch.from_numpy(X0h).to(dev)
    W1 = torch.from_numpy(W1h).to(dev)
    W2 = torch.from_numpy(W2h).to(dev)
    Z1 = X0 @ W1
    del X0
    out = {"workload": "configs[4] 2-layer GCN forward on the config-3 graph, SpMM stages only",
           "N": dw3.N, "nnz": dw3.nnz, "stages": []}
    for mode, W in (("bucket", 64), ("fastrand", 64), ("full", 0)):
        d1 = DeviceWorkload(dw3.w, dev, X=Z1, F=256)
        r1 = per_call_table(d1, [(mode, W)], 10, flush, 3)[0]
        H1 = torch.relu(d1.Y)
        Z2 = H1 @ W2                                        # [N x 41], row stride 41
        d2 = DeviceWorkload(dw3.w, dev, X=Z2, F=41)
        r2 = per_call_table(d2, [(mode, W)], 10, flush, 3)[0]
        for F, r in ((256, r1), (41, r2)):
            r = dict(r, F=F)
            r.pop("speedup_vs_full", None)
            out["stages"].append(r)
            log(f"  cfg5 F={F:3d} {mode:8s} W={W:3d}: {r['ms']:.3f} ms  {r['eff_GBps']:.0f} GB/s "
                f"({100 * r['frac_hbm_peak']:.1f}% of peak)")
        del d1, d2, H1, Z2
    full = {s["F"]: s["ms"] for s in out["stages"] if s["mode"] == "full"}
    for s in out["stages"]:
        s["speedup_vs_full"] = round(full[s["F"]] / s["ms"], 2)
    return out


if __name__ == "__main__":
    sys.exit(main())
