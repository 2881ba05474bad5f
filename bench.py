#!/usr/bin/env python3
"""Benchmark of the ES-SpMM hot path on one MI355X.

A *step* is one pass of the whole hot path over one synthetic graph: for every
sampling width W of the configuration, es_spmm in bucket and in fastrand mode,
plus the full (unsampled) product -- Algorithm 1 of the paper end to end, and
the exact CSR SpMM it is compared with.  Inputs are resident in HBM before the
timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4|3|2|5]
                    [--main-only] [--no-cpu-baseline] [--calibrate] [--calibrate-gather]
                    [--mark-calls] [--only sweep|backward|aux]

Three byte counts per call (N rows, F columns, nnz_kept sampled entries):
  B_eff  = 4(N+1) + 8 nnz_kept + 4F nnz_kept + 4F N     one row of X per kept entry: what the
                                                         kernel requests when nothing is reused
  B_min  = 4(N+1) + 8 nnz_kept + 4F distinct + 4F N     every distinct kept column's row of X once:
                                                         the compulsory HBM traffic
  traffic                                                what rocprofv3 counted leaving the L2s
                                                         (profiles/traffic.json, written by
                                                         rocprof_summary.py; not measured here)
value   = sum of B_eff over the step / wall time of the step ("effective bandwidth": it counts
          re-reads that caches serve, so it may exceed the HBM peak -- then `cache_served` says so)
roofline.frac = B_min rate / 8 TB/s, the only one of the three that is a fraction of HBM peak.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")

CONFIG_TEXT = {
    2: "configs[1] mid-size citation-like graph: N=170k, power-law degree mean 14, F=128",
    3: "configs[2] dense social-like graph: N=233k, power-law degree mean 490, F=64",
    4: "configs[3] large co-purchase-like graph: N=2.45M, mean degree 50, F=128 (100 padded)",
}


def log(msg: str) -> None:
    print(msg, file=sys.stderr, flush=True)


# --------------------------------------------------------------------------
# byte counts
# --------------------------------------------------------------------------
def algorithmic_bytes(N: int, nnz_kept: int, F: int) -> int:
    """B_eff: row pointers, sampled (column, value) pairs, one row of X per kept entry, Y once."""
    return 4 * (N + 1) + 8 * nnz_kept + 4 * F * nnz_kept + 4 * F * N


def compulsory_bytes(N: int, nnz_kept: int, F: int, distinct_cols: int) -> int:
    """B_min: as B_eff, but every distinct kept column's row of X counted once."""
    return 4 * (N + 1) + 8 * nnz_kept + 4 * F * min(N, distinct_cols) + 4 * F * N


def sector_adjusted_bytes(N: int, nnz_kept: int, nnz_kept_strided: int, F: int, L: int) -> int:
    """B_eff with the 8 bytes per sampled entry replaced by two fetch units of L
    bytes (one of colidx, one of vals) for the entries FastRand reads at stride
    577 (rows longer than W); contiguous reads keep their 8 bytes."""
    return (4 * (N + 1) + 8 * (nnz_kept - nnz_kept_strided) + 2 * L * nnz_kept_strided
            + 4 * F * nnz_kept + 4 * F * N)


def line_floor_bytes(N: int, nnz_kept: int, F: int, ldx: int, L: int) -> int:
    """B_eff with each gathered row of X counted as the whole L-byte lines it
    touches: a row of 4F bytes starting at byte 4*ldx*c touches
    ceil((start mod L + 4F) / L) lines; averaged over the start offsets that
    occur (multiples of gcd(4*ldx, L)).  What a kernel moves at least when no
    line is ever shared between two gathers."""
    from math import gcd
    step = gcd(4 * ldx, L)
    offs = range(0, L, step)
    lines = sum(-(-(o + 4 * F) // L) for o in offs) / len(offs)
    return int(4 * (N + 1) + 8 * nnz_kept + lines * L * nnz_kept + 4 * F * N)


def kernel_source_hash() -> str:
    """Hash of the kernel sources; profiles/traffic.json carries the hash it was measured at."""
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2104_10716_amd", "csrc")
    for name in sorted(os.listdir(src)):
        if name.endswith((".h", ".hip")):
            h.update(name.encode())
            h.update(open(os.path.join(src, name), "rb").read())
    return h.hexdigest()[:16]


def load_traffic(key: str):
    """Per-call counter traffic of workload `key` from profiles/traffic.json, or ({}, meta)."""
    try:
        with open(TRAFFIC_FILE) as fh:
            doc = json.load(fh)
    except (OSError, ValueError):
        return {}, {"file": None}
    entry = doc.get("workloads", {}).get(key, {})
    meta = {"file": "profiles/traffic.json", "measured_at_source_hash": entry.get("source_hash"),
            "current_source_hash": kernel_source_hash(),
            "fetch_granularity_bytes": doc.get("fetch_granularity_bytes")}
    meta["stale"] = meta["measured_at_source_hash"] != meta["current_source_hash"]
    return entry.get("calls", {}), meta


# --------------------------------------------------------------------------
# workload on the device
# --------------------------------------------------------------------------
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
        # caller-owned workspace of es_spmm_ws (lets the library run its column-partitioned
        # product where it decides to); allocated once, outside every timed region
        import paper_2104_10716_amd as es
        self.ws = torch.empty(max(1, es.es_spmm_workspace_bytes(self.N) // 4), dtype=torch.int32, device=dev)
        self._distinct = {}

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

    def nnz_kept_strided(self, mode, W):
        """Kept entries FastRand reads at stride 577: those of rows longer than W."""
        if mode != "fastrand":
            return 0
        return int(W * int((self.deg > W).sum()))

    def distinct_kept_columns(self, mode, W):
        """Number of distinct columns among the kept entries (for B_min).  Counted
        on the device from the library's own sampled-graph export, outside any
        timed region."""
        import torch
        import paper_2104_10716_amd as es
        key = (mode, W)
        if key not in self._distinct:
            flags = torch.zeros(self.N, dtype=torch.bool, device=self.rowptr.device)
            if mode == "full":
                flags[self.colidx.long()] = True
            else:
                orp, oci, _ = es.es_spmm_materialize(self.rowptr, self.colidx, None, W, mode, 0)
                kept = int(orp[-1].item())
                flags[oci[:kept].long()] = True
                del orp, oci
            self._distinct[key] = int(flags.sum().item())
            torch.cuda.empty_cache()
        return self._distinct[key]

    def launch(self, mode, W, seed=0):
        import paper_2104_10716_amd as es
        es.es_spmm_ws(self.rowptr, self.colidx, self.vals, self.X, self.Y, W, mode, seed, "none", None, self.ws,
                      F=self.F)


def call_label(mode, W):
    return f"{mode}:{W}"


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


def rates_row(dw, mode, W, ms, traffic_calls, L):
    """The three rates of one call at `ms` milliseconds."""
    kept = dw.nnz_kept(mode, W)
    B_eff = algorithmic_bytes(dw.N, kept, dw.F)
    B_min = compulsory_bytes(dw.N, kept, dw.F, dw.distinct_kept_columns(mode, W))
    eff = B_eff / (ms * 1e6)
    row = {"nnz_kept": kept, "gflops": round(2.0 * kept * dw.F / (ms * 1e6), 1),
           "eff_GBps": round(eff, 1), "eff_over_hbm_peak": round(eff / HBM_PEAK_GBPS, 4),
           "min_GBps": round(B_min / (ms * 1e6), 1),
           "hbm_frac_compulsory": round(B_min / (ms * 1e6) / HBM_PEAK_GBPS, 4)}
    if L:
        B_sec = sector_adjusted_bytes(dw.N, kept, dw.nnz_kept_strided(mode, W), dw.F, L)
        row["eff_sector_adjusted_GBps"] = round(B_sec / (ms * 1e6), 1)
        ldx = int(dw.X.stride(0))
        if (4 * ldx) % L or (4 * dw.F) % L:                    # rows do not tile whole lines (F = 41, 64, ...)
            B_line = line_floor_bytes(dw.N, kept, dw.F, ldx, L)
            row["line_floor_bytes"] = B_line
            row["line_floor_over_B_eff"] = round(B_line / B_eff, 3)
            row["line_floor_GBps"] = round(B_line / (ms * 1e6), 1)
    t = traffic_calls.get(call_label(mode, W))
    if t:
        tb = t["fetch_bytes"] + t["write_bytes"]
        row["traffic_GBps"] = round(tb / (ms * 1e6), 1)
        row["traffic_over_B_eff"] = round(tb / B_eff, 3)
        row["l2_hit_pct"] = t.get("l2_hit_pct")
    # the kernel requested more than HBM can deliver in that time, or the counters saw
    # clearly fewer bytes leave the L2s than it requested: caches served the difference
    row["cache_served"] = bool(eff > HBM_PEAK_GBPS or (t and row["traffic_over_B_eff"] < 0.9))
    return row


def per_call_table(dw, calls, reps, flush, cold_reps, traffic_calls=None, L=None):
    rows = []
    t_full = None
    for mode, W in calls:
        for _ in range(2):
            dw.launch(mode, W)
        med, mn = time_call(dw, mode, W, reps)
        cold = time_call(dw, mode, W, cold_reps, flush)[0] if flush is not None and cold_reps else None
        row = {"mode": mode, "W": W, "ms": round(med, 4), "ms_min": round(mn, 4),
               "ms_cold": None if cold is None else round(cold, 4)}
        row.update(rates_row(dw, mode, W, med, traffic_calls or {}, L))
        rows.append(row)
        if mode == "full":
            t_full = med
    for r in rows:
        r["speedup_vs_full"] = round(t_full / r["ms"], 2) if t_full else None
    return rows


def log_rows(tag, rows):
    for r in rows:
        log(f"  {tag} {r['mode']:8s} W={r['W']:4d}: {r['ms']:.3f} ms | B_eff {r['eff_GBps']:.0f} GB/s "
            f"({r['eff_over_hbm_peak']:.2f}x HBM peak{', cache-served' if r['cache_served'] else ''}) | "
            f"B_min {r['min_GBps']:.0f} GB/s ({100 * r['hbm_frac_compulsory']:.1f}% of HBM peak)"
            + (f" | L2-miss traffic {r['traffic_GBps']:.0f} GB/s" if "traffic_GBps" in r else "")
            + (f" | x{r['speedup_vs_full']} vs full" if r.get("speedup_vs_full") else ""))


# --------------------------------------------------------------------------
# CPU baseline: the oracle as it stands, on the GPU machine's host cores
# --------------------------------------------------------------------------
def cpu_baseline(dw, calls, target_seconds=12.0, max_passes=6):
    """The oracle, as it stands, on the same workload: every call of the sweep on
    a random subset of rows sized from a short probe so that about
    `target_seconds` of CPU work are timed (whole passes over all rows, repeated,
    when the host is fast enough), at all cores; then the same on one core with a
    proportionally smaller subset.  GB/s of the same B_eff byte count as `value`."""
    import numpy as np
    import oracle
    w = dw.w
    Xh = w.X if tuple(dw.X.shape) == tuple(w.X.shape) else dw.X.cpu().numpy()
    cores = oracle.threads()
    order = np.random.default_rng(0).permutation(dw.N).astype(np.int64)

    def run(rows_):
        total = 0
        t0 = time.perf_counter()
        for mode, W in calls:
            oracle.spmm(w.rowptr, w.colidx, w.vals, Xh, dw.F, W, mode, 0, rows=rows_, want_denom=False)
            kept = int((dw.deg[rows_] if mode == "full" else np.minimum(dw.deg[rows_], W)).sum())
            total += algorithmic_bytes(rows_.size, kept, dw.F)
        return total, time.perf_counter() - t0

    def sized(threads):
        oracle.set_threads(threads)
        probe = np.sort(order[:max(1, dw.N // 100)])
        run(probe[: max(1, probe.size // 10)])                    # first touch: threads, page cache
        _, dt = run(probe)                                        # 1 % of the rows sizes the sample
        frac = min(1.0, target_seconds / max(dt, 1e-3) / 100.0)
        rows = np.sort(order[:max(1, int(dw.N * frac))])
        total = dt_sum = 0.0
        passes = 0
        while passes < max_passes and (passes == 0 or (frac >= 1.0 and dt_sum < target_seconds)):
            b, dt = run(rows)
            total += b
            dt_sum += dt
            passes += 1
        return total / dt_sum / 1e9, dt_sum, rows.size, passes

    v, dt, nrows, passes = sized(cores)
    out = {"value": round(v, 3), "unit": "GB/s", "cores": cores, "kind": "oracle", "seconds": round(dt, 2),
           "sample": f"{passes} pass(es) over {nrows} random rows of {dw.N} ({100.0 * nrows / dw.N:.2f}%), every "
                     f"call of the sweep, fp64 accumulation, B_eff bytes of those rows"}
    v1, dt1, nrows1, passes1 = sized(1)
    oracle.set_threads(cores)
    out["single_core_value"] = round(v1, 3)
    out["single_core_sample"] = f"{passes1} pass(es) over {nrows1} rows, {dt1:.1f} s"
    return out


# --------------------------------------------------------------------------
# calibration legs (context figures; their kernels carry names rocprof_summary.py looks for)
# --------------------------------------------------------------------------
def calibrate_counters(dev):
    """Kernels of known traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE:
    three 1 GiB device-to-device copies, then three runs of the sampler export
    (es_materialize_kernel, FastRand W=16) on a graph of 65 536 rows of 2 000
    entries each, whose strided reads of colidx and vals touch a number of
    32 / 64 / 128-byte blocks computed here: the fetch granularity L is the block
    size whose count matches the counter."""
    import numpy as np
    import torch
    import paper_2104_10716_amd as es
    src = torch.ones(256 * 1024 * 1024, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst
    rows, n, W = 65536, 2000, 16
    rowptr = (torch.arange(rows + 1, dtype=torch.int64, device=dev) * n).to(torch.int32)
    colidx = torch.zeros(rows * n, dtype=torch.int32, device=dev)
    vals = torch.ones(rows * n, dtype=torch.float32, device=dev)
    out = es.es_spmm_materialize(rowptr, colidx, vals, W, "fastrand", 0)
    for _ in range(2):
        es.es_spmm_materialize(rowptr, colidx, vals, W, "fastrand", 0, *out)
    torch.cuda.synchronize()
    pos = (np.arange(W, dtype=np.int64) * 577) % n                      # Equation 2, seed 0
    byte_off = (np.arange(rows, dtype=np.int64)[:, None] * n + pos[None, :]) * 4
    blocks = {str(L): int(np.unique(byte_off // L).size) * 2 for L in (32, 64, 128)}   # colidx + vals
    del rowptr, colidx, vals, out
    torch.cuda.empty_cache()
    return {"copy_bytes_each_way": 1 << 30, "strided_probe": {"rows": rows, "row_length": n, "W": W,
            "sampled_entries": rows * W, "blocks_touched": blocks, "rowptr_bytes": 4 * (rows + 1),
            "written_bytes": rows * W * 8}}


def calibrate_gather(dev):
    """What the machine sustains on random row gathers, measured with the
    library's own exact product: graphs of N rows with 64 uniformly random
    columns each, unit values, table = X of N x F floats.  `roaming`: columns
    anywhere in the table; `own_eighth`: a row's columns lie in the eighth of the
    table its own position falls in, so each XCD (which walks a contiguous range
    of rows) touches one eighth of X."""
    import torch
    import paper_2104_10716_amd as es
    deg = 64
    out = []
    g = torch.Generator(device=dev)
    g.manual_seed(99)
    for F in (64, 128, 256):
        for mb in (8, 16, 32, 64, 128, 256, 1024):
            N = (mb << 20) // (4 * F)
            rowptr = (torch.arange(N + 1, dtype=torch.int64, device=dev) * deg).to(torch.int32)
            X = torch.ones((N, F), dtype=torch.float32, device=dev)
            Y = torch.empty_like(X)
            row = {"F": F, "table_MB": mb, "rows": N}
            for kind in ("roaming", "own_eighth"):
                cols = torch.randint(0, N, (N * deg,), dtype=torch.int64, device=dev, generator=g)
                if kind == "own_eighth":
                    share = N // 8
                    owner = (torch.arange(N, device=dev) // share).clamp(max=7).repeat_interleave(deg)
                    cols = owner * share + cols % share
                cols = cols.to(torch.int32)
                t = _time_fn(lambda: es.es_spmm(rowptr, cols, None, X, Y, 0, "full"), reps=5, warm=2)
                row[kind + "_GBps"] = round(algorithmic_bytes(N, N * deg, F) / (t * 1e6), 1)
                del cols
            out.append(row)
            log(f"  gather calibration F={F} table {mb} MB: roaming {row['roaming_GBps']:.0f} GB/s, "
                f"own eighth per XCD {row['own_eighth_GBps']:.0f} GB/s")
            del rowptr, X, Y
            torch.cuda.empty_cache()
    return out


# --------------------------------------------------------------------------
def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, choices=(2, 3, 4, 5))
    ap.add_argument("--feature-width", type=int, default=41, choices=(41, 256),
                    help="config 5 only: which SpMM stage of the 2-layer GCN forward to time")
    ap.add_argument("--main-only", action="store_true",
                    help="only the timed sweep of --config (what the rocprofv3 summaries profile)")
    ap.add_argument("--only", choices=("sweep", "backward", "aux", "calls"), default="sweep",
                    help="backward / aux: run only the transposed-product or the sampled-graph export "
                         "kernels of --config a few times (for rocprofv3) and print their timings; "
                         "calls: only the per-call timing table of --config (also for builds of the "
                         "library loaded through ES_SPMM_LIBRARY)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="first run kernels of known traffic (1 GiB copies, a strided-read probe) that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--calibrate-gather", action="store_true",
                    help="also time random row gathers of 8 MB - 1 GB tables (context for the rates)")
    ap.add_argument("--mark-calls", action="store_true",
                    help="launch a tiny int16 fill before every es_spmm call so that a counter run's "
                         "dispatch list can be cut into calls (adds launch gaps: not for timing)")
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

    calibration = calibrate_counters(dev) if args.calibrate else None

    t0 = time.perf_counter()
    w = make_workload(3 if args.config == 5 else args.config)
    log(f"config {args.config}: N={w.N} nnz={w.nnz} F={w.F} generated in {time.perf_counter() - t0:.1f}s")
    if args.config == 5:
        dw = gcn_stage_workload(w, dev, args.feature_width)
        calls = dw.calls((64,))
        workload_text = (f"configs[4] 2-layer GCN forward on the config-3 graph, SpMM stage at "
                         f"F={args.feature_width} (row stride {args.feature_width})")
        traffic_key = f"config5:F{args.feature_width}"
    else:
        dw = DeviceWorkload(w, dev)
        calls = dw.calls(w.Ws)
        workload_text = CONFIG_TEXT[args.config]
        traffic_key = f"config{args.config}"

    if args.only != "sweep":
        if args.only == "calls":
            rows = per_call_table(dw, calls, 20, None, 0)
            log_rows(f"cfg{args.config}", rows)
        else:
            rows = (backward_table(dw, dev, [c for c in calls if c[0] != "full"][:6]) if args.only == "backward"
                    else aux_table(dw, dev, calls))
        print(json.dumps({"workload": workload_text, "only": args.only, "result": rows}), flush=True)
        return 0

    traffic_calls, traffic_meta = load_traffic(traffic_key)
    L = traffic_meta.get("fetch_granularity_bytes")
    # counts for the byte formulas, outside the timed region
    kept = {c: dw.nnz_kept(*c) for c in calls}
    distinct = {c: dw.distinct_kept_columns(*c) for c in calls}
    step_B_eff = sum(algorithmic_bytes(dw.N, kept[c], dw.F) for c in calls)
    step_B_min = sum(compulsory_bytes(dw.N, kept[c], dw.F, distinct[c]) for c in calls)
    step_flops = sum(2 * kept[c] * dw.F for c in calls)
    have_traffic = all(call_label(*c) in traffic_calls for c in calls)
    step_traffic = (sum(traffic_calls[call_label(*c)]["fetch_bytes"] + traffic_calls[call_label(*c)]["write_bytes"]
                        for c in calls) if have_traffic else None)

    # which kernel serves each call (as rocprofv3 names it, template arguments cut to the lane count)
    def kernel_of(mode, W):
        info = es.es_spmm_launch_info(dw.N, dw.nnz, dw.F, W, mode, ldx=dw.X.stride(0), ldy=dw.Y.stride(0),
                                      aligned16=(dw.F % 4 == 0 and dw.X.stride(0) % 4 == 0))
        if info["column_ranges"] > 1:
            base = "es_spmm_part_flat_kernel" if info["flattened"] else "es_spmm_part_kernel"
        else:
            base = "es_spmm_flat_kernel" if info["flattened"] else "es_spmm_kernel"
        return f"{base}<{info['lanes_per_row']}, ...>"
    call_kernels = {call_label(*c): kernel_of(*c) for c in calls}
    names = list(call_kernels.values())
    main_kernel = max(set(names), key=names.count)

    marker = torch.empty(1, dtype=torch.int16, device=dev)      # fill_ on it: FillFunctor<short>, used nowhere else

    def step():
        for i, (mode, W) in enumerate(calls):
            if args.mark_calls:
                marker.fill_(i)
            dw.launch(mode, W)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)       # on torch's current stream, where es_spmm launches
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
    kernel_ms = ev_ms / launches                      # mean es_spmm call duration, HIP events
    eff = step_B_eff / len(calls) / (kernel_ms * 1e6)
    cmin = step_B_min / len(calls) / (kernel_ms * 1e6)
    log(f"step: {ms_per_step:.3f} ms wall, {ev_ms / args.steps:.3f} ms by events; B_eff {step_B_eff / 1e9:.3f} GB "
        f"-> {step_B_eff / (ms_per_step * 1e6):.0f} GB/s effective; B_min {step_B_min / 1e9:.3f} GB -> "
        f"{cmin:.0f} GB/s compulsory")

    roofline = {
        "bound": "hbm", "unit": "GB/s", "peak": HBM_PEAK_GBPS,
        # compulsory bytes: the only count that is HBM traffic by construction, so the only
        # one reported as a fraction of the HBM peak
        "achieved": round(cmin, 1), "frac": round(cmin / HBM_PEAK_GBPS, 4),
        "bytes": "B_min: rowptr + kept (column, value) pairs + each DISTINCT kept column's row of X once + Y once",
        "bytes_per_launch": int(step_B_min / len(calls)),
        "kernel": main_kernel, "kernel_of_call": call_kernels, "launch_ms": round(kernel_ms, 5),
        "traffic": None if step_traffic is None else int(step_traffic / len(calls)),
        "traffic_source": traffic_meta,
        "rates_GBps": {
            "effective_B_eff": round(eff, 1),
            "compulsory_B_min": round(cmin, 1),
            "l2_miss_traffic": None if step_traffic is None
            else round(step_traffic / len(calls) / (kernel_ms * 1e6), 1)},
        "effective_bytes_per_launch": int(step_B_eff / len(calls)),
        "effective_over_hbm_peak": round(eff / HBM_PEAK_GBPS, 4),
        "cache_served": bool(eff > HBM_PEAK_GBPS or (step_traffic is not None and step_traffic < 0.9 * step_B_eff)),
        "served_by": "per-XCD 4 MB L2 and the 256 MB Infinity Cache: B_eff counts one row of X per kept "
                     "entry, the counters see only L2 misses, HBM sees only what the Infinity Cache misses",
    }
    result = {
        "metric": "es_spmm effective bandwidth (B_eff algorithmic bytes / time) over the W sweep "
                  "{bucket,fastrand} + full SpMM",
        "value": round(step_B_eff / (ms_per_step * 1e6), 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "gflops": round(step_flops / (ms_per_step * 1e6), 1),
        "config": {"workload": workload_text, "N": dw.N, "nnz": dw.nnz, "F": dw.F,
                   "W": sorted({W for _, W in calls if W}), "modes": ["bucket", "fastrand", "full"], "seed": 0,
                   "calls_per_step": len(calls), "call_order": [call_label(*c) for c in calls]},
        "roofline": roofline,
    }
    if calibration is not None:
        result["calibration"] = calibration

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(dw, calls)
        log(f"cpu baseline: {result['cpu_baseline']}")

    if args.calibrate_gather:
        result["gather_calibration"] = calibrate_gather(dev)

    if not args.main_only:
        flush = torch.empty(256 * 1024 * 1024, dtype=torch.float32, device=dev)   # 1 GiB
        flush.zero_()
        result["calls"] = per_call_table(dw, calls, 20, flush, 5, traffic_calls, L)
        log_rows(f"cfg{args.config}", result["calls"])
        extra = [tiny_config1(dev)]
        for cfg in (2, 3, 4):
            if cfg == args.config:
                continue
            del dw
            torch.cuda.empty_cache()
            t0 = time.perf_counter()
            w = make_workload(cfg)
            log(f"config {cfg}: N={w.N} nnz={w.nnz} F={w.F} generated in {time.perf_counter() - t0:.1f}s")
            dw = DeviceWorkload(w, dev)
            tc, tm = load_traffic(f"config{cfg}")
            rows = per_call_table(dw, dw.calls(w.Ws), 10, flush, 3, tc, L)
            extra.append({"workload": CONFIG_TEXT[cfg], "N": dw.N, "nnz": dw.nnz, "F": dw.F, "calls": rows,
                          "traffic_source": tm})
            log_rows(f"cfg{cfg}", rows)
            if cfg == 3:
                big = per_call_table(dw, [("bucket", 1792), ("bucket", 2304), ("fastrand", 1792),
                                          ("full", 0)], 5, None, 0)
                extra.append({"workload": "config-3 graph at the widths the paper needs for Bucket on its "
                                          "densest graph (S = 1792, 2304)", "calls": big[:-1]})
                log_rows("cfg3", big[:-1])
                extra.append(presampled_ablation(dw, dev))
                extra.append(unweighted_norm_table(dw, dev))
                extra.append(backward_table(dw, dev, ((("fastrand", 16), ("fastrand", 64), ("bucket", 64),
                                                       ("fastrand", 256)))))
                extra.append(gcn_feature_sweep(dw, dev, flush))
        result["extra"] = extra

    print(json.dumps(result), flush=True)
    return 0


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
    import paper_2104_10716_amd as es
    out = {"workload": f"pre-sampled graph ablation (paper Section 5.6) on the same graph, F={dw.F}",
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


def aux_table(dw, dev, calls):
    """The sampled-graph export kernels on their own (scan + es_materialize_kernel)."""
    import paper_2104_10716_amd as es
    out = {"workload": "es_spmm_materialize on the same graph", "rows": []}
    for mode, W in calls:
        bufs = es.es_spmm_materialize(dw.rowptr, dw.colidx, dw.vals, W, mode, 0)
        t = _time_fn(lambda: es.es_spmm_materialize(dw.rowptr, dw.colidx, dw.vals, W, mode, 0, *bufs), reps=5)
        out["rows"].append({"mode": mode, "W": W, "materialize_ms": round(t, 4), "kept": dw.nnz_kept(mode, W)})
        log(f"  materialise {mode:8s} W={W:4d}: {t:.3f} ms")
        del bufs
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
        t_norm = _time_fn(lambda: es.es_spmm_ws(dw.rowptr, dw.colidx, None, dw.X, Y2, W, mode, 0,
                                                "inv_degree", None, dw.ws, F=dw.F))
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
    tg = es.es_spmm_transpose_graph(dw.rowptr, dw.colidx, dw.vals)
    t_graph = _time_fn(lambda: es.es_spmm_transpose_graph(dw.rowptr, dw.colidx, dw.vals), reps=3, warm=1)
    out["transpose_graph_once_ms"] = round(t_graph, 4)
    log(f"  backward: transposed graph for the pull kernel, built once per graph: {t_graph:.3f} ms")
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
        t_inv = _time_fn(lambda: es.es_spmm_backward_pull(dw.rowptr, tg, dw.X, dX, W, mode, 0, F=dw.F))
        out["rows"].append({"mode": mode, "W": W, "forward_ms": round(t_fwd, 4),
                            "backward_pull_ms": round(t_inv, 4),
                            "backward_atomic_ms": round(t_bwd, 4), "sampled_transpose_build_ms": round(t_build, 4),
                            "full_product_on_sampled_transpose_ms": round(t_pull, 4)})
        log(f"  backward {mode:8s} W={W:3d}: pull over the transposed graph {t_inv:.3f} ms | atomic scatter "
            f"{t_bwd:.3f} ms | sampled transpose build {t_build:.3f} ms + product on it {t_pull:.3f} ms | "
            f"forward {t_fwd:.3f} ms")
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
    t256, _ = load_traffic("config5:F256")
    t41, _ = load_traffic("config5:F41")
    for mode, W in (("bucket", 64), ("fastrand", 64), ("full", 0)):
        d1 = DeviceWorkload(dw3.w, dev, X=Z1, F=256)
        r1 = per_call_table(d1, [(mode, W)], 10, flush, 3, t256)[0]
        H1 = torch.relu(d1.Y)
        Z2 = H1 @ W2                                        # [N x 41], row stride 41
        d2 = DeviceWorkload(dw3.w, dev, X=Z2, F=41)
        r2 = per_call_table(d2, [(mode, W)], 10, flush, 3, t41)[0]
        for F, r in ((256, r1), (41, r2)):
            r = dict(r, F=F)
            r.pop("speedup_vs_full", None)
            out["stages"].append(r)
        del d1, d2, H1, Z2
    full = {s["F"]: s["ms"] for s in out["stages"] if s["mode"] == "full"}
    for s in out["stages"]:
        s["speedup_vs_full"] = round(full[s["F"]] / s["ms"], 2)
    for F in (256, 41):
        log_rows(f"cfg5 F={F}", [s for s in out["stages"] if s["F"] == F])
    return out


if __name__ == "__main__":
    sys.exit(main())
