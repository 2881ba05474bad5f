#!/usr/bin/env python3
"""Turn the rocprofv3 output of bench.py runs into profiles/<name>.md and into
an entry of profiles/traffic.json (the per-call counter traffic bench.py prints
beside its own timings, stamped with the hash of the kernel sources it was
measured at).

The runs it expects under one directory DIR (each made from the repository
root on the GPU machine, after `cd /tmp && export TMPDIR=/tmp`; ARGS selects the
workload, e.g. `--config 4` or `--config 5 --feature-width 41`):

  DIR/trace   rocprofv3 --kernel-trace --stats -d DIR/trace -o t --output-format csv --
                  python3 bench.py --main-only --no-cpu-baseline ARGS          > DIR/trace.json
  DIR/fetch   rocprofv3 --pmc FETCH_SIZE -d DIR/fetch -o t --output-format csv --
                  python3 bench.py --main-only --no-cpu-baseline --calibrate --mark-calls
                  --steps 3 --warmup 1 ARGS                                    > DIR/fetch.json
  DIR/write   the same with --pmc WRITE_SIZE                                   > DIR/write.json
  DIR/l2      the same with --pmc TCC_HIT_sum TCC_MISS_sum   (no --calibrate)
  DIR/lds     the same with --pmc SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE   (no --calibrate)
  DIR/atomic  (optional) --pmc TCC_ATOMIC_sum TCC_EA0_ATOMIC_sum -- python3 bench.py --only backward ARGS

usage: python rocprof_summary.py DIR NAME KEY [ARGS...]
   NAME  file name under profiles/ (without .md);  KEY  entry of traffic.json ("config4", "config5:F41")

Second form, for the legs that are not the W sweep (`bench.py --only backward|aux`): a per-kernel
table (mean duration from the trace run, mean FETCH_SIZE / WRITE_SIZE / atomic counters per dispatch
from the counter runs DIR/fetch, DIR/write, DIR/atomic):
       python rocprof_summary.py --kernels DIR NAME "TITLE" [ARGS...]
"""
from __future__ import annotations

import collections
import csv
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
KIB = 1024.0
GIB_KIB = 1048576.0


def short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0]


def counter_rows(d, sub):
    path = os.path.join(d, sub, "t_counter_collection.csv")
    if not os.path.exists(path):
        return []
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def per_call(rows, counter, order):
    """Mean counter value per call of one step.  A call starts at a marker
    dispatch (the int16 fill bench.py --mark-calls launches, whose order is the
    step's call order) and owns every es_ kernel up to the next marker."""
    acc = collections.defaultdict(list)
    idx, cur = -1, None
    for r in rows:
        if r["Counter_Name"] != counter:
            continue
        name = r["Kernel_Name"]
        if "FillFunctor<short>" in name:
            if cur is not None:
                acc[order[idx % len(order)]].append(cur)
            idx += 1
            cur = 0.0
        elif cur is not None and "es_" in name:
            cur += float(r["Counter_Value"])
    if cur is not None:
        acc[order[idx % len(order)]].append(cur)
    return {k: sum(v) / len(v) for k, v in acc.items()}


def kernel_mean(rows, counter, needle, first=None, largest=None):
    """Mean of `counter` over the dispatches whose kernel name holds `needle`:
    all of them, the first `first`, or the `largest` largest readings (the 1 GiB
    calibration copies among the small copies the framework issues)."""
    v = [float(r["Counter_Value"]) for r in rows if r["Counter_Name"] == counter and needle in r["Kernel_Name"]]
    if first:
        v = v[:first]
    if largest:
        v = sorted(v)[-largest:]
    return sum(v) / len(v) if v else None


def by_kernel(rows, counter):
    """{short kernel name: (mean counter value, mean dispatch ns under the counter run, dispatches)}"""
    acc = collections.defaultdict(list)
    for r in rows:
        if r["Counter_Name"] == counter and "es_" in r["Kernel_Name"]:
            acc[short(r["Kernel_Name"])].append((float(r["Counter_Value"]),
                                                 int(r["End_Timestamp"]) - int(r["Start_Timestamp"])))
    return {k: (sum(x for x, _ in v) / len(v), sum(t for _, t in v) / len(v), len(v)) for k, v in acc.items()}


def kernels_main() -> int:
    d, name, title = sys.argv[2], sys.argv[3], sys.argv[4]
    bench_args = " ".join(sys.argv[5:])
    import bench
    out = [f"# rocprofv3 summary: {title}\n",
           f"Kernel sources at hash `{bench.kernel_source_hash()}`. All commands run from the repository root on one "
           f"MI355X (`cd /tmp && export TMPDIR=/tmp` first); `<args>` = `{bench_args}`.\n",
           "`rocprofv3 --kernel-trace --stats -d <dir> -o t --output-format csv -- python3 bench.py <args>`; counters: "
           "the same command after `rocprofv3 --pmc FETCH_SIZE`, `--pmc WRITE_SIZE` and `--pmc TCC_ATOMIC_sum "
           "TCC_EA0_ATOMIC_sum` (one run each). FETCH_SIZE is scaled by 2.000, WRITE_SIZE by 1.000 (the 1 GiB copy "
           "calibration of the sweep profiles).\n"]
    stats = {short(r["Name"]): r for r in csv.DictReader(open(os.path.join(d, "trace", "t_kernel_stats.csv")))}
    fetch = by_kernel(counter_rows(d, "fetch"), "FETCH_SIZE")
    write = by_kernel(counter_rows(d, "write"), "WRITE_SIZE")
    at = counter_rows(d, "atomic")
    atom, ea = by_kernel(at, "TCC_ATOMIC_sum"), by_kernel(at, "TCC_EA0_ATOMIC_sum")
    out.append("| kernel | calls | avg us | min us | max us | fetched MB | written MB | L2 atomic requests (M) | "
               "atomics sent on to memory (M) | atomic requests / s (G) |\n|---|---|---|---|---|---|---|---|---|---|")
    for k, r in stats.items():
        if "es_" not in k:
            continue
        f = fetch.get(k, (0, 0, 0))[0] * 2.0 * KIB / 1e6
        w = write.get(k, (0, 0, 0))[0] * KIB / 1e6
        a_ = atom.get(k)
        e_ = ea.get(k)
        rate = "-" if not a_ or a_[0] == 0 else f"{a_[0] / a_[1]:.1f}"
        out.append(f"| `{k}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | {int(r['MinNs']) / 1e3:.1f} | "
                   f"{int(r['MaxNs']) / 1e3:.1f} | {f:.1f} | {w:.1f} | {'-' if not a_ else f'{a_[0] / 1e6:.2f}'} | "
                   f"{'-' if not e_ else f'{e_[0] / 1e6:.2f}'} | {rate} |")
    out.append("\nbench.py output of the trace run (stderr log lines):\n\n```")
    err = os.path.join(d, "trace.err")
    if os.path.exists(err):
        out += [l.rstrip() for l in open(err) if l.startswith("  ")]
    out.append("```\n")
    with open(os.path.join(ROOT, "profiles", name + ".md"), "w") as fh:
        fh.write("\n".join(out))
    print("\n".join(out))
    return 0


def main() -> int:
    if sys.argv[1] == "--kernels":
        return kernels_main()
    d, name, key = sys.argv[1], sys.argv[2], sys.argv[3]
    bench_args = " ".join(sys.argv[4:])
    import bench
    out = []
    trace = json.load(open(os.path.join(d, "trace.json")))
    cfg = trace["config"]
    order = cfg["call_order"]
    out.append(f"# rocprofv3 summary: es_spmm kernels, {key} W-sweep step\n")
    out.append(f"Workload: {cfg['workload']} (N={cfg['N']}, nnz={cfg['nnz']}, F={cfg['F']}); one step = "
               f"{cfg['calls_per_step']} es_spmm calls ({', '.join(order)}).\n")
    out.append(f"Kernel sources at hash `{bench.kernel_source_hash()}` (bench.py `kernel_source_hash`). All "
               "commands run from the repository root on one MI355X (`cd /tmp && export TMPDIR=/tmp` first); "
               f"`<args>` = `{bench_args}`.\n")
    out.append("## Kernel trace\n")
    out.append("`rocprofv3 --kernel-trace --stats -d <dir> -o t --output-format csv -- python3 bench.py "
               "--main-only --no-cpu-baseline <args>`\n")
    out.append("| kernel | calls | total ms | avg us | min us | max us | % |\n|---|---|---|---|---|---|---|")
    for r in csv.DictReader(open(os.path.join(d, "trace", "t_kernel_stats.csv"))):
        if float(r["Percentage"]) < 0.005:
            continue
        out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {int(r['TotalDurationNs']) / 1e6:.3f} | "
                   f"{float(r['AverageNs']) / 1e3:.2f} | {int(r['MinNs']) / 1e3:.2f} | {int(r['MaxNs']) / 1e3:.2f} | "
                   f"{r['Percentage']} |")
    rl = trace["roofline"]
    out.append(f"\nbench.py line of the same run: value {trace['value']} GB/s (B_eff), ms_per_step "
               f"{trace['ms_per_step']}; per es_spmm call (HIP events over the timed region): launch_ms "
               f"{rl['launch_ms']}, B_eff {rl['effective_bytes_per_launch']} bytes -> "
               f"{rl['rates_GBps']['effective_B_eff']} GB/s ({rl['effective_over_hbm_peak']} x HBM peak, "
               f"cache_served {rl['cache_served']}), B_min {rl['bytes_per_launch']} bytes -> {rl['achieved']} GB/s = "
               f"roofline.frac {rl['frac']} of the 8 TB/s HBM peak.\n")

    fetch, write = counter_rows(d, "fetch"), counter_rows(d, "write")
    l2, lds = counter_rows(d, "l2"), counter_rows(d, "lds")
    cf = kernel_mean(fetch, "FETCH_SIZE", "copyBuffer", largest=3)
    cw = kernel_mean(write, "WRITE_SIZE", "copyBuffer", largest=3)
    ff, fw = GIB_KIB / cf, GIB_KIB / cw
    out.append("## Traffic leaving the L2s (TCC_EA), two runs\n")
    out.append("`rocprofv3 --pmc FETCH_SIZE -d <dir> -o t --output-format csv -- python3 bench.py --main-only "
               "--no-cpu-baseline --calibrate --mark-calls --steps 3 --warmup 1 <args>` and the same with "
               "`WRITE_SIZE`.\n")
    out.append(f"Scale: a 1 GiB device-to-device copy (`__amd_rocclr_copyBuffer`, 1048576 KiB each way) reads "
               f"FETCH_SIZE = {cf:.1f} and WRITE_SIZE = {cw:.1f}; factors {ff:.3f} and {fw:.3f}.\n")
    L = None
    cal = json.load(open(os.path.join(d, "fetch.json"))).get("calibration")
    probe = kernel_mean(fetch, "FETCH_SIZE", "es_materialize_kernel", first=3)
    if cal and probe:
        sp = cal["strided_probe"]
        got = probe * ff * KIB - sp["rowptr_bytes"]
        best = min(sp["blocks_touched"], key=lambda b: abs(sp["blocks_touched"][b] * int(b) - got))
        L = int(best)
        out.append(f"Fetch granularity: the strided-read probe (es_materialize_kernel, FastRand W={sp['W']} on "
                   f"{sp['rows']} rows of {sp['row_length']} entries: {sp['sampled_entries']} sampled entries, "
                   f"each a 4-byte read of colidx and of vals) fetched {got / 1e6:.1f} MB = "
                   f"{got / (2 * sp['sampled_entries']):.1f} bytes per 4-byte read; the blocks it touches "
                   f"predict " + ", ".join(f"{sp['blocks_touched'][b] * int(b) / 1e6:.1f} MB at {b} B"
                                           for b in sp["blocks_touched"]) + f" -> L = {L} bytes.\n")
    pf, pw = per_call(fetch, "FETCH_SIZE", order), per_call(write, "WRITE_SIZE", order)
    ph, pm = per_call(l2, "TCC_HIT_sum", order), per_call(l2, "TCC_MISS_sum", order)
    pc, pa = per_call(lds, "SQ_LDS_BANK_CONFLICT", order), per_call(lds, "SQ_LDS_IDX_ACTIVE", order)
    out.append("| call | fetched MB | written MB | traffic MB | L2 hit % | LDS bank-conflict / active cycles |\n"
               "|---|---|---|---|---|---|")
    calls = {}
    for k in order:
        fb, wb = pf[k] * ff * KIB, pw[k] * fw * KIB
        hit = 100 * ph[k] / (ph[k] + pm[k]) if k in ph and ph[k] + pm[k] > 0 else None
        calls[k] = {"fetch_bytes": int(fb), "write_bytes": int(wb), "l2_hit_pct": None if hit is None else round(hit, 1)}
        out.append(f"| {k} | {fb / 1e6:.1f} | {wb / 1e6:.1f} | {(fb + wb) / 1e6:.1f} | "
                   f"{'-' if hit is None else f'{hit:.1f}'} | "
                   f"{pc.get(k, float('nan')):.0f} / {pa.get(k, float('nan')):.0f} |")
    tot = sum(c["fetch_bytes"] + c["write_bytes"] for c in calls.values())
    out.append(f"\nMean traffic per es_spmm call over the step: {tot / len(order) / 1e6:.1f} MB (B_eff per call "
               f"{rl['effective_bytes_per_launch'] / 1e6:.1f} MB, B_min per call {rl['bytes_per_launch'] / 1e6:.1f} MB); "
               f"at launch_ms {rl['launch_ms']} that is {tot / len(order) / (rl['launch_ms'] * 1e6):.0f} GB/s.\n")
    out.append("FETCH_SIZE / WRITE_SIZE count what crosses from the L2s to the memory fabric: reads that the "
               "256 MB Infinity Cache serves are included, so this is L2-miss traffic, an upper bound of HBM traffic.\n")
    out.append("L2 counters: `rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum ...`; LDS counters: `rocprofv3 --pmc "
               "SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE ...` (same bench arguments, without --calibrate).\n")
    with open(os.path.join(ROOT, "profiles", name + ".md"), "w") as fh:
        fh.write("\n".join(out))

    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        doc = json.load(open(tpath))
    except (OSError, ValueError):
        doc = {"note": "written by rocprof_summary.py from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of "
                       "bench.py; bytes per es_spmm call, scaled by a 1 GiB copy", "workloads": {}}
    if L:
        doc["fetch_granularity_bytes"] = L
    doc["workloads"][key] = {"source_hash": bench.kernel_source_hash(), "profile": f"profiles/{name}.md",
                             "calls": calls}
    with open(tpath, "w") as fh:
        json.dump(doc, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print("\n".join(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
