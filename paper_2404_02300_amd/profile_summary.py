"""Turn rocprofv3 output (CSV) into the short text summaries under profiles/ and
into profiles/traffic.json, the per-kernel HBM bytes bench.py reports as
`roofline.traffic`.

    python -m paper_2404_02300_amd.profile_summary <workload> --trace DIR [--fetch DIR --write DIR] [--mfma DIR]
                                                   [--bench JSON] [--note TEXT]

DIR is the `-d` directory of one rocprofv3 run of `bench.py --workload <workload>`:
  --trace  rocprofv3 --kernel-trace --stats --output-format csv -d DIR -o trace -- python3 bench.py ...
  --fetch  rocprofv3 --pmc FETCH_SIZE        --output-format csv -d DIR -o pmc   -- python3 bench.py ... --calibrate-copy
  --write  rocprofv3 --pmc WRITE_SIZE        (same command)
  --mfma   rocprofv3 --pmc MfmaUtil          (same command, without --calibrate-copy)
The counter runs start with one plain 1 GiB device copy (`--calibrate-copy`); what the two
counters read for it gives the bytes per count (FETCH_SIZE and WRITE_SIZE are specified in
KiB, but one FETCH_SIZE count is 2 KiB on this machine) and is checked here, not assumed.

traffic.json carries a hash of the kernel sources it was measured with; bench.py reports the
figures only while the sources still hash to the same value and prints null otherwise.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os
import re
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
PROFILES = os.path.join(ROOT, "profiles")
TRAFFIC = os.path.join(PROFILES, "traffic.json")
GIB = float(1 << 30)


def sources_hash() -> str:
    """sha256 over the HIP sources and internal header the library is built from."""
    h = hashlib.sha256()
    for p in sorted(glob.glob(os.path.join(HERE, "csrc", "*"))):
        if p.endswith((".hip", ".h")):
            h.update(os.path.basename(p).encode())
            h.update(open(p, "rb").read())
    return h.hexdigest()[:16]


def short_name(n: str) -> str:
    n = re.sub(r"sdt::\(anonymous namespace\)::", "", n)
    n = re.sub(r"\(anonymous namespace\)::", "", n)
    n = re.sub(r"^void ", "", n)
    return re.sub(r"\(.*$", "", n)


def _find(d: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    if not hits:
        raise FileNotFoundError(f"no *{suffix} under {d}")
    return hits[0]


def _grid(r: dict) -> int:
    if r.get("Grid_Size"):
        return int(r["Grid_Size"])
    g = 1
    for k in ("Grid_Size_X", "Grid_Size_Y", "Grid_Size_Z"):
        g *= max(1, int(r.get(k) or 1))
    return g


def kernel_key(name: str, grid: int) -> str:
    return f"{short_name(name)} [{grid} threads]"


def is_ours(key: str) -> bool:
    return not (key.startswith("at::") or key.startswith("__amd") or key.startswith("void at::"))


def read_trace(d: str):
    """[(key, calls, total_us, avg_us, percent)] sorted by total time, per (kernel, launch size)."""
    rows = list(csv.DictReader(open(_find(d, "kernel_trace.csv"))))
    agg = collections.OrderedDict()
    for r in rows:
        agg.setdefault(kernel_key(r["Kernel_Name"], _grid(r)), []).append(
            (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    tot = sum(sum(v) for v in agg.values()) or 1.0
    out = [(k, len(v), sum(v), sum(v) / len(v), 100 * sum(v) / tot) for k, v in agg.items()]
    out.sort(key=lambda t: -t[2])
    return out


def read_counter(d: str):
    """{key: [values per dispatch]} of a one-counter --pmc run, in dispatch order."""
    rows = list(csv.DictReader(open(_find(d, "counter_collection.csv"))))
    agg = collections.OrderedDict()
    for r in rows:
        agg.setdefault(kernel_key(r["Kernel_Name"], _grid(r)), []).append(float(r["Counter_Value"]))
    return agg


def calibrate(counter: dict, what: str) -> float:
    """Bytes per count, from the plain 1 GiB device copy of `bench.py --calibrate-copy`: the runtime's
    buffer-copy kernel (the largest of its dispatches; the small ones are host uploads of a few bytes)."""
    best = 0.0
    for k, v in counter.items():
        if k.startswith("__amd_rocclr_copyBuffer"):
            best = max(best, max(v))
    if best <= 0:
        raise ValueError(f"{what}: no calibration copy found (run bench.py with --calibrate-copy)")
    per = GIB / best
    # the copy moves exactly 1 GiB each way; the factor must be a whole number of KiB within 1 %
    kib = per / 1024.0
    if kib < 0.99 or abs(kib - round(kib)) > 0.01 * round(kib):
        raise ValueError(f"{what}: calibration gives {kib:.3f} KiB per count, not a whole number")
    return float(round(kib)) * 1024.0


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("workload")
    ap.add_argument("--trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--mfma")
    ap.add_argument("--bench", help="the JSON line bench.py printed for the same workload and build (not under the profiler)")
    ap.add_argument("--command", default=None, help="the bench.py arguments of the profiled runs (for the record)")
    ap.add_argument("--note", default=None)
    ap.add_argument("--out", default=None, help="summary file name under profiles/ (default: derived from the workload)")
    a = ap.parse_args(argv)
    w = a.workload
    cmd = a.command or f"--workload {w} --steps 20 --no-cpu-baseline --serial --reps 1"
    L = [f"rocprofv3 summaries, bench.py {cmd}, one MI355X; kernel sources hash {sources_hash()}.", ""]
    if a.note:
        L += [a.note, ""]
    if a.trace:
        L += ["command (cwd /tmp, TMPDIR=/tmp):",
              f"  rocprofv3 --kernel-trace --stats --output-format csv -d {a.trace} -o trace -- python3 bench.py {cmd}",
              "Kernel durations in microseconds from the kernel trace, grouped by kernel and launch size "
              "(under the tracer kernels of different streams are serialised).", "",
              f"{'kernel [grid]':76s} {'calls':>6s} {'total_us':>12s} {'avg_us':>10s} {'%':>6s}"]
        for k, c, t, avg, pct in read_trace(a.trace):
            if is_ours(k):
                L.append(f"{k[:76]:76s} {c:6d} {t:12.1f} {avg:10.2f} {pct:6.2f}")
        L.append("")
    if a.bench:
        b = json.loads(open(a.bench).read().strip().splitlines()[-1])
        r = b["roofline"]
        L += [f"bench.py (same build, not under the tracer): {b['value']} {b['unit']}, {b['ms_per_step']} ms per step "
              f"(median of {b.get('repetitions', 1)} repetitions).",
              f"bench.py roofline entry: {r.get('kernel')}: {r['achieved']} {r['unit']} = {r['frac']} of {r['peak']}, "
              f"HIP-event duration {r.get('avg_launch_us')} us per launch.", ""]
    traffic_entry = None
    if a.fetch and a.write:
        fetch, write = read_counter(a.fetch), read_counter(a.write)
        fb, wb = calibrate(fetch, "FETCH_SIZE"), calibrate(write, "WRITE_SIZE")
        L += ["HBM traffic counters (two more runs, one counter each; cwd /tmp, TMPDIR=/tmp):",
              f"  rocprofv3 --pmc FETCH_SIZE --output-format csv -d {a.fetch} -o pmc -- python3 bench.py {cmd} --calibrate-copy",
              f"  rocprofv3 --pmc WRITE_SIZE --output-format csv -d {a.write} -o pmc -- python3 bench.py {cmd} --calibrate-copy",
              f"Calibration on the plain 1 GiB device copy of the same runs: {fb / 1024:.0f} KiB per FETCH_SIZE count, "
              f"{wb / 1024:.0f} KiB per WRITE_SIZE count.",
              f"{'kernel [grid]':64s} {'n':>4s} {'FETCH avg':>14s} {'WRITE avg':>14s} {'read MB':>10s} {'written MB':>10s}"]
        kernels = {}
        for k, f in fetch.items():
            if not is_ours(k):
                continue
            wv = write.get(k, [0.0])
            fa, wa = sum(f) / len(f), sum(wv) / len(wv)
            kernels[k] = {"read_bytes": fa * fb, "written_bytes": wa * wb, "dispatches": len(f)}
            L.append(f"{k[:64]:64s} {len(f):4d} {fa:14.1f} {wa:14.1f} {fa * fb / 1e6:10.1f} {wa * wb / 1e6:10.1f}")
        L.append("")
        traffic_entry = {"sources_hash": sources_hash(), "bench_args": cmd,
                         "bytes_per_count": {"FETCH_SIZE": fb, "WRITE_SIZE": wb}, "kernels": kernels}
    if a.mfma:
        util = read_counter(a.mfma)
        L += ["Matrix-core utilisation counter (one more run):",
              f"  rocprofv3 --pmc MfmaUtil --output-format csv -d {a.mfma} -o pmc -- python3 bench.py {cmd}",
              "MfmaUtil = sum(SQ_VALU_MFMA_BUSY_CYCLES) / (max(GRBM_GUI_ACTIVE) * number of SIMDs) * 100, per dispatch; "
              "kernels that use the matrix cores:",
              f"{'kernel [grid]':76s} {'n':>4s} {'MfmaUtil avg %':>15s} {'max %':>8s}"]
        for k, v in util.items():
            if is_ours(k) and max(v) > 0.25:
                L.append(f"{k[:76]:76s} {len(v):4d} {sum(v) / len(v):15.1f} {max(v):8.1f}")
        L.append("")
    os.makedirs(PROFILES, exist_ok=True)
    name = a.out or ("fullgraph_layer_kernels.txt" if w == "fullgraph" else
                     f"stage_{w}_at_scale.txt" if w in ("sampling", "gather") else f"train_step_{w}_kernels.txt")
    open(os.path.join(PROFILES, name), "w").write("\n".join(L))
    print("\n".join(L))
    if traffic_entry is not None:
        table = json.load(open(TRAFFIC)) if os.path.exists(TRAFFIC) else {}
        traffic_entry["summary"] = "profiles/" + name
        table[w] = traffic_entry
        json.dump(table, open(TRAFFIC, "w"), indent=1, sort_keys=True)
        print(f"wrote {TRAFFIC} entry '{w}' ({len(traffic_entry['kernels'])} kernels)")


def measured_traffic(workload: str, kernel_substr: str, grid_threads=None):
    """Read + written HBM bytes per launch of the kernel whose key contains `kernel_substr` (and, if
    given, was launched with `grid_threads` threads), from profiles/traffic.json -- or None when the
    file has no such entry or was measured with other kernel sources than the ones in the tree."""
    if not os.path.exists(TRAFFIC):
        return None
    e = json.load(open(TRAFFIC)).get(workload)
    if not e or e.get("sources_hash") != sources_hash():
        return None
    hits = [(k, v) for k, v in e["kernels"].items() if kernel_substr in k and
            (grid_threads is None or k.endswith(f"[{grid_threads} threads]"))]
    if not hits:
        return None
    k, v = max(hits, key=lambda kv: kv[1]["read_bytes"] + kv[1]["written_bytes"])
    return {"bytes": v["read_bytes"] + v["written_bytes"], "read": v["read_bytes"], "written": v["written_bytes"],
            "kernel": k, "from": e.get("summary"), "sources_hash": e["sources_hash"]}


if __name__ == "__main__":
    main(sys.argv[1:])
