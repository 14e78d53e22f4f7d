"""Turns rocprofv3 output of `bench.py` into the short summaries kept under profiles/.

Usage (after the three rocprofv3 runs named below wrote their CSVs under <dir>/kt, <dir>/fetch and <dir>/write):

    python -m paper_2512_09277_amd.rocprof_summary --dir out/prof --routing metro --rank 2 \\
        --workload deepseek_v3_decode --bench-args "--only-metro --no-cpu-baseline --no-hip-graph --rank 2 --steps 20 --warmup 5 --calibration-copy"

writes profiles/hot_path_<workload>_<routing>_rocprofv3.md (kernel-trace statistics and HBM-side bytes per
dispatch) and profiles/ffn_traffic_<workload>.json (the two FFN kernels' bytes per launch, with the rank, the
routing and a hash of the kernel sources they were measured on; bench.py prints them as `roofline.traffic`
only while all three still match its own run).

If <dir>/l2 exists (a fourth run, `--pmc TCC_REQ_sum TCC_HIT_sum TCC_MISS_sum TCC_EA0_RDREQ_sum`), the summary also
lists the L2's requests, hits and misses per launch of the FFN kernels and the rate at which the misses (128 B
each) were served over the kernel-trace duration.

Byte counters are scaled by what the same counter reads for bench.py's `--calibration-copy` (one plain
1 GiB device-to-device copy): FETCH_SIZE and WRITE_SIZE are in KiB per dispatch.
"""
from __future__ import annotations

import argparse
import csv
import glob
import hashlib
import json
import os
import statistics

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GIB_KIB = 1048576.0


def short(name: str) -> str:
    name = name.replace("metro::(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0]


def find(dirname: str, pattern: str) -> str:
    hits = glob.glob(os.path.join(dirname, "**", pattern), recursive=True)
    if not hits:
        raise SystemExit(f"no {pattern} under {dirname}")
    return hits[0]


def counter_rows(path: str, counter: str):
    rows = [r for r in csv.DictReader(open(path)) if r["Counter_Name"] == counter]
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def calibration(fetch_rows, write_rows):
    """Counter readings of the 1 GiB calibration copy.  It is the plain copy (copyBuffer) before this library's
    first kernel whose WRITE_SIZE is 1 GiB to within 1 % (that counter reads a plain copy exactly); the same
    dispatch id in the FETCH_SIZE run (the same program, so the same dispatch sequence) gives the fetch reading."""
    hit = None
    for r in write_rows:
        if "metro::" in r["Kernel_Name"]:
            break
        if "copyBuffer" in r["Kernel_Name"] and abs(float(r["Counter_Value"]) - GIB_KIB) < 0.01 * GIB_KIB:
            hit = r
    if hit is None:
        raise SystemExit("no calibration copy found: run bench.py with --calibration-copy")
    same = [r for r in fetch_rows if r["Dispatch_Id"] == hit["Dispatch_Id"] and "copyBuffer" in r["Kernel_Name"]]
    if not same:
        raise SystemExit("the FETCH_SIZE run has no plain copy at the calibration copy's dispatch id")
    return float(same[0]["Counter_Value"]), float(hit["Counter_Value"])


def per_kernel(rows):
    d = {}
    for r in rows:
        if "metro::" in r["Kernel_Name"]:
            d.setdefault(short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    return d


L2_COUNTERS = ("TCC_REQ_sum", "TCC_HIT_sum", "TCC_MISS_sum", "TCC_EA0_RDREQ_sum")


def l2_table(path: str, stats, cmd):
    """L2 (TCC) requests per launch of the FFN kernels, summed over the 8 XCDs' L2s.  A request is one 128-byte
    line; a miss becomes one read request to the fabric (TCC_EA0_RDREQ), so misses x 128 B should equal the scaled
    FETCH_SIZE above, and misses x 128 B / duration is the rate at which the fabric filled the L2s."""
    avg_ns = {short(r["Name"]): float(r["AverageNs"]) for r in stats}
    vals = {c: per_kernel(counter_rows(path, c)) for c in L2_COUNTERS}
    lines = ["", "L2 requests per dispatch (128-byte lines, all XCDs), from a fourth run:", "",
             "    " + cmd("--pmc " + " ".join(L2_COUNTERS), "l2"), "",
             "| kernel | requests | hits | misses | fabric read requests | miss bytes | miss bytes / avg duration |",
             "|---|---|---|---|---|---|---|"]
    for k in vals["TCC_REQ_sum"]:
        if not k.startswith("ffn_mfma_kernel"):
            continue
        req, hit, miss, ea = (statistics.mean(vals[c][k]) for c in L2_COUNTERS)
        lines.append(f"| {k} | {req:.4g} | {hit:.4g} | {miss:.4g} | {ea:.4g} | {miss * 128:.4g} | "
                     f"{miss * 128 / avg_ns[k]:.0f} GB/s |")
    return lines


def source_sha16() -> str:
    h = hashlib.sha256()
    for name in ("ffn.hip", "device_utils.h", "host_utils.h"):
        with open(os.path.join(ROOT, "paper_2512_09277_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--dir", required=True)
    ap.add_argument("--routing", required=True, choices=["metro", "token_balanced"])
    ap.add_argument("--rank", type=int, required=True)
    ap.add_argument("--workload", default="deepseek_v3_decode")
    ap.add_argument("--bench-args", required=True, help="the arguments bench.py was run with under rocprofv3")
    ap.add_argument("--no-json", action="store_true", help="do not write profiles/ffn_traffic_<workload>.json")
    args = ap.parse_args()

    stats = [r for r in csv.DictReader(open(find(os.path.join(args.dir, "kt"), "*kernel_stats.csv"))) if "metro::" in r["Name"]]
    fetch = counter_rows(find(os.path.join(args.dir, "fetch"), "*counter_collection.csv"), "FETCH_SIZE")
    write = counter_rows(find(os.path.join(args.dir, "write"), "*counter_collection.csv"), "WRITE_SIZE")
    cf, cw = calibration(fetch, write)
    ff, wf = GIB_KIB / cf, GIB_KIB / cw
    f, w = per_kernel(fetch), per_kernel(write)

    cmd = lambda opts, sub: (f"rocprofv3 {opts} --output-format csv -d {args.dir}/{sub} -o {sub} -- python3 bench.py "
                             f"{args.bench_args}")
    lines = [f"# rocprofv3 summary: hot path of {args.workload}, {args.routing} routing, rank {args.rank}", "",
             f"Kernel source hash (ffn.hip, device_utils.h, host_utils.h): `{source_sha16()}`.",
             "Commands (run from /tmp with TMPDIR=/tmp on the MI355X box, one rocprofv3 run each):", "",
             "    " + cmd("--kernel-trace --stats", "kt"), "    " + cmd("--pmc FETCH_SIZE", "fetch"),
             "    " + cmd("--pmc WRITE_SIZE", "write"),
             f"    python -m paper_2512_09277_amd.rocprof_summary --dir {args.dir} --routing {args.routing} --rank {args.rank} "
             f"--workload {args.workload} --bench-args \"...\"", "",
             "Kernel trace (every launch of a hot-path kernel in that run is on the same rank and routing, so the",
             "average is the per-launch duration" + ("; the gate kernels come from bench.py's separate gate timing loop"
                                                     if any("gate_" in r["Name"] and "gate_up" not in r["Name"] for r in stats)
                                                     else "") + "):", "",
             "| kernel | calls | avg ns | min ns | max ns | stddev |", "|---|---|---|---|---|---|"]
    for r in stats:
        lines.append(f"| {short(r['Name'])} | {r['Calls']} | {float(r['AverageNs']):.0f} | {r['MinNs']} | {r['MaxNs']} | "
                     f"{float(r['StdDev']):.0f} |")
    lines += ["", "HBM-side bytes per dispatch.  Calibration: the plain 1 GiB copy reads FETCH_SIZE "
              f"{cf:.1f} KiB and WRITE_SIZE {cw:.1f} KiB", f"for 1048576 KiB read and written: scale factors {ff:.3f} (fetch) and "
              f"{wf:.3f} (write).", "",
              "| kernel | dispatches | FETCH_SIZE KiB (raw avg) | WRITE_SIZE KiB (raw avg) | scaled fetch bytes | scaled write bytes |",
              "|---|---|---|---|---|---|"]
    out = {}
    for k in f:
        fa, wa = statistics.mean(f[k]), statistics.mean(w.get(k, [0.0]))
        fb, wb = fa * 1024 * ff, wa * 1024 * wf
        lines.append(f"| {k} | {len(f[k])} | {fa:.1f} | {wa:.1f} | {fb:.4g} | {wb:.4g} |")
        out[k] = dict(fetch_bytes=round(fb), write_bytes=round(wb))
    l2_dir = os.path.join(args.dir, "l2")
    if os.path.isdir(l2_dir):
        lines += l2_table(find(l2_dir, "*counter_collection.csv"), stats, cmd)
    text = "\n".join(lines) + "\n"
    md = os.path.join(ROOT, "profiles", f"hot_path_{args.workload}_{args.routing}_rocprofv3.md")
    open(md, "w").write(text)
    print(text)
    if not args.no_json:
        rec = dict(workload=args.workload, routing=args.routing, rank=args.rank, ffn_source_sha16=source_sha16(),
                   fetch_scale=round(ff, 4), write_scale=round(wf, 4), gate_up=out["ffn_mfma_kernel<true>"],
                   down=out["ffn_mfma_kernel<false>"], per_kernel=out,
                   summary=os.path.relpath(md, ROOT))
        with open(os.path.join(ROOT, "profiles", f"ffn_traffic_{args.workload}.json"), "w") as fh:
            json.dump(rec, fh, indent=1)
            fh.write("\n")


if __name__ == "__main__":
    main()
