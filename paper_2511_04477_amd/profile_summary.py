"""Turn the CSV output of a few rocprofv3 runs of bench.py into a short Markdown summary under profiles/
and refresh profiles/hbm_traffic.txt (the table bench.py reads `roofline.traffic` from).

The runs (on the MI355X machine, from /tmp with TMPDIR=/tmp; W = gate70b, q4096, gate70b_colblock, gate70b_w8, gate70b_w2):

    rocprofv3 --kernel-trace --stats --output-format csv -d D/trace -o kt -- python3 bench.py --trace-pass  > D/trace.log
    rocprofv3 --kernel-trace --stats --output-format csv -d D/kt    -o kt -- python3 bench.py --pmc-pass --pmc-workload W > D/kt.log
    rocprofv3 --pmc FETCH_SIZE  --output-format csv -d D/fetch -o pmc -- python3 bench.py --pmc-pass --pmc-workload W
    rocprofv3 --pmc WRITE_SIZE  --output-format csv -d D/write -o pmc -- python3 bench.py --pmc-pass --pmc-workload W
    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY
              --output-format csv -d D/sq -o pmc -- python3 bench.py --pmc-pass --pmc-workload W

then

    python3 -m paper_2511_04477_amd.profile_summary --dir D --workload W --out profiles/NAME.md

The trace run (only for gate70b, the benchmark's headline workload) replays the very graphs the benchmark
times, so its per-kernel average is the launch duration under the timed conditions; the --pmc-pass runs
launch every kernel once per weight copy with plain stream launches.  FETCH_SIZE and WRITE_SIZE are
scaled by what the same counter reads for a plain 64 MiB copy kernel in the same run.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TRAFFIC = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
LAYOUT = {"gate70b": ("group-layout", "spqt_gemv_", 0.515625), "q4096": ("group-layout", "spqt_gemv_", 0.515625),
          "gate70b_colblock": ("column-block", "spqt_cb_gemv_kernel", 0.5625),
          "gate70b_w8": ("8-bit column-block", "spqt_cb8_gemv_kernel", 1.0625),
          "gate70b_w2": ("2-bit column-block", "spqt_cb2_gemv_kernel", 0.3125)}


def short(name: str) -> str:
    return name.replace("void (anonymous namespace)::", "").replace("(anonymous namespace)::", "").split("(")[0]


def find(d: str, suffix: str) -> str:
    hits = glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True)
    if not hits:
        raise FileNotFoundError(f"no *{suffix} under {d}")
    return hits[0]


def info_line(path: str, key: str) -> dict:
    for line in open(path):
        if line.startswith('{"' + key + '"'):
            return json.loads(line)
    raise ValueError(f"{path}: no {key} line")


def stats(d: str, want) -> list:
    rows = []
    for r in csv.DictReader(open(find(d, "kernel_stats.csv"))):
        if want(r["Name"]):
            rows.append((short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]), int(float(r["MinNs"])), int(float(r["MaxNs"]))))
    return rows


def counters(d: str, kname: str) -> dict:
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(find(d, "counter_collection.csv"))):
        k = r["Kernel_Name"]
        if kname in k or "spqt_gather" in k:
            key = short(k)
        elif "copy_kernel" in k and "anonymous" in k and "at::" not in k:
            key = "copy_kernel"
        else:
            continue
        acc[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: sum(v) / len(v) for c, v in d2.items()} for k, d2 in acc.items()}


def is_dense(kernel: str) -> bool:
    return "<4, true" in kernel


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.splitlines()[0])
    ap.add_argument("--dir", required=True, help="folder holding trace/ kt/ fetch/ write/ sq/ and the logs")
    ap.add_argument("--workload", required=True, choices=sorted(LAYOUT))
    ap.add_argument("--out", required=True)
    ap.add_argument("--traffic", default=TRAFFIC, help="the traffic table to refresh (default: profiles/hbm_traffic.txt)")
    args = ap.parse_args(argv)
    D, W = args.dir, args.workload
    lay, kname, bytes_per_weight = LAYOUT[W]
    info = info_line(os.path.join(D, "kt.log"), "pmc_pass")
    M, K = info["M"], info["K"]
    L = [f"# rocprofv3 summary: {lay} GEMV kernels on {M} x {K}, 50 % activation sparsity", "",
         f"Workload: {M} x {K} {'int8' if 'w8' in W else ('2-bit' if 'w2' in W else 'int4')}, x ~ Laplace(0,1) fp16, threshold = 50 % quantile, batch 1; "
         f"{info['launches_per_kernel']} rotated weight copies. Kept bytes per sparse launch: {info['kept_bytes_per_launch']:,.0f}; "
         f"dense bytes: {info['dense_bytes_per_launch']:,.0f}.", "",
         "All commands run on the MI355X box from /tmp with TMPDIR=/tmp; summarized by",
         f"`python3 -m paper_2511_04477_amd.profile_summary --dir D --workload {W} --out {os.path.relpath(args.out, ROOT)}`.", ""]

    trace_log = os.path.join(D, "trace.log")
    if os.path.exists(trace_log):
        tinfo = info_line(trace_log, "trace_pass")
        L += ["## Kernel durations under the benchmark's own graph replay", "",
              "    rocprofv3 --kernel-trace --stats --output-format csv -d D/trace -o kt -- python3 bench.py --trace-pass", "",
              "The program replays the four graphs of the headline workload exactly as bench.py times them (back-to-back launches "
              "from a HIP graph, rotated copies); HIP events of the same run, per launch: "
              + ", ".join(f"{k} {v} us" for k, v in tinfo["events_us"].items()) + ".", "",
              "| kernel | calls | average ns | min ns | max ns | GB/s on its algorithmic bytes | fraction of 8 TB/s |", "|---|---|---|---|---|---|---|"]
        for name, calls, avg, mn, mx in stats(os.path.join(D, "trace"), lambda n: "spqt_" in n):
            if "gather" in name:
                L.append(f"| {name} | {calls} | {avg:.0f} | {mn} | {mx} | - | - |")
                continue
            b = tinfo["dense_bytes_per_launch"] if is_dense(name) else tinfo["kept_bytes_per_launch"]
            L.append(f"| {name} | {calls} | {avg:.0f} | {mn} | {mx} | {b / avg:.0f} | {b / avg / 8000:.3f} |")
        L.append("")

    L += ["## Kernel durations, isolated stream launches", "",
          f"    rocprofv3 --kernel-trace --stats --output-format csv -d D/kt -o kt -- python3 bench.py --pmc-pass --pmc-workload {W}", "",
          "Every kernel launched once per weight copy with plain stream launches: the profiler brackets every dispatch and the GPU "
          "idles between them, so these read higher than back-to-back launches from a HIP graph do.", "",
          "| kernel | calls | average ns | min ns | max ns | GB/s on its algorithmic bytes |", "|---|---|---|---|---|---|"]
    for name, calls, avg, mn, mx in stats(os.path.join(D, "kt"), lambda n: kname in n or "spqt_gather" in n or ("copy_kernel" in n and "anonymous" in n and "at::" not in n)):
        if "copy_kernel" in name:
            gb = f"{2 * info['copy_bytes'] / avg:.0f} (read + write)"
        elif "gather" in name:
            gb = "-"
        else:
            gb = f"{(info['dense_bytes_per_launch'] if is_dense(name) else info['kept_bytes_per_launch']) / avg:.0f}"
        L.append(f"| {name} | {calls} | {avg:.0f} | {mn} | {mx} | {gb} |")
    if lay == "group-layout":
        L += ["", "spqt_gemv_list_kernel<4>: list-driven sparse kernel with row-aligned passes (spqt_gemv with an index list, one activation row).",
              "spqt_gemv_kernel<wavefronts per workgroup, DENSE, BATCH, FUSED>: <4, true, 1, 0> dense, <4, false, 1, 1> one launch with static",
              "column ranges (spqt_gemv_fused), <4, false, 1, 0> list-driven with one-group passes (SPQT_CFG_GROUP_PASSES, an ablation).",
              "spqt_gemv_bal_kernel<4>: one launch with even shares of the kept columns (SPQT_CFG_EVEN_SHARES)."]

    f, w, sq = (counters(os.path.join(D, x), kname) for x in ("fetch", "write", "sq"))
    fs, ws = 65536.0 / f["copy_kernel"]["FETCH_SIZE"], 65536.0 / w["copy_kernel"]["WRITE_SIZE"]
    L += ["", "## Hardware counters (one run per counter set, same program)", "",
          f"    rocprofv3 --pmc FETCH_SIZE --output-format csv -d D/fetch -o pmc -- python3 bench.py --pmc-pass --pmc-workload {W}",
          "    rocprofv3 --pmc WRITE_SIZE ...",
          "    rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_WAVES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY ...", "",
          f"Counter scaling from the 64 MiB copy kernel: FETCH_SIZE reads {f['copy_kernel']['FETCH_SIZE']:.0f} KiB (x{fs:.3f} to true bytes), "
          f"WRITE_SIZE {w['copy_kernel']['WRITE_SIZE']:.0f} KiB (x{ws:.3f}).", "",
          "| kernel | HBM read bytes | HBM written bytes | read+write / algorithmic | VALU wave-instr | VALU lane-ops per weight | SALU | LDS | VMEM reads | waves |",
          "|---|---|---|---|---|---|---|---|---|---|"]
    traffic_rows = {}
    for k in sorted(sq):
        if kname not in k:
            continue
        b = info["dense_bytes_per_launch"] if is_dense(k) else info["kept_bytes_per_launch"]
        weights = b / bytes_per_weight
        rd, wr = f[k]["FETCH_SIZE"] * fs * 1024, w[k]["WRITE_SIZE"] * ws * 1024
        q = sq[k]
        L.append(f"| {k} | {rd:,.0f} | {wr:,.0f} | {(rd + wr) / b:.3f} | {q['SQ_INSTS_VALU']:,.0f} | {q['SQ_INSTS_VALU'] * 64 / weights:.2f} | "
                 f"{q['SQ_INSTS_SALU']:,.0f} | {q['SQ_INSTS_LDS']:,.0f} | {q['SQ_INSTS_VMEM_RD']:,.0f} | {q['SQ_WAVES']:,.0f} |")
        traffic_rows[k.split("<")[0] + ("_dense" if is_dense(k) else "") + ("_one_launch" if "false, 1, 1>" in k else "")
                     + ("_group_passes" if "false, 1, 0>" in k else "")] = int(rd + wr)
    L += ["", "VALU lane-ops per weight = VALU wave-instructions (matrix-core instructions included) x 64 / weights multiplied. "
          "The chip issues 39.3 T lane-ops/s (256 CUs x 4 SIMD x 16 lanes x 2.4 GHz)."]
    with open(args.out, "w") as fh:
        fh.write("\n".join(L) + "\n")
    print("\n".join(L))

    # refresh the traffic table: one line per (kernel, M, K, sparsity)
    keep = []
    if os.path.exists(args.traffic):
        for line in open(args.traffic):
            fl = line.split()
            if line.startswith("#") or len(fl) < 5:
                continue
            if (fl[0] in traffic_rows) and (int(fl[1]), int(fl[2])) == (M, K):
                continue
            keep.append(line.rstrip("\n"))
    for kern, nbytes in sorted(traffic_rows.items()):
        keep.append(f"{kern} {M} {K} 0.5 {nbytes} {os.path.relpath(args.out, ROOT)}")
    with open(args.traffic, "w") as fh:
        fh.write("# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size), written by\n"
                 "# python3 -m paper_2511_04477_amd.profile_summary; columns: kernel M K sparsity bytes source\n")
        fh.write("\n".join(sorted(keep)) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
