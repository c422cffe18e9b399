"""The script that turns rocprofv3's CSV output into profiles/*.md and profiles/hbm_traffic.txt, on synthetic
CSVs with known answers: `roofline.traffic` in the benchmark line is whatever this arithmetic says, so the
counter scaling (what FETCH_SIZE / WRITE_SIZE read for a plain 64 MiB copy), the per-kernel averages and the
naming of the traffic rows are pinned here.  No GPU, no profiler."""
import csv
import json
import os

from paper_2511_04477_amd import profile_summary


def write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w", newline="") as fh:
        w = csv.writer(fh)
        w.writerow(header)
        w.writerows(rows)


def test_summary_and_traffic_table_from_synthetic_csvs(tmp_path):
    D = str(tmp_path / "prof")
    LIST = "void (anonymous namespace)::spqt_gemv_list_kernel<4>(unsigned char const*, int)"
    DENSE = "void (anonymous namespace)::spqt_gemv_kernel<4, true, 1, 0>(unsigned char const*, int)"
    COPY = "(anonymous namespace)::copy_kernel(unsigned int*, unsigned int const*, unsigned long)"
    GATHER = "void (anonymous namespace)::spqt_gather_kernel<1, false>(unsigned short const*)"
    kept, dense = 60_000_000, 120_000_000
    os.makedirs(D)
    with open(os.path.join(D, "kt.log"), "w") as fh:
        fh.write("noise\n" + json.dumps({"pmc_pass": True, "workload": "gate70b", "M": 28672, "K": 8192, "copy_bytes": 64 << 20,
                                          "launches_per_kernel": 8, "kept_bytes_per_launch": kept,
                                          "dense_bytes_per_launch": dense, "y_bytes_per_launch": 4 * 28672}) + "\n")
    write_csv(os.path.join(D, "kt", "kt_kernel_stats.csv"), ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
              [[LIST, 8, 160000, 20000.0, 40, 19000, 21000, 1], [DENSE, 8, 240000, 30000.0, 50, 29000, 31000, 1],
               [COPY, 8, 160000, 20000.0, 5, 19000, 21000, 1], [GATHER, 16, 48000, 3000.0, 5, 2900, 3100, 1],
               ["void at::native::copy_kernel<float>(float*)", 3, 3, 1.0, 0, 1, 1, 0]])
    cc = ["Correlation_Id", "Dispatch_Id", "Agent_Id", "Kernel_Name", "Counter_Name", "Counter_Value"]
    # FETCH_SIZE reads half the true KiB on the copy (32768 for 64 MiB): factor 2; two launches of the list kernel average to 29000 KiB
    write_csv(os.path.join(D, "fetch", "pmc_counter_collection.csv"), cc,
              [[1, 1, 0, COPY, "FETCH_SIZE", 32768], [2, 2, 0, LIST, "FETCH_SIZE", 28000], [3, 3, 0, LIST, "FETCH_SIZE", 30000],
               [4, 4, 0, DENSE, "FETCH_SIZE", 58000], [5, 5, 0, GATHER, "FETCH_SIZE", 8]])
    write_csv(os.path.join(D, "write", "pmc_counter_collection.csv"), cc,
              [[1, 1, 0, COPY, "WRITE_SIZE", 65536], [2, 2, 0, LIST, "WRITE_SIZE", 500], [3, 3, 0, DENSE, "WRITE_SIZE", 600],
               [4, 4, 0, GATHER, "WRITE_SIZE", 16]])
    sq_names = ["SQ_INSTS_VALU", "SQ_INSTS_SALU", "SQ_INSTS_LDS", "SQ_INSTS_VMEM_RD", "SQ_WAVES", "SQ_BUSY_CYCLES", "SQ_WAVE_CYCLES", "SQ_WAIT_INST_ANY"]
    rows = []
    for kern, valu in ((LIST, 3_000_000), (DENSE, 6_000_000), (COPY, 10)):
        for n in sq_names:
            rows.append([1, 1, 0, kern, n, valu if n == "SQ_INSTS_VALU" else 896])
    write_csv(os.path.join(D, "sq", "pmc_counter_collection.csv"), cc, rows)

    out = str(tmp_path / "summary.md")
    traffic = str(tmp_path / "traffic.txt")
    with open(traffic, "w") as fh:
        fh.write("# old header\nspqt_gemv_list_kernel 28672 8192 0.5 1 stale.md\nspqt_gemv_list_kernel 4096 4096 0.5 777 other.md\n")
    assert profile_summary.main(["--dir", D, "--workload", "gate70b", "--out", out, "--traffic", traffic]) == 0

    md = open(out).read()
    assert "| spqt_gemv_list_kernel<4> | 8 | 20000 | 19000 | 21000 | 3000 |" in md          # 60e6 B / 20000 ns = 3000 GB/s
    assert "| spqt_gemv_kernel<4, true, 1, 0> | 8 | 30000 | 29000 | 31000 | 4000 |" in md   # dense bytes
    assert "at::native" not in md
    assert "x2.000 to true bytes" in md and "(x1.000)" in md
    table = {}
    for line in open(traffic):
        if not line.startswith("#"):
            f = line.split()
            table[(f[0], int(f[1]), int(f[2]))] = int(f[4])
    # list kernel: 29000 KiB x 2 read + 500 KiB written; the stale row of the same shape is replaced, the other shape's kept
    assert table[("spqt_gemv_list_kernel", 28672, 8192)] == (29000 * 2 + 500) * 1024
    assert table[("spqt_gemv_kernel_dense", 28672, 8192)] == (58000 * 2 + 600) * 1024
    assert table[("spqt_gemv_list_kernel", 4096, 4096)] == 777
    # VALU lane-ops per weight: 3e6 wave-instructions x 64 / (kept bytes / 0.515625 bytes per weight)
    assert f"{3_000_000 * 64 / (kept / 0.515625):.2f}" in md
