#!/usr/bin/env python3
"""Benchmark of the SpQt hot path on one MI355X.

A step is one pass of the whole hot path over one activation vector: spqt_gather (threshold + index
compaction) followed by the load-balanced sparse int4 GEMV, batch 1.  The headline workload is the
largest single-GPU configuration: the 70B-shaped MLP gate projection (28672 x 8192, group 128) at 50 %
activation sparsity.  Weight buffers rotate over independently seeded copies whose total size is
several times the 256 MB Infinity Cache, so no launch re-reads cached weights.

Prints ONE JSON line (the fields are built in main() below): the headline step, the GEMV-only kernel
time with its roofline fraction, the dense kernel, the one-launch kernels, a sweep over the other
configurations' shapes and sparsities, the decoder-layer sequences of configurations 3 and 4, what
trivial kernels reach on this machine, and the CPU oracle timed on the same workload.  `--full` adds the
side studies of bench_studies.py.  `--gpus` above 1 is refused: this build is a one-GPU kernel path.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

from bench_support import (HBM_PEAK_GBPS, ROOT, Workload, calibrate, kept_bytes, layer_sequence, time_sequence)

HEADLINE = dict(config=5, tensor="gate", M=28672, K=8192, dist="laplace", sparsity=0.5)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def measured_traffic(kernel, M, K, sparsity):
    """HBM bytes per launch of `kernel` on this workload as the hardware counters saw them, from the table
    the profile summarizer keeps under profiles/ (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE, each scaled
    by what the same counter reads for a plain copy of known size); None when the table has no such row."""
    try:
        for line in open(TRAFFIC_FILE):
            f = line.split()
            if len(f) >= 5 and not line.startswith("#") and f[0] == kernel and (int(f[1]), int(f[2])) == (M, K) \
                    and abs(float(f[3]) - sparsity) < 1e-9:
                return int(float(f[4]))
    except OSError:
        pass
    return None


class CpuBaseline:
    """The cpu_baseline leg: the ONLY code in this file that touches oracle/.  It times the oracle
    as it stands on the host cores, and it hands out the oracle's results for the workloads being
    timed, so that a GPU number is only reported for outputs that match the oracle.  With --no-cpu
    the leg is off: nothing under oracle/ is imported and the GPU results go unchecked here (the
    test suite covers parity)."""

    def __init__(self, enabled):
        self.enabled = enabled

    def gather(self, x_np, thr):
        import oracle
        return oracle.gather(x_np, thr)

    def gemv(self, case, x_np, thr):
        import oracle
        return oracle.gemv(case["q_rowmajor"], case["scales"], x_np, thr)[0]

    def gemv_rows(self, case, x_np, thr, rows):
        import oracle
        return oracle.gemv_rows(case["q_rowmajor"], case["scales"], x_np, thr, rows)[0]

    def colblock(self, W_rows, x_np, thr):
        """Column-block reference on a subset of whole 256-row tiles of fp32 weights."""
        from oracle import colblock as cb
        q, s = cb.quantize(W_rows)
        return cb.gemv(q, s, x_np, thr)[0]

    def colblock_w8(self, W_rows, x_np, thr):
        """8-bit column-block reference on a subset of whole 128-row block-rows of fp32 weights."""
        from oracle import colblock_w8 as c8
        q, s = c8.quantize(W_rows)
        return c8.gemv(q, s, x_np, thr)[0]

    def colblock_w2(self, W_rows, x_np, thr):
        """2-bit column-block reference on a subset of whole 512-row block-rows of fp32 weights."""
        from oracle import colblock_w2 as c2
        c, s = c2.quantize(W_rows)
        return c2.gemv(c, s, x_np, thr)[0]

    def colblock_k(self, W_rows, x_np, thr):
        """K-quant column-block reference on a subset of whole 256-row tiles of fp32 weights."""
        from oracle import colblock_k as ck
        return ck.gemv(ck.quantize(W_rows), x_np, thr)[0]

    def quantization_error(self):
        """Bytes against accuracy of the weight formats on the same synthetic fp32 matrices (2048 x 4096;
        x ~ Laplace(0,1), dense product): relative RMS error of the dequantized weights and of y = W x
        against the unquantized fp64 product.  Two matrices: plain N(0, 0.02^2), and the workload
        module's matrix in which every 64th COLUMN is 8 times larger (an input channel with outlier
        weights: blocks along a column keep it to itself, groups along a row all contain one).  The
        group layout carries whatever the model's quantizer produced (it is a repack); here its source
        is made with the plain symmetric rule s = max|w| / 7 over G consecutive weights of a ROW, the
        counterpart of the column-block rule.  Host only (NumPy and the oracles); says nothing about
        trained weights."""
        import numpy as np
        from oracle import colblock as cb, colblock_k as ck, colblock_w8 as c8, colblock_w2 as c2
        from workloads import make_fp_weights, make_x
        M, K = 2048, 4096
        x = make_x(K, "laplace", 424243)[0].astype(np.float64)

        def rel(a, b):
            return float(np.sqrt(np.mean((a - b) ** 2) / np.mean(b ** 2)))

        def row_groups(Wf, G):      # symmetric int4 along K, fp16 scale per (row, G columns)
            w = Wf.reshape(M, K // G, G)
            s = (np.max(np.abs(w), axis=2) / np.float32(7.0)).astype(np.float16).astype(np.float32)
            with np.errstate(divide="ignore", invalid="ignore"):
                q = np.where(s[:, :, None] > 0, np.clip(np.rint(w / s[:, :, None]), -8, 7), 0)
            return (q * s[:, :, None]).reshape(M, K).astype(np.float64)

        rows = []
        plain = (np.random.default_rng(424244).standard_normal((M, K)) * 0.02).astype(np.float32)
        for label, Wf in (("gaussian", plain), ("gaussian, every 64th column x8", make_fp_weights(M, K, 424242))):
            W = Wf.astype(np.float64)
            y = W @ x
            q4, s4 = cb.quantize(Wf)
            q8, s8 = c8.quantize(Wf)
            q2, s2 = c2.quantize(Wf)
            forms = [("group layout, 128 along K", 4 + 16 / 128, row_groups(Wf, 128)),
                     ("group layout, 64 along K", 4 + 16 / 64, row_groups(Wf, 64)),
                     ("column blocks of 32 rows", 4 + 16 / 32, cb.dequant(q4, s4)),
                     ("column blocks, 6-bit scales and minima", 4.5, ck.dequant(ck.quantize(Wf))),
                     ("column blocks of 32 rows, 8-bit", 8 + 16 / 32, c8.dequant(q8, s8)),
                     ("column blocks of 32 rows, 2-bit", 2 + 16 / 32, c2.dequant(q2, s2))]
            rows += [{"weights": label, "format": name, "bits_per_weight": round(bits, 3),
                      "rel_rms_weight_error": round(rel(Wd, W), 5), "rel_rms_gemv_error": round(rel(Wd @ x, y), 5)}
                     for name, bits, Wd in forms]
        return rows

    @staticmethod
    def close(got, ref):
        import numpy as np
        err = np.abs(np.asarray(got, dtype=np.float64) - ref)
        return bool(np.all(err <= 1e-2 + 2e-3 * np.abs(ref))), float(err.max())

    def time_gemv(self, case, x_np, thr, threads, runs=5):
        """Median over `runs` oracle GEMVs (after one warm-up) on `threads` threads (0 = all the host's):
        (median us per GEMV, threads used)."""
        import oracle
        all_threads = oracle.threads()
        oracle.set_threads(threads or all_threads)
        used = oracle.threads()
        oracle.gemv(case["q_rowmajor"], case["scales"], x_np, thr)       # warm
        times = []
        for _ in range(runs):
            t0 = time.perf_counter()
            oracle.gemv(case["q_rowmajor"], case["scales"], x_np, thr)
            times.append(time.perf_counter() - t0)
        oracle.set_threads(all_threads)
        times.sort()
        return times[len(times) // 2] * 1e6, used


def sweep_row(torch, spqt, np, config, tensor, m, k, dist, s, batch, K_steps, use_graph, reuse=None):
    """One row of the sweep: GEMV only, dense, gather + GEMV and the one-launch kernel on one shape and sparsity."""
    from workloads import CONFIG_SCALE_RANGE
    w = reuse or Workload(torch, spqt, m, k, dist, CONFIG_SCALE_RANGE[config], config, tensor, s, batch=batch,
                          min_copies=8 if config == 5 else 2)
    steps = max(w.copies * 4, min(K_steps, 1600))
    t_g = time_sequence(torch, w.gemv_only, w.copies, steps, w.copies, use_graph)
    t_d = time_sequence(torch, w.dense_only, w.copies, steps, w.copies, use_graph)
    t_s = time_sequence(torch, w.step, w.copies, steps, w.copies, use_graph)
    t_f = time_sequence(torch, w.fused if batch == 1 else w.fused_rows, w.copies, steps, w.copies, use_graph)
    t_r = time_sequence(torch, w.step_own_sets, w.copies, steps, w.copies, use_graph) if batch > 1 else None
    t_fo = time_sequence(torch, w.fused_rows_own_sets, w.copies, steps, w.copies, use_graph) if batch > 1 else None
    gb = w.mean_kept_bytes / (t_g * 1e-6) / 1e9
    return {"config": config, "tensor": tensor, "M": m, "K": k, "batch": batch, "sparsity_per_row": s,
            "kept_frac": round(float(np.mean(w.n_ns)) / k, 4),
            "us_gemv": round(t_g, 3), "us_dense": round(t_d, 3), "us_gather_plus_gemv": round(t_s, 3),
            "us_fused": None if t_f is None else round(t_f, 3),
            "us_gather_rows_plus_gemv": None if t_r is None else round(t_r, 3),
            "us_fused_own_sets": None if t_fo is None else round(t_fo, 3),
            "GBps_kept": round(gb, 1), "frac_of_8TBps": round(gb / HBM_PEAK_GBPS, 4),
            "dense_GBps": round(w.dense_bytes / (t_d * 1e-6) / 1e9, 1),
            "speedup_vs_dense": round(t_d / t_g, 3), "fused_speedup_vs_dense": None if t_f is None else round(t_d / t_f, 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1600)
    ap.add_argument("--warmup", type=int, default=160)
    ap.add_argument("--eager", action="store_true", help="plain stream launches instead of HIP graph replay")
    ap.add_argument("--no-sweep", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--full", action="store_true", help="also the side studies (bench_studies.py)")
    ap.add_argument("--trace-pass", action="store_true",
                    help="for rocprofv3 --kernel-trace: only the headline workload's four graphs (GEMV only, dense, "
                         "gather + GEMV, one launch), replayed exactly as the benchmark times them; prints their "
                         "HIP-event times")
    ap.add_argument("--pmc-pass", action="store_true",
                    help="for hardware-counter runs: launch only a 64 MiB calibration copy (x8) and the kernels "
                         "of --pmc-workload once per weight copy, eagerly, and exit")
    ap.add_argument("--pmc-workload", choices=["gate70b", "q4096", "gate70b_colblock", "gate70b_w8", "gate70b_w2"], default="gate70b",
                    help="with --pmc-pass: 28672x8192 group layout (the headline), 4096x4096 group layout, "
                         "28672x8192 column-block layout, 28672x8192 8-bit column-block layout, all at 50 %%")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU kernel path; run with --gpus 1 "
              "(sharding across GPUs is not implemented)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2511_04477_amd as spqt
    from workloads import CONFIG_SCALE_RANGE

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    spqt.lib()
    use_graph = not args.eager
    K_steps, W = args.steps, args.warmup

    if args.pmc_pass:
        import bench_studies
        if args.pmc_workload == "q4096":
            bench_studies.pmc_pass_small(torch, spqt)
        else:
            bench_studies.pmc_pass_large(torch, spqt, args.pmc_workload)
        return

    # ---------------- headline: config 5 gate, 28672 x 8192, 50 % --------------------------
    H = HEADLINE
    M, K = H["M"], H["K"]
    wl = Workload(torch, spqt, M, K, H["dist"], CONFIG_SCALE_RANGE[H["config"]], H["config"], H["tensor"], H["sparsity"],
                  min_copies=8)
    cpu = CpuBaseline(enabled=not args.no_cpu and not args.trace_pass)
    ok, max_err = wl.check_copy0(cpu)
    if not ok:
        print(f"bench.py: parity check against the oracle FAILED (max err {max_err})", file=sys.stderr)
        sys.exit(1)
    if cpu.enabled:     # the one-launch kernels too
        ref = cpu.gemv(wl.case0, wl.x_np[0:1], wl.thr[0])
        for fn, want in ((wl.fused, ref), (wl.fused_even_shares, ref), (wl.dense_only, cpu.gemv(wl.case0, wl.x_np[0:1], 0.0))):
            wl.y[0].fill_(float("nan"))
            fn(0)
            torch.cuda.synchronize()
            if not cpu.close(wl.y[0].cpu().numpy(), want)[0]:
                print(f"bench.py: parity check of {fn.__name__} FAILED", file=sys.stderr)
                sys.exit(1)
    us_step = time_sequence(torch, wl.step, wl.copies, K_steps, W, use_graph, exact_warmup=True)
    side_steps = max(K_steps, 1600)
    us_gemv = time_sequence(torch, wl.gemv_only, wl.copies, side_steps, W, use_graph)
    us_dense = time_sequence(torch, wl.dense_only, wl.copies, side_steps, W, use_graph)
    us_fused = time_sequence(torch, wl.fused, wl.copies, side_steps, W, use_graph)
    if args.trace_pass:
        print(json.dumps({"trace_pass": True, "M": M, "K": K, "sparsity": H["sparsity"], "copies": wl.copies,
                          "kept_bytes_per_launch": wl.mean_kept_bytes, "dense_bytes_per_launch": wl.dense_bytes,
                          "events_us": {"gather_plus_gemv": round(us_step, 3), "spqt_gemv_list_kernel": round(us_gemv, 3),
                                        "dense": round(us_dense, 3), "one_launch_static_ranges": round(us_fused, 3)}}))
        return
    us_gather = time_sequence(torch, wl.gather_only, wl.copies, side_steps, W, use_graph)
    us_even = time_sequence(torch, wl.fused_even_shares, wl.copies, side_steps, W, use_graph)
    us_step_eager = time_sequence(torch, wl.step, wl.copies, min(K_steps, 800), min(W, 200), False) if args.full else None

    achieved = wl.mean_kept_bytes / (us_gemv * 1e-6) / 1e9
    out = {
        "metric": "us per GEMV (spqt_gather + sparse int4 GEMV), 50% activation sparsity, batch 1",
        "value": round(us_step, 3),
        "unit": "us/GEMV",
        "n_gpus": 1, "steps": K_steps, "warmup": W,
        "ms_per_step": round(us_step * 1e-3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int4 weights x fp16 activations, fp32 accumulate",
        "data": "synthetic",
        "config": {"workload": "configs[4] gate: 28672x8192 int4 group-128 (70B MLP gate/up), scales fp16 U(0.003,0.015), "
                               "x~Laplace(0,1) fp16, threshold=50% quantile, batch 1 (the largest single-GPU configuration)",
                   "M": M, "K": K, "sparsity": H["sparsity"], "copies_rotated": wl.copies,
                   "rotated_MB": round(wl.copies * spqt.spqt_packed_bytes(M, K) / 1e6, 1),
                   "launch": "hipgraph replay" if use_graph else "stream launches",
                   "step": "spqt_gather + spqt_gemv (two launches, index list in HBM)",
                   "mean_n_ns": float(np.mean(wl.n_ns))},
        "effective_GBps_kept_bytes": round(wl.mean_kept_bytes / (us_step * 1e-6) / 1e9, 1),
        "us_gemv_only": round(us_gemv, 3), "us_gather_only": round(us_gather, 3),
        "us_dense_gemv": round(us_dense, 3), "speedup_vs_dense": round(us_dense / us_gemv, 3),
        "ideal_speedup_vs_dense": round(wl.dense_bytes / wl.mean_kept_bytes, 3),
        "us_step_stream_launches": None if us_step_eager is None else round(us_step_eager, 3),
        "us_one_launch_step": round(us_fused, 3),
        "one_launch_effective_GBps_kept_bytes": round(wl.mean_kept_bytes / (us_fused * 1e-6) / 1e9, 1),
        "one_launch_speedup_vs_dense": round(us_dense / us_fused, 3),
        "us_one_launch_even_shares_step": round(us_even, 3),
        "oracle_max_abs_err": max_err,
        "roofline": {"bound": "hbm", "kernel": "spqt_gemv_list_kernel", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "bytes_per_launch": wl.mean_kept_bytes, "us_per_launch": round(us_gemv, 3),
                     # kept bytes plus x, the index list and y: what the launch must touch at all
                     "bytes_per_launch_with_x_idx_y": wl.mean_kept_bytes + 2 * K + 4 * float(np.mean(wl.n_ns)) + 4 * M,
                     "traffic": measured_traffic("spqt_gemv_list_kernel", M, K, H["sparsity"])},
    }

    # ---------------- context: what trivial kernels reach on this machine ----------------------
    t_empty, t_read, read_bytes, big_gbps = calibrate(torch, wl.mean_kept_bytes)
    out["context"] = {"empty_launch_us": round(t_empty, 3),
                      "plain_read_same_bytes_us": round(t_read, 3), "plain_read_bytes": read_bytes,
                      "plain_read_1GiB_GBps": round(big_gbps, 1),
                      "gemv_frac_of_plain_read_rate": round(achieved / big_gbps, 4),
                      "gemv_us_over_plain_read_us": round(us_gemv / t_read, 3),
                      "note": "plain streaming read of the same byte count, cold, same graph-replay timing: the practical floor for one launch"}

    # ---------------- sweeps ---------------------------------------------------------------
    if not args.no_sweep:
        rows = [(5, "down", 8192, 28672, "laplace", [0.5], 1),
                (2, "q", 4096, 4096, "laplace", [0.0, 0.25, 0.4, 0.5, 0.65], 1)]
        if args.full:
            rows += [(3, "gate", 11008, 4096, "laplace", [0.4, 0.5], 1),
                     (3, "down", 4096, 11008, "silu_product", [0.4, 0.5], 1),
                     (4, "k", 1024, 4096, "laplace", [0.5], 1),
                     (4, "gate", 14336, 4096, "laplace", [0.5], 1),
                     (4, "down", 4096, 14336, "laplace", [0.5], 1),
                     (5, "gate", 28672, 8192, "laplace", [0.3, 0.7], 1),
                     (5, "down", 8192, 28672, "laplace", [0.3, 0.7], 1),
                     (5, "gate", 28672, 8192, "laplace", [0.3, 0.5, 0.7], 4),
                     (5, "down", 8192, 28672, "laplace", [0.5], 4),
                     (2, "q", 4096, 4096, "laplace", [0.5], 4)]
        sweep = [sweep_row(torch, spqt, np, H["config"], H["tensor"], M, K, H["dist"], H["sparsity"], 1, K_steps, use_graph, reuse=wl)]
        del wl.packed[1:]           # the headline's rotated copies are no longer needed
        torch.cuda.empty_cache()
        for config, tensor, m, k, dist, sps, batch in rows:
            for s in sps:
                sweep.append(sweep_row(torch, spqt, np, config, tensor, m, k, dist, s, batch, K_steps, use_graph))
                torch.cuda.empty_cache()
        out["sweep"] = sweep
        # decoder-layer GEMV sequences with spqt_gather time included: Llama-3-8B full layer over 32 rotated
        # layers (configuration 4), Llama-2-7B MLP over 16 (configuration 3), 70B-shaped MLP over 8
        # (configuration 5), all at 50 %
        seq_modes = ("strict", "shared", "fused", "merged_gather_gemv", "merged_fused", "dense", "merged_dense")
        out["layer_sequences"] = [layer_sequence(torch, spqt, 4, 32, 0.5, use_graph, modes=None if args.full else seq_modes),
                                  layer_sequence(torch, spqt, 3, 16, 0.5, use_graph, modes=None if args.full else seq_modes),
                                  layer_sequence(torch, spqt, 5, 8, 0.5, use_graph, modes=None if args.full else seq_modes)]
        if args.full:
            import bench_studies as st
            out["layer_sequences"].append(layer_sequence(torch, spqt, 3, 16, 0.4, use_graph))
            out["colblock_layout"] = st.colblock_rows(torch, spqt, use_graph, cpu)
            out["ablations"] = st.ablations(torch, spqt, use_graph, cpu)
            if cpu.enabled:
                out["quantization_error"] = cpu.quantization_error()
            out["rowmajor_baseline"] = st.rowmajor_baseline(torch, spqt, use_graph, cpu)
            out["eight_bit_layout"] = st.eight_bit_rows(torch, spqt, use_graph, cpu)
            out["two_bit_layout"] = st.two_bit_rows(torch, spqt, use_graph, cpu)
            out["merged_gate_up_70b"] = st.merged_gate_up_70b(torch, spqt, use_graph, cpu)
            out["dense_shape_sweep"] = st.dense_shape_sweep(torch, spqt, use_graph)
            out["speedup_grid"] = st.speedup_grid(torch, spqt, use_graph)

    # ---------------- CPU oracle baseline on the headline workload -------------------------
    if cpu.enabled:
        us_all, cores = cpu.time_gemv(wl.case0, wl.x_np[0:1], wl.thr[0], threads=0, runs=7)
        us_one, _ = cpu.time_gemv(wl.case0, wl.x_np[0:1], wl.thr[0], threads=1, runs=5)
        rm_bytes = M * K // 2 + M * (K // 128) * 2
        out["cpu_baseline"] = {"value": round(us_all, 1), "unit": "us/GEMV", "cores": cores, "kind": "oracle",
                               "sample": f"median of 7 oracle GEMVs (mask + dequantize the row-major row + dot, fp64) on copy 0 of "
                                         f"the same {M}x{K} 50% workload, all host threads; single_thread_us is the median of 5 on one thread",
                               "single_thread_us": round(us_one, 1),
                               "GBps_kept_bytes": round(wl.mean_kept_bytes / (us_all * 1e-6) / 1e9, 2),
                               "GBps_rowmajor_bytes_read": round(rm_bytes / (us_all * 1e-6) / 1e9, 2)}
        if args.full:
            from workloads import make_case, quantile_threshold
            others = []
            for config, tensor in ((2, "q"), (3, "gate"), (4, "gate"), (5, "down")):
                case = make_case(config, tensor, want_q=False)
                thr = quantile_threshold(case["x"], 0.5)
                us, cores = cpu.time_gemv(case, case["x"], thr, threads=0, runs=5)
                us1, _ = cpu.time_gemv(case, case["x"], thr, threads=1, runs=5)
                others.append({"config": config, "tensor": tensor, "M": case["M"], "K": case["K"], "sparsity": 0.5,
                               "us_per_gemv": round(us, 1), "single_thread_us": round(us1, 1), "cores": cores})
                del case
            out["cpu_baseline_other_shapes"] = others
    print(json.dumps(out))


if __name__ == "__main__":
    main()
