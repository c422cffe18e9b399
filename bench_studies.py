"""Side studies of the benchmark (bench.py --full): ablations, comparison kernels, other layouts and
shapes, and the hardware-counter passes the profile summaries are made from.  The headline run does not
need this module.  The CPU-oracle leg reaches it only as the `cpu` object bench.py hands in.
"""
from __future__ import annotations

import json
import sys

from bench_support import (HBM_PEAK_GBPS, ROTATE_BYTES, Calib, Workload, kept_bytes, time_sequence)


def ablations(torch, spqt, use_graph, cpu):
    """Section 6.3's question on this hardware, on the 70B gate shape at 50 %: what do the index
    list's even split (Section 4.2.3) and the compaction buy?  Two activation patterns: iid
    Laplace (kept columns spread evenly) and a clustered one (7 of 8 kept columns in the first
    half of K), three kernels: list-balanced (spqt_gather + spqt_gemv), static column ranges
    with in-kernel test and compaction (spqt_gemv_fused), the same without compaction, and the one-launch
    kernel that counts the kept columns first and splits them evenly (SPQT_CFG_EVEN_SHARES).  Also the
    list-balanced kernel with one-group passes instead of row-aligned ones (SPQT_CFG_GROUP_PASSES)."""
    import numpy as np
    from workloads import CONFIG_SCALE_RANGE
    M, K, s = 28672, 8192, 0.5
    rows = []
    for dist in ("laplace", "laplace_clustered"):
        w = Workload(torch, spqt, M, K, dist, CONFIG_SCALE_RANGE[5], 5, "gate", s)
        # copy 0 against the oracle in every mode (the clustered pattern is not covered elsewhere at this size)
        if cpu.enabled:
            ref = cpu.gemv(w.case0, w.x_np[0:1], w.thr[0])
            for fn in (w.step, w.gemv_group_passes, w.fused, w.fused_even_shares, w.fused_no_compaction):
                w.y[0].fill_(float("nan"))
                fn(0)
                torch.cuda.synchronize()
                if not cpu.close(w.y[0].cpu().numpy(), ref)[0]:
                    print(f"bench.py: ablation parity check FAILED ({dist}, {fn.__name__})", file=sys.stderr)
                    sys.exit(1)
        steps = w.copies * 40
        t = {name: time_sequence(torch, fn, w.copies, steps, w.copies, use_graph)
             for name, fn in (("list_balanced_gemv", w.gemv_only), ("list_balanced_gemv_group_passes", w.gemv_group_passes),
                              ("gather_plus_list_balanced_gemv", w.step),
                              ("static_ranges_compacted", w.fused), ("even_shares_one_launch", w.fused_even_shares),
                              ("static_ranges_no_compaction", w.fused_no_compaction), ("dense", w.dense_only))}
        rows.append({"M": M, "K": K, "sparsity": s, "activations": dist,
                     "kept_frac": round(float(np.mean(w.n_ns)) / K, 4),
                     "us": {k: round(v, 3) for k, v in t.items()},
                     "speedup_vs_dense": {k: round(t["dense"] / v, 3) for k, v in t.items() if k != "dense"}})
        del w
        torch.cuda.empty_cache()
    return rows


def rowmajor_baseline(torch, spqt, use_graph, cpu):
    """Sections 6.1 and 6.3 on this hardware: the same int4 GEMV read from the ROW-MAJOR source
    layout - dense (the row-wise baseline the zigzag dense kernel should be on par with) and with
    the naive per-weight sparsity test (no byte of a row-major line can be skipped) - next to the
    zigzag kernels, at 50 % on the headline and the 70B gate shape.  Copy 0 of every mode is
    checked against the oracle."""
    import numpy as np
    from workloads import CONFIG_SCALE_RANGE
    calib = Calib(torch)
    dev = torch.device("cuda:0")
    rows = []
    for config, tensor, M, K in ((2, "q", 4096, 4096), (5, "gate", 28672, 8192)):
        w = Workload(torch, spqt, M, K, "laplace", CONFIG_SCALE_RANGE[config], config, tensor, 0.5)
        lo, hi = CONFIG_SCALE_RANGE[config]
        # row-major copies: copy 0 is the seeded source of the packed copy 0, the others random codes
        q = [torch.from_numpy(w.case0["q_rowmajor"]).to(dev)]
        sc = [torch.from_numpy(np.ascontiguousarray(w.case0["scales"])).to(dev)]
        g = torch.Generator(device=dev)
        g.manual_seed(4242 + M)
        for _ in range(1, w.copies):
            q.append(torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device=dev, generator=g))
            sc.append((torch.rand((M, K // 128), device=dev, generator=g) * (hi - lo) + lo).to(torch.float16))
        y = torch.zeros((w.copies, M), dtype=torch.float32, device=dev)

        def rm_dense(i):
            calib.rowmajor_gemv(q[i], sc[i], M, K, w.x[i], 0.0, 0, y[i])

        def rm_skip(i):
            calib.rowmajor_gemv(q[i], sc[i], M, K, w.x[i], w.thr[i], 1, y[i])

        if cpu.enabled:
            for fn, thr in ((rm_dense, 0.0), (rm_skip, w.thr[0])):
                y[0].fill_(float("nan"))
                fn(0)
                torch.cuda.synchronize()
                if not cpu.close(y[0].cpu().numpy(), cpu.gemv(w.case0, w.x_np[0:1], thr))[0]:
                    print(f"bench.py: row-major baseline parity check FAILED ({fn.__name__})", file=sys.stderr)
                    sys.exit(1)
        steps = max(w.copies * 8, 400)
        t = {name: time_sequence(torch, fn, w.copies, steps, w.copies, use_graph)
             for name, fn in (("rowmajor_dense", rm_dense), ("rowmajor_naive_skip", rm_skip),
                              ("zigzag_dense", w.dense_only), ("zigzag_static_ranges_no_compaction", w.fused_no_compaction),
                              ("zigzag_list_balanced_gemv", w.gemv_only), ("zigzag_gather_plus_gemv", w.step))}
        rows.append({"M": M, "K": K, "sparsity": 0.5, "kept_frac": round(float(np.mean(w.n_ns)) / K, 4),
                     "us": {k: round(v, 3) for k, v in t.items()},
                     "speedup_vs_rowmajor_dense": {k: round(t["rowmajor_dense"] / v, 3) for k, v in t.items() if k != "rowmajor_dense"}})
        del w, q, sc, y
        torch.cuda.empty_cache()
    return rows


def merged_gate_up_70b(torch, spqt, use_graph, cpu):
    """Config 5's gate and up projections as ONE matrix (57344 x 8192; both consume the same x, paper
    Section 5: they share a threshold): what one launch reaches when it has twice the bytes to amortize
    its fixed costs over.  Copy 0 is the two seeded tensors stacked and is checked against the oracle on
    sampled rows; the other copies are random packed bytes."""
    import numpy as np
    from workloads import CONFIG_SCALE_RANGE, make_case, make_x, quantile_threshold, seed_for, KIND_X
    dev = torch.device("cuda:0")
    K, Mh = 8192, 28672
    M = 2 * Mh
    gate, up = make_case(5, "gate", want_q=False), make_case(5, "up", want_q=False)
    q = np.concatenate([gate["q_rowmajor"], up["q_rowmajor"]], axis=0)
    sc = np.concatenate([gate["scales"], up["scales"]], axis=0)
    del gate, up
    pbytes = spqt.spqt_packed_bytes(M, K)
    copies = max(2, -(-ROTATE_BYTES // pbytes))
    T, NG = M // 256, K // 128
    lo, hi = CONFIG_SCALE_RANGE[5]
    packed = [torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)]
    g = torch.Generator(device=dev)
    g.manual_seed(9301)
    for _ in range(1, copies):
        buf = torch.randint(0, 256, (T * NG, spqt.CHUNK_BYTES), dtype=torch.uint8, device=dev, generator=g)
        s16 = (torch.rand((T * NG, 256), device=dev, generator=g) * (hi - lo) + lo).to(torch.float16)
        buf[:, :512] = s16.view(torch.uint8)
        packed.append(buf.reshape(-1))
    x_np = make_x(K, "laplace", seed_for(5, 0, "gate", KIND_X))
    x = torch.from_numpy(x_np[0]).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y = torch.empty(M, dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    rows = []
    sample = np.unique(np.concatenate([np.arange(0, 512), np.arange(Mh - 256, Mh + 256), np.arange(M - 512, M)]))
    for s in (0.5, 0.7):
        thr = quantile_threshold(x_np, s)
        spqt.spqt_gather(x, thr, idx, cnt)
        torch.cuda.synchronize()
        n = int(cnt.item())
        if cpu.enabled:
            ref = cpu.gemv_rows({"q_rowmajor": q, "scales": sc}, x_np, thr, sample)
            for name, call in (("list", lambda: spqt.spqt_gemv(packed[0], M, K, x, idx, cnt, y, ws)),
                               ("fused", lambda: spqt.spqt_gemv_fused(packed[0], M, K, x, thr, y, ws))):
                y.fill_(float("nan"))
                call()
                torch.cuda.synchronize()
                if not cpu.close(y.cpu().numpy()[sample], ref)[0]:
                    print(f"bench.py: merged gate|up parity check FAILED ({name}, s={s})", file=sys.stderr)
                    sys.exit(1)
        fns = {"us_gemv": lambda i: spqt.spqt_gemv(packed[i], M, K, x, idx, cnt, y, ws),
               "us_dense": lambda i: spqt.spqt_gemv(packed[i], M, K, x, None, None, y, ws),
               "us_gather_plus_gemv": lambda i: (spqt.spqt_gather(x, thr, idx, cnt),
                                                 spqt.spqt_gemv(packed[i], M, K, x, idx, cnt, y, ws)),
               "us_fused": lambda i: spqt.spqt_gemv_fused(packed[i], M, K, x, thr, y, ws)}
        t = {k: time_sequence(torch, f, copies, 800, 200, use_graph) for k, f in fns.items()}
        kept = kept_bytes(M, K, n)
        rows.append({"M": M, "K": K, "sparsity": s, "kept_frac": round(n / K, 4), **{k: round(v, 3) for k, v in t.items()},
                     "GBps_kept": round(kept / (t["us_gemv"] * 1e-6) / 1e9, 1),
                     "frac_of_8TBps": round(kept / (t["us_gemv"] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                     "dense_GBps": round(pbytes / (t["us_dense"] * 1e-6) / 1e9, 1),
                     "dense_frac_of_8TBps": round(pbytes / (t["us_dense"] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                     "speedup_vs_dense": round(t["us_dense"] / t["us_gemv"], 3)})
    del packed
    torch.cuda.empty_cache()
    return rows


def other_width_rows(torch, spqt, use_graph, cpu, bits):
    """The 8-bit or 2-bit flavour of the column-block layout (block-rows of 128 or 512 rows, one column
    still one 128-byte run) on the headline and the 70B gate shape at 50 % and dense.  Copy 0 is
    quantized from seeded fp32 weights by the library and checked against the NumPy oracle on sampled
    block-rows; the other copies are random codes under valid fp16 scales."""
    import numpy as np
    from workloads import make_fp_weights, make_x, quantile_threshold
    dev = torch.device("cuda:0")
    if bits == 8:
        tile_rows, chunk_bytes, seed = 128, spqt.CB8_CHUNK_BYTES, 9100
        packed_bytes, quantize, gemv, reference = spqt.spqt_cb8_packed_bytes, spqt.spqt_cb8_quantize, spqt.spqt_cb8_gemv, cpu.colblock_w8
        one_launch, rows_fn = spqt.spqt_cb8_gemv_fused, spqt.spqt_cb8_gemv_rows
    else:
        tile_rows, chunk_bytes, seed = 512, spqt.CB2_CHUNK_BYTES, 9200
        packed_bytes, quantize, gemv, reference = spqt.spqt_cb2_packed_bytes, spqt.spqt_cb2_quantize, spqt.spqt_cb2_gemv, cpu.colblock_w2
        one_launch, rows_fn = spqt.spqt_cb2_gemv_fused, spqt.spqt_cb2_gemv_rows
    scale_bytes = 128 * 2 * (tile_rows // 32)
    rows = []
    for M, K in ((4096, 4096), (28672, 8192)):
        pbytes = packed_bytes(M, K)
        copies = max(2, -(-ROTATE_BYTES // pbytes))
        T, NC = M // tile_rows, K // 128
        W0 = make_fp_weights(M, K, seed + M)
        packed = [torch.from_numpy(quantize(W0)).to(dev)]
        g = torch.Generator(device=dev)
        g.manual_seed(seed + 1 + M)
        for _ in range(1, copies):
            buf = torch.randint(0, 256, (T * NC, chunk_bytes), dtype=torch.uint8, device=dev, generator=g)
            sc = (torch.rand((T * NC, scale_bytes // 2), device=dev, generator=g) * 0.0008 + 0.0003).to(torch.float16)
            buf[:, :scale_bytes] = sc.view(torch.uint8)
            packed.append(buf.reshape(-1))
        tiles = np.unique(np.array([0, T // 2, T - 1]))
        sample = (tiles[:, None] * tile_rows + np.arange(tile_rows)[None, :]).ravel()
        W0_sample = W0[sample].copy()
        del W0
        x_np = make_x(K, "laplace", seed + 2 + M)
        thr = quantile_threshold(x_np, 0.5)
        x = torch.from_numpy(x_np[0]).to(dev)
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        y = torch.empty(M, dtype=torch.float32, device=dev)
        ws = spqt.new_workspace(M, K)
        spqt.spqt_gather(x, thr, idx, cnt)
        torch.cuda.synchronize()
        n = int(cnt.item())
        if cpu.enabled:
            y.fill_(float("nan"))
            gemv(packed[0], M, K, x, idx, cnt, y, ws)
            torch.cuda.synchronize()
            want = reference(W0_sample, x_np, thr)
            ok = cpu.close(y.cpu().numpy()[sample], want)[0]
            y.fill_(float("nan"))
            one_launch(packed[0], M, K, x, thr, y, ws)
            torch.cuda.synchronize()
            if not (ok and cpu.close(y.cpu().numpy()[sample], want)[0]):
                print(f"bench.py: {bits}-bit column-block parity check FAILED ({M}x{K})", file=sys.stderr)
                sys.exit(1)
        fns = {"us_gemv": lambda i: gemv(packed[i], M, K, x, idx, cnt, y, ws),
               "us_dense": lambda i: gemv(packed[i], M, K, x, None, None, y, ws),
               "us_gather_plus_gemv": lambda i: (spqt.spqt_gather(x, thr, idx, cnt),
                                                 gemv(packed[i], M, K, x, idx, cnt, y, ws)),
               "us_one_launch": lambda i: one_launch(packed[i], M, K, x, thr, y, ws)}
        # two activation rows on the union of their kept columns (each row 50 %: the union keeps about 75 %)
        x2_np = np.concatenate([x_np, make_x(K, "laplace", seed + 3 + M)], axis=0)
        x2 = torch.from_numpy(x2_np).to(dev)
        idx2 = torch.empty(K, dtype=torch.int32, device=dev)
        cnt2 = torch.zeros(1, dtype=torch.int32, device=dev)
        y2 = torch.empty(2 * M, dtype=torch.float32, device=dev)
        ws2 = spqt.new_workspace(M, K, 2)
        spqt.spqt_gather(x2, thr, idx2, cnt2)
        fns["us_two_rows_union"] = lambda i: rows_fn(packed[i], M, K, x2, idx2, cnt2, y2, ws2)
        t = {k: time_sequence(torch, f, copies, max(copies * 4, 800), copies, use_graph) for k, f in fns.items()}
        kept = n * (M * bits // 8 + M // 16)
        rows.append({"M": M, "K": K, "sparsity": 0.5, "kept_frac": round(n / K, 4), "bits_per_weight": bits + 0.5,
                     "kept_bytes": kept, **{k: round(v, 3) for k, v in t.items()},
                     "GBps_kept": round(kept / (t["us_gemv"] * 1e-6) / 1e9, 1),
                     "frac_of_8TBps": round(kept / (t["us_gemv"] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                     "dense_GBps": round(pbytes / (t["us_dense"] * 1e-6) / 1e9, 1),
                     "speedup_vs_dense": round(t["us_dense"] / t["us_gemv"], 3)})
        del packed
        torch.cuda.empty_cache()
    return rows


def eight_bit_rows(torch, spqt, use_graph, cpu):
    return other_width_rows(torch, spqt, use_graph, cpu, 8)


def two_bit_rows(torch, spqt, use_graph, cpu):
    return other_width_rows(torch, spqt, use_graph, cpu, 2)


def colblock_rows(torch, spqt, use_graph, cpu, full=True):
    """The column-block variant of the layout (the paper's own grouping, Section 4.1.2: 32-row
    blocks along a column, scales skipped with their column) on the headline and 70B shapes.
    Copy 0 is quantized from seeded fp32 weights by the library and checked against the
    NumPy oracle on sampled 256-row tiles; the other copies are random packed bytes."""
    import numpy as np
    from workloads import make_fp_weights, make_x, quantile_threshold
    dev = torch.device("cuda:0")
    rows = []
    L, C = "laplace", "laplace_clustered"     # C: 7 of 8 kept columns in the first half of K
    shapes = ((4096, 4096, ((0.5, L),)), (28672, 8192, ((0.3, L), (0.5, L), (0.7, L), (0.5, C))),
              (8192, 28672, ((0.5, L),)))
    for M, K, sps in (shapes if full else shapes[:1]):
        pbytes = spqt.spqt_cb_packed_bytes(M, K)
        copies = max(2, -(-ROTATE_BYTES // pbytes))
        T, NC = M // 256, K // 128
        W0 = make_fp_weights(M, K, 9000 + M)
        packed = [torch.from_numpy(spqt.spqt_cb_quantize(W0)).to(dev)]
        g = torch.Generator(device=dev)
        g.manual_seed(9001 + M)
        for _ in range(1, copies):
            buf = torch.randint(0, 256, (T * NC, spqt.CB_CHUNK_BYTES), dtype=torch.uint8, device=dev, generator=g)
            sc = (torch.rand((T * NC, 1024), device=dev, generator=g) * 0.015 + 0.005).to(torch.float16)
            buf[:, :2048] = sc.view(torch.uint8)
            packed.append(buf.reshape(-1))
        tiles = np.unique(np.array([0, T // 2, T - 1]))
        sample = (tiles[:, None] * 256 + np.arange(256)[None, :]).ravel()
        W0_sample = W0[sample].copy()
        packed_k0 = torch.from_numpy(spqt.spqt_cbk_quantize(W0)).to(dev) if cpu.enabled else None
        del W0
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        y = torch.empty(M, dtype=torch.float32, device=dev)
        ws = spqt.new_workspace(M, K)
        for s, dist in sps:
            x_np = make_x(K, dist, 9002 + M)
            thr = quantile_threshold(x_np, s)
            x = torch.from_numpy(x_np[0]).to(dev)
            spqt.spqt_gather(x, thr, idx, cnt)
            torch.cuda.synchronize()
            n = int(cnt.item())
            if cpu.enabled:
                ref = cpu.colblock(W0_sample, x_np, thr)
                for name, call in (("list", lambda: spqt.spqt_cb_gemv(packed[0], M, K, x, idx, cnt, y, ws)),
                                   ("fused", lambda: spqt.spqt_cb_gemv_fused(packed[0], M, K, x, thr, y, ws))):
                    y.fill_(float("nan"))
                    call()
                    torch.cuda.synchronize()
                    if not cpu.close(y.cpu().numpy()[sample], ref)[0]:
                        print(f"bench.py: column-block parity check FAILED ({M}x{K}, {name})", file=sys.stderr)
                        sys.exit(1)
            fns = {"us_gemv": lambda i: spqt.spqt_cb_gemv(packed[i], M, K, x, idx, cnt, y, ws),
                   "us_dense": lambda i: spqt.spqt_cb_gemv(packed[i], M, K, x, None, None, y, ws),
                   "us_gather_plus_gemv": lambda i: (spqt.spqt_gather(x, thr, idx, cnt),
                                                     spqt.spqt_cb_gemv(packed[i], M, K, x, idx, cnt, y, ws)),
                   "us_fused": lambda i: spqt.spqt_cb_gemv_fused(packed[i], M, K, x, thr, y, ws)}
            t = {k: time_sequence(torch, f, copies, max(copies * 4, 800), copies, use_graph) for k, f in fns.items()}
            kept = n * (M // 2 + M // 16)
            rows.append({"M": M, "K": K, "sparsity": s, "activations": dist, "kept_frac": round(n / K, 4),
                         "bits_per_weight": 4.5, "kept_bytes": kept,
                         **{k: round(v, 3) for k, v in t.items()},
                         "GBps_kept": round(kept / (t["us_gemv"] * 1e-6) / 1e9, 1),
                         "frac_of_8TBps": round(kept / (t["us_gemv"] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                         "dense_GBps": round(pbytes / (t["us_dense"] * 1e-6) / 1e9, 1),
                         "speedup_vs_dense": round(t["us_dense"] / t["us_gemv"], 3),
                         "fused_speedup_vs_dense": round(t["us_dense"] / t["us_fused"], 3)})
        if M == 28672:      # four activation rows sharing the union list (config 5's batch-4 case)
            xb_np = make_x(K, "laplace", 9003 + M, 4)
            thr = quantile_threshold(xb_np, 0.5)
            xb = torch.from_numpy(xb_np).to(dev)
            yb = torch.empty((4, M), dtype=torch.float32, device=dev)
            wsb = spqt.new_workspace(M, K, 4)
            spqt.spqt_gather(xb, thr, idx, cnt)
            torch.cuda.synchronize()
            n = int(cnt.item())
            if cpu.enabled:
                from_ref = []
                spqt.spqt_cb_gemv(packed[0], M, K, xb, idx, cnt, yb, wsb)
                torch.cuda.synchronize()
                for b in range(4):      # the union set with each row's own values == that row with the others' dropped columns kept
                    from_ref.append(cpu.colblock(W0_sample, np.where(np.any(~(np.abs(xb_np.astype(np.float32)) < np.float32(thr)), axis=0), xb_np[b], 0).astype(np.float16)[None, :], 0.0))
                    if not cpu.close(yb[b].cpu().numpy()[sample], from_ref[b])[0]:
                        print(f"bench.py: column-block batch-4 parity check FAILED (row {b})", file=sys.stderr)
                        sys.exit(1)
            t_s = time_sequence(torch, lambda i: spqt.spqt_cb_gemv(packed[i], M, K, xb, idx, cnt, yb, wsb), copies, max(copies * 4, 400), copies, use_graph)
            t_d = time_sequence(torch, lambda i: spqt.spqt_cb_gemv(packed[i], M, K, xb, None, None, yb, wsb), copies, max(copies * 4, 400), copies, use_graph)
            rows.append({"M": M, "K": K, "batch": 4, "sparsity_per_row": 0.5, "activations": L, "kept_frac": round(n / K, 4),
                         "us_gemv": round(t_s, 3), "us_dense": round(t_d, 3), "speedup_vs_dense": round(t_d / t_s, 3)})
        # K-quant flavour (6-bit block scales and minima under fp16 superblock scales): copy 0 quantized
        # by the library and checked, then timed on the rotating buffers with their headers rewritten
        # (finite superblock scales; any 6-bit fields and codes are valid)
        x_np = make_x(K, L, 9002 + M)
        thr = quantile_threshold(x_np, 0.5)
        x = torch.from_numpy(x_np[0]).to(dev)
        spqt.spqt_gather(x, thr, idx, cnt)
        torch.cuda.synchronize()
        n = int(cnt.item())
        if cpu.enabled:
            ref = cpu.colblock_k(W0_sample, x_np, thr)
            y.fill_(float("nan"))
            spqt.spqt_cbk_gemv(packed_k0, M, K, x, idx, cnt, y, ws)
            torch.cuda.synchronize()
            if not cpu.close(y.cpu().numpy()[sample], ref)[0]:
                print(f"bench.py: K-quant column-block parity check FAILED ({M}x{K})", file=sys.stderr)
                sys.exit(1)
            del packed_k0
        for buf in packed:
            hdr = buf.view(T * NC, spqt.CB_CHUNK_BYTES)[:, :2048].view(torch.float16).view(T * NC, 128, 8)
            hdr[:, :, 0] = 0.0005
            hdr[:, :, 1] = 0.0004
        t_ks = time_sequence(torch, lambda i: spqt.spqt_cbk_gemv(packed[i], M, K, x, idx, cnt, y, ws), copies, max(copies * 4, 800), copies, use_graph)
        t_kd = time_sequence(torch, lambda i: spqt.spqt_cbk_gemv(packed[i], M, K, x, None, None, y, ws), copies, max(copies * 4, 800), copies, use_graph)
        rows.append({"M": M, "K": K, "format": "k-quant", "sparsity": 0.5, "activations": L, "kept_frac": round(n / K, 4),
                     "us_gemv": round(t_ks, 3), "us_dense": round(t_kd, 3), "speedup_vs_dense": round(t_kd / t_ks, 3)})
        del packed
        torch.cuda.empty_cache()
    return rows


def speedup_grid(torch, spqt, use_graph):
    """Sparse-over-dense speed-up against sparsity on the GEMV shapes of the paper's kernel
    micro-benchmark (Section 6.3: Llama-3-8B, Llama-2-13B and Llama-2-70B projections at 25 / 40 /
    50 %), for both layouts; random packed bytes, iid Laplace activations, gather time not included."""
    import numpy as np
    from workloads import make_x, quantile_threshold
    dev = torch.device("cuda:0")
    shapes = [("llama-3-8b", 4096, 4096), ("llama-3-8b", 14336, 4096), ("llama-3-8b", 4096, 14336),
              ("llama-2-13b", 5120, 5120), ("llama-2-13b", 13824, 5120), ("llama-2-13b", 5120, 13824),
              ("llama-2-70b", 8192, 8192), ("llama-2-70b", 28672, 8192), ("llama-2-70b", 8192, 28672)]
    rows = []
    for model, M, K in shapes:
        T, NC = M // 256, K // 128
        x_np = make_x(K, "laplace", 9200 + M + K)
        x = torch.from_numpy(x_np[0]).to(dev)
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        y = torch.empty(M, dtype=torch.float32, device=dev)
        ws = spqt.new_workspace(M, K)
        for layout, chunk, nscale, gemv in (("group", spqt.CHUNK_BYTES, 256, spqt.spqt_gemv),
                                            ("colblock", spqt.CB_CHUNK_BYTES, 1024, spqt.spqt_cb_gemv)):
            pbytes = T * NC * chunk
            copies = max(2, -(-ROTATE_BYTES // pbytes))
            g = torch.Generator(device=dev)
            g.manual_seed(9201 + M + K)
            packed = []
            for _ in range(copies):
                buf = torch.randint(0, 256, (T * NC, chunk), dtype=torch.uint8, device=dev, generator=g)
                sc = (torch.rand((T * NC, nscale), device=dev, generator=g) * 0.015 + 0.005).to(torch.float16)
                buf[:, :2 * nscale] = sc.view(torch.uint8)
                packed.append(buf.reshape(-1))
            steps = max(copies * 4, 400)
            t_dense = time_sequence(torch, lambda i: gemv(packed[i], M, K, x, None, None, y, ws), copies, steps, copies, use_graph)
            row = {"model": model, "M": M, "K": K, "layout": layout, "us_dense": round(t_dense, 3), "sparse": []}
            for sp in (0.25, 0.4, 0.5):
                thr = quantile_threshold(x_np, sp)
                spqt.spqt_gather(x, thr, idx, cnt)
                torch.cuda.synchronize()
                t_sparse = time_sequence(torch, lambda i: gemv(packed[i], M, K, x, idx, cnt, y, ws), copies, steps, copies, use_graph)
                row["sparse"].append({"sparsity": sp, "us": round(t_sparse, 3), "speedup_vs_dense": round(t_dense / t_sparse, 3)})
            rows.append(row)
            del packed
            torch.cuda.empty_cache()
    return rows


def dense_shape_sweep(torch, spqt, use_graph):
    """The dense zigzag kernel on the 15 shapes of the paper's dense micro-benchmark
    (Section 6.3, dense GEMV comparison: m in {2048, 4096, 8192} x k in {1024 ... 16384}); random packed bytes."""
    dev = torch.device("cuda:0")
    rows = []
    for M in (2048, 4096, 8192):
        for K in (1024, 2048, 4096, 8192, 16384):
            pbytes = spqt.spqt_packed_bytes(M, K)
            copies = max(2, -(-ROTATE_BYTES // pbytes))
            g = torch.Generator(device=dev)
            g.manual_seed(1000 * M + K)
            T, NG = M // 256, K // 128
            packed = []
            for _ in range(copies):
                buf = torch.randint(0, 256, (T * NG, spqt.CHUNK_BYTES), dtype=torch.uint8, device=dev, generator=g)
                sc = (torch.rand((T * NG, 256), device=dev, generator=g) * 0.015 + 0.005).to(torch.float16)
                buf[:, :512] = sc.view(torch.uint8)
                packed.append(buf.reshape(-1))
            x = torch.randn(K, device=dev, generator=g).to(torch.float16)
            y = torch.empty(M, dtype=torch.float32, device=dev)
            ws = spqt.new_workspace(M, K)
            fn = lambda i: spqt.spqt_gemv(packed[i], M, K, x, None, None, y, ws)
            us = time_sequence(torch, fn, copies, copies * 4, copies, use_graph)
            rows.append({"M": M, "K": K, "us_dense": round(us, 3), "GBps": round(pbytes / (us * 1e-6) / 1e9, 1),
                         "GFLOPS": round(2.0 * M * K / (us * 1e-6) / 1e9, 1)})
            del packed
            torch.cuda.empty_cache()
    return rows


def pmc_pass_small(torch, spqt):
    """Hardware-counter pass on 4096 x 4096 at 50 %: 8 plain copies of 64 MiB for counter scaling, then the
    list-driven sparse kernel once per weight copy, eagerly."""
    from workloads import CONFIG_SCALE_RANGE
    M, K = 4096, 4096
    wl = Workload(torch, spqt, M, K, "laplace", CONFIG_SCALE_RANGE[2], 2, "q", 0.5)
    cal = Calib(torch)
    a = torch.empty(64 << 20, dtype=torch.uint8, device="cuda:0").random_(0, 256)
    b = torch.empty_like(a)
    for _ in range(8):
        cal.copy(b, a, 64 << 20)
    for fn in (wl.gemv_only, wl.dense_only, wl.fused):
        for i in range(wl.copies):
            fn(i)
    torch.cuda.synchronize()
    print(json.dumps({"pmc_pass": True, "workload": "q4096", "M": M, "K": K, "copy_bytes": 64 << 20, "launches_per_kernel": wl.copies,
                      "kept_bytes_per_launch": wl.mean_kept_bytes, "dense_bytes_per_launch": wl.dense_bytes, "y_bytes_per_launch": 4 * M}))


def pmc_pass_large(torch, spqt, which):
    """Hardware-counter pass on the 70B gate shape (28672 x 8192, 50 %): 8 plain copies of 64 MiB
    for counter scaling, then the sparse, dense and one-launch kernels once per weight copy."""
    import numpy as np
    from workloads import CONFIG_SCALE_RANGE, make_x, quantile_threshold
    M, K, s = 28672, 8192, 0.5
    cal = Calib(torch)
    dev = torch.device("cuda:0")
    a = torch.empty(64 << 20, dtype=torch.uint8, device=dev).random_(0, 256)
    b = torch.empty_like(a)
    for _ in range(8):
        cal.copy(b, a, 64 << 20)
    if which == "gate70b":
        wl = Workload(torch, spqt, M, K, "laplace", CONFIG_SCALE_RANGE[5], 5, "gate", s, min_copies=8)
        for fn in (wl.gemv_only, wl.gemv_group_passes, wl.dense_only, wl.fused, wl.fused_even_shares, wl.gather_only):
            for i in range(wl.copies):
                fn(i)
        kept, dense, copies = wl.mean_kept_bytes, wl.dense_bytes, wl.copies
    elif which in ("gate70b_w8", "gate70b_w2"):
        if which == "gate70b_w8":
            bits, tile_rows, chunk_bytes = 8, 128, spqt.CB8_CHUNK_BYTES
            packed_bytes, gemv = spqt.spqt_cb8_packed_bytes, spqt.spqt_cb8_gemv
        else:
            bits, tile_rows, chunk_bytes = 2, 512, spqt.CB2_CHUNK_BYTES
            packed_bytes, gemv = spqt.spqt_cb2_packed_bytes, spqt.spqt_cb2_gemv
        scale_bytes = 128 * 2 * (tile_rows // 32)
        pbytes = packed_bytes(M, K)
        copies = max(2, -(-ROTATE_BYTES // pbytes))
        T, NC = M // tile_rows, K // 128
        g = torch.Generator(device=dev)
        g.manual_seed(9201)
        packed = []
        for _ in range(copies):
            buf = torch.randint(0, 256, (T * NC, chunk_bytes), dtype=torch.uint8, device=dev, generator=g)
            sc = (torch.rand((T * NC, scale_bytes // 2), device=dev, generator=g) * 0.0008 + 0.0003).to(torch.float16)
            buf[:, :scale_bytes] = sc.view(torch.uint8)
            packed.append(buf.reshape(-1))
        x_np = make_x(K, "laplace", 9202)
        thr = quantile_threshold(x_np, s)
        x = torch.from_numpy(x_np[0]).to(dev)
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        y = torch.empty(M, dtype=torch.float32, device=dev)
        ws = spqt.new_workspace(M, K)
        spqt.spqt_gather(x, thr, idx, cnt)
        torch.cuda.synchronize()
        for i in range(copies):
            gemv(packed[i], M, K, x, idx, cnt, y, ws)
        for i in range(copies):
            gemv(packed[i], M, K, x, None, None, y, ws)
        kept, dense = int(cnt.item()) * (M * bits // 8 + M // 16), pbytes
    else:
        pbytes = spqt.spqt_cb_packed_bytes(M, K)
        copies = max(2, -(-ROTATE_BYTES // pbytes))
        T, NC = M // 256, K // 128
        g = torch.Generator(device=dev)
        g.manual_seed(9101)
        packed = []
        for _ in range(copies):
            buf = torch.randint(0, 256, (T * NC, spqt.CB_CHUNK_BYTES), dtype=torch.uint8, device=dev, generator=g)
            sc = (torch.rand((T * NC, 1024), device=dev, generator=g) * 0.015 + 0.005).to(torch.float16)
            buf[:, :2048] = sc.view(torch.uint8)
            packed.append(buf.reshape(-1))
        x_np = make_x(K, "laplace", 9102)
        thr = quantile_threshold(x_np, s)
        x = torch.from_numpy(x_np[0]).to(dev)
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        y = torch.empty(M, dtype=torch.float32, device=dev)
        ws = spqt.new_workspace(M, K)
        spqt.spqt_gather(x, thr, idx, cnt)
        torch.cuda.synchronize()
        for i in range(copies):
            spqt.spqt_cb_gemv(packed[i], M, K, x, idx, cnt, y, ws)
        for i in range(copies):
            spqt.spqt_cb_gemv(packed[i], M, K, x, None, None, y, ws)
        for i in range(copies):
            spqt.spqt_cb_gemv_fused(packed[i], M, K, x, thr, y, ws)
        kept, dense = int(cnt.item()) * (M // 2 + M // 16), pbytes
    torch.cuda.synchronize()
    print(json.dumps({"pmc_pass": True, "workload": which, "M": M, "K": K, "copy_bytes": 64 << 20, "launches_per_kernel": copies,
                      "kept_bytes_per_launch": kept, "dense_bytes_per_launch": dense, "y_bytes_per_launch": 4 * M}))


