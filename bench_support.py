"""Shared pieces of the benchmark: rotating workloads, graph capture and timing, the calibration kernels.

Used by bench.py (the headline run) and bench_studies.py (the side studies behind --full).  Nothing here
touches the CPU oracle.
"""
from __future__ import annotations

import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X published HBM3E peak
INFINITY_CACHE_BYTES = 256 << 20
ROTATE_BYTES = 3 * INFINITY_CACHE_BYTES   # rotate over at least this many bytes of weights


def kept_bytes(M, K, n_ns, groups_touched=None):
    """Algorithmic HBM bytes of one sparse GEMV: the 128-byte runs of the kept columns plus the
    fp16 scales of every (row, group) that has a kept column."""
    ng = K // 128 if groups_touched is None else groups_touched
    return n_ns * M // 2 + ng * M * 2


class Workload:
    """Rotating set of packed weight copies + per-copy activations, thresholds and index lists
    for one (M, K) shape at one sparsity."""

    def __init__(self, torch, spqt, M, K, dist, scale_range, config, tensor, sparsity, copies=None, batch=1, min_copies=2):
        import numpy as np
        from workloads import make_case, make_x, quantile_threshold, seed_for, KIND_X
        self.torch, self.spqt, self.M, self.K = torch, spqt, M, K
        self.sparsity = sparsity
        self.batch = batch
        dev = torch.device("cuda:0")
        pbytes = spqt.spqt_packed_bytes(M, K)
        self.copies = copies or max(min_copies, -(-ROTATE_BYTES // pbytes))
        lo, hi = scale_range
        T, NG = M // 256, K // 128
        # copy 0: the seeded row-major tensors of the workload module, repacked by the library
        self.case0 = make_case(config, tensor, layer=0, want_q=False)
        self.packed = [torch.from_numpy(spqt.spqt_pack(self.case0["q_rowmajor"], self.case0["scales"])).to(dev)]
        # other copies: independently seeded random codes and scales drawn directly in packed
        # form on the GPU (any byte is a valid pair of codes; scale area gets fp16 U(lo, hi))
        for layer in range(1, self.copies):
            g = torch.Generator(device=dev)
            g.manual_seed(seed_for(config, layer, tensor))
            buf = torch.randint(0, 256, (T * NG, spqt.CHUNK_BYTES), dtype=torch.uint8, device=dev, generator=g)
            sc = (torch.rand((T * NG, 256), device=dev, generator=g) * (hi - lo) + lo).to(torch.float16)
            buf[:, :512] = sc.view(torch.uint8)
            self.packed.append(buf.reshape(-1))
        xs, thr = [], []
        self.dist = dist
        for layer in range(self.copies):
            x = make_x(K, dist, seed_for(config, layer, tensor, KIND_X), batch)
            xs.append(x[0] if batch == 1 else x)
            thr.append(quantile_threshold(x, sparsity))
        self.x_np = np.stack(xs)
        self.thr = thr
        self.x = torch.from_numpy(self.x_np).to(dev)
        self.idx = torch.zeros((self.copies, K), dtype=torch.int32, device=dev)
        self.cnt = torch.zeros((self.copies, 1), dtype=torch.int32, device=dev)
        self.y = torch.zeros((self.copies, M) if batch == 1 else (self.copies, batch, M), dtype=torch.float32, device=dev)
        self.ws = spqt.new_workspace(M, K, batch)
        self.x_masked = torch.zeros_like(self.x) if batch > 1 else None
        for i in range(self.copies):
            spqt.spqt_gather(self.x[i], self.thr[i], self.idx[i], self.cnt[i])
        torch.cuda.synchronize()
        self.n_ns = self.cnt.cpu().numpy().ravel()
        self.mean_kept_bytes = float(np.mean([kept_bytes(M, K, int(n)) for n in self.n_ns]))
        self.dense_bytes = kept_bytes(M, K, K)

    # one step of the hot path on copy i
    def step(self, i):
        self.spqt.spqt_gather(self.x[i], self.thr[i], self.idx[i], self.cnt[i])
        self.spqt.spqt_gemv(self.packed[i], self.M, self.K, self.x[i], self.idx[i], self.cnt[i], self.y[i], self.ws)

    def step_own_sets(self, i):
        """Several rows, each keeping its own set: union list + per-row zeroed copy of x."""
        self.spqt.spqt_gather_rows(self.x[i], self.thr[i], self.idx[i], self.cnt[i], self.x_masked[i])
        self.spqt.spqt_gemv(self.packed[i], self.M, self.K, self.x_masked[i], self.idx[i], self.cnt[i], self.y[i], self.ws)

    def gemv_only(self, i):
        self.spqt.spqt_gemv(self.packed[i], self.M, self.K, self.x[i], self.idx[i], self.cnt[i], self.y[i], self.ws)

    def gemv_group_passes(self, i):
        """The index-list kernel whose passes hold columns of one quantization group (an ablation)."""
        self.spqt.spqt_gemv(self.packed[i], self.M, self.K, self.x[i], self.idx[i], self.cnt[i], self.y[i], self.ws,
                            flags=self.spqt.CFG_GROUP_PASSES)

    def gather_only(self, i):
        self.spqt.spqt_gather(self.x[i], self.thr[i], self.idx[i], self.cnt[i])

    def fused(self, i):
        self.spqt.spqt_gemv_fused(self.packed[i], self.M, self.K, self.x[i], self.thr[i], self.y[i], self.ws)

    def fused_even_shares(self, i):
        """One launch, every wavefront an even share of the kept columns (counted inside the kernel)."""
        self.spqt.spqt_gemv_fused(self.packed[i], self.M, self.K, self.x[i], self.thr[i], self.y[i], self.ws,
                                  flags=self.spqt.CFG_EVEN_SHARES)

    def fused_rows(self, i):
        """Several rows in one launch, union of the kept sets."""
        self.spqt.spqt_gemv_fused_rows(self.packed[i], self.M, self.K, self.x[i], self.thr[i], self.y[i], self.ws)

    def fused_rows_own_sets(self, i):
        """Several rows in one launch, each summing over its own kept set."""
        self.spqt.spqt_gemv_fused_rows(self.packed[i], self.M, self.K, self.x[i], self.thr[i], self.y[i], self.ws, own_sets=True)

    def fused_no_compaction(self, i):
        self.spqt.spqt_gemv_fused(self.packed[i], self.M, self.K, self.x[i], self.thr[i], self.y[i], self.ws,
                                  flags=self.spqt.CFG_NO_COMPACTION)

    def dense_only(self, i):
        self.spqt.spqt_gemv(self.packed[i], self.M, self.K, self.x[i], None, None, self.y[i], self.ws)

    def check_copy0(self, cpu):
        """Parity of copy 0 against the oracle (through the cpu_baseline leg) in exactly this launch
        configuration; (True, None) when the leg is off."""
        import numpy as np
        if not cpu.enabled:
            return True, None
        self.step(0)
        self.torch.cuda.synchronize()
        ref_idx, n = cpu.gather(self.x_np[0:1], self.thr[0])
        ref = cpu.gemv(self.case0, self.x_np[0:1], self.thr[0])
        ok_idx = int(self.cnt[0].item()) == n and np.array_equal(self.idx[0, :n].cpu().numpy(), ref_idx)
        ok_y, max_err = cpu.close(self.y[0].cpu().numpy(), ref)
        return ok_idx and ok_y, max_err


def make_graph(torch, fn, n):
    """Capture fn(0..n-1) back to back into one HIP graph."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(n):
            fn(i)
    return g


def time_sequence(torch, fn, copies, steps, warmup, use_graph=True, exact_warmup=False):
    """Average microseconds per call of fn over exactly `steps` calls (after `warmup` untimed
    ones), rotating the copy index; HIP events on the launch stream bracket the timed region.
    Side measurements get at least 200 warm-up calls and at least 30 ms of them (a first
    measurement on an idle GPU otherwise reads 5-10 % high); the headline passes exact_warmup and
    gets `warmup` rounded up to whole rotations.  Every graph that is timed has been replayed once
    before the timed region (a graph's first launch uploads it)."""
    if not exact_warmup:
        warmup = max(warmup, 200)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn(0)                       # first launch of a kernel loads its code object: not under capture
    torch.cuda.synchronize()
    if use_graph:
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            full = make_graph(torch, fn, copies)
            rem_n = steps % copies
            rem = make_graph(torch, fn, rem_n) if rem_n else None
            if rem is not None:
                rem.replay()
            for _ in range(max(1, -(-warmup // copies))):
                full.replay()
            torch.cuda.synchronize()
            if not exact_warmup:    # and at least 30 ms of them: after seconds of host work the clocks are down
                t0 = time.perf_counter()
                while time.perf_counter() - t0 < 0.03:
                    full.replay()
                    torch.cuda.synchronize()
            start.record()
            for _ in range(steps // copies):
                full.replay()
            if rem is not None:
                rem.replay()
            stop.record()
            torch.cuda.synchronize()
    else:
        for k in range(warmup):
            fn(k % copies)
        torch.cuda.synchronize()
        start.record()
        for k in range(steps):
            fn(k % copies)
        stop.record()
        torch.cuda.synchronize()
    return start.elapsed_time(stop) * 1e3 / steps


class Calib:
    """ctypes face of libspqt_calib.so: plain streaming read / copy / empty launch, used to put the
    GEMV numbers next to what a trivial kernel reaches on the same box."""

    def __init__(self, torch):
        import ctypes
        self.torch = torch
        path = os.path.join(ROOT, "paper_2511_04477_amd", "libspqt_calib.so")
        L = ctypes.CDLL(path)
        vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        L.spqt_calib_read.argtypes = [vp, sz, vp, i32, i32, vp]
        L.spqt_calib_copy.argtypes = [vp, vp, sz, i32, vp]
        L.spqt_calib_empty.argtypes = [vp]
        L.spqt_calib_rowmajor_gemv.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_float, i32, vp, vp]
        self.L = L
        self.sink = torch.zeros(1, dtype=torch.int32, device="cuda:0")

    def stream(self):
        return self.torch.cuda.current_stream().cuda_stream

    def empty(self, _i=0):
        self.L.spqt_calib_empty(self.stream())

    def read(self, buf, offset, nbytes, blocks=0, unroll=4):
        self.L.spqt_calib_read(buf.data_ptr() + offset, nbytes, self.sink.data_ptr(), blocks, unroll, self.stream())

    def rowmajor_gemv(self, q, scales, M, K, x, thr, skip, y):
        rc = self.L.spqt_calib_rowmajor_gemv(q.data_ptr(), scales.data_ptr(), M, K, x.data_ptr(), float(thr), int(skip),
                                             y.data_ptr(), self.stream())
        if rc != 0:
            raise RuntimeError(f"spqt_calib_rowmajor_gemv failed ({rc})")

    def copy(self, dst, src, nbytes):
        self.L.spqt_calib_copy(dst.data_ptr(), src.data_ptr(), nbytes, 0, self.stream())


def calibrate(torch, nbytes_like):
    """(empty-launch us, us of a plain cold streaming read of ~nbytes_like bytes, GB/s of a 1 GiB read)."""
    cal = Calib(torch)
    big = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").random_(0, 256)
    t_empty = time_sequence(torch, cal.empty, 100, 2000, 200, True)
    size = max(1 << 20, (int(nbytes_like) + 65535) // 65536 * 65536)
    k = (1 << 30) // size
    blocks = max(64, min(4096, size // 16 // 256 // 2))
    t_small = time_sequence(torch, lambda i: cal.read(big, (i % k) * size, size, blocks, 2), k, 2 * k, k, True)
    t_big = time_sequence(torch, lambda i: cal.read(big, 0, 1 << 30, 8192, 4), 2, 6, 2, True)
    del big
    torch.cuda.empty_cache()
    return t_empty, t_small, size, (1 << 30) / (t_big * 1e-6) / 1e9


def layer_sequence(torch, spqt, config, layers, sparsity, use_graph=True, reps=5, modes=None):
    """Decoder-layer GEMV sequence (configs 3 and 4): every projection of every layer has its own
    independently seeded weights and a threshold calibrated offline (separate 64*K draw) for the
    requested sparsity; activations are per input site (attention input, o input, MLP input,
    down input).  One HIP graph holds the whole multi-layer pass.  Returns per-mode timings.
    Modes: strict = one spqt_gather + spqt_gemv per projection; shared = one gather per input site
    (threshold sharing, paper Section 5); fused = one launch per projection; merged_* = projections that
    read the same activations stacked into one matrix; dense / merged_dense = the dense kernel; cb_* = the
    merged matrices in the column-block layout."""
    import numpy as np
    from workloads import (CONFIG_SHAPES, CONFIG_SCALE_RANGE, KIND_CALIB, KIND_X, calibrated_threshold,
                           make_x, seed_for)
    dev = torch.device("cuda:0")
    shapes = CONFIG_SHAPES[config]
    lo, hi = CONFIG_SCALE_RANGE[config]
    site_of = {"q": "attn", "k": "attn", "v": "attn", "o": "o", "gate": "mlp", "up": "mlp", "down": "down"}
    thr = {name: calibrated_threshold(K, dist, sparsity, seed_for(config, 0, name, KIND_CALIB))
           for name, M, K, dist in shapes}
    L = []          # per layer: list of (name, M, K, packed, x, thr, idx, cnt, y, site)
    kept_bytes_total, dense_bytes_total, n_gemv = 0.0, 0.0, 0
    ws = {}
    for layer in range(layers):
        xs = {}
        items = []
        for name, M, K, dist in shapes:
            site = site_of[name]
            if site not in xs:
                xv = make_x(K, dist, seed_for(config, layer, name, KIND_X))
                xs[site] = torch.from_numpy(xv[0]).to(dev)
            g = torch.Generator(device=dev)
            g.manual_seed(seed_for(config, layer, name))
            T, NG = M // 256, K // 128
            buf = torch.randint(0, 256, (T * NG, spqt.CHUNK_BYTES), dtype=torch.uint8, device=dev, generator=g)
            sc = (torch.rand((T * NG, 256), device=dev, generator=g) * (hi - lo) + lo).to(torch.float16)
            buf[:, :512] = sc.view(torch.uint8)
            if (M, K) not in ws:
                ws[(M, K)] = spqt.new_workspace(M, K)
            idx = torch.zeros(K, dtype=torch.int32, device=dev)
            cnt = torch.zeros(1, dtype=torch.int32, device=dev)
            y = torch.zeros(M, dtype=torch.float32, device=dev)
            items.append((name, M, K, buf.reshape(-1), xs[site], thr[name], idx, cnt, y, site))
        L.append(items)
    # Projections that read the same activations, packed as ONE matrix: block-rows are the
    # storage unit of the layout, so concatenating packed buffers along M is concatenating bytes.
    # {q,k,v} and {gate,up} then share one threshold, as in the paper's customized mode (Section 5).
    merged = []
    for items in L:
        groups, order = {}, []
        for it in items:
            if it[9] not in groups:
                groups[it[9]] = []
                order.append(it[9])
            groups[it[9]].append(it)
        mitems = []
        for site in order:
            g_items = groups[site]
            Mtot = sum(it[1] for it in g_items)
            K = g_items[0][2]
            pk = torch.cat([it[3] for it in g_items]) if len(g_items) > 1 else g_items[0][3]
            if (Mtot, K) not in ws:
                ws[(Mtot, K)] = spqt.new_workspace(Mtot, K)
            y = torch.zeros(Mtot, dtype=torch.float32, device=dev)
            mitems.append((Mtot, K, pk, g_items[0][4], g_items[0][5], g_items[0][6], g_items[0][7], y))
        merged.append(mitems)

    all_modes = ("strict", "shared", "fused", "merged_gather_gemv", "merged_fused", "dense", "merged_dense",
                 "cb_merged_gather_gemv", "cb_merged_fused", "cb_merged_dense")
    modes = all_modes if modes is None else tuple(modes)
    # The same merged matrices in the column-block layout (random packed bytes of that format).
    cb_merged = []
    for li, mitems in enumerate(merged if any(m.startswith("cb_") for m in modes) else []):
        row = []
        for mi, (Mtot, K, pk, x, t, idx, cnt, y) in enumerate(mitems):
            g = torch.Generator(device=dev)
            g.manual_seed(seed_for(config, li, "w") + 7000 + mi)
            T, NC = Mtot // 256, K // 128
            buf = torch.randint(0, 256, (T * NC, spqt.CB_CHUNK_BYTES), dtype=torch.uint8, device=dev, generator=g)
            sc = (torch.rand((T * NC, 1024), device=dev, generator=g) * (hi - lo) + lo).to(torch.float16)
            buf[:, :2048] = sc.view(torch.uint8)
            row.append(buf.reshape(-1))
        cb_merged.append(row)

    # achieved kept counts (one eager pass)
    for items in L:
        for name, M, K, pk, x, t, idx, cnt, y, site in items:
            spqt.spqt_gather(x, t, idx, cnt)
    torch.cuda.synchronize()
    for items in L:
        for name, M, K, pk, x, t, idx, cnt, y, site in items:
            kept_bytes_total += kept_bytes(M, K, int(cnt.item()))
            dense_bytes_total += kept_bytes(M, K, K)
            n_gemv += 1

    def run(mode):
        if mode.startswith("cb_"):
            for mitems, cbrow in zip(merged, cb_merged):
                for (Mtot, K, pk, x, t, idx, cnt, y), cpk in zip(mitems, cbrow):
                    if mode == "cb_merged_fused":
                        spqt.spqt_cb_gemv_fused(cpk, Mtot, K, x, t, y, ws[(Mtot, K)])
                    elif mode == "cb_merged_dense":
                        spqt.spqt_cb_gemv(cpk, Mtot, K, x, None, None, y, ws[(Mtot, K)])
                    else:
                        spqt.spqt_gather(x, t, idx, cnt)
                        spqt.spqt_cb_gemv(cpk, Mtot, K, x, idx, cnt, y, ws[(Mtot, K)])
            return
        if mode.startswith("merged"):
            for mitems in merged:
                for Mtot, K, pk, x, t, idx, cnt, y in mitems:
                    if mode == "merged_fused":
                        spqt.spqt_gemv_fused(pk, Mtot, K, x, t, y, ws[(Mtot, K)])
                    elif mode == "merged_dense":
                        spqt.spqt_gemv(pk, Mtot, K, x, None, None, y, ws[(Mtot, K)])
                    else:
                        spqt.spqt_gather(x, t, idx, cnt)
                        spqt.spqt_gemv(pk, Mtot, K, x, idx, cnt, y, ws[(Mtot, K)])
            return
        for items in L:
            done_sites = {}
            for name, M, K, pk, x, t, idx, cnt, y, site in items:
                w = ws[(M, K)]
                if mode == "dense":
                    spqt.spqt_gemv(pk, M, K, x, None, None, y, w)
                elif mode == "fused":
                    spqt.spqt_gemv_fused(pk, M, K, x, t, y, w)
                elif mode == "strict":          # one gather per projection
                    spqt.spqt_gather(x, t, idx, cnt)
                    spqt.spqt_gemv(pk, M, K, x, idx, cnt, y, w)
                else:                           # "shared": one gather per input site (threshold sharing)
                    if site not in done_sites:
                        spqt.spqt_gather(x, t, idx, cnt)
                        done_sites[site] = (idx, cnt)
                    si, sc_ = done_sites[site]
                    spqt.spqt_gemv(pk, M, K, x, si, sc_, y, w)

    out = {"config": config, "layers": layers, "gemvs_per_layer": len(shapes), "sparsity_target": sparsity,
           "packed_MB": round(dense_bytes_total / 1e6, 1), "kept_MB": round(kept_bytes_total / 1e6, 1)}
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for mode in modes:
        run(mode)
        torch.cuda.synchronize()
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            if use_graph:
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    run(mode)
                fn = g.replay
            else:
                fn = lambda: run(mode)
            fn()
            torch.cuda.synchronize()
            start.record()
            for _ in range(reps):
                fn()
            stop.record()
            torch.cuda.synchronize()
        us_pass = start.elapsed_time(stop) * 1e3 / reps
        nbytes = dense_bytes_total if mode.endswith("dense") else kept_bytes_total
        if mode.startswith("cb_"):
            nbytes *= 0.5625 / 0.515625          # 4.5 instead of 4.125 bits per weight
        gbps = nbytes / (us_pass * 1e-6) / 1e9
        out[mode] = {"us_per_layer": round(us_pass / layers, 2), "us_per_gemv": round(us_pass / n_gemv, 3),
                     "GBps": round(gbps, 1), "frac_of_8TBps": round(gbps / HBM_PEAK_GBPS, 4)}
    def ratio(a, b):
        return round(out[a]["us_per_layer"] / out[b]["us_per_layer"], 3) if a in out and b in out else None
    out["speedup_strict_vs_dense"] = ratio("dense", "strict")
    out["speedup_fused_vs_dense"] = ratio("dense", "fused")
    out["speedup_merged_fused_vs_merged_dense"] = ratio("merged_dense", "merged_fused")
    out["speedup_cb_merged_fused_vs_cb_merged_dense"] = ratio("cb_merged_dense", "cb_merged_fused")
    out["launches_per_layer"] = {"strict": 2 * len(shapes), "shared": len(shapes) + len(merged[0]), "fused": len(shapes),
                                 "merged_gather_gemv": 2 * len(merged[0]), "merged_fused": len(merged[0]), "dense": len(shapes), "merged_dense": len(merged[0])}
    return out
