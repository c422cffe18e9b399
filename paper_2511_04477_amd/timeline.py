"""Per-wavefront timeline of one GEMV launch, from the stamped build of the kernels.

    python -m paper_2511_04477_amd.timeline --M 28672 --K 8192 --sparsity 0.5 --kernel list

loads libspqt_timeline.so (the product kernels compiled with -DSPQT_TIMELINE=1: every wavefront stamps
the 100 MHz wall clock at fixed points and writes the stamps out at its end), runs the chosen kernel over
rotated weight copies so that the weights come from HBM, stamps the last launch and prints a Markdown
summary: for every point the minimum, median and maximum over the wavefronts, in microseconds after the
first wavefront's start.  The stamped build waits for the first pass's weights before it goes on (to
be able to stamp their arrival); the product build does not, so the stamped launch is a little slower.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

import numpy as np

POINTS = ["start", "share known", "first pass issued", "first weights", "loop done", "LDS reduced", "end"]


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.splitlines()[0])
    ap.add_argument("--M", type=int, default=28672)
    ap.add_argument("--K", type=int, default=8192)
    ap.add_argument("--sparsity", type=float, default=0.5)
    ap.add_argument("--kernel", choices=["list", "fused", "dense", "fused_static"], default="list")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--waves", type=int, default=0)
    ap.add_argument("--copies", type=int, default=0, help="rotated weight copies (0: enough for 1 GiB)")
    args = ap.parse_args(argv)

    import torch
    from . import binding as B
    from . import build as build_mod
    if not os.path.exists(build_mod.TIMELINE_LIB):
        print(f"{build_mod.TIMELINE_LIB} is not built; run `python -m paper_2511_04477_amd.build`", file=sys.stderr)
        return 2
    B.LIB_PATH = build_mod.TIMELINE_LIB
    import paper_2511_04477_amd as spqt
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    from workloads import make_x, quantile_threshold

    M, K, s = args.M, args.K, args.sparsity
    dev = torch.device("cuda:0")
    L = spqt.lib()
    setter = {"list": "spqt_timeline_set_list", "fused": "spqt_timeline_set_bal", "dense": "spqt_timeline_set_gemv",
              "fused_static": "spqt_timeline_set_gemv"}[args.kernel]
    set_buf = getattr(L, setter)
    set_buf.argtypes = [ctypes.c_void_p]
    T, NG = (M + 255) // 256, K // 128
    one = T * NG * 16896
    copies = args.copies or max(3, -(-(1 << 30) // one))
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    packed = []
    for _ in range(copies):     # any byte is a valid pair of codes; the scale area gets fp16 U(0.003, 0.015)
        buf = torch.randint(0, 256, (T * NG, 16896), dtype=torch.uint8, device=dev, generator=gen)
        sc = (torch.rand((T * NG, 256), device=dev, generator=gen) * 0.012 + 0.003).to(torch.float16)
        buf[:, :512] = sc.view(torch.uint8)
        packed.append(buf.reshape(-1))
    x_np = make_x(K, "laplace", 77)
    thr = quantile_threshold(x_np, s)
    x = torch.from_numpy(x_np[0]).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y = torch.empty(M, dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    kind = {"list": True, "fused": True, "dense": False, "fused_static": True}[args.kernel]
    d_splits, d_waves = spqt.spqt_default_cfg(M, K, 1, kind)
    S, W = args.splits or d_splits, args.waves or d_waves
    grid = 8 * ((T + 7) // 8) * S
    stamps = torch.zeros(grid * W * 8, dtype=torch.int64, device=dev)

    def go(i):
        if args.kernel == "list":
            spqt.spqt_gather(x, thr, idx, cnt)
            spqt.spqt_gemv(packed[i], M, K, x, idx, cnt, y, ws, splits=S, waves=W)
        elif args.kernel == "dense":
            spqt.spqt_gemv(packed[i], M, K, x, None, None, y, ws, splits=S, waves=W)
        elif args.kernel == "fused":
            spqt.spqt_gemv_fused(packed[i], M, K, x, thr, y, ws, splits=S, waves=W, flags=spqt.CFG_EVEN_SHARES)
        else:
            spqt.spqt_gemv_fused(packed[i], M, K, x, thr, y, ws, splits=S, waves=W)

    for rep in range(2):                # warm rotation: code, x, idx stay hot; weights rotate out of the caches
        for i in range(copies):
            go(i)
    torch.cuda.synchronize()
    rc = set_buf(stamps.data_ptr())
    assert rc == 0, rc
    for i in range(copies - 1):
        go(i)
    stamps.zero_()
    go(copies - 1)
    torch.cuda.synchronize()
    set_buf(None)

    d = stamps.cpu().numpy().reshape(grid * W, 8)
    d = d[d[:, 0] > 0]
    t0 = d[:, 0].min()
    us = lambda col: 0.01 * (col.astype(np.float64) - t0)
    print(f"### {args.kernel} kernel, {M} x {K}, sparsity {s}, {S} workgroups per block-row x {W} wavefronts "
          f"({len(d)} wavefronts stamped, {copies} rotated copies)\n")
    print("| point | min us | median us | max us |")
    print("|---|---|---|---|")
    for j, name in enumerate(POINTS):
        col = d[:, j][d[:, j] > 0]
        if col.size == 0:
            continue
        v = us(col)
        print(f"| {name} | {v.min():.2f} | {np.median(v):.2f} | {v.max():.2f} |")
    red = d[(d[:, 7] & 1) == 1]
    if red.size:
        v = us(red[:, 6])
        print(f"| end, reducing workgroups only | {v.min():.2f} | {np.median(v):.2f} | {v.max():.2f} |")
    hw = (d[:, 7] >> 8) & 0xFFFFFFFF
    xcc = (d[:, 7] >> 40) & 15
    cu = (hw >> 8) & 15
    sh = (hw >> 12) & 1
    se = (hw >> 13) & 7
    cuid = ((xcc * 8 + se) * 2 + sh) * 16 + cu
    ids, per_cu = np.unique(cuid, return_counts=True)
    print(f"\nCUs used: {len(ids)}; wavefronts per CU: min {per_cu.min()}, median {int(np.median(per_cu))}, max {per_cu.max()}")
    # how uneven the wavefronts finish their loops: inside a workgroup, and between workgroups
    full = stamps.cpu().numpy().reshape(grid, W, 8)
    full = full[full[:, 0, 0] > 0]
    if full.shape[0]:
        done = 0.01 * (full[:, :, 4].astype(np.float64) - t0)
        inside = done.max(axis=1) - done.min(axis=1)
        last = done.max(axis=1)
        print(f"loop done, spread inside a workgroup (last - first wavefront): median {np.median(inside):.2f} us, max {inside.max():.2f} us; "
              f"last wavefront of a workgroup: min {last.min():.2f}, median {np.median(last):.2f}, max {last.max():.2f} us")
    # where the slow wavefronts are: by XCD, by position inside the workgroup, by split index of the block-row
    done_all = us(d[:, 4])
    print("loop done, median per XCD: " + ", ".join(f"{np.median(done_all[xcc == i]):.2f}" for i in sorted(set(xcc.tolist()))))
    start_all = us(d[:, 0])
    print("start, median per XCD: " + ", ".join(f"{np.median(start_all[xcc == i]):.2f}" for i in sorted(set(xcc.tolist()))))
    if full.shape[0]:
        print("loop done, median per wavefront index in the workgroup: " + ", ".join(f"{np.median(done[:, w]):.2f}" for w in range(W)))
        print("start, median per wavefront index in the workgroup: " + ", ".join(f"{np.median(0.01 * (full[:, w, 0] - t0)):.2f}" for w in range(W)))
    if (d[:, 3] > 0).all():      # kernels without a "first weights" stamp leave it zero
        stream = us(d[:, 4]) - us(d[:, 3])
        print(f"first weights -> loop done per wavefront: median {np.median(stream):.2f} us, max {stream.max():.2f} us")
    return 0


if __name__ == "__main__":
    sys.exit(main())
