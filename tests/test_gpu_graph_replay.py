"""Every GEMV entry point captured in a HIP graph and replayed: the benchmark times graph replays, and callers
under graph capture are whom spqt_gemv_static is for.  Each replay - with unrelated eager work and a
synchronization before it, and the outputs overwritten in between - must reproduce the eager result bit for
bit (the kernels clear with fill kernels, never with memset nodes, and leave the exchange area zero)."""
import numpy as np
import pytest

from workloads import make_fp_weights, make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

M, K = 2048, 2048


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2511_04477_amd as spqt
    assert torch.cuda.is_available(), "these tests need the MI355X"
    spqt.lib()
    return torch, spqt, torch.device("cuda:0")


def entry_points(torch, spqt, dev):
    """name -> (packed tensor, callable(x, thr, idx, cnt, y, ws), rows of x)"""
    w = make_weights(M, K, 5150)
    Wf = make_fp_weights(M, K, 5151)
    up = lambda a: torch.from_numpy(a).to(dev)
    group = up(spqt.spqt_pack(w["q_rowmajor"], w["scales"]))
    cb, cbk = up(spqt.spqt_cb_quantize(Wf)), up(spqt.spqt_cbk_quantize(Wf))
    cb8, cb2 = up(spqt.spqt_cb8_quantize(Wf)), up(spqt.spqt_cb2_quantize(Wf))
    E = {}
    E["spqt_gemv"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_gemv(group, M, K, x, idx, cnt, y, ws), 1)
    E["spqt_gemv dense"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_gemv(group, M, K, x, None, None, y, ws), 1)
    E["spqt_gemv 4 rows"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_gemv(group, M, K, x, idx, cnt, y, ws), 4)
    E["spqt_gemv_static"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_gemv_static(group, M, K, x, idx, cnt, y), 1)
    E["spqt_gemv_fused"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_gemv_fused(group, M, K, x, thr, y, ws), 1)
    E["spqt_gemv_fused even shares"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_gemv_fused(
        group, M, K, x, thr, y, ws, flags=spqt.CFG_EVEN_SHARES), 1)
    E["spqt_gemv_fused_rows"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_gemv_fused_rows(group, M, K, x, thr, y, ws), 3)
    E["spqt_cb_gemv"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb_gemv(cb, M, K, x, idx, cnt, y, ws), 1)
    E["spqt_cb_gemv_fused"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb_gemv_fused(cb, M, K, x, thr, y, ws), 1)
    E["spqt_cbk_gemv"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cbk_gemv(cbk, M, K, x, idx, cnt, y, ws), 2)
    E["spqt_cb8_gemv"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb8_gemv(cb8, M, K, x, idx, cnt, y, ws), 1)
    E["spqt_cb8_gemv_fused"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb8_gemv_fused(cb8, M, K, x, thr, y, ws), 1)
    E["spqt_cb8_gemv_rows"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb8_gemv_rows(cb8, M, K, x, idx, cnt, y, ws), 4)
    E["spqt_cb2_gemv"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb2_gemv(cb2, M, K, x, idx, cnt, y, ws), 1)
    E["spqt_cb2_gemv_fused"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb2_gemv_fused(cb2, M, K, x, thr, y, ws), 1)
    E["spqt_cb2_gemv_rows"] = (lambda x, thr, idx, cnt, y, ws: spqt.spqt_cb2_gemv_rows(cb2, M, K, x, idx, cnt, y, ws), 3)
    return E


def test_every_entry_point_replays_from_a_graph(gpu):
    torch, spqt, dev = gpu
    E = entry_points(torch, spqt, dev)
    ws = spqt.new_workspace(M, K, 4)           # one workspace for all of them, as a caller would have
    for name, (call, rows) in E.items():
        print("graph replay:", name, flush=True)
        x_np = make_x(K, "laplace", 5200 + rows, batch=rows)
        thr = quantile_threshold(x_np, 0.5)
        x = torch.from_numpy(x_np if rows > 1 else x_np[0].copy()).to(dev)
        idx = torch.zeros(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        y = torch.zeros(rows * M, dtype=torch.float32, device=dev)

        def run():
            spqt.spqt_gather(x, thr, idx, cnt)
            call(x, thr, idx, cnt, y, ws)

        run()
        torch.cuda.synchronize()
        eager = y.cpu().numpy().copy()
        assert np.isfinite(eager).all() and np.abs(eager).max() > 0
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run()
        for rep in range(4):
            y.fill_(float("nan"))
            idx.fill_(-1)
            cnt.fill_(-1)
            other = torch.randn(1 << 16, device=dev).sum()     # unrelated eager work between the replays
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy().view(np.uint32), eager.view(np.uint32)), (name, rep)
            assert float(other) == float(other)
        # the exchange area is all zero again, whatever ran
        assert int(torch.count_nonzero(ws).item()) == 0, name
        del g
