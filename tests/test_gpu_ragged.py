"""GPU parity for output counts M that are not a multiple of the block height (256 rows): the last
block-row is zero-padded in the packed form and the kernels must write exactly M outputs per
activation row - nothing past them.  All three weight formats, through the C ABI, against the
oracles on the same seeded inputs; tolerance |y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref|."""
import numpy as np
import pytest

import oracle
from oracle import colblock as cb, colblock_k as ck
from workloads import make_fp_weights, make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3
CANARY = 12345.0


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2511_04477_amd as spqt
    assert torch.cuda.is_available(), "these tests need the MI355X"
    spqt.lib()
    return torch, spqt, torch.device("cuda:0")


def say(*a):
    print(*a, flush=True)


def assert_close(got, ref, what):
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {int(bad.sum())} outputs off, max err {err.max():.3e}"


def run(gpu, kind, packed_np, M, K, x_np, thr, mode, splits, waves):
    """One GEMV on the GPU; y sits inside a larger buffer filled with a canary value so that a
    write outside [batch][M] shows.  mode: 'list', 'dense' or 'fused'."""
    torch, spqt, dev = gpu
    packed = torch.from_numpy(packed_np).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    batch = x.shape[0]
    xx = x if batch > 1 else x[0]
    buf = torch.full((batch * M + 512,), CANARY, dtype=torch.float32, device=dev)
    y = buf[256:256 + batch * M].view(batch, M)
    yy = y if batch > 1 else y[0]
    ws = spqt.new_workspace(M, K, batch)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    if mode == "list":
        spqt.spqt_gather(xx, thr, idx, cnt)
    li, lc = (idx, cnt) if mode == "list" else (None, None)
    if kind == "g128":
        if mode == "fused":
            spqt.spqt_gemv_fused(packed, M, K, xx, thr, yy, ws, splits=splits, waves=waves)
        else:
            spqt.spqt_gemv(packed, M, K, xx, li, lc, yy, ws, splits=splits, waves=waves)
    elif kind == "cb":
        if mode == "fused":
            spqt.spqt_cb_gemv_fused(packed, M, K, xx, thr, yy, ws, splits=splits, waves=waves)
        else:
            spqt.spqt_cb_gemv(packed, M, K, xx, li, lc, yy, ws, splits=splits, waves=waves)
    else:
        spqt.spqt_cbk_gemv(packed, M, K, xx, li, lc, yy, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:256] == CANARY) and np.all(out[256 + batch * M:] == CANARY), "write outside y"
    return out[256:256 + batch * M].reshape(batch, M)


@pytest.mark.parametrize("M", [1, 100, 257, 300, 1000, 2047])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (5, 2), (16, 4)])
def test_ragged_group128(gpu, M, splits, waves):
    import paper_2511_04477_amd as spqt
    K = 1024
    Mp = 256 * ((M + 255) // 256)
    w = make_weights(Mp, K, 6100 + M)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    packed = spqt.spqt_pack(q, sc)
    x = make_x(K, "laplace", 6101 + M)
    for s, mode in ((0.5, "list"), (0.0, "dense"), (0.5, "fused"), (1.0, "list")):
        thr = quantile_threshold(x, s) if s < 1.0 else float("inf")
        say(f"ragged g128 M={M} splits={splits} waves={waves} mode={mode} s={s}")
        ref = oracle.gemv(q, sc, x, 0.0 if mode == "dense" else thr)
        assert_close(run(gpu, "g128", packed, M, K, x, thr, mode, splits, waves), ref, f"g128 {mode}")


@pytest.mark.parametrize("M", [100, 300, 1000])
def test_ragged_group128_batch4(gpu, M):
    import paper_2511_04477_amd as spqt
    K = 2048
    Mp = 256 * ((M + 255) // 256)
    w = make_weights(Mp, K, 6200 + M)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    packed = spqt.spqt_pack(q, sc)
    x = make_x(K, "laplace", 6201 + M, batch=4)
    thr = quantile_threshold(x, 0.5)
    say(f"ragged g128 batch 4 M={M}")
    ref = oracle.gemv(q, sc, x, thr)
    assert_close(run(gpu, "g128", packed, M, K, x, thr, "list", 0, 0), ref, "g128 batch 4")
    assert_close(run(gpu, "g128", packed, M, K, x, thr, "dense", 3, 4), oracle.gemv(q, sc, x, 0.0), "g128 batch 4 dense")


@pytest.mark.parametrize("M", [1, 31, 300, 1000, 2047])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (5, 2), (16, 4)])
def test_ragged_column_block(gpu, M, splits, waves):
    import paper_2511_04477_amd as spqt
    K = 1024
    Mp = 256 * ((M + 255) // 256)
    W = make_fp_weights(Mp, K, 6300 + M)[:M].copy()
    packed = spqt.spqt_cb_quantize(W)
    q, s = cb.quantize(cb.pad_rows(W))
    x = make_x(K, "laplace", 6301 + M)
    for sp, mode in ((0.5, "list"), (0.0, "dense"), (0.5, "fused")):
        thr = quantile_threshold(x, sp)
        say(f"ragged cb M={M} splits={splits} waves={waves} mode={mode}")
        ref = cb.gemv(q, s, x, 0.0 if mode == "dense" else thr)[:, :M]
        assert_close(run(gpu, "cb", packed, M, K, x, thr, mode, splits, waves), ref, f"cb {mode}")
    xb = make_x(K, "laplace", 6302 + M, batch=3)
    thr = quantile_threshold(xb, 0.5)
    assert_close(run(gpu, "cb", packed, M, K, xb, thr, "list", splits, waves), cb.gemv(q, s, xb, thr)[:, :M], "cb batch 3")


@pytest.mark.parametrize("M", [1, 300, 1000])
@pytest.mark.parametrize("splits,waves", [(0, 0), (5, 2), (16, 4)])
def test_ragged_kquant(gpu, M, splits, waves):
    import paper_2511_04477_amd as spqt
    K = 1024
    Mp = 256 * ((M + 255) // 256)
    W = make_fp_weights(Mp, K, 6400 + M)[:M].copy()
    packed = spqt.spqt_cbk_quantize(W)
    p = ck.quantize(ck.pad_rows(W))
    x = make_x(K, "laplace", 6401 + M)
    for sp, mode in ((0.5, "list"), (0.0, "dense")):
        thr = quantile_threshold(x, sp)
        say(f"ragged cbk M={M} splits={splits} waves={waves} mode={mode}")
        ref = ck.gemv(p, x, 0.0 if mode == "dense" else thr)[:, :M]
        assert_close(run(gpu, "cbk", packed, M, K, x, thr, mode, splits, waves), ref, f"cbk {mode}")
