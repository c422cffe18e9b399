"""GPU parity of two options around the GEMV, through the C ABI, against the oracles:

* per-row kept sets for several activation rows (spqt_gather_rows: union list + a copy of x
  with each row's own dropped entries zeroed) - every row must equal the batch-1 oracle result
  of that row alone;
* fp16 output (SPQT_CFG_Y_FP16) - the oracle's value within the usual tolerance, and exactly
  the fp32 output of the same launch shape rounded to nearest even.

Tolerance |y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref| (fp16 rounding, 2^-11 relative, fits inside)."""
import numpy as np
import pytest

import oracle
from oracle import colblock as cb, colblock_k as ck
from workloads import make_fp_weights, make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3


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


def gather_rows(gpu, x_np, thr):
    torch, spqt, dev = gpu
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    K = x.shape[-1]
    idx = torch.full((K,), -7, dtype=torch.int32, device=dev)
    cnt = torch.full((1,), -7, dtype=torch.int32, device=dev)
    xm = torch.full_like(x, float("nan"))
    spqt.spqt_gather_rows(x, thr, idx, cnt, xm)
    torch.cuda.synchronize()
    return x, idx, cnt, xm


@pytest.mark.parametrize("K", [128, 4096, 8192, 28672])
@pytest.mark.parametrize("batch", [1, 2, 3, 4])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9])
def test_gather_rows_list_and_masked_copy_bit_exact(gpu, K, batch, sparsity):
    x = make_x(K, "laplace", 7000 + K + batch, batch=batch)
    thr = quantile_threshold(x, sparsity)
    say(f"gather_rows K={K} batch={batch} s={sparsity}")
    _, idx, cnt, xm = gather_rows(gpu, x, thr)
    ref, n = oracle.gather(x, thr)
    assert int(cnt.cpu()[0]) == n and np.array_equal(idx.cpu().numpy()[:n], ref)
    assert np.all(idx.cpu().numpy()[n:] == -7)
    want = x.view(np.uint16).copy()
    for b in range(batch):
        want[b][~oracle.mask(x[b:b + 1], thr)] = 0          # a row's own dropped entries become +0
    assert np.array_equal(xm.cpu().numpy().view(np.uint16), want)


def test_gather_rows_ties_signed_zero_and_special_values(gpu):
    x = np.zeros((2, 256), dtype=np.float16)
    x[0, :8] = [0.5, -0.5, 0.25, 0.0, -0.0, 0.75, 0.4995, -0.4995]
    x[1, :8] = [0.1, 0.5, -0.6, np.nan, np.inf, -np.inf, -0.0, 0.0]
    for thr in (0.5, 0.0, float("inf")):
        _, idx, cnt, xm = gather_rows(gpu, x, thr)
        ref, n = oracle.gather(x, thr)
        assert int(cnt.cpu()[0]) == n and np.array_equal(idx.cpu().numpy()[:n], ref)
        want = x.view(np.uint16).copy()
        for b in range(2):
            want[b][~oracle.mask(x[b:b + 1], thr)] = 0
        assert np.array_equal(xm.cpu().numpy().view(np.uint16), want), thr


@pytest.mark.parametrize("batch", [2, 4])
@pytest.mark.parametrize("M,K", [(512, 1024), (1000, 4096)])
def test_rows_keep_their_own_sets(gpu, batch, M, K):
    """y[b] of the union-list GEMV fed the masked copy == the batch-1 oracle of row b alone."""
    torch, spqt, dev = gpu
    Mp = 256 * ((M + 255) // 256)
    w = make_weights(Mp, K, 7100 + M + K)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    W = make_fp_weights(Mp, K, 7101 + M + K)[:M].copy()
    x = make_x(K, "laplace", 7102 + M + K + batch, batch=batch)
    thr = quantile_threshold(x, 0.6)
    say(f"per-row sets M={M} K={K} batch={batch}")
    _, idx, cnt, xm = gather_rows(gpu, x, thr)
    ws = spqt.new_workspace(M, K, batch)
    y = torch.full((batch, M), float("nan"), dtype=torch.float32, device=dev)

    packed = torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)
    spqt.spqt_gemv(packed, M, K, xm, idx, cnt, y, ws)
    torch.cuda.synchronize()
    ref = np.concatenate([oracle.gemv(q, sc, x[b:b + 1], thr) for b in range(batch)], axis=0)
    assert_close(y.cpu().numpy(), ref, "g128 per-row")
    union = oracle.gemv(q, sc, x, thr)
    assert np.abs(union - ref).max() > 1e-3, "the union result must differ, or the test shows nothing"

    packed = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
    y.fill_(float("nan"))
    spqt.spqt_cb_gemv(packed, M, K, xm, idx, cnt, y, ws)
    torch.cuda.synchronize()
    qc, s = cb.quantize(cb.pad_rows(W))
    ref = np.concatenate([cb.gemv(qc, s, x[b:b + 1], thr) for b in range(batch)], axis=0)[:, :M]
    assert_close(y.cpu().numpy(), ref, "cb per-row")


@pytest.mark.parametrize("M,K", [(512, 1024), (999, 2048)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 2), (6, 4)])
def test_fp16_output(gpu, M, K, splits, waves):
    torch, spqt, dev = gpu
    Mp = 256 * ((M + 255) // 256)
    w = make_weights(Mp, K, 7200 + M + K)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    W = make_fp_weights(Mp, K, 7201 + M + K)[:M].copy()
    x1 = make_x(K, "laplace", 7202 + M + K)
    x3 = make_x(K, "laplace", 7203 + M + K, batch=3)
    say(f"fp16 y M={M} K={K} splits={splits} waves={waves}")
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)

    def both(call, batch):
        """Run `call(y)` with an fp32 and an fp16 y (canaries around the fp16 one)."""
        y32 = torch.full((batch, M), float("nan"), dtype=torch.float32, device=dev)
        buf = torch.full((batch * M + 64,), 77.0, dtype=torch.float16, device=dev)
        y16 = buf[32:32 + batch * M].view(batch, M)
        call(y32 if batch > 1 else y32[0])
        call(y16 if batch > 1 else y16[0])
        torch.cuda.synchronize()
        out = buf.cpu().numpy()
        assert np.all(out[:32] == 77.0) and np.all(out[32 + batch * M:] == 77.0), "write outside y"
        a, b = y32.cpu().numpy(), out[32:32 + batch * M].reshape(batch, M)
        assert np.array_equal(a.astype(np.float16).view(np.uint16), b.view(np.uint16)), "fp16 y != RNE(fp32 y)"
        return b

    for x_np, batch in ((x1, 1), (x3, 3)):
        thr = quantile_threshold(x_np, 0.5)
        x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
        xx = x if batch > 1 else x[0]
        ws = spqt.new_workspace(M, K, batch)
        spqt.spqt_gather(xx, thr, idx, cnt)
        packed = torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)
        got = both(lambda y: spqt.spqt_gemv(packed, M, K, xx, idx, cnt, y, ws, splits=splits, waves=waves), batch)
        assert_close(got, oracle.gemv(q, sc, x_np, thr), "g128 fp16")
        got = both(lambda y: spqt.spqt_gemv(packed, M, K, xx, None, None, y, ws, splits=splits, waves=waves), batch)
        assert_close(got, oracle.gemv(q, sc, x_np, 0.0), "g128 dense fp16")
        packed_cb = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
        qc, s = cb.quantize(cb.pad_rows(W))
        got = both(lambda y: spqt.spqt_cb_gemv(packed_cb, M, K, xx, idx, cnt, y, ws, splits=splits, waves=waves), batch)
        assert_close(got, cb.gemv(qc, s, x_np, thr)[:, :M], "cb fp16")
        if batch == 1:
            got = both(lambda y: spqt.spqt_gemv_fused(packed, M, K, xx, thr, y, ws, splits=splits, waves=waves), 1)
            assert_close(got, oracle.gemv(q, sc, x_np, thr), "g128 fused fp16")
            got = both(lambda y: spqt.spqt_cb_gemv_fused(packed_cb, M, K, xx, thr, y, ws, splits=splits, waves=waves), 1)
            assert_close(got, cb.gemv(qc, s, x_np, thr)[:, :M], "cb fused fp16")
            packed_k = torch.from_numpy(spqt.spqt_cbk_quantize(W)).to(dev)
            p = ck.quantize(ck.pad_rows(W))
            got = both(lambda y: spqt.spqt_cbk_gemv(packed_k, M, K, xx, idx, cnt, y, ws, splits=splits, waves=waves), 1)
            assert_close(got, ck.gemv(p, x_np, thr)[:, :M], "cbk fp16")
