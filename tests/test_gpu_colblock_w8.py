"""GPU parity of the 8-bit column-block GEMV (spqt_cb8_gemv, through the C ABI) against the NumPy
oracle oracle/colblock_w8.py on the same seeded inputs.  The packed bytes come from the library's
host quantizer, which the CPU tests pin bit for bit to the oracle's; outputs must satisfy
|y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref| elementwise (fp32 accumulation vs the fp64 oracle)."""
import numpy as np
import pytest

from oracle import colblock_w8 as c8
from workloads import make_fp_weights, make_x, quantile_threshold

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


def run(gpu, packed_np, M, K, x_np, thr, dense=False, splits=0, waves=0, half=False):
    torch, spqt, dev = gpu
    packed = torch.from_numpy(packed_np).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    dt = torch.float16 if half else torch.float32
    buf = torch.full((M + 256,), 321.0, dtype=dt, device=dev)
    y = buf[128:128 + M]
    ws = spqt.new_workspace(M, K)
    if dense:
        spqt.spqt_cb8_gemv(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_cb8_gemv(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:128] == 321.0) and np.all(out[128 + M:] == 321.0), "write outside y"
    return out[128:128 + M][None, :]


@pytest.mark.parametrize("M,K", [(128, 128), (512, 1024), (1024, 4096), (2048, 1152), (1, 256), (300, 1024), (1000, 2048)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (2, 4), (7, 2), (16, 4), (64, 1)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_cb8_sparse_gemv(gpu, M, K, splits, waves, sparsity):
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(128 * ((M + 127) // 128), K, 8800 + M + K)[:M].copy()
    x = make_x(K, "laplace", 8801 + M + K)
    thr = quantile_threshold(x, sparsity) if sparsity < 1.0 else float("inf")
    say(f"cb8 M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    q, s = c8.quantize(c8.pad_rows(W))
    ref = c8.gemv(q, s, x, thr)[:, :M]
    assert_close(run(gpu, spqt.spqt_cb8_quantize(W), M, K, x, thr, splits=splits, waves=waves), ref, "cb8 sparse")


@pytest.mark.parametrize("M,K", [(128, 128), (1024, 2048), (768, 640), (999, 1024)])
def test_cb8_dense_kernel_threshold_zero_and_fp16_output(gpu, M, K):
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(128 * ((M + 127) // 128), K, 8900 + M + K)[:M].copy()
    x = make_x(K, "laplace", 8901 + M + K)
    packed = spqt.spqt_cb8_quantize(W)
    q, s = c8.quantize(c8.pad_rows(W))
    ref = c8.gemv(q, s, x, 0.0)[:, :M]
    say(f"cb8 dense M={M} K={K}")
    d32 = run(gpu, packed, M, K, x, 0.0, dense=True)
    assert_close(d32, ref, "cb8 dense")
    assert_close(run(gpu, packed, M, K, x, 0.0), ref, "cb8 thr=0")
    d16 = run(gpu, packed, M, K, x, 0.0, dense=True, half=True)
    assert np.array_equal(d16.view(np.uint16), d32.astype(np.float16).view(np.uint16)), "fp16 y != RNE(fp32 y)"


def test_cb8_exact_arithmetic_is_bit_exact(gpu):
    """Small-integer x and power-of-two scales: every product and partial sum is exactly
    representable in fp32 (the bias term included), so the GPU must equal the oracle bit for bit."""
    import paper_2511_04477_amd as spqt
    M, K = 512, 512
    rng = np.random.default_rng(77)
    q0 = rng.integers(-127, 128, size=(M, K)).astype(np.int16)
    q0.reshape(M // 32, 32, K)[:, 0, :] = 127
    s0 = (2.0 ** rng.integers(-8, -5, size=(M // 32, K))).astype(np.float32)
    W = (q0.astype(np.float32) * np.repeat(s0, 32, axis=0)).astype(np.float32)
    x = rng.integers(-2, 3, size=(1, K)).astype(np.float16)
    q, s = c8.quantize(W)
    assert np.array_equal(q, q0)
    ref = c8.gemv(q, s, x, 1.0)
    got = run(gpu, spqt.spqt_cb8_quantize(W), M, K, x, 1.0, splits=4, waves=4)
    assert np.array_equal(got.astype(np.float64), ref)


def test_cb8_column_probe(gpu):
    """x = c * e_k: y must be c * (column k of the dequantized matrix) exactly, for every k."""
    import paper_2511_04477_amd as spqt
    M, K = 256, 256
    W = make_fp_weights(M, K, 8950)
    packed = spqt.spqt_cb8_quantize(W)
    q, s = c8.quantize(W)
    Wd = c8.dequant(q, s)
    for k in list(range(0, K, 5)) + [K - 1]:
        e = np.zeros((1, K), dtype=np.float16)
        e[0, k] = 2.0
        got = run(gpu, packed, M, K, e, 1.0, splits=2, waves=2)
        assert np.array_equal(got[0].astype(np.float64), 2.0 * Wd[:, k]), k


def test_cb8_full_size_sampled_tiles_and_repeat(gpu):
    """The 70B gate shape in the default launch configuration, checked on sampled block-rows; a
    second call on the same workspace must give the same bits (fixed summation order)."""
    torch, spqt, dev = gpu
    M, K = 28672, 8192
    W = make_fp_weights(M, K, 8960)
    x = make_x(K, "laplace", 8961)
    thr = quantile_threshold(x, 0.5)
    packed = torch.from_numpy(spqt.spqt_cb8_quantize(W)).to(dev)
    xd = torch.from_numpy(x[0].copy()).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y = torch.zeros(M, dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    spqt.spqt_gather(xd, thr, idx, cnt)
    spqt.spqt_cb8_gemv(packed, M, K, xd, idx, cnt, y, ws)
    torch.cuda.synchronize()
    first = y.cpu().numpy().copy()
    y.zero_()
    spqt.spqt_cb8_gemv(packed, M, K, xd, idx, cnt, y, ws)
    torch.cuda.synchronize()
    assert np.array_equal(first.view(np.uint32), y.cpu().numpy().view(np.uint32))
    for t in (0, 111, 223):
        rows = slice(128 * t, 128 * t + 128)
        q, s = c8.quantize(W[rows])
        assert_close(first[None, rows], c8.gemv(q, s, x, thr), f"block-row {t}")


def run_one_launch(gpu, packed_np, M, K, x_np, thr, splits=0, waves=0, half=False):
    torch, spqt, dev = gpu
    packed = torch.from_numpy(packed_np).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    buf = torch.full((M + 256,), 321.0, dtype=torch.float16 if half else torch.float32, device=dev)
    y = buf[128:128 + M]
    spqt.spqt_cb8_gemv_fused(packed, M, K, x, thr, y, spqt.new_workspace(M, K), splits=splits, waves=waves)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:128] == 321.0) and np.all(out[128 + M:] == 321.0), "write outside y"
    return out[128:128 + M][None, :]


@pytest.mark.parametrize("M,K", [(128, 128), (512, 1024), (1024, 4096), (1, 256), (300, 1024), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (2, 4), (7, 2), (16, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_cb8_one_launch(gpu, M, K, splits, waves, sparsity):
    """Gather and GEMV in one launch: the oracle's y for the same threshold (no list exists to compare)."""
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(128 * ((M + 127) // 128), K, 9008 + M + K)[:M].copy()
    x = make_x(K, "laplace", 9108 + M + K)
    thr = quantile_threshold(x, sparsity) if sparsity < 1.0 else float("inf")
    say(f"cb8 one launch M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    q, s = c8.quantize(c8.pad_rows(W))
    ref = c8.gemv(q, s, x, thr)[:, :M]
    got = run_one_launch(gpu, spqt.spqt_cb8_quantize(W), M, K, x, thr, splits=splits, waves=waves)
    assert_close(got, ref, "cb8 one launch")


def test_cb8_one_launch_clustered_ties_and_fp16(gpu):
    """Kept columns all in one corner of x (whole units empty), entries equal to the threshold (kept), fp16 y."""
    import paper_2511_04477_amd as spqt
    M, K = 384, 1024
    W = make_fp_weights(M, K, 9308)
    x = np.zeros((1, K), dtype=np.float16)
    rng = np.random.default_rng(9408)
    x[0, 640:768] = rng.standard_normal(128).astype(np.float16)
    x[0, 5] = 0.5
    x[0, 1023] = -0.5
    thr = 0.5
    q, s = c8.quantize(W)
    ref = c8.gemv(q, s, x, thr)
    assert c8.keep_mask(x, thr)[5] and c8.keep_mask(x, thr)[1023]
    say("cb8 one launch clustered")
    packed = spqt.spqt_cb8_quantize(W)
    got = run_one_launch(gpu, packed, M, K, x, thr, splits=4, waves=4)
    assert_close(got, ref, "clustered")
    h = run_one_launch(gpu, packed, M, K, x, thr, splits=4, waves=4, half=True)
    assert np.array_equal(h.view(np.uint16), got.astype(np.float16).view(np.uint16))


def run_rows(gpu, packed_np, M, K, x_np, thr, dense=False, splits=0, waves=0, half=False):
    torch, spqt, dev = gpu
    B = x_np.shape[0]
    packed = torch.from_numpy(packed_np).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    buf = torch.full((B * M + 256,), 321.0, dtype=torch.float16 if half else torch.float32, device=dev)
    y = buf[128:128 + B * M]
    ws = spqt.new_workspace(M, K, B)
    if dense:
        spqt.spqt_cb8_gemv_rows(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_cb8_gemv_rows(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:128] == 321.0) and np.all(out[128 + B * M:] == 321.0), "write outside y"
    return out[128:128 + B * M].reshape(B, M)


@pytest.mark.parametrize("M,K", [(128, 128), (512, 1024), (1024, 2048), (300, 1024)])
@pytest.mark.parametrize("batch", [2, 3, 4])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (3, 2), (8, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9])
def test_cb8_several_rows_on_the_union_list(gpu, M, K, batch, splits, waves, sparsity):
    """Several activation rows share the union of their kept columns and one pass over the weights:
    every listed column contributes to every row, as the oracle's batch form does."""
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(128 * ((M + 127) // 128), K, 9508 + M + K)[:M].copy()
    x = make_x(K, "laplace", 9608 + M + K, batch=batch)
    thr = quantile_threshold(x, sparsity)
    say(f"cb8 rows M={M} K={K} batch={batch} splits={splits} waves={waves} s={sparsity}")
    q, s = c8.quantize(c8.pad_rows(W))
    ref = c8.gemv(q, s, x, thr)[:, :M]
    assert_close(run_rows(gpu, spqt.spqt_cb8_quantize(W), M, K, x, thr, splits=splits, waves=waves), ref, "cb8 rows")


def test_cb8_rows_dense_fp16_and_limits(gpu):
    """Dense mode with several rows, fp16 output, one row through the rows entry point equals the batch-1 entry
    point bit for bit, and a row count past the limit is refused."""
    torch, spqt, dev = gpu
    M, K = 256, 1024
    W = make_fp_weights(M, K, 9708)
    x = make_x(K, "laplace", 9709, batch=4)
    packed = spqt.spqt_cb8_quantize(W)
    q, s = c8.quantize(W)
    say("cb8 rows dense")
    d32 = run_rows(gpu, packed, M, K, x, 0.0, dense=True)
    assert_close(d32, c8.gemv(q, s, x, 0.0), "rows dense")
    d16 = run_rows(gpu, packed, M, K, x, 0.0, dense=True, half=True)
    assert np.array_equal(d16.view(np.uint16), d32.astype(np.float16).view(np.uint16))
    thr = quantile_threshold(x[0:1], 0.5)
    one = run_rows(gpu, packed, M, K, x[0:1], thr, splits=4, waves=4)
    assert np.array_equal(one.view(np.uint32), run(gpu, packed, M, K, x[0:1], thr, splits=4, waves=4).view(np.uint32))
    xb = torch.zeros((5, K), dtype=torch.float16, device=dev)
    yb = torch.zeros((5) * M, dtype=torch.float32, device=dev)
    with pytest.raises(spqt.SpqtError):
        spqt.spqt_cb8_gemv_rows(torch.from_numpy(packed).to(dev), M, K, xb, None, None, yb, spqt.new_workspace(M, K, 4))
