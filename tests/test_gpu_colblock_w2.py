"""GPU parity of the 2-bit column-block GEMV (spqt_cb2_gemv, through the C ABI) against the NumPy
oracle oracle/colblock_w2.py on the same seeded inputs.  The packed bytes come from the library's
host quantizer, which the CPU tests pin bit for bit to the oracle's; outputs must satisfy
|y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref| elementwise (fp32 accumulation vs the fp64 oracle)."""
import numpy as np
import pytest

from oracle import colblock_w2 as c2
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


def padded(M):
    return 512 * ((M + 511) // 512)


def run(gpu, packed_np, M, K, x_np, thr, dense=False, splits=0, waves=0, half=False, ws=None):
    torch, spqt, dev = gpu
    packed = torch.from_numpy(packed_np).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    dt = torch.float16 if half else torch.float32
    buf = torch.full((M + 256,), 321.0, dtype=dt, device=dev)
    y = buf[128:128 + M]
    if ws is None:
        ws = spqt.new_workspace(M, K)
    if dense:
        spqt.spqt_cb2_gemv(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_cb2_gemv(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:128] == 321.0) and np.all(out[128 + M:] == 321.0), "write outside y"
    return out[128:128 + M][None, :]


@pytest.mark.parametrize("M,K", [(512, 128), (1024, 1024), (2048, 4096), (1536, 1152), (1, 256), (300, 1024), (1000, 2048)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (2, 4), (7, 2), (16, 4), (3, 1)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_cb2_sparse_gemv(gpu, M, K, splits, waves, sparsity):
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(padded(M), K, 9800 + M + K)[:M].copy()
    x = make_x(K, "laplace", 9801 + M + K)
    thr = quantile_threshold(x, sparsity) if sparsity < 1.0 else float("inf")
    say(f"cb2 M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    c, s = c2.quantize(c2.pad_rows(W))
    ref = c2.gemv(c, s, x, thr)[:, :M]
    assert_close(run(gpu, spqt.spqt_cb2_quantize(W), M, K, x, thr, splits=splits, waves=waves), ref, "cb2 sparse")


@pytest.mark.parametrize("M,K", [(512, 128), (1024, 2048), (1536, 640), (999, 1024)])
def test_cb2_dense_kernel_threshold_zero_and_fp16_output(gpu, M, K):
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(padded(M), K, 9900 + M + K)[:M].copy()
    x = make_x(K, "laplace", 9901 + M + K)
    packed = spqt.spqt_cb2_quantize(W)
    c, s = c2.quantize(c2.pad_rows(W))
    ref = c2.gemv(c, s, x, 0.0)[:, :M]
    say(f"cb2 dense M={M} K={K}")
    d32 = run(gpu, packed, M, K, x, 0.0, dense=True)
    assert_close(d32, ref, "cb2 dense")
    assert_close(run(gpu, packed, M, K, x, 0.0), ref, "cb2 thr=0")
    d16 = run(gpu, packed, M, K, x, 0.0, dense=True, half=True)
    assert np.array_equal(d16.view(np.uint16), d32.astype(np.float16).view(np.uint16)), "fp16 y != RNE(fp32 y)"


def test_cb2_exact_arithmetic_is_bit_exact(gpu):
    """Small-integer x and power-of-two scales: every product and partial sum is exactly
    representable in fp32 (the level offset of 1.5 scales included), so the GPU must equal the oracle
    bit for bit - whatever order it sums in."""
    import paper_2511_04477_amd as spqt
    M, K = 1024, 512
    rng = np.random.default_rng(78)
    c0 = rng.integers(0, 4, size=(M, K)).astype(np.uint8)
    c0.reshape(M // 32, 32, K)[:, 0, :] = 3
    s0 = (2.0 ** rng.integers(-8, -5, size=(M // 32, K))).astype(np.float32)
    W = ((c0.astype(np.float32) - np.float32(1.5)) * np.repeat(s0, 32, axis=0)).astype(np.float32)
    x = rng.integers(-2, 3, size=(1, K)).astype(np.float16)
    c, s = c2.quantize(W)
    assert np.array_equal(c, c0)
    ref = c2.gemv(c, s, x, 1.0)
    say("cb2 exact arithmetic")
    for splits, waves in ((4, 4), (1, 1), (0, 0)):
        got = run(gpu, spqt.spqt_cb2_quantize(W), M, K, x, 1.0, splits=splits, waves=waves)
        assert np.array_equal(got.astype(np.float64), ref), (splits, waves)


def test_cb2_column_probe(gpu):
    """x = a * e_k: y must be a * (column k of the dequantized matrix) exactly, for every k - each of the
    512 rows of a block-row picks its own 2-bit field and its own block's scale."""
    import paper_2511_04477_amd as spqt
    M, K = 1024, 256
    W = make_fp_weights(M, K, 9950)
    packed = spqt.spqt_cb2_quantize(W)
    c, s = c2.quantize(W)
    Wd = c2.dequant(c, s)
    say("cb2 column probe")
    for k in list(range(0, K, 5)) + [K - 1]:
        e = np.zeros((1, K), dtype=np.float16)
        e[0, k] = 2.0
        got = run(gpu, packed, M, K, e, 1.0, splits=2, waves=2)
        assert np.array_equal(got[0].astype(np.float64), 2.0 * Wd[:, k]), k


def test_cb2_every_code_at_every_field(gpu):
    """One column whose 512 rows cycle through the four codes with a shift per row, scale 1: the 16 field
    positions of a dword each see all four codes, the three fields above the mantissa bits included."""
    import paper_2511_04477_amd as spqt
    M, K = 512, 128
    W = np.zeros((M, K), dtype=np.float32)
    for k in range(4):
        codes = (np.arange(M) + k) % 4
        codes.reshape(16, 32)[:, 0] = 3 if k % 2 == 0 else 0     # an outer level in every block: scale 1
        W[:, k] = codes.astype(np.float32) - 1.5
    c, s = c2.quantize(W)
    assert np.all(s[:, :4].astype(np.float32) == 1.0)
    say("cb2 fields")
    for k in range(4):
        e = np.zeros((1, K), dtype=np.float16)
        e[0, k] = 1.0
        got = run(gpu, spqt.spqt_cb2_quantize(W), M, K, e, 0.5, splits=1, waves=1)
        assert np.array_equal(got[0], W[:, k]), k


def test_cb2_shares_a_workspace_with_the_other_kernels(gpu):
    """The exchange area is left all zero by every call, so one workspace serves 4-bit, 8-bit and 2-bit
    calls in any order."""
    torch, spqt, dev = gpu
    from oracle import colblock as c4
    M, K = 2048, 2048
    W = make_fp_weights(M, K, 9970)
    x = make_x(K, "laplace", 9971)
    thr = quantile_threshold(x, 0.5)
    ws = spqt.new_workspace(M, K)
    c, s = c2.quantize(W)
    ref2 = c2.gemv(c, s, x, thr)
    q, s4 = c4.quantize(W)
    ref4 = c4.gemv(q, s4, x, thr)
    p2 = spqt.spqt_cb2_quantize(W)
    p4 = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
    xd = torch.from_numpy(x[0].copy()).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y4 = torch.zeros(M, dtype=torch.float32, device=dev)
    say("cb2 shared workspace")
    for rep in range(3):
        assert_close(run(gpu, p2, M, K, x, thr, splits=4, ws=ws), ref2, f"2-bit, round {rep}")
        spqt.spqt_gather(xd, thr, idx, cnt)
        spqt.spqt_cb_gemv(p4, M, K, xd, idx, cnt, y4, ws, splits=8)
        torch.cuda.synchronize()
        assert_close(y4.cpu().numpy()[None, :], ref4, f"4-bit, round {rep}")


def test_cb2_full_size_sampled_tiles_and_repeat(gpu):
    """The 70B gate shape in the default launch configuration, checked on sampled block-rows; a
    second call on the same workspace must give the same bits (fixed summation order)."""
    torch, spqt, dev = gpu
    M, K = 28672, 8192
    W = make_fp_weights(M, K, 9960)
    x = make_x(K, "laplace", 9961)
    thr = quantile_threshold(x, 0.5)
    packed = torch.from_numpy(spqt.spqt_cb2_quantize(W)).to(dev)
    xd = torch.from_numpy(x[0].copy()).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y = torch.zeros(M, dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    say("cb2 full size")
    spqt.spqt_gather(xd, thr, idx, cnt)
    spqt.spqt_cb2_gemv(packed, M, K, xd, idx, cnt, y, ws)
    torch.cuda.synchronize()
    first = y.cpu().numpy().copy()
    y.zero_()
    spqt.spqt_cb2_gemv(packed, M, K, xd, idx, cnt, y, ws)
    torch.cuda.synchronize()
    assert np.array_equal(first.view(np.uint32), y.cpu().numpy().view(np.uint32))
    for t in (0, 27, 55):
        rows = slice(512 * t, 512 * t + 512)
        c, s = c2.quantize(W[rows])
        assert_close(first[None, rows], c2.gemv(c, s, x, thr), f"block-row {t}")
    yd = torch.zeros(M, dtype=torch.float32, device=dev)
    spqt.spqt_cb2_gemv(packed, M, K, xd, None, None, yd, ws)
    torch.cuda.synchronize()
    for t in (3, 40):
        rows = slice(512 * t, 512 * t + 512)
        c, s = c2.quantize(W[rows])
        assert_close(yd.cpu().numpy()[None, rows], c2.gemv(c, s, x, 0.0), f"dense block-row {t}")


def run_one_launch(gpu, packed_np, M, K, x_np, thr, splits=0, waves=0, half=False):
    torch, spqt, dev = gpu
    packed = torch.from_numpy(packed_np).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    buf = torch.full((M + 256,), 321.0, dtype=torch.float16 if half else torch.float32, device=dev)
    y = buf[128:128 + M]
    spqt.spqt_cb2_gemv_fused(packed, M, K, x, thr, y, spqt.new_workspace(M, K), splits=splits, waves=waves)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:128] == 321.0) and np.all(out[128 + M:] == 321.0), "write outside y"
    return out[128:128 + M][None, :]


@pytest.mark.parametrize("M,K", [(512, 128), (1024, 1024), (2048, 4096), (1, 256), (300, 1024), (1536, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (2, 4), (7, 2), (16, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_cb2_one_launch(gpu, M, K, splits, waves, sparsity):
    """Gather and GEMV in one launch: the oracle's y for the same threshold (no list exists to compare)."""
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(512 * ((M + 511) // 512), K, 9002 + M + K)[:M].copy()
    x = make_x(K, "laplace", 9102 + M + K)
    thr = quantile_threshold(x, sparsity) if sparsity < 1.0 else float("inf")
    say(f"cb2 one launch M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    q, s = c2.quantize(c2.pad_rows(W))
    ref = c2.gemv(q, s, x, thr)[:, :M]
    got = run_one_launch(gpu, spqt.spqt_cb2_quantize(W), M, K, x, thr, splits=splits, waves=waves)
    assert_close(got, ref, "cb2 one launch")


def test_cb2_one_launch_clustered_ties_and_fp16(gpu):
    """Kept columns all in one corner of x (whole units empty), entries equal to the threshold (kept), fp16 y."""
    import paper_2511_04477_amd as spqt
    M, K = 1536, 1024
    W = make_fp_weights(M, K, 9302)
    x = np.zeros((1, K), dtype=np.float16)
    rng = np.random.default_rng(9402)
    x[0, 640:768] = rng.standard_normal(128).astype(np.float16)
    x[0, 5] = 0.5
    x[0, 1023] = -0.5
    thr = 0.5
    q, s = c2.quantize(W)
    ref = c2.gemv(q, s, x, thr)
    assert c2.keep_mask(x, thr)[5] and c2.keep_mask(x, thr)[1023]
    say("cb2 one launch clustered")
    packed = spqt.spqt_cb2_quantize(W)
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
        spqt.spqt_cb2_gemv_rows(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_cb2_gemv_rows(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:128] == 321.0) and np.all(out[128 + B * M:] == 321.0), "write outside y"
    return out[128:128 + B * M].reshape(B, M)


@pytest.mark.parametrize("M,K", [(512, 128), (1024, 1024), (2048, 2048), (300, 1024)])
@pytest.mark.parametrize("batch", [2, 3])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (3, 2), (8, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9])
def test_cb2_several_rows_on_the_union_list(gpu, M, K, batch, splits, waves, sparsity):
    """Several activation rows share the union of their kept columns and one pass over the weights:
    every listed column contributes to every row, as the oracle's batch form does."""
    import paper_2511_04477_amd as spqt
    W = make_fp_weights(512 * ((M + 511) // 512), K, 9502 + M + K)[:M].copy()
    x = make_x(K, "laplace", 9602 + M + K, batch=batch)
    thr = quantile_threshold(x, sparsity)
    say(f"cb2 rows M={M} K={K} batch={batch} splits={splits} waves={waves} s={sparsity}")
    q, s = c2.quantize(c2.pad_rows(W))
    ref = c2.gemv(q, s, x, thr)[:, :M]
    assert_close(run_rows(gpu, spqt.spqt_cb2_quantize(W), M, K, x, thr, splits=splits, waves=waves), ref, "cb2 rows")


def test_cb2_rows_dense_fp16_and_limits(gpu):
    """Dense mode with several rows, fp16 output, one row through the rows entry point equals the batch-1 entry
    point bit for bit, and a row count past the limit is refused."""
    torch, spqt, dev = gpu
    M, K = 1024, 1024
    W = make_fp_weights(M, K, 9702)
    x = make_x(K, "laplace", 9703, batch=3)
    packed = spqt.spqt_cb2_quantize(W)
    q, s = c2.quantize(W)
    say("cb2 rows dense")
    d32 = run_rows(gpu, packed, M, K, x, 0.0, dense=True)
    assert_close(d32, c2.gemv(q, s, x, 0.0), "rows dense")
    d16 = run_rows(gpu, packed, M, K, x, 0.0, dense=True, half=True)
    assert np.array_equal(d16.view(np.uint16), d32.astype(np.float16).view(np.uint16))
    thr = quantile_threshold(x[0:1], 0.5)
    one = run_rows(gpu, packed, M, K, x[0:1], thr, splits=4, waves=4)
    assert np.array_equal(one.view(np.uint32), run(gpu, packed, M, K, x[0:1], thr, splits=4, waves=4).view(np.uint32))
    xb = torch.zeros((4, K), dtype=torch.float16, device=dev)
    yb = torch.zeros((4) * M, dtype=torch.float32, device=dev)
    with pytest.raises(spqt.SpqtError):
        spqt.spqt_cb2_gemv_rows(torch.from_numpy(packed).to(dev), M, K, xb, None, None, yb, spqt.new_workspace(M, K, 4))
