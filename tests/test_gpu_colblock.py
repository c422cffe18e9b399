"""GPU parity of the column-block GEMV (spqt_cb_gemv, through the C ABI) against the NumPy oracle
oracle/colblock.py on the same seeded inputs.  The packed bytes come from the library's host
quantizer, which the CPU tests pin bit for bit to the oracle's; outputs must satisfy
|y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref| elementwise (fp32 accumulation vs the fp64 oracle)."""
import numpy as np
import pytest

from oracle import colblock as cb
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


def gpu_cb_gemv(gpu, W, x_np, thr, dense=False, splits=0, waves=0, packed=None):
    torch, spqt, dev = gpu
    M, K = W.shape
    if packed is None:
        packed = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    y = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    if dense:
        spqt.spqt_cb_gemv(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_cb_gemv(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    return y.cpu().numpy()[None, :]


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1024, 4096), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (2, 4), (7, 2), (16, 4), (64, 1)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_cb_sparse_gemv(gpu, M, K, splits, waves, sparsity):
    W = make_fp_weights(M, K, 8100 + M + K)
    x = make_x(K, "laplace", 8101 + M + K)
    thr = quantile_threshold(x, sparsity)
    say(f"cb M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    q, s = cb.quantize(W)
    ref = cb.gemv(q, s, x, thr)
    assert_close(gpu_cb_gemv(gpu, W, x, thr, splits=splits, waves=waves), ref, "cb sparse")


def gpu_cb_gemv_fused(gpu, W, x_np, thr, splits=0, waves=0, packed=None):
    torch, spqt, dev = gpu
    M, K = W.shape
    if packed is None:
        packed = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    y = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    spqt.spqt_cb_gemv_fused(packed, M, K, x, thr, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    return y.cpu().numpy()[None, :]


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1024, 4096), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (2, 4), (7, 2), (16, 4), (64, 1)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_cb_fused_gemv(gpu, M, K, splits, waves, sparsity):
    """One launch: threshold, in-wave compaction and the column-block GEMV."""
    W = make_fp_weights(M, K, 8700 + M + K)
    x = make_x(K, "laplace_clustered" if sparsity == 0.9 else "laplace", 8701 + M + K)
    thr = quantile_threshold(x, sparsity)
    say(f"cb fused M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    q, s = cb.quantize(W)
    ref = cb.gemv(q, s, x, thr)
    assert_close(gpu_cb_gemv_fused(gpu, W, x, thr, splits=splits, waves=waves), ref, "cb fused")


def test_cb_fused_ties_empty_units_and_exact(gpu):
    M, K = 1024, 2048
    W = make_fp_weights(M, K, 8800)
    x = make_x(K, "laplace", 8801)
    x[0, 0:512] = 0            # empty 64-column units
    x[0, 700] = 3.0
    x[0, 1024:1152] = 2.0      # two full units
    x[0, 1500] = 0.75          # a tie with the threshold is kept
    thr = 0.75
    q, s = cb.quantize(W)
    ref = cb.gemv(q, s, x, thr)
    for splits, waves in [(0, 0), (1, 1), (5, 4), (16, 2)]:
        assert_close(gpu_cb_gemv_fused(gpu, W, x, thr, splits=splits, waves=waves), ref, f"cb fused {splits}x{waves}")
    rng = np.random.default_rng(8802)
    q0 = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    q0.reshape(M // 32, 32, K)[:, 0, :] = 7
    s0 = (2.0 ** rng.integers(-8, -3, size=(M // 32, K))).astype(np.float32)
    We = q0.astype(np.float32) * np.repeat(s0, 32, axis=0)
    xi = rng.integers(-4, 5, size=(1, K)).astype(np.float16)
    qe, se = cb.quantize(We)
    got = gpu_cb_gemv_fused(gpu, We, xi, 2.0)
    assert np.array_equal(got.astype(np.float64), cb.gemv(qe, se, xi, 2.0))


@pytest.mark.parametrize("batch", [2, 3, 4])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 4), (5, 2), (16, 4)])
def test_cb_batch_rows_share_one_pass(gpu, batch, splits, waves):
    """Batch 2-4: union index list, every row its own x values on the union set."""
    torch, spqt, dev = gpu
    M, K = 1024, 2048
    W = make_fp_weights(M, K, 8900 + batch)
    x_np = make_x(K, "laplace", 8901 + batch, batch=batch)
    thr = 0.9
    q, s = cb.quantize(W)
    ref = cb.gemv(q, s, x_np, thr)
    packed = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
    x = torch.from_numpy(x_np).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    spqt.spqt_gather(x, thr, idx, cnt)
    ws = spqt.new_workspace(M, K, batch)
    y = torch.full((batch, M), float("nan"), dtype=torch.float32, device=dev)
    spqt.spqt_cb_gemv(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy(), ref, f"cb batch {batch} sparse")
    yd = torch.full((batch, M), float("nan"), dtype=torch.float32, device=dev)
    spqt.spqt_cb_gemv(packed, M, K, x, None, None, yd, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    assert_close(yd.cpu().numpy(), cb.gemv(q, s, x_np, 0.0), f"cb batch {batch} dense")
    # identical rows must reproduce the batch-1 result bit for bit
    xi = torch.from_numpy(np.repeat(x_np[0:1], batch, axis=0).copy()).to(dev)
    spqt.spqt_gather(xi, thr, idx, cnt)
    spqt.spqt_cb_gemv(packed, M, K, xi, idx, cnt, y, ws, splits=splits, waves=waves)
    y1 = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
    spqt.spqt_cb_gemv(packed, M, K, xi[0].contiguous(), idx, cnt, y1, spqt.new_workspace(M, K), splits=splits, waves=waves)
    torch.cuda.synchronize()
    for b in range(batch):
        assert np.array_equal(y[b].cpu().numpy(), y1.cpu().numpy()), b


@pytest.mark.parametrize("M,K", [(256, 128), (1024, 2048), (768, 640)])
def test_cb_dense_kernel_and_threshold_zero(gpu, M, K):
    W = make_fp_weights(M, K, 8200 + M + K)
    x = make_x(K, "normal", 8201 + M + K)
    q, s = cb.quantize(W)
    ref = cb.gemv(q, s, x, 0.0)
    for splits, waves in [(0, 0), (1, 4), (5, 2)]:
        say(f"cb dense M={M} K={K} {splits}x{waves}")
        d = gpu_cb_gemv(gpu, W, x, 0.0, dense=True, splits=splits, waves=waves)
        z = gpu_cb_gemv(gpu, W, x, 0.0, dense=False, splits=splits, waves=waves)
        assert_close(d, ref, "cb dense")
        assert np.array_equal(d, z), "index-free kernel and threshold 0 must agree bit for bit"


def test_cb_exact_arithmetic_is_bit_exact(gpu):
    """Power-of-two scales, codes that hit them exactly, small integer x: every product and
    partial sum is representable, so any summation order gives the oracle's result exactly."""
    M, K = 512, 1024
    rng = np.random.default_rng(8300)
    q0 = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    q0.reshape(M // 32, 32, K)[:, 0, :] = 7
    s0 = (2.0 ** rng.integers(-8, -3, size=(M // 32, K))).astype(np.float32)
    W = q0.astype(np.float32) * np.repeat(s0, 32, axis=0)
    x = rng.integers(-4, 5, size=(1, K)).astype(np.float16)
    q, s = cb.quantize(W)
    assert np.array_equal(q, q0)
    ref = cb.gemv(q, s, x, 2.0)
    for splits, waves in [(0, 0), (3, 4), (16, 1)]:
        got = gpu_cb_gemv(gpu, W, x, 2.0, splits=splits, waves=waves)
        assert np.array_equal(got.astype(np.float64), ref), f"{splits}x{waves}"


def test_cb_column_probe(gpu):
    """x = c e_k reads exactly column k: y = c * dequant(W)[:, k] - any address mix-up shows."""
    torch, spqt, dev = gpu
    M, K = 512, 384
    W = make_fp_weights(M, K, 8400)
    q, s = cb.quantize(W)
    Wd = cb.dequant(q, s)
    packed = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
    for k in list(range(0, K, 7)) + [K - 1]:
        e = np.zeros((1, K), dtype=np.float16)
        e[0, k] = -1.5
        got = gpu_cb_gemv(gpu, W, e, 0.5, packed=packed)[0].astype(np.float64)
        want = (-1.5 * Wd[:, k]).astype(np.float32).astype(np.float64)
        assert np.array_equal(got, want), k


def test_cb_clustered_and_reproducible(gpu):
    M, K = 1024, 2048
    W = make_fp_weights(M, K, 8500)
    x = make_x(K, "laplace_clustered", 8501)
    x[0, 0:300] = 0
    x[0, 1000] = 0.75            # a tie with the threshold is kept
    thr = 0.75
    q, s = cb.quantize(W)
    ref = cb.gemv(q, s, x, thr)
    first = None
    for rep in range(10):
        got = gpu_cb_gemv(gpu, W, x, thr)
        assert_close(got, ref, "cb clustered")
        first = got if first is None else first
        assert np.array_equal(got, first), "results must be reproducible"


def test_cb_full_size_sampled_rows(gpu):
    """The benchmark's shapes in the default launch configuration, checked on sampled 256-row
    tiles (the oracle computes any subset of tiles independently)."""
    torch, spqt, dev = gpu
    for M, K in [(4096, 4096), (28672, 8192), (8192, 28672)]:
        say(f"cb full size {M}x{K}")
        W = make_fp_weights(M, K, 8600 + M)
        x = make_x(K, "laplace", 8601 + M)
        thr = quantile_threshold(x, 0.5)
        packed = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
        got = gpu_cb_gemv(gpu, W, x, thr, packed=packed)[0]
        gotd = gpu_cb_gemv(gpu, W, x, thr, dense=True, packed=packed)[0]
        gotf = gpu_cb_gemv_fused(gpu, W, x, thr, packed=packed)[0]
        rng = np.random.default_rng(M)
        tiles = np.unique(np.concatenate([[0, M // 256 - 1], rng.integers(0, M // 256, size=3)]))
        rows = (tiles[:, None] * 256 + np.arange(256)[None, :]).ravel()
        q, s = cb.quantize(W[rows])           # blocks are quantized independently of each other
        assert_close(got[rows][None, :], cb.gemv(q, s, x, thr), f"cb {M}x{K} sparse")
        assert_close(gotd[rows][None, :], cb.gemv(q, s, x, 0.0), f"cb {M}x{K} dense")
        assert_close(gotf[rows][None, :], cb.gemv(q, s, x, thr), f"cb {M}x{K} fused")
        del packed
        del W


def test_cb_hip_graph_replay_matches_eager(gpu):
    """A whole little sequence (workspace init, gather, list-driven, dense and one-launch column-block
    GEMVs plus the group-layout one-launch GEMV on the same x) captured in one HIP graph and replayed
    with eager work and synchronizations in between: every replay reproduces the eager results."""
    torch, spqt, dev = gpu
    from workloads import make_weights
    import oracle
    M, K = 1024, 2048
    W = make_fp_weights(M, K, 9300)
    gw = make_weights(M, K, 9301)
    x_np = make_x(K, "laplace", 9302)
    thr = quantile_threshold(x_np, 0.5)
    packed = torch.from_numpy(spqt.spqt_cb_quantize(W)).to(dev)
    gpacked = torch.from_numpy(spqt.spqt_pack(gw["q_rowmajor"], gw["scales"])).to(dev)
    x = torch.from_numpy(x_np[0]).to(dev)
    idx = torch.zeros(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    ys = [torch.zeros(M, dtype=torch.float32, device=dev) for _ in range(4)]
    ws = spqt.new_workspace(M, K)

    def run():
        spqt.spqt_workspace_init(ws)          # a fill kernel, safe under capture
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_cb_gemv(packed, M, K, x, idx, cnt, ys[0], ws, splits=8)
        spqt.spqt_cb_gemv(packed, M, K, x, None, None, ys[1], ws, splits=4)
        spqt.spqt_cb_gemv_fused(packed, M, K, x, thr, ys[2], ws, splits=8)
        spqt.spqt_gemv_fused(gpacked, M, K, x, thr, ys[3], ws, splits=8)

    run()
    torch.cuda.synchronize()
    eager = [y.cpu().numpy().copy() for y in ys]
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for rep in range(5):
        for y in ys:
            y.fill_(float("nan"))
        idx.fill_(-1)
        scratch = torch.randn(1 << 16, device=dev).sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for j, y in enumerate(ys):
            assert np.array_equal(y.cpu().numpy(), eager[j]), (rep, j)
        assert float(scratch) == float(scratch)
    q, s = cb.quantize(W)
    assert_close(eager[0][None, :], cb.gemv(q, s, x_np, thr), "graph: cb list")
    assert_close(eager[1][None, :], cb.gemv(q, s, x_np, 0.0), "graph: cb dense")
    assert_close(eager[2][None, :], cb.gemv(q, s, x_np, thr), "graph: cb fused")
    assert_close(eager[3][None, :], oracle.gemv(gw["q_rowmajor"], gw["scales"], x_np, thr), "graph: group fused")


# ------------------------------------------------------------------ K-quant flavour (spqt_cbk_*)

def gpu_cbk_gemv(gpu, W, x_np, thr, dense=False, splits=0, waves=0, packed=None):
    torch, spqt, dev = gpu
    M, K = W.shape
    if packed is None:
        packed = torch.from_numpy(spqt.spqt_cbk_quantize(W)).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    y = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    if dense:
        spqt.spqt_cbk_gemv(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_cbk_gemv(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    return y.cpu().numpy()[None, :]


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1024, 4096), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (7, 2), (16, 4), (64, 1)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_cbk_sparse_gemv(gpu, M, K, splits, waves, sparsity):
    from oracle import colblock_k as ck
    W = make_fp_weights(M, K, 9400 + M + K)
    W += np.float32(0.01)          # off-centre weights: the minima matter
    x = make_x(K, "laplace", 9401 + M + K)
    thr = quantile_threshold(x, sparsity)
    say(f"cbk M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    ref = ck.gemv(ck.quantize(W), x, thr)
    assert_close(gpu_cbk_gemv(gpu, W, x, thr, splits=splits, waves=waves), ref, "cbk sparse")


def test_cbk_dense_exact_and_probe(gpu):
    from oracle import colblock_k as ck
    torch, spqt, dev = gpu
    M, K = 512, 384
    W = make_fp_weights(M, K, 9500) - np.float32(0.02)
    p = ck.quantize(W)
    x = make_x(K, "normal", 9501)
    for splits, waves in [(0, 0), (3, 4)]:
        d = gpu_cbk_gemv(gpu, W, x, 0.0, dense=True, splits=splits, waves=waves)
        z = gpu_cbk_gemv(gpu, W, x, 0.0, dense=False, splits=splits, waves=waves)
        assert_close(d, ck.gemv(p, x, 0.0), "cbk dense")
        assert np.array_equal(d, z)
    # column probe: x = c e_k gives c * value[:, k] exactly (one product, one subtraction per row)
    Wd = ck.dequant(p)
    packed = torch.from_numpy(spqt.spqt_cbk_quantize(W)).to(dev)
    for k in list(range(0, K, 11)) + [K - 1]:
        e = np.zeros((1, K), dtype=np.float16)
        e[0, k] = 2.0
        got = gpu_cbk_gemv(gpu, W, e, 1.0, packed=packed)[0].astype(np.float64)
        assert np.array_equal(got, (2.0 * Wd[:, k]).astype(np.float32).astype(np.float64)), k
    # exactly representable superblocks and small integer x: bit-exact whatever the summation order
    rng = np.random.default_rng(9502)
    T = M // 256
    d16 = (2.0 ** rng.integers(-10, -6, size=(T, K))).astype(np.float32)
    sc = rng.integers(16, 64, size=(M // 32, K)); sc.reshape(T, 8, K)[:, 0, :] = 63
    mq = rng.integers(0, 64, size=(M // 32, K)); mq.reshape(T, 8, K)[:, 1, :] = 63
    q = rng.integers(0, 16, size=(M, K)); q.reshape(M // 32, 32, K)[:, 0, :] = 0; q.reshape(M // 32, 32, K)[:, 1, :] = 15
    se = np.repeat(d16, 8, axis=0) * sc
    me = np.repeat(d16 / 4, 8, axis=0) * mq
    We = (np.repeat(se, 32, axis=0) * q - np.repeat(me, 32, axis=0)).astype(np.float32)
    xi = rng.integers(-4, 5, size=(1, K)).astype(np.float16)
    pe = ck.quantize(We)
    assert np.array_equal(pe["q"], q)
    got = gpu_cbk_gemv(gpu, We, xi, 2.0)
    assert np.array_equal(got.astype(np.float64), ck.gemv(pe, xi, 2.0))


def test_cbk_full_size_sampled_tiles(gpu):
    from oracle import colblock_k as ck
    torch, spqt, dev = gpu
    for M, K in [(4096, 4096), (28672, 8192)]:
        say(f"cbk full size {M}x{K}")
        W = make_fp_weights(M, K, 9600 + M) + np.float32(0.005)
        x = make_x(K, "laplace", 9601 + M)
        thr = quantile_threshold(x, 0.5)
        packed = torch.from_numpy(spqt.spqt_cbk_quantize(W)).to(dev)
        got = gpu_cbk_gemv(gpu, W, x, thr, packed=packed)[0]
        gotd = gpu_cbk_gemv(gpu, W, x, thr, dense=True, packed=packed)[0]
        tiles = np.unique(np.array([0, M // 512, M // 256 - 1]))
        rows = (tiles[:, None] * 256 + np.arange(256)[None, :]).ravel()
        p = ck.quantize(W[rows])
        assert_close(got[rows][None, :], ck.gemv(p, x, thr), f"cbk {M}x{K} sparse")
        assert_close(gotd[rows][None, :], ck.gemv(p, x, 0.0), f"cbk {M}x{K} dense")
        del W, packed


@pytest.mark.parametrize("batch", [2, 3, 4])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 4), (5, 2), (16, 4)])
def test_cbk_batch_rows_share_one_pass(gpu, batch, splits, waves):
    """K-quant flavour with several activation rows: the union list, every row its own values."""
    from oracle import colblock_k as ck
    torch, spqt, dev = gpu
    M, K = 768, 1024
    W = make_fp_weights(M, K, 9700) + np.float32(0.01)
    x_np = make_x(K, "laplace", 9701 + batch, batch=batch)
    thr = quantile_threshold(x_np, 0.6)
    say(f"cbk batch={batch} splits={splits} waves={waves}")
    packed = torch.from_numpy(spqt.spqt_cbk_quantize(W)).to(dev)
    x = torch.from_numpy(x_np).to(dev)
    y = torch.full((batch, M), float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K, batch)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    spqt.spqt_gather(x, thr, idx, cnt)
    spqt.spqt_cbk_gemv(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    p = ck.quantize(W)
    assert_close(y.cpu().numpy(), ck.gemv(p, x_np, thr), "cbk batch")
    y.fill_(float("nan"))
    spqt.spqt_cbk_gemv(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy(), ck.gemv(p, x_np, 0.0), "cbk batch dense")


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1024, 4096), (300, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (7, 2), (16, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9])
def test_cbk_fused_gemv(gpu, M, K, splits, waves, sparsity):
    """K-quant flavour, threshold inside the kernel: same result as gather + list-driven GEMV."""
    from oracle import colblock_k as ck
    torch, spqt, dev = gpu
    W = make_fp_weights(256 * ((M + 255) // 256), K, 9800 + M + K)[:M].copy() + np.float32(0.01)
    x_np = make_x(K, "laplace", 9801 + M + K)
    thr = quantile_threshold(x_np, sparsity)
    say(f"cbk fused M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    packed = torch.from_numpy(spqt.spqt_cbk_quantize(W)).to(dev)
    x = torch.from_numpy(x_np[0].copy()).to(dev)
    y = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    spqt.spqt_cbk_gemv_fused(packed, M, K, x, thr, y, ws, splits=splits, waves=waves)
    torch.cuda.synchronize()
    ref = ck.gemv(ck.quantize(ck.pad_rows(W)), x_np, thr)[:, :M]
    assert_close(y.cpu().numpy()[None, :], ref, "cbk fused")
