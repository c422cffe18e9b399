"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Index lists and packed bytes must match bit for bit; outputs must satisfy
|y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref| elementwise (fp32 accumulation vs the fp64 oracle).
"""
import numpy as np
import pytest

import oracle
from workloads import make_case, make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3
EVEN_SHARES = 16     # SPQT_CFG_EVEN_SHARES


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2511_04477_amd as spqt
    assert torch.cuda.is_available(), "these tests need the MI355X"
    spqt.lib()   # raises if the HIP library is not built: there is no fallback
    return torch, spqt, torch.device("cuda:0")


def say(*a):
    print(*a, flush=True)


def gpu_gather(gpu, x_np, thr, poison=-7):
    torch, spqt, dev = gpu
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    K = x.shape[-1]
    idx = torch.full((K + 64,), poison, dtype=torch.int32, device=dev)
    cnt = torch.full((2,), poison, dtype=torch.int32, device=dev)
    spqt.spqt_gather(x if x.shape[0] > 1 else x[0], thr, idx, cnt)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), cnt.cpu().numpy()


def gpu_gemv(gpu, w, x_np, thr, dense=False, splits=0, waves=0, packed=None, flags=0):
    torch, spqt, dev = gpu
    M, K = w["q_rowmajor"].shape[0], w["q_rowmajor"].shape[1] * 2
    if packed is None:
        packed = torch.from_numpy(spqt.spqt_pack(w["q_rowmajor"], w["scales"])).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    batch = x.shape[0]
    xx = x if batch > 1 else x[0]
    y = torch.full((batch, M), float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K, batch)
    if dense:
        spqt.spqt_gemv(packed, M, K, xx, None, None, y if batch > 1 else y[0], ws, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(xx, thr, idx, cnt)
        spqt.spqt_gemv(packed, M, K, xx, idx, cnt, y if batch > 1 else y[0], ws, splits=splits, waves=waves, flags=flags)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def assert_close(got, ref, what=""):
    err = np.abs(got.astype(np.float64) - ref)
    bound = ATOL + RTOL * np.abs(ref)
    bad = np.argwhere(err > bound)
    assert bad.size == 0, f"{what}: {bad.shape[0]} outputs out of tolerance, first {bad[0]}, max err {err.max():.4g}"
    return float(err.max())


# ------------------------------------------------------------------------------ gather

@pytest.mark.parametrize("K", [128, 1024, 4096, 8192, 11008, 14336, 28672, 65536])
@pytest.mark.parametrize("sparsity", [0.0, 0.25, 0.5, 0.65, 0.97])
def test_gather_bit_exact(gpu, K, sparsity):
    x = make_x(K, "laplace", 9000 + K)
    thr = quantile_threshold(x, sparsity)
    say(f"gather K={K} s={sparsity} thr={thr}")
    idx, cnt = gpu_gather(gpu, x, thr)
    ref, n = oracle.gather(x, thr)
    assert cnt[0] == n and cnt[1] == -7
    assert np.array_equal(idx[:n], ref)
    assert np.all(idx[n:] == -7), "entries past n_ns must stay untouched"


def test_gather_edge_thresholds_and_ties(gpu):
    x = make_x(4096, "normal", 9100)
    idx, cnt = gpu_gather(gpu, x, 0.0)
    assert cnt[0] == 4096 and np.array_equal(idx[:4096], np.arange(4096))
    idx, cnt = gpu_gather(gpu, x, float("inf"))
    assert cnt[0] == 0 and np.all(idx == -7)
    xt = np.zeros((1, 256), dtype=np.float16)
    xt[0, :7] = [0.5, -0.5, 0.25, 0.0, -0.0, 0.75, 0.4995]
    xt[0, 100] = np.nan
    xt[0, 200] = np.inf
    for thr in (0.5, 0.0, float("inf"), 0.25):
        idx, cnt = gpu_gather(gpu, xt, thr)
        ref, n = oracle.gather(xt, thr)
        assert cnt[0] == n and np.array_equal(idx[:n], ref), thr


def test_gather_batch_union(gpu):
    x = make_x(8192, "laplace", 9200, batch=4)
    for s in (0.3, 0.5, 0.7):
        thr = quantile_threshold(x, s)
        idx, cnt = gpu_gather(gpu, x, thr)
        ref, n = oracle.gather(x, thr)
        assert cnt[0] == n and np.array_equal(idx[:n], ref)


def test_gather_is_reproducible(gpu):
    x = make_x(28672, "laplace", 9300)
    thr = quantile_threshold(x, 0.5)
    first = gpu_gather(gpu, x, thr)
    for _ in range(10):
        again = gpu_gather(gpu, x, thr)
        assert np.array_equal(first[0], again[0]) and np.array_equal(first[1], again[1])


# ------------------------------------------------------------------------------ packed bytes

def test_packed_bytes_on_device_equal_reference_packer(gpu):
    torch, spqt, dev = gpu
    case = make_case(1, "w")
    packed = torch.from_numpy(spqt.spqt_pack(case["q_rowmajor"], case["scales"])).to(dev)
    assert np.array_equal(packed.cpu().numpy(), oracle.pack(case["q_rowmajor"], case["scales"]))


# ------------------------------------------------------------------------------ gemv values

@pytest.mark.parametrize("sparsity", [0.0, 0.25, 0.4, 0.5, 0.65, 0.9, 1.0])
def test_config1_sparse_gemv(gpu, sparsity):
    case = make_case(1, "w")
    thr = quantile_threshold(case["x"], sparsity)
    say(f"config1 s={sparsity}")
    got = gpu_gemv(gpu, case, case["x"], thr)
    ref = oracle.gemv(case["q_rowmajor"], case["scales"], case["x"], thr)
    assert_close(got, ref, f"config1 s={sparsity}")
    if sparsity == 1.0:
        assert np.all(got == 0.0), "n_ns == 0 must still write zeros"


@pytest.mark.parametrize("M,K", [(256, 128), (256, 256), (768, 640), (512, 1024), (1024, 4096), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (1, 4), (2, 2), (3, 4), (5, 1), (8, 4), (64, 2)])
def test_launch_shapes_and_ragged_sizes(gpu, M, K, splits, waves):
    w = make_weights(M, K, 7000 + M + K)
    x = make_x(K, "laplace", 7001 + M + K)
    thr = quantile_threshold(x, 0.5)
    say(f"M={M} K={K} splits={splits} waves={waves}")
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    assert_close(gpu_gemv(gpu, w, x, thr, splits=splits, waves=waves), ref, "sparse")
    ref0 = oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0)
    assert_close(gpu_gemv(gpu, w, x, 0.0, dense=True, splits=splits, waves=waves), ref0, "dense")


def test_threshold_zero_equals_dense_kernel_bitwise(gpu):
    """thr = 0 lists every column, so the list kernel with one-group passes must do exactly what the
    index-free dense kernel does in the same launch shape (same partition, same order) - identical
    bits.  The default list kernel (row-aligned passes) sums in another order: equal within tolerance."""
    import paper_2511_04477_amd as spqt
    case = make_case(1, "w")
    for splits, waves in ((1, 4), (2, 4), (4, 2)):
        a = gpu_gemv(gpu, case, case["x"], 0.0, splits=splits, waves=waves, flags=spqt.CFG_GROUP_PASSES)
        b = gpu_gemv(gpu, case, case["x"], 0.0, dense=True, splits=splits, waves=waves)
        assert np.array_equal(a, b), (splits, waves)
        c = gpu_gemv(gpu, case, case["x"], 0.0, splits=splits, waves=waves)
        assert_close(c, b.astype(np.float64), "row-aligned passes at threshold 0")


def test_exact_arithmetic_case_is_bit_exact(gpu):
    """Integer x, power-of-two scales: every product and partial sum is exactly representable
    in fp32, so the GPU must equal the oracle bit for bit whatever its summation order."""
    M, K = 512, 1024
    rng = np.random.default_rng(5)
    w = make_weights(M, K, 31)
    w["scales"] = (2.0 ** rng.integers(-6, -2, size=(M, K // 128))).astype(np.float16)
    x = rng.integers(-4, 5, size=(1, K)).astype(np.float16)
    for thr in (0.0, 2.0, 3.0):
        ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
        got = gpu_gemv(gpu, w, x, thr)
        assert np.array_equal(got.astype(np.float64), ref), thr
    got = gpu_gemv(gpu, w, x, 0.0, dense=True)
    assert np.array_equal(got.astype(np.float64), oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0))


@pytest.mark.parametrize("batch", [1, 4])
def test_subnormal_and_extreme_activations(gpu, batch):
    """fp16 subnormal x must count exactly (2^-24 times a small integer times a code is exact in
    fp32, and with power-of-two scales so is every partial sum), and x near the fp16 maximum must
    neither overflow nor lose more than fp32 accumulation must (the bound scales with the size of
    the terms, offset-binary bias included: 16 * scale * |x| per weight): the multiply stage feeds
    raw fp16 bits to the matrix cores."""
    M, K = 512, 512
    rng = np.random.default_rng(77 + batch)
    w = make_weights(M, K, 33)
    w["scales"] = (2.0 ** rng.integers(-6, -2, size=(M, K // 128))).astype(np.float16)
    tiny = (rng.integers(-7, 8, size=(batch, K)).astype(np.float64) * 2.0 ** -24).astype(np.float16)
    assert np.all(np.abs(tiny.astype(np.float64)) < 6.2e-5)      # all subnormal (or zero)
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], tiny, 0.0)
    for dense in (False, True):
        got = gpu_gemv(gpu, w, tiny, 0.0, dense=dense)
        assert np.array_equal(got.astype(np.float64), ref), dense
    big = make_x(K, "laplace", 78, batch=batch)
    big[:, ::17] = np.float16(60000.0) * np.sign(big[:, ::17].astype(np.float32) + 0.5).astype(np.float16)
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], big, 0.5)
    got = gpu_gemv(gpu, w, big, 0.5)
    err = np.abs(got.astype(np.float64) - ref)
    terms = (16.0 * np.repeat(w["scales"].astype(np.float64), 128, axis=1)) @ np.abs(big.astype(np.float64)).T   # [M, batch]
    assert np.all(np.isfinite(got)) and np.all(err <= ATOL + 1e-5 * terms.T), (err / terms.T).max()


def test_column_probe(gpu):
    """x = c * e_k  =>  y = c * dequant(W[:, k]) exactly; catches any address-mapping error."""
    torch, spqt, dev = gpu
    M, K = 512, 384
    w = make_weights(M, K, 41)
    Wd = oracle.dequant(w["q_rowmajor"], w["scales"])
    packed = torch.from_numpy(spqt.spqt_pack(w["q_rowmajor"], w["scales"])).to(dev)
    for k in list(range(0, K, 7)) + [127, 128, 255, 256, K - 1]:
        x = np.zeros((1, K), dtype=np.float16)
        x[0, k] = -1.5
        got = gpu_gemv(gpu, w, x, 1.0, packed=packed)[0].astype(np.float64)
        want = (-1.5 * Wd[:, k])
        assert np.array_equal(got, want.astype(np.float32).astype(np.float64)), k


def test_clustered_sparsity(gpu):
    """Kept columns bunched into a few groups, empty groups, a group with a single kept
    column, and a list whose slices straddle group boundaries."""
    M, K = 1024, 2048
    w = make_weights(M, K, 61)
    x = make_x(K, "laplace", 62)
    x[0, 0:512] = 0            # four empty groups
    x[0, 640:768] = 0
    x[0, 700] = 3.0            # a group with one kept column
    x[0, 1024:1152] = 2.0      # a full group
    thr = 0.75
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    for splits, waves in [(0, 0), (1, 1), (7, 4), (16, 2)]:
        assert_close(gpu_gemv(gpu, w, x, thr, splits=splits, waves=waves), ref, f"clustered {splits}x{waves}")


def test_gemv_is_reproducible(gpu):
    case = make_case(1, "w")
    thr = quantile_threshold(case["x"], 0.5)
    first = gpu_gemv(gpu, case, case["x"], thr)
    for _ in range(20):
        assert np.array_equal(first, gpu_gemv(gpu, case, case["x"], thr))


def test_batch4_union(gpu):
    M, K = 512, 1024
    w = make_weights(M, K, 71)
    x = make_x(K, "laplace", 72, batch=4)
    for s in (0.0, 0.3, 0.5, 0.7):
        thr = quantile_threshold(x, s)
        ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
        assert_close(gpu_gemv(gpu, w, x, thr), ref, f"batch4 s={s}")
    x1 = np.ascontiguousarray(np.repeat(x[:1], 4, axis=0))
    thr = quantile_threshold(x1, 0.5)
    # four equal rows: the batch kernel must give each of them what the same kernel gives one row
    import paper_2511_04477_amd as spqt
    y4 = gpu_gemv(gpu, w, x1, thr, splits=2, waves=4)
    y1 = gpu_gemv(gpu, w, x1[:1], thr, splits=2, waves=4, flags=spqt.CFG_GROUP_PASSES)
    assert all(np.array_equal(y4[b], y4[0]) for b in range(4))
    assert_close(y4[:1], y1.astype(np.float64), "batch 4 row vs the one-row kernel")


@pytest.mark.parametrize("batch", [2, 3, 4])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (3, 4), (8, 2)])
def test_batch_rows_share_one_pass(gpu, batch, splits, waves):
    """Several activation rows over the union index list, multi-group slices and several
    workgroups per block-row; also the dense kernel and per-row consistency with batch 1."""
    M, K = 1024, 2048
    w = make_weights(M, K, 81)
    x = make_x(K, "laplace", 82 + batch, batch=batch)
    thr = quantile_threshold(x, 0.6)
    say(f"batch={batch} splits={splits} waves={waves}")
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    assert_close(gpu_gemv(gpu, w, x, thr, splits=splits, waves=waves), ref, "batch sparse")
    ref0 = oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0)
    assert_close(gpu_gemv(gpu, w, x, 0.0, dense=True, splits=splits, waves=waves), ref0, "batch dense")


def gpu_gemv_fused(gpu, w, x_np, thr, splits=0, waves=0, packed=None, flags=0):
    torch, spqt, dev = gpu
    M, K = w["q_rowmajor"].shape[0], w["q_rowmajor"].shape[1] * 2
    if packed is None:
        packed = torch.from_numpy(spqt.spqt_pack(w["q_rowmajor"], w["scales"])).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)[0]
    y = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)
    spqt.spqt_gemv_fused(packed, M, K, x, thr, y, ws, splits=splits, waves=waves, flags=flags)
    torch.cuda.synchronize()
    return y.cpu().numpy()[None, :]


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1024, 4096), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (2, 4), (7, 2), (16, 4), (64, 1)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_fused_gather_gemv(gpu, M, K, splits, waves, sparsity):
    """The one-launch path (threshold + in-wave compaction + GEMV) against the oracle."""
    w = make_weights(M, K, 7100 + M + K)
    x = make_x(K, "laplace", 7101 + M + K)
    thr = quantile_threshold(x, sparsity)
    say(f"fused M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    assert_close(gpu_gemv_fused(gpu, w, x, thr, splits=splits, waves=waves), ref, "fused")


@pytest.mark.parametrize("M,K", [(256, 128), (1024, 4096), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (7, 2), (16, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_fused_even_shares(gpu, M, K, splits, waves, sparsity):
    """The one-launch kernel that counts the kept columns first and gives every wavefront an even share."""
    _, spqt, _ = gpu
    w = make_weights(M, K, 7200 + M + K)
    x = make_x(K, "laplace", 7201 + M + K)
    thr = quantile_threshold(x, sparsity)
    say(f"fused even shares M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    got = gpu_gemv_fused(gpu, w, x, thr, splits=splits, waves=waves, flags=spqt.CFG_EVEN_SHARES)
    assert_close(got, ref, "fused, even shares")


@pytest.mark.parametrize("M,K,dist", [(512, 1024, "laplace"), (1024, 4096, "laplace_clustered"), (768, 8192, "laplace"),
                                      (256, 32768, "laplace"), (2048, 1152, "normal")])
@pytest.mark.parametrize("sparsity", [0.0, 0.3, 0.5, 0.97, 1.0])
def test_fused_equals_gather_then_list_kernel_bitwise(gpu, M, K, dist, sparsity):
    """One launch with SPQT_CFG_EVEN_SHARES (list built inside the kernel) and spqt_gather + spqt_gemv perform the same
    arithmetic in the same order when their launch shapes agree: the outputs are equal bit for bit, and
    both are within the oracle's tolerance."""
    w = make_weights(M, K, 7400 + M + K)
    x = make_x(K, dist, 7401 + M + K)
    thr = float("inf") if sparsity == 1.0 else quantile_threshold(x, sparsity)
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    for splits, waves in [(0, 0), (1, 1), (3, 2), (16, 4), (64, 4)]:
        say(f"fused vs list M={M} K={K} {dist} s={sparsity} {splits}x{waves}")
        a = gpu_gemv_fused(gpu, w, x, thr, splits=splits, waves=waves, flags=EVEN_SHARES)
        b = gpu_gemv(gpu, w, x, thr, splits=splits, waves=waves)
        assert_close(a, ref, "one launch")
        assert np.array_equal(a, b), f"one launch != gather + list kernel at {splits}x{waves}"


def test_fused_clustered_ties_and_exact(gpu):
    M, K = 1024, 2048
    w = make_weights(M, K, 61)
    x = make_x(K, "laplace", 62)
    x[0, 0:512] = 0            # empty groups and empty 64-column units
    x[0, 640:768] = 0
    x[0, 700] = 3.0            # a group with one kept column
    x[0, 1024:1152] = 2.0      # a full group
    x[0, 1500] = 0.75          # a tie with the threshold is kept
    thr = 0.75
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    for splits, waves in [(0, 0), (1, 1), (5, 4), (16, 2)]:
        assert_close(gpu_gemv_fused(gpu, w, x, thr, splits=splits, waves=waves), ref, f"fused clustered {splits}x{waves}")
    # exact-arithmetic inputs: bit-for-bit
    rng = np.random.default_rng(5)
    w["scales"] = (2.0 ** rng.integers(-6, -2, size=(M, K // 128))).astype(np.float16)
    xi = rng.integers(-4, 5, size=(1, K)).astype(np.float16)
    for thr in (0.0, 2.0, 3.0):
        ref = oracle.gemv(w["q_rowmajor"], w["scales"], xi, thr)
        assert np.array_equal(gpu_gemv_fused(gpu, w, xi, thr).astype(np.float64), ref), thr


@pytest.mark.parametrize("M,K", [(256, 128), (1024, 4096), (2048, 1152)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (7, 2), (16, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9, 1.0])
def test_fused_without_compaction(gpu, M, K, splits, waves, sparsity):
    """The ablation mode (in-kernel test, dropped columns keep their slot with x = 0) computes
    the same GEMV."""
    _, spqt, _ = gpu
    w = make_weights(M, K, 7300 + M + K)
    x = make_x(K, "laplace_clustered", 7301 + M + K)
    thr = quantile_threshold(x, sparsity)
    say(f"fused-nocompact M={M} K={K} splits={splits} waves={waves} s={sparsity}")
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    got = gpu_gemv_fused(gpu, w, x, thr, splits=splits, waves=waves, flags=spqt.CFG_NO_COMPACTION)
    assert_close(got, ref, "fused without compaction")


def test_fused_full_size_headline(gpu):
    torch, spqt, dev = gpu
    case = make_case(2, "q", want_q=False)
    packed = torch.from_numpy(spqt.spqt_pack(case["q_rowmajor"], case["scales"])).to(dev)
    for s in (0.0, 0.25, 0.5, 0.65):
        thr = quantile_threshold(case["x"], s)
        ref = oracle.gemv(case["q_rowmajor"], case["scales"], case["x"], thr)
        assert_close(gpu_gemv_fused(gpu, case, case["x"], thr, packed=packed), ref, f"fused cfg2 s={s}")


@pytest.mark.parametrize("tensor", ["gate", "down"])
def test_fused_full_size_70b(gpu, tensor):
    """The 70B MLP shapes through both one-launch kernels in the library's default launch shape."""
    torch, spqt, dev = gpu
    case = make_case(5, tensor, want_q=False)
    packed = torch.from_numpy(spqt.spqt_pack(case["q_rowmajor"], case["scales"])).to(dev)
    for s in (0.3, 0.5, 0.7):
        thr = quantile_threshold(case["x"], s)
        say(f"fused full size cfg5/{tensor} s={s}")
        ref = oracle.gemv(case["q_rowmajor"], case["scales"], case["x"], thr)
        assert_close(gpu_gemv_fused(gpu, case, case["x"], thr, packed=packed), ref, f"fused cfg5/{tensor} s={s}")
        got = gpu_gemv_fused(gpu, case, case["x"], thr, packed=packed, flags=EVEN_SHARES)
        assert_close(got, ref, f"fused, even shares cfg5/{tensor} s={s}")
        splits, waves = spqt.spqt_default_cfg(case["M"], case["K"], 1, True)
        assert np.array_equal(got, gpu_gemv(gpu, case, case["x"], thr, packed=packed)), "one launch != gather + list kernel"


def test_longest_supported_k(gpu):
    """K = 65536 (the gather's limit), one block-row: list-driven, dense and one-launch paths."""
    M, K = 256, 65536
    w = make_weights(M, K, 93)
    x = make_x(K, "laplace", 94)
    thr = quantile_threshold(x, 0.5)
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    idx, cnt = gpu_gather(gpu, x, thr)
    ref_idx, n = oracle.gather(x, thr)
    assert int(cnt[0]) == n and np.array_equal(idx[:n], ref_idx)
    for splits, waves in [(0, 0), (64, 4), (3, 2)]:
        assert_close(gpu_gemv(gpu, w, x, thr, splits=splits, waves=waves), ref, f"K=65536 {splits}x{waves}")
        assert_close(gpu_gemv_fused(gpu, w, x, thr, splits=splits, waves=waves), ref, f"K=65536 fused {splits}x{waves}")
    assert_close(gpu_gemv(gpu, w, x, 0.0, dense=True), oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0), "K=65536 dense")


def test_one_workspace_serves_any_sequence_of_shapes_and_kernels(gpu):
    """The reducer of a block-row puts every exchange word it consumed back to zero, so one workspace may
    serve calls of different M, K, launch shape and kernel in any order: after every call the whole
    workspace reads as zeros again and the result is that of a fresh workspace."""
    torch, spqt, dev = gpu
    shapes = [(1024, 2048), (2048, 1024), (300, 1024), (1024, 2048), (512, 4096)]
    ws = spqt.new_workspace(2048, 4096, 2)
    cases = {}
    for (M, K) in set(shapes):
        w = make_weights(M, K, 91 + M + K)
        x_np = make_x(K, "laplace", 92 + M, batch=2)
        thr = quantile_threshold(x_np[:1], 0.5)
        cases[(M, K)] = (w, x_np, thr, torch.from_numpy(spqt.spqt_pack(w["q_rowmajor"], w["scales"])).to(dev),
                         oracle.gemv(w["q_rowmajor"], w["scales"], x_np[:1], thr),
                         oracle.gemv(w["q_rowmajor"], w["scales"], x_np, thr),
                         oracle.gemv(w["q_rowmajor"], w["scales"], x_np[:1], 0.0))
    launch = [(8, 2), (16, 4), (3, 1), (5, 4), (64, 1)]
    for call, (M, K) in enumerate(shapes):
        w, x_np, thr, packed, ref1, ref2, ref_dense = cases[(M, K)]
        splits, waves = launch[call]
        say(f"shared workspace call {call}: {M}x{K} splits={splits} waves={waves}")
        x1 = torch.from_numpy(x_np[0]).to(dev)
        x2 = torch.from_numpy(x_np).to(dev)
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        y = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
        spqt.spqt_gather(x1, thr, idx, cnt)
        spqt.spqt_gemv(packed, M, K, x1, idx, cnt, y, ws, splits=splits, waves=waves)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy()[None, :], ref1, f"list, call {call}")
        assert int(torch.count_nonzero(ws).item()) == 0, "exchange words must be back to zero"
        y.fill_(float("nan"))
        spqt.spqt_gemv(packed, M, K, x1, None, None, y, ws, splits=splits, waves=waves)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy()[None, :], ref_dense, f"dense, call {call}")
        y.fill_(float("nan"))
        spqt.spqt_gemv_fused(packed, M, K, x1, thr, y, ws, splits=min(splits, K // 64), waves=waves)
        torch.cuda.synchronize()
        assert_close(y.cpu().numpy()[None, :], ref1, f"one launch, call {call}")
        y2 = torch.full((2, M), float("nan"), dtype=torch.float32, device=dev)
        spqt.spqt_gather(x2, thr, idx, cnt)
        spqt.spqt_gemv(packed, M, K, x2, idx, cnt, y2, ws, splits=splits, waves=waves)
        torch.cuda.synchronize()
        assert_close(y2.cpu().numpy(), ref2, f"two rows, call {call}")
        assert int(torch.count_nonzero(ws).item()) == 0, "exchange words must be back to zero"


def test_hip_graph_replay_matches_eager(gpu):
    """gather + GEMV captured in one HIP graph and replayed, with eager work and
    synchronizations between the replays: every replay must reproduce the eager result."""
    torch, spqt, dev = gpu
    case = make_case(1, "w")
    M, K = case["M"], case["K"]
    packed = torch.from_numpy(spqt.spqt_pack(case["q_rowmajor"], case["scales"])).to(dev)
    xs = [make_x(K, "normal", 8800 + i)[0] for i in range(3)]
    thr = [quantile_threshold(v, 0.5) for v in xs]
    x = torch.from_numpy(xs[0]).to(dev)
    idx = torch.zeros(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y = torch.zeros(M, dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K)

    def run():
        spqt.spqt_gather(x, thr[0], idx, cnt)
        spqt.spqt_gemv(packed, M, K, x, idx, cnt, y, ws)

    run()
    torch.cuda.synchronize()
    eager = {0: y.cpu().numpy().copy()}
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for rep in range(5):
        y.fill_(float("nan"))
        idx.fill_(-1)
        # unrelated eager work on the same buffers' neighbours and a sync between replays
        scratch = torch.randn(1 << 16, device=dev).sum()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy(), eager[0]), rep
        assert float(scratch) == float(scratch)
    ref = oracle.gemv(case["q_rowmajor"], case["scales"], xs[0][None, :], thr[0])
    assert_close(y.cpu().numpy()[None, :], ref, "graph replay")


# ------------------------------------------------------------------------------ full sizes

FULL = [(2, "q", [0.0, 0.25, 0.4, 0.5, 0.65]),
        (3, "gate", [0.4, 0.5]), (3, "down", [0.4, 0.5]),
        (4, "k", [0.5]), (4, "gate", [0.5]), (4, "down", [0.5]),
        (5, "gate", [0.3, 0.5, 0.7]), (5, "down", [0.3, 0.5, 0.7])]


@pytest.mark.parametrize("config,tensor,sparsities", FULL)
def test_full_size_default_launch(gpu, config, tensor, sparsities):
    """Benchmark shapes in the launch configuration the benchmark times (library default)."""
    torch, spqt, dev = gpu
    case = make_case(config, tensor, want_q=False)
    say(f"full config={config} tensor={tensor} M={case['M']} K={case['K']}")
    packed_np = spqt.spqt_pack(case["q_rowmajor"], case["scales"])
    packed = torch.from_numpy(packed_np).to(dev)
    for s in sparsities:
        thr = quantile_threshold(case["x"], s)
        ref = oracle.gemv(case["q_rowmajor"], case["scales"], case["x"], thr)
        got = gpu_gemv(gpu, case, case["x"], thr, packed=packed)
        e = assert_close(got, ref, f"cfg{config}/{tensor} s={s}")
        say(f"   s={s}: max|err|={e:.3e}")
    ref = oracle.gemv(case["q_rowmajor"], case["scales"], case["x"], 0.0)
    assert_close(gpu_gemv(gpu, case, case["x"], 0.0, dense=True, packed=packed), ref, "dense")


@pytest.mark.parametrize("tensor", ["gate", "down"])
def test_full_size_four_rows_union_list(gpu, tensor):
    """The 70B MLP shapes with 4 activation rows: spqt_gather(batch 4) gives the union list, spqt_gemv(batch 4)
    consumes it in the library's default launch shape - the calls and shape the benchmark times.  The index
    list is compared whole; the outputs on 640 sampled rows (the last block-row included) that the oracle
    computes one by one."""
    torch, spqt, dev = gpu
    case = make_case(5, tensor, batch=4, want_q=False)
    M, K = case["M"], case["K"]
    q, sc, x_np = case["q_rowmajor"], case["scales"], case["x"]
    packed = torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)
    rng = np.random.default_rng(9970 + M)
    rows = np.unique(np.concatenate([rng.choice(M - 256, size=512, replace=False), np.arange(M - 128, M)]))
    x = torch.from_numpy(x_np).to(dev)
    idx = torch.full((K,), -7, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    ws = spqt.new_workspace(M, K, 4)
    for s in (0.3, 0.5, 0.7):
        thr = quantile_threshold(x_np, s)
        say(f"four rows, full size: {tensor} {M}x{K} s={s}")
        y = torch.full((4, M), float("nan"), dtype=torch.float32, device=dev)
        idx.fill_(-7)
        spqt.spqt_gather(x, thr, idx, cnt)
        spqt.spqt_gemv(packed, M, K, x, idx, cnt, y, ws)
        torch.cuda.synchronize()
        ref_idx, n = oracle.gather(x_np, thr)
        assert int(cnt.item()) == n and np.array_equal(idx[:n].cpu().numpy(), ref_idx)
        got = y.cpu().numpy()
        assert not np.isnan(got).any()
        e = assert_close(got[:, rows], oracle.gemv_rows(q, sc, x_np, thr, rows), f"{tensor} 4 rows s={s}")
        say(f"   kept {n}/{K}, max|err|={e:.3e}")


# ------------------------------------------------------------------------------ pinned corner behaviour

def test_non_finite_activation_makes_every_output_nan(gpu):
    """A kept Inf (or NaN) activation: the offset-binary bias (-8 * sum of kept x) meets the products'
    opposite infinity, so every output is NaN in every kernel - the behaviour the header states.  The
    oracle (w * x per weight) is non-finite in every row as well."""
    M, K = 512, 1024
    w = make_weights(M, K, 8801)
    for bad in (np.inf, -np.inf, np.nan):
        x = make_x(K, "laplace", 8802)
        x[0, 300] = bad
        thr = quantile_threshold(x[:, :256], 0.5)
        ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
        assert not np.isfinite(ref).any()
        for got in (gpu_gemv(gpu, w, x, thr), gpu_gemv(gpu, w, x, 0.0, dense=True), gpu_gemv_fused(gpu, w, x, thr),
                    gpu_gemv_fused(gpu, w, x, thr, flags=EVEN_SHARES), gpu_gemv(gpu, w, x, thr, flags=8)):
            assert np.isnan(got).all(), bad


def test_matrix_cores_take_fp16_subnormals_unflushed(gpu):
    """The multiply feeds the 4-bit codes to v_mfma_f32_4x4x4_16B_f16 as fp16 SUBNORMALS (code * 2^-24).  Were
    subnormal inputs flushed to zero, every product would vanish and y would be -8 * scale * sum(x) for every
    row.  Codes 1 (q = -7) and 15 (q = +7) with scale 1 and x = 1 on the kept columns: y = -7 n or +7 n exactly."""
    M, K = 512, 1024
    q = np.empty((M, K // 2), dtype=np.uint8)
    q[0::2] = 0x99          # two's-complement nibble 9 = -7 in every position: stored code 1
    q[1::2] = 0x77          # +7: stored code 15
    w = {"q_rowmajor": q, "scales": np.ones((M, K // 128), dtype=np.float16)}
    x = np.zeros((1, K), dtype=np.float16)
    kept = np.arange(0, K, 3)
    x[0, kept] = 1.0
    want = np.where(np.arange(M) % 2 == 0, -7.0, 7.0) * len(kept)
    assert np.array_equal(oracle.gemv(q, w["scales"], x, 0.5)[0], want)
    for got in (gpu_gemv(gpu, w, x, 0.5), gpu_gemv(gpu, w, x, 0.0, dense=True), gpu_gemv_fused(gpu, w, x, 0.5),
                gpu_gemv_fused(gpu, w, x, 0.5, flags=EVEN_SHARES), gpu_gemv(gpu, w, np.repeat(x, 3, axis=0), 0.5)):
        assert np.array_equal(got.astype(np.float64), np.broadcast_to(want, got.shape))


@pytest.mark.parametrize("M", [1, 255, 257, 1000, 3000, 5000, 9000])
@pytest.mark.parametrize("K", [128, 384, 1152, 5120, 9216])
def test_default_launch_shape_off_the_tuned_shapes(gpu, M, K):
    """The launch shape the library picks (spqt_default_cfg) on shapes it was not tuned on - ragged M, K that
    is no power of two, very flat and very tall matrices - through every batch-1 entry point, against the oracle."""
    torch, spqt, dev = gpu
    Mp = 256 * ((M + 255) // 256)
    full = make_weights(Mp, K, 8900 + M + K)
    w = {"q_rowmajor": np.ascontiguousarray(full["q_rowmajor"][:M]), "scales": np.ascontiguousarray(full["scales"][:M])}
    x = make_x(K, "laplace", 8901 + M + K)
    thr = quantile_threshold(x, 0.5)
    say(f"off-grid default launch M={M} K={K} cfg={spqt.spqt_default_cfg(M, K, 1, True)} dense cfg={spqt.spqt_default_cfg(M, K, 1, False)}")
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    assert_close(gpu_gemv(gpu, w, x, thr), ref, "list")
    assert_close(gpu_gemv_fused(gpu, w, x, thr), ref, "one launch")
    assert_close(gpu_gemv_fused(gpu, w, x, thr, flags=EVEN_SHARES), ref, "one launch, even shares")
    assert_close(gpu_gemv(gpu, w, x, 0.0, dense=True), oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0), "dense")
    # and the allocation-free entry point, which uses the same default shape with the static scratch
    packed = torch.from_numpy(spqt.spqt_pack(w["q_rowmajor"], w["scales"])).to(dev)
    xd = torch.from_numpy(x[0]).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y = torch.full((M,), float("nan"), dtype=torch.float32, device=dev)
    spqt.spqt_gather(xd, thr, idx, cnt)
    spqt.spqt_gemv_static(packed, M, K, xd, idx, cnt, y)
    torch.cuda.synchronize()
    assert_close(y.cpu().numpy()[None, :], ref, "static scratch")
