"""GPU parity of the group-layout kernels with quantization groups of 64 columns (the layout's other
group size), through the C ABI, against the oracle on the same seeded inputs.  Packed bytes must equal
the oracle packer's; outputs must satisfy |y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref| elementwise."""
import numpy as np
import pytest

import oracle
from workloads import make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3
G = 64


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2511_04477_amd as spqt
    assert torch.cuda.is_available(), "these tests need the MI355X"
    spqt.lib()
    return torch, spqt, torch.device("cuda:0")


def assert_close(got, ref, what):
    err = np.abs(got.astype(np.float64) - ref)
    bad = err > ATOL + RTOL * np.abs(ref)
    assert not bad.any(), f"{what}: {int(bad.sum())} outputs off, max err {err.max():.3e}"


def run(gpu, w, M, K, x_np, thr, mode, splits=0, waves=0):
    torch, spqt, dev = gpu
    packed_np = spqt.spqt_pack(w["q_rowmajor"], w["scales"], group=G)
    assert np.array_equal(packed_np, oracle.pack(w["q_rowmajor"], w["scales"], group=G))
    packed = torch.from_numpy(packed_np).to(dev)
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    batch = x.shape[0]
    xx = x if batch > 1 else x[0]
    y = torch.full((batch, M), float("nan"), dtype=torch.float32, device=dev)
    yy = y if batch > 1 else y[0]
    ws = spqt.new_workspace(M, K, batch)
    if mode == "fused":
        spqt.spqt_gemv_fused(packed, M, K, xx, thr, yy, ws, group=G, splits=splits, waves=waves)
    elif mode == "dense":
        spqt.spqt_gemv(packed, M, K, xx, None, None, yy, ws, group=G, splits=splits, waves=waves)
    else:
        idx = torch.empty(K, dtype=torch.int32, device=dev)
        cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        spqt.spqt_gather(xx, thr, idx, cnt)
        spqt.spqt_gemv(packed, M, K, xx, idx, cnt, yy, ws, group=G, splits=splits, waves=waves)
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1024, 4096), (300, 1152), (4096, 4096)])
@pytest.mark.parametrize("splits,waves", [(0, 0), (1, 1), (7, 2), (16, 4)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9])
def test_group64_all_modes(gpu, M, K, splits, waves, sparsity):
    w = make_weights(M, K, 6600 + M + K, group=G)
    x = make_x(K, "laplace", 6601 + M + K)
    thr = quantile_threshold(x, sparsity)
    print(f"group 64 M={M} K={K} splits={splits} waves={waves} s={sparsity}", flush=True)
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr, group=G)
    assert_close(run(gpu, w, M, K, x, thr, "list", splits, waves), ref, "list")
    assert_close(run(gpu, w, M, K, x, thr, "fused", splits, waves), ref, "fused")
    if sparsity == 0.0:
        assert_close(run(gpu, w, M, K, x, thr, "dense", splits, waves), ref, "dense")


@pytest.mark.parametrize("batch", [2, 4])
def test_group64_batch(gpu, batch):
    M, K = 768, 2048
    w = make_weights(M, K, 6700, group=G)
    x = make_x(K, "laplace", 6701 + batch, batch=batch)
    thr = quantile_threshold(x, 0.5)
    assert_close(run(gpu, w, M, K, x, thr, "list"), oracle.gemv(w["q_rowmajor"], w["scales"], x, thr, group=G), "batch list")
    assert_close(run(gpu, w, M, K, x, thr, "dense", 3, 4), oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0, group=G), "batch dense")


def test_group64_exact_arithmetic_is_bit_exact(gpu):
    M, K = 512, 1024
    rng = np.random.default_rng(65)
    w = make_weights(M, K, 6800, group=G)
    w["scales"] = (2.0 ** rng.integers(-6, -2, size=(M, K // G))).astype(np.float16)
    x = rng.integers(-4, 5, size=(1, K)).astype(np.float16)
    for thr in (0.0, 2.0):
        ref = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr, group=G)
        assert np.array_equal(run(gpu, w, M, K, x, thr, "list").astype(np.float64), ref)
        assert np.array_equal(run(gpu, w, M, K, x, thr, "fused").astype(np.float64), ref)
