"""The allocation-free entry point (spqt_gemv_static) against spqt_gemv with a caller's workspace:
same kernels and launch shape, so the outputs must be equal bit for bit; both are also held to the
oracle's tolerance.  Two calls in a row on the GPU's one static array, the second on a smaller input."""
import ctypes

import numpy as np
import pytest

import oracle
from workloads import make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3


def _one(torch, spqt, dev, M, K, batch, seed, dense):
    w = make_weights(M, K, seed)
    x_np = make_x(K, "laplace", seed + 1, batch=batch)
    thr = quantile_threshold(x_np, 0.5)
    packed = torch.from_numpy(spqt.spqt_pack(w["q_rowmajor"], w["scales"])).to(dev)
    x = torch.from_numpy(x_np if batch > 1 else x_np[0]).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    spqt.spqt_gather(x, thr, idx, cnt)
    shape = (batch, M) if batch > 1 else (M,)
    y_ws = torch.full(shape, float("nan"), dtype=torch.float32, device=dev)
    y_st = torch.full(shape, float("nan"), dtype=torch.float32, device=dev)
    ws = spqt.new_workspace(M, K, batch)
    spqt.spqt_gemv(packed, M, K, x, None if dense else idx, None if dense else cnt, y_ws, ws)
    # straight through the C ABI: plain pointers and sizes
    rc = spqt.lib().spqt_gemv_static(packed.data_ptr(), M, K, 128, x.data_ptr(), batch,
                                     None if dense else idx.data_ptr(), None if dense else cnt.data_ptr(),
                                     y_st.data_ptr(), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, spqt.spqt_status_str(rc)
    torch.cuda.synchronize()
    a, b = y_ws.cpu().numpy().reshape(batch, M), y_st.cpu().numpy().reshape(batch, M)
    assert np.array_equal(a, b), f"{M}x{K} batch {batch}: static scratch and caller workspace differ"
    ref = oracle.gemv(w["q_rowmajor"], w["scales"], x_np, 0.0 if dense else thr)
    err = np.abs(b.astype(np.float64) - ref)
    assert np.all(err <= ATOL + RTOL * np.abs(ref)), float(err.max())


def test_static_scratch_matches_workspace_two_calls_second_smaller():
    import torch
    import paper_2511_04477_amd as spqt
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    splits, _ = spqt.spqt_default_cfg(4096, 4096, 1, True)
    assert splits > 1, "the first case must really use the exchange words"
    for (M, K, batch, dense) in [(4096, 4096, 1, False), (1024, 2048, 1, False),    # second call: smaller input
                                 (2048, 1024, 4, False), (1280, 1024, 1, True), (300, 512, 2, False)]:
        print(f"static scratch: {M}x{K} batch {batch} dense={dense}", flush=True)
        _one(torch, spqt, dev, M, K, batch, 4400 + M + K + batch, dense)


def test_static_scratch_rejects_what_does_not_fit():
    import torch
    import paper_2511_04477_amd as spqt
    dev = torch.device("cuda:0")
    M, K = 8192, 28672            # 32 block-rows x 16 workgroups x 4 rows x 256 words of 8 bytes = 4 MiB > the array
    splits, _ = spqt.spqt_default_cfg(M, K, 4, True)
    assert 256 + (M // 256) * 256 * splits * 4 * 8 > (2 << 20) + 256
    one = torch.zeros(16, dtype=torch.uint8, device=dev)
    p = one.data_ptr()
    assert spqt.lib().spqt_gemv_static(p, M, K, 128, p, 4, p, p, p, None) == -4       # SPQT_ESIZE, on the host, nothing launched
    assert spqt.lib().spqt_gemv_static(p, 100, 100, 128, p, 1, None, None, p, None) == -2     # SPQT_ESHAPE
    torch.cuda.synchronize()
