"""GPU parity of the benchmark's comparison kernel (int4 GEMV on the row-major source layout,
dense and with the naive per-weight sparsity test) against the oracle: a baseline that computed
something else would make the speed-up tables meaningless.  Same tolerance as the product path."""
import ctypes
import os

import numpy as np
import pytest

import oracle
from workloads import make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def calib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    L = ctypes.CDLL(os.path.join(ROOT, "paper_2511_04477_amd", "libspqt_calib.so"))
    vp = ctypes.c_void_p
    L.spqt_calib_rowmajor_gemv.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int64, vp, ctypes.c_float,
                                           ctypes.c_int, vp, vp]
    return torch, L


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1000, 4096), (4096, 11008), (37, 28672)])
@pytest.mark.parametrize("sparsity", [0.0, 0.5, 0.9])
def test_rowmajor_baseline_matches_oracle(calib, M, K, sparsity):
    torch, L = calib
    dev = torch.device("cuda:0")
    Mp = 256 * ((M + 255) // 256)
    w = make_weights(Mp, K, 7700 + M + K)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    x = make_x(K, "laplace", 7701 + M + K)
    thr = quantile_threshold(x, sparsity)
    print(f"rowmajor baseline M={M} K={K} s={sparsity}", flush=True)
    qd = torch.from_numpy(q).to(dev)
    sd = torch.from_numpy(np.ascontiguousarray(sc)).to(dev)
    xd = torch.from_numpy(x[0].copy()).to(dev)
    st = torch.cuda.current_stream().cuda_stream
    for skip, t in ((0, 0.0), (1, thr)):
        buf = torch.full((M + 128,), 55.0, dtype=torch.float32, device=dev)
        y = buf[64:64 + M]
        rc = L.spqt_calib_rowmajor_gemv(qd.data_ptr(), sd.data_ptr(), M, K, xd.data_ptr(), t, skip, y.data_ptr(), st)
        assert rc == 0
        torch.cuda.synchronize()
        out = buf.cpu().numpy()
        assert np.all(out[:64] == 55.0) and np.all(out[64 + M:] == 55.0), "write outside y"
        ref = oracle.gemv(q, sc, x, t)[0]
        err = np.abs(out[64:64 + M].astype(np.float64) - ref)
        assert np.all(err <= ATOL + RTOL * np.abs(ref)), f"skip={skip}: max err {err.max():.3e}"
