"""The bounded wait of the exchange between the workgroups of a block-row, on the GPU: what happens when a
reducer abandons its wait.  libspqt_giveup.so is the group-layout GEMV built with silent producers and a wait
of a handful of polls, so the give-up path runs on every launch that has several workgroups per block-row
while every kernel still ends normally.  Expected: the affected outputs are NaN (never silently wrong), the
workspace's poison flag is raised, every later call on that workspace - from the product library too - yields
NaN until spqt_workspace_init clears it, and after the init the product library is right again."""
import ctypes
import os

import numpy as np
import pytest

import oracle
from workloads import make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2511_04477_amd as spqt
    assert torch.cuda.is_available(), "these tests need the MI355X"
    spqt.lib()
    path = os.path.join(os.path.dirname(spqt.__file__), "libspqt_giveup.so")
    assert os.path.exists(path), "libspqt_giveup.so is not built (python -m paper_2511_04477_amd.build)"
    G = ctypes.CDLL(path)
    vp, i64, i32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
    G.spqt_gemv_ex.argtypes = [vp, i64, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp, ctypes.POINTER(spqt.LaunchCfg)]
    G.spqt_gemv_fused.argtypes = [vp, i64, i64, i32, vp, ctypes.c_float, vp, vp, sz, vp, ctypes.POINTER(spqt.LaunchCfg)]
    return torch, spqt, torch.device("cuda:0"), G


def test_abandoned_wait_gives_nan_and_poisons_the_workspace(gpu):
    torch, spqt, dev, G = gpu
    M, K = 1024, 2048
    case = make_weights(M, K, 4242)
    x_np = make_x(K, "laplace", 4243)
    thr = quantile_threshold(x_np, 0.5)
    ref = oracle.gemv(case["q_rowmajor"], case["scales"], x_np, thr)[0]
    packed = torch.from_numpy(spqt.spqt_pack(case["q_rowmajor"], case["scales"])).to(dev)
    x = torch.from_numpy(x_np[0].copy()).to(dev)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    spqt.spqt_gather(x, thr, idx, cnt)
    ws = spqt.new_workspace(M, K)
    y = torch.zeros(M, dtype=torch.float32, device=dev)

    def close(y_t):
        got = y_t.cpu().numpy().astype(np.float64)
        return bool(np.all(np.abs(got - ref) <= 1e-2 + 2e-3 * np.abs(ref)))

    def flag():
        return int(ws[:4].view(torch.int32).item())

    def give_up_call(splits, fused=False):
        cfg = spqt.LaunchCfg(splits, 4, 0)
        args = (packed.data_ptr(), M, K, 128, x.data_ptr())
        if fused:
            rc = G.spqt_gemv_fused(*args, ctypes.c_float(thr), y.data_ptr(), ws.data_ptr(), ws.numel(), None, ctypes.byref(cfg))
        else:
            rc = G.spqt_gemv_ex(*args, 1, idx.data_ptr(), cnt.data_ptr(), y.data_ptr(), ws.data_ptr(), ws.numel(), None,
                                ctypes.byref(cfg))
        assert rc == 0
        torch.cuda.synchronize()

    print("give-up: one workgroup per block-row needs no exchange", flush=True)
    give_up_call(1)
    assert close(y) and flag() == 0

    for fused in (False, True):
        print(f"give-up: four workgroups per block-row, fused={fused}", flush=True)
        spqt.spqt_workspace_init(ws)
        y.zero_()
        give_up_call(4, fused)
        assert bool(torch.isnan(y).all()), "an abandoned wait must leave NaN, not a partial sum"
        assert flag() == 1, "the poison flag must be raised"
        # nothing but the flag is left in the workspace: the reducer zeroed what it polled, the producers wrote nothing
        assert int(torch.count_nonzero(ws[256:]).item()) == 0

        print("give-up: the product library on the poisoned workspace", flush=True)
        y.zero_()
        spqt.spqt_gemv(packed, M, K, x, idx, cnt, y, ws, splits=4, waves=4)
        torch.cuda.synchronize()
        assert bool(torch.isnan(y).all()), "a poisoned workspace must keep yielding NaN"
        y.zero_()
        spqt.spqt_gemv(packed, M, K, x, idx, cnt, y, ws, splits=1, waves=4)      # no exchange, no flag to read
        torch.cuda.synchronize()
        assert close(y)

        print("give-up: after spqt_workspace_init", flush=True)
        spqt.spqt_workspace_init(ws)
        assert flag() == 0
        y.zero_()
        spqt.spqt_gemv(packed, M, K, x, idx, cnt, y, ws, splits=4, waves=4)
        torch.cuda.synchronize()
        assert close(y)
