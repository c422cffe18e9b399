"""GPU parity of the one-launch kernel for several activation rows (spqt_gemv_fused_rows) against the
oracle, through the C ABI: the union mode against the oracle's union GEMV (a column is visited if any row
keeps it, every row takes every visited column), the own-sets mode against the oracle's batch-1 result
of every row alone.  Tolerance |y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref|."""
import numpy as np
import pytest

import oracle
from workloads import make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3
CANARY = 12288.0    # exact in fp16 too


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
    bad = ~(err <= ATOL + RTOL * np.abs(ref))
    assert not bad.any(), f"{what}: {int(bad.sum())} outputs off, max err {np.nanmax(err):.3e}"


def run(gpu, packed, M, K, group, x_np, thr, own, splits=0, y_half=False):
    """y sits inside a larger buffer filled with a canary so that a write outside [batch][M] shows."""
    torch, spqt, dev = gpu
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    batch = x.shape[0]
    dt = torch.float16 if y_half else torch.float32
    buf = torch.full((batch * M + 512,), CANARY, dtype=dt, device=dev)
    y = buf[256:256 + batch * M].view(batch, M)
    ws = spqt.new_workspace(M, K, batch)
    for rep in range(2):    # twice on one workspace: the epochs advance
        spqt.spqt_gemv_fused_rows(packed, M, K, x if batch > 1 else x[0], thr, y if batch > 1 else y[0], ws, own_sets=own,
                                  group=group, splits=splits)
    torch.cuda.synchronize()
    out = buf.float().cpu().numpy()
    assert np.all(out[:256] == CANARY) and np.all(out[256 + batch * M:] == CANARY), "write outside y"
    return out[256:256 + batch * M].reshape(batch, M)


def own_sets_reference(q, sc, x, thr, group):
    """Row b alone through the oracle's batch-1 GEMV."""
    return np.stack([oracle.gemv(q, sc, x[b:b + 1], thr, group=group)[0] for b in range(x.shape[0])])


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1000, 2048), (2048, 4096), (300, 8192)])
@pytest.mark.parametrize("batch", [2, 3, 4])
@pytest.mark.parametrize("group", [128, 64])
def test_fused_rows_match_oracle(gpu, M, K, batch, group):
    torch, spqt, dev = gpu
    Mp = 256 * ((M + 255) // 256)
    w = make_weights(Mp, K, 9900 + M + K, group=group)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    packed = torch.from_numpy(spqt.spqt_pack(q, sc, group)).to(dev)
    x = make_x(K, "laplace", 9901 + M + batch, batch=batch)
    for s in (0.0, 0.5, 0.9, 1.0):
        thr = 0.0 if s == 0.0 else (float("inf") if s == 1.0 else quantile_threshold(x, s))
        ref_union = oracle.gemv(q, sc, x, thr, group=group)
        ref_own = own_sets_reference(q, sc, x, thr, group)
        for splits in (0, 1, 5, 16):
            say(f"fused rows M={M} K={K} batch={batch} group={group} s={s} splits={splits}")
            assert_close(run(gpu, packed, M, K, group, x, thr, False, splits), ref_union, f"union s={s} splits={splits}")
            assert_close(run(gpu, packed, M, K, group, x, thr, True, splits), ref_own, f"own sets s={s} splits={splits}")


def test_fused_rows_full_size_and_fp16_output(gpu):
    """The 70B gate shape, 4 rows, default launch shape; fp16 output is the fp32 output rounded."""
    torch, spqt, dev = gpu
    from workloads import make_case
    case = make_case(5, "gate", batch=4, want_q=False)
    M, K = case["M"], case["K"]
    q, sc, x = case["q_rowmajor"], case["scales"], case["x"]
    packed = torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)
    thr = quantile_threshold(x, 0.5)
    say(f"fused rows full size M={M} K={K}")
    rows = np.random.default_rng(9950).choice(M, size=512, replace=False)
    rows.sort()
    got_u = run(gpu, packed, M, K, 128, x, thr, False)
    got_o = run(gpu, packed, M, K, 128, x, thr, True)
    assert_close(got_u[:, rows], oracle.gemv_rows(q, sc, x, thr, rows), "union, sampled rows")
    ref_o = np.stack([oracle.gemv_rows(q, sc, x[b:b + 1], thr, rows)[0] for b in range(4)])
    assert_close(got_o[:, rows], ref_o, "own sets, sampled rows")
    half = run(gpu, packed, M, K, 128, x, thr, True, y_half=True)
    assert np.array_equal(half, got_o.astype(np.float16).astype(np.float32)), "fp16 output is the fp32 output rounded"


def test_fused_rows_batch1_and_equal_rows(gpu):
    """batch 1 forwards to the one-row kernel; four equal rows give four equal results in both modes."""
    torch, spqt, dev = gpu
    M, K = 1024, 2048
    w = make_weights(M, K, 9960)
    q, sc = w["q_rowmajor"], w["scales"]
    packed = torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)
    x1 = make_x(K, "laplace", 9961)
    thr = quantile_threshold(x1, 0.6)
    ref = oracle.gemv(q, sc, x1, thr)
    assert_close(run(gpu, packed, M, K, 128, x1, thr, False), ref, "batch 1")
    x4 = np.ascontiguousarray(np.repeat(x1, 4, axis=0))
    for own in (False, True):
        y4 = run(gpu, packed, M, K, 128, x4, thr, own)
        assert all(np.array_equal(y4[b], y4[0]) for b in range(4))
        assert_close(y4[:1], ref, f"equal rows own={own}")
