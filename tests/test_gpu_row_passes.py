"""GPU parity for the two ways the index-list GEMV for one activation row consumes its list - row-aligned
passes (the default: only a row of 8 slots must be of one quantization group) and one-group passes
(SPQT_CFG_GROUP_PASSES) - against the oracle: |y_gpu - y_ref| <= 1e-2 + 2e-3 * |y_ref| on the same
seeded inputs.  Sparsities from 0 to 1 put from one to many groups into a pass; the hand-made lists
cover what a threshold on iid activations never produces."""
import numpy as np
import pytest

import oracle
from workloads import make_weights, make_x, quantile_threshold

pytestmark = pytest.mark.gpu

ATOL, RTOL = 1e-2, 2e-3
CANARY = 12288.0


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


def run(gpu, packed, M, K, group, x_np, thr, splits, waves, idx_np=None, flags=0):
    torch, spqt, dev = gpu
    x = torch.from_numpy(np.ascontiguousarray(x_np)).to(dev)
    buf = torch.full((M + 512,), CANARY, dtype=torch.float32, device=dev)
    y = buf[256:256 + M]
    ws = spqt.new_workspace(M, K, 1)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    if idx_np is None:
        spqt.spqt_gather(x, thr, idx, cnt)
    else:
        idx[:len(idx_np)] = torch.from_numpy(idx_np.astype(np.int32)).to(dev)
        cnt.fill_(len(idx_np))
    for rep in range(2):    # twice on one workspace: the epochs advance
        spqt.spqt_gemv(packed, M, K, x, idx, cnt, y, ws, group=group, splits=splits, waves=waves, flags=flags)
    torch.cuda.synchronize()
    out = buf.cpu().numpy()
    assert np.all(out[:256] == CANARY) and np.all(out[256 + M:] == CANARY), "write outside y"
    return out[256:256 + M]


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (1000, 2048), (2048, 4096), (4096, 4096), (300, 8192)])
@pytest.mark.parametrize("group", [128, 64])
def test_list_passes_match_oracle(gpu, M, K, group):
    torch, spqt, dev = gpu
    Mp = 256 * ((M + 255) // 256)
    w = make_weights(Mp, K, 9600 + M + K, group=group)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    packed = torch.from_numpy(spqt.spqt_pack(q, sc, group)).to(dev)
    x = make_x(K, "laplace", 9601 + M)
    for s in (0.0, 0.3, 0.5, 0.7, 0.9, 0.97, 0.995, 1.0):
        thr = 0.0 if s == 0.0 else (float("inf") if s == 1.0 else quantile_threshold(x, s))
        ref = oracle.gemv(q, sc, x, thr, group=group)[0]
        for splits, waves in ((0, 0), (1, 1), (3, 2), (16, 4)):
            for flags in (0, spqt.CFG_GROUP_PASSES):
                say(f"list passes M={M} K={K} group={group} s={s} splits={splits} waves={waves} flags={flags}")
                assert_close(run(gpu, packed, M, K, group, x, thr, splits, waves, flags=flags), ref,
                             f"s={s} splits={splits} waves={waves} flags={flags}")


def test_list_passes_clustered_and_unordered_lists(gpu):
    """Lists that are not what a threshold on iid activations gives: whole groups kept and whole groups
    dropped, one kept column per group, and a caller-made list in descending order."""
    torch, spqt, dev = gpu
    M, K = 1024, 4096
    w = make_weights(M, K, 9700)
    q, sc = w["q_rowmajor"], w["scales"]
    packed = torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)
    x = make_x(K, "laplace", 9701)
    xf = x.astype(np.float64)[0]
    Wd = oracle.dequant(q, sc)
    lists = {
        "every other group": np.concatenate([np.arange(g * 128, g * 128 + 128) for g in range(0, K // 128, 2)]),
        "one per group": np.arange(5, K, 128),
        "nine per group": np.concatenate([np.arange(g * 128 + 3, g * 128 + 12) for g in range(K // 128)]),
        "descending": np.arange(K - 1, -1, -3),
        "single column": np.array([K - 1]),
    }
    for name, lst in lists.items():
        ref = Wd[:, lst] @ xf[lst]
        for splits, waves in ((0, 0), (1, 4), (7, 1)):
            for flags in (0, spqt.CFG_GROUP_PASSES):
                say(f"list '{name}' splits={splits} waves={waves} flags={flags}")
                assert_close(run(gpu, packed, M, K, 128, x, 0.0, splits, waves, idx_np=lst, flags=flags), ref, name)


def test_one_workspace_across_kernels_and_launch_shapes(gpu):
    """Calls of every group-layout kernel, in launch shapes that lay the exchanged words out differently
    (any number of workgroups per block-row), alternate on ONE workspace with the same M: the tags
    must keep words left by earlier calls from being taken for this call's."""
    torch, spqt, dev = gpu
    M, K = 2816, 2048          # 11 block-rows
    w = make_weights(M, K, 9800)
    q, sc = w["q_rowmajor"], w["scales"]
    packed = torch.from_numpy(spqt.spqt_pack(q, sc)).to(dev)
    ws = spqt.new_workspace(M, K, 1)
    idx = torch.empty(K, dtype=torch.int32, device=dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    y = torch.empty(M, dtype=torch.float32, device=dev)
    rng = np.random.default_rng(9801)
    shapes = [(0, 0), (16, 4), (5, 4), (3, 2), (64, 1), (7, 4), (2, 1), (13, 2)]
    for it in range(24):
        x_np = make_x(K, "laplace", 9802 + it)
        thr = quantile_threshold(x_np, float(rng.uniform(0.1, 0.95)))
        x = torch.from_numpy(x_np[0]).to(dev)
        splits, waves = shapes[int(rng.integers(len(shapes)))]
        kind = ("rows", "groups", "dense", "fused")[it % 4]
        say(f"shared workspace it={it} kind={kind} splits={splits} waves={waves}")
        y.fill_(float("nan"))
        if kind == "fused":
            spqt.spqt_gemv_fused(packed, M, K, x, thr, y, ws, splits=splits, waves=waves)
        elif kind == "dense":
            spqt.spqt_gemv(packed, M, K, x, None, None, y, ws, splits=splits, waves=waves)
        else:
            spqt.spqt_gather(x, thr, idx, cnt)
            spqt.spqt_gemv(packed, M, K, x, idx, cnt, y, ws, splits=splits, waves=waves,
                           flags=spqt.CFG_GROUP_PASSES if kind == "groups" else 0)
        torch.cuda.synchronize()
        ref = oracle.gemv(q, sc, x_np, 0.0 if kind == "dense" else thr)[0]
        assert_close(y.cpu().numpy(), ref, f"it={it} {kind} {splits}x{waves}")
