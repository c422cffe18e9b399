"""Pins for the K-quant column-block oracle (oracle/colblock_k.py), none of which re-uses its
formulas: exactly representable superblocks, error bounds, special blocks, symmetries, a
pure-Python cross-check, independent NumPy expressions, closed-form byte and bit positions.
Format: paper Section 4.1.1 (Q4_K: 256-weight superblocks of eight 32-weight blocks, 6-bit block
scales and minima, 16-bit superblock scales) on the column-wise superblocks of Section 4.1.2."""
import numpy as np
import pytest

from oracle import colblock_k as ck
from workloads import make_fp_weights, make_x, quantile_threshold


def representable(M, K, seed):
    """W = (d*sc)*q - dmin*m with power-of-two d, dmin = d/4, sc in 16..63 and m in 0..63 reaching 63
    in every superblock, and q covering 0 and 15 in every block: the quantizer must recover all of it."""
    rng = np.random.default_rng(seed)
    T = M // 256
    d = (2.0 ** rng.integers(-12, -6, size=(T, K))).astype(np.float16)
    dmin = (d.astype(np.float32) / 4).astype(np.float16)
    sc = rng.integers(16, 64, size=(M // 32, K)).astype(np.uint8)
    m = rng.integers(0, 64, size=(M // 32, K)).astype(np.uint8)
    sc.reshape(T, 8, K)[:, 3, :] = 63
    m.reshape(T, 8, K)[:, 5, :] = 63
    q = rng.integers(0, 16, size=(M, K)).astype(np.uint8)
    q.reshape(M // 32, 32, K)[:, 0, :] = 0
    q.reshape(M // 32, 32, K)[:, 1, :] = 15
    se = np.repeat(d.astype(np.float32), 8, axis=0) * sc
    me = np.repeat(dmin.astype(np.float32), 8, axis=0) * m
    W = (np.repeat(se, 32, axis=0) * q - np.repeat(me, 32, axis=0)).astype(np.float32)
    return W, {"q": q, "sc": sc, "m": m, "d": d, "dmin": dmin}


def test_representable_superblocks_quantize_exactly():
    W, p0 = representable(512, 256, 1)
    p = ck.quantize(W)
    for key in ("q", "sc", "m"):
        assert np.array_equal(p[key], p0[key]), key
    for key in ("d", "dmin"):
        assert np.array_equal(p[key].view(np.uint16), p0[key].view(np.uint16)), key
    assert np.array_equal(ck.dequant(p), W.astype(np.float64))


def test_ranges_and_error_bound():
    W = make_fp_weights(512, 384, 2)
    p = ck.quantize(W)
    assert p["q"].max() <= 15 and p["sc"].max() <= 63 and p["m"].max() <= 63
    d = np.repeat(p["d"].astype(np.float64), 256, axis=0)
    dm = np.repeat(p["dmin"].astype(np.float64), 256, axis=0)
    se = d * np.repeat(p["sc"].astype(np.float64), 32, axis=0)
    err = np.abs(ck.dequant(p) - W.astype(np.float64))
    # half a step of the effective scale, plus what rounding the block scale / minimum to 6 bits and
    # the superblock scales to fp16 can move the ends of the block's range
    bound = 0.5 * se + (0.5 + 63 * 2.0 ** -11) * dm + 15 * (0.5 + 63 * 2.0 ** -11) * d + 1e-12
    assert np.all(err <= bound)
    # and the quantization really is 4-bit fine: typical error well under a step
    assert np.median(err / np.maximum(se, 1e-30)) < 0.3
    # every superblock uses the top of both 6-bit ranges
    assert np.all(p["sc"].reshape(-1, 8, 384).max(axis=1)[p["d"].astype(np.float32) > 0] == 63)


def test_special_blocks():
    W = make_fp_weights(256, 128, 3)
    W[:, 5] = 0.0                                   # a whole zero superblock
    W[0:32, 9] = np.abs(W[0:32, 9]) + 0.01          # an all-positive block: minimum 0
    W[32:64, 9] = -np.abs(W[32:64, 9]) - 0.01       # an all-negative block: its top code stands for <= 0
    p = ck.quantize(W)
    assert p["d"].view(np.uint16)[0, 5] == 0 and p["dmin"].view(np.uint16)[0, 5] == 0 and np.all(p["q"][:, 5] == 0)
    assert np.all(ck.dequant(p)[:, 5] == 0)
    assert p["m"][0, 9] == 0
    d = ck.dequant(p)
    assert np.all(d[0:32, 9] >= 0) and np.all(d[32:64, 9] <= 1e-12)


def test_scaling_by_two_keeps_every_code():
    W = make_fp_weights(256, 256, 4)
    a, b = ck.quantize(W), ck.quantize(W * np.float32(2.0))
    for key in ("q", "sc", "m"):
        assert np.array_equal(a[key], b[key]), key
    assert np.array_equal(b["d"].astype(np.float32), a["d"].astype(np.float32) * 2)
    assert np.array_equal(b["dmin"].astype(np.float32), a["dmin"].astype(np.float32) * 2)


def test_quantizer_against_pure_python():
    W = make_fp_weights(256, 128, 5)
    p = ck.quantize(W)
    rng = np.random.default_rng(6)
    near_tie = lambda r: abs(abs(r - np.floor(r)) - 0.5) < 1e-4
    for _ in range(60):
        k = int(rng.integers(0, 128))
        col = [float(v) for v in W[:, k]]
        sb, mb = [], []
        for b in range(8):
            blk = col[32 * b:32 * b + 32]
            lo, hi = min(min(blk), 0.0), max(max(blk), 0.0)
            sb.append(float(np.float32(np.float32(hi) - np.float32(lo)) / np.float32(15)))
            mb.append(-lo)
        d = float(np.float16(np.float32(max(sb)) / np.float32(63)))
        dm = float(np.float16(np.float32(max(mb)) / np.float32(63)))
        assert d == float(p["d"][0, k]) and dm == float(p["dmin"][0, k])
        for b in range(8):
            if near_tie(sb[b] / d) or near_tie(mb[b] / dm):
                continue
            sc = max(0, min(63, int(round(sb[b] / d))))
            m = max(0, min(63, int(round(mb[b] / dm))))
            assert sc == int(p["sc"][b, k]) and m == int(p["m"][b, k])
            se, me = d * sc, dm * m
            for r in range(32):
                ratio = (col[32 * b + r] + me) / se if se > 0 else 0.0
                if near_tie(ratio):
                    continue
                assert int(p["q"][32 * b + r, k]) == max(0, min(15, int(round(ratio))))


def case(M, K, seed, s=0.5):
    p = ck.quantize(make_fp_weights(M, K, seed))
    x = make_x(K, "laplace", seed + 1)
    return p, x, quantile_threshold(x, s)


def test_gemv_threshold_zero_is_dense_product():
    p, x, _ = case(512, 256, 10)
    d = np.repeat(p["d"].astype(np.float64), 8, axis=0)
    dm = np.repeat(p["dmin"].astype(np.float64), 8, axis=0)
    Wd = (p["q"].reshape(-1, 32, 256) * (d * p["sc"])[:, None, :] - (dm * p["m"])[:, None, :]).reshape(512, 256)
    assert np.allclose(ck.gemv(p, x, 0.0)[0], Wd @ x[0].astype(np.float64), rtol=1e-12, atol=1e-12)


def test_gemv_threshold_inf_definition_and_brute_force():
    p, x, thr = case(256, 128, 11)
    assert np.all(ck.gemv(p, x, float("inf")) == 0)
    xz = x.copy()
    xz[np.abs(xz.astype(np.float32)) < np.float32(thr)] = 0
    assert np.allclose(ck.gemv(p, x, thr), ck.gemv(p, xz, 0.0), rtol=1e-12, atol=1e-12)
    got = ck.gemv(p, x, thr)[0]
    for mrow in range(0, 256, 19):
        acc = 0.0
        for k in range(128):
            if not (abs(float(np.float32(x[0, k]))) < float(np.float32(thr))):
                b = mrow // 32
                val = float(p["d"][0, k]) * int(p["sc"][b, k]) * int(p["q"][mrow, k]) - float(p["dmin"][0, k]) * int(p["m"][b, k])
                acc += val * float(x[0, k])
        assert abs(acc - got[mrow]) <= 1e-9 * max(1.0, abs(acc))


def test_gemv_column_probe():
    p, x, _ = case(256, 128, 12)
    Wd = ck.dequant(p)
    for k in range(128):
        e = np.zeros((1, 128), dtype=np.float16)
        e[0, k] = 2.5
        assert np.array_equal(ck.gemv(p, e, 1.0)[0], 2.5 * Wd[:, k])


def test_pack_round_trip_and_size():
    assert ck.packed_bytes(256, 128) == 18432
    p, _, _ = case(512, 384, 13)
    pk = ck.pack(p)
    assert pk.nbytes == ck.packed_bytes(512, 384)
    back = ck.unpack(pk, 512, 384)
    for key in ("q", "sc", "m"):
        assert np.array_equal(back[key], p[key]), key
    for key in ("d", "dmin"):
        assert np.array_equal(back[key].view(np.uint16), p[key].view(np.uint16)), key


def test_pack_closed_form_positions():
    M, K = 512, 256
    NC = K // 128
    zero = {"q": np.zeros((M, K), np.uint8), "sc": np.zeros((M // 32, K), np.uint8), "m": np.zeros((M // 32, K), np.uint8),
            "d": np.zeros((M // 256, K), np.float16), "dmin": np.zeros((M // 256, K), np.float16)}
    assert not ck.pack(zero).any()
    rng = np.random.default_rng(14)
    for _ in range(30):
        mrow, k = int(rng.integers(0, M)), int(rng.integers(0, K))
        chunk = ((mrow // 256) * NC + k // 128) * 18432
        head = chunk + 16 * (k % 128)
        p = {key: v.copy() for key, v in zero.items()}
        p["q"][mrow, k] = 11
        nz = np.flatnonzero(ck.pack(p))
        at = chunk + 2048 + (k % 128) * 128 + (mrow % 256) // 2
        assert nz.tolist() == [at] and int(ck.pack(p)[at]) == 11 << (4 * (mrow % 2))
        p = {key: v.copy() for key, v in zero.items()}
        p["d"].view(np.uint16)[mrow // 256, k] = 0xBEEF
        p["dmin"].view(np.uint16)[mrow // 256, k] = 0x1234
        pk = ck.pack(p)
        assert np.flatnonzero(pk).tolist() == [head, head + 1, head + 2, head + 3]
        assert pk[head:head + 4].tolist() == [0xEF, 0xBE, 0x34, 0x12]
        b = (mrow % 256) // 32
        for field, base in (("sc", 0), ("m", 48)):
            p = {key: v.copy() for key, v in zero.items()}
            p[field][mrow // 32, k] = 63
            pk = ck.pack(p)
            value = 0
            for byte in range(12):
                value |= int(pk[head + 4 + byte]) << (8 * byte)
            assert value == 63 << (base + 6 * b)
            assert not pk[:head + 4].any() and not pk[head + 16:].any()


@pytest.mark.parametrize("M,K", [(255, 128), (256, 100)])
def test_bad_shapes(M, K):
    with pytest.raises(ValueError):
        ck.packed_bytes(M, K)
