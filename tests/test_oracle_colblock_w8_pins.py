"""Pins for the 8-bit column-block oracle (oracle/colblock_w8.py): each test checks it against
something other than its own formula - exactly representable inputs, error bounds, symmetries,
hand-made rounding cases, pure-Python brute force, independent NumPy expressions, closed-form byte
positions, and the 4-bit oracle (a finer grid must not be less accurate).  The paper (Section
4.1.3) only states that the layout carries over to other bit-widths; format and rule are this
build's reading, stated in the oracle's header."""
import numpy as np
import pytest

from oracle import colblock as cb4
from oracle import colblock_w8 as cb
from workloads import make_fp_weights, make_x, quantile_threshold


def representable(M, K, seed):
    """W = q0 * s0 with max|q0| = 127 in every block and power-of-two s0: quantization must be exact."""
    rng = np.random.default_rng(seed)
    q0 = rng.integers(-127, 128, size=(M, K)).astype(np.int16)
    q0.reshape(M // 32, 32, K)[:, 0, :] = 127 * rng.choice([-1, 1], size=(M // 32, K))
    s0 = (2.0 ** rng.integers(-12, -5, size=(M // 32, K))).astype(np.float16)
    W = (q0.astype(np.float32) * np.repeat(s0.astype(np.float32), 32, axis=0)).astype(np.float32)
    return W, q0, s0


def test_representable_matrix_quantizes_exactly():
    W, q0, s0 = representable(256, 256, 1)
    q, s = cb.quantize(W)
    assert np.array_equal(q, q0)
    assert np.array_equal(s.view(np.uint16), s0.view(np.uint16))
    assert np.array_equal(cb.dequant(q, s), W.astype(np.float64))


def test_error_bound_code_range_and_finer_than_four_bits():
    W = make_fp_weights(512, 384, 2)
    q, s = cb.quantize(W)
    assert q.min() >= -128 and q.max() <= 127
    sf = np.repeat(s.astype(np.float64), 32, axis=0)
    err = np.abs(cb.dequant(q, s) - W.astype(np.float64))
    # half a step, plus what rounding the scale to fp16 (relative 2^-11) can push the largest weight
    assert np.all(err <= 0.5 * sf + 127.0 * sf * 2.0 ** -11 + 1e-12)
    assert np.all(np.max(np.abs(q.reshape(-1, 32, 384)), axis=1)[s.astype(np.float32) > 0] == 127)
    q4, s4 = cb4.quantize(W)
    err4 = np.abs(cb4.dequant(q4, s4) - W.astype(np.float64))
    assert np.sqrt(np.mean(err ** 2)) < np.sqrt(np.mean(err4 ** 2)) / 10     # 127/7 = 18 times finer steps


def test_zero_and_tiny_blocks():
    W = make_fp_weights(128, 128, 3)
    W[0:32, 5] = 0.0
    W[32:64, 9] = np.float32(1e-9)        # max/127 rounds to fp16 zero
    q, s = cb.quantize(W)
    assert s[0, 5] == 0 and np.all(q[0:32, 5] == 0)
    assert s[1, 9] == 0 and np.all(q[32:64, 9] == 0)
    d = cb.dequant(q, s)
    assert np.all(d[0:32, 5] == 0) and np.all(d[32:64, 9] == 0)


def test_scale_and_sign_symmetry():
    W = make_fp_weights(128, 256, 4)
    q, s = cb.quantize(W)
    q2, s2 = cb.quantize(W * np.float32(2.0))
    assert np.array_equal(q2, q) and np.array_equal(s2.astype(np.float32), s.astype(np.float32) * 2)
    qn, sn = cb.quantize(-W)
    assert np.array_equal(sn.view(np.uint16), s.view(np.uint16)) and np.array_equal(qn, -q)


def test_ties_round_to_even():
    W = np.zeros((128, 128), dtype=np.float32)
    vals = [127.0, 2.5, 3.5, -2.5, 0.5, 1.5, -0.5, -126.5, 126.5, -127.0, 100.5, -101.5]
    W[: len(vals), 0] = vals                      # scale = 127/127 = 1 exactly
    q, s = cb.quantize(W)
    assert float(s[0, 0]) == 1.0
    assert q[: len(vals), 0].tolist() == [127, 2, 4, -2, 0, 2, 0, -126, 126, -127, 100, -102]


def test_quantizer_against_pure_python():
    W = make_fp_weights(128, 128, 5)
    q, s = cb.quantize(W)
    rng = np.random.default_rng(6)
    for _ in range(300):
        b, k = int(rng.integers(0, 4)), int(rng.integers(0, 128))
        col = [float(v) for v in W[32 * b:32 * b + 32, k]]
        amax = max(abs(v) for v in col)
        sc = float(np.float16(np.float32(amax) / np.float32(127.0)))
        assert sc == float(s[b, k])
        for r, v in enumerate(col):
            ratio = v / sc
            if abs(abs(ratio - np.floor(ratio)) - 0.5) < 1e-3:
                continue                      # too close to a tie for a double-precision cross-check
            assert int(q[32 * b + r, k]) == max(-128, min(127, int(round(ratio))))


def case(M, K, seed, s=0.5):
    W = make_fp_weights(M, K, seed)
    q, sc = cb.quantize(W)
    x = make_x(K, "laplace", seed + 1)
    return q, sc, x, quantile_threshold(x, s)


def test_gemv_threshold_zero_is_dense_product():
    q, sc, x, _ = case(256, 256, 10)
    Wd = (q.reshape(-1, 32, 256).astype(np.float64) * sc.astype(np.float64)[:, None, :]).reshape(256, 256)
    assert np.allclose(cb.gemv(q, sc, x, 0.0)[0], Wd @ x[0].astype(np.float64), rtol=1e-12, atol=1e-12)


def test_gemv_threshold_inf_is_zero_and_definition():
    q, sc, x, thr = case(128, 256, 11)
    assert np.all(cb.gemv(q, sc, x, float("inf")) == 0)
    xz = x.copy()
    xz[np.abs(xz.astype(np.float32)) < np.float32(thr)] = 0
    assert np.allclose(cb.gemv(q, sc, x, thr), cb.gemv(q, sc, xz, 0.0), rtol=1e-12, atol=1e-12)
    kept = np.flatnonzero(~(np.abs(x[0].astype(np.float32)) < np.float32(thr)))
    assert np.array_equal(np.flatnonzero(cb.keep_mask(x, thr)), kept) and 0 < kept.size < 256


def test_gemv_brute_force_pure_python():
    q, sc, x, thr = case(128, 128, 12)
    got = cb.gemv(q, sc, x, thr)[0]
    xs = [float(v) for v in x[0]]
    for m in range(0, 128, 9):
        acc = 0.0
        for k in range(128):
            if not (abs(float(np.float32(x[0, k]))) < float(np.float32(thr))):
                acc += int(q[m, k]) * float(sc[m // 32, k]) * xs[k]
        assert abs(acc - got[m]) <= 1e-9 * max(1.0, abs(acc))


def test_gemv_column_probe_and_additivity():
    q, sc, x, _ = case(128, 128, 13)
    for k in range(128):
        e = np.zeros((1, 128), dtype=np.float16)
        e[0, k] = -1.5
        want = -1.5 * q[:, k].astype(np.float64) * np.repeat(sc[:, k].astype(np.float64), 32)
        assert np.array_equal(cb.gemv(q, sc, e, 0.5)[0], want)
    a, b = x.copy(), x.copy()
    a[0, 64:] = 0
    b[0, :64] = 0
    assert np.allclose(cb.gemv(q, sc, a, 0.0) + cb.gemv(q, sc, b, 0.0), cb.gemv(q, sc, x, 0.0), rtol=1e-12, atol=1e-12)


def test_gemv_approaches_the_unquantized_product():
    """An 8-bit grid reproduces W x to about a percent of a 4-bit grid's error."""
    W = make_fp_weights(256, 512, 14)
    x = make_x(512, "laplace", 15)
    exact = W.astype(np.float64) @ x[0].astype(np.float64)
    q, s = cb.quantize(W)
    q4, s4 = cb4.quantize(W)
    e8 = np.abs(cb.gemv(q, s, x, 0.0)[0] - exact)
    e4 = np.abs(cb4.gemv(q4, s4, x, 0.0)[0] - exact)
    assert np.sqrt(np.mean(e8 ** 2)) < np.sqrt(np.mean(e4 ** 2)) / 10
    assert np.sqrt(np.mean(e8 ** 2)) < 1e-2 * np.sqrt(np.mean(exact ** 2))


def test_pack_size_and_round_trip():
    assert cb.packed_bytes(128, 128) == 17408
    assert cb.packed_bytes(4096, 4096) == 4096 * 4096 + (4096 // 32) * 4096 * 2
    q, sc, _, _ = case(384, 384, 16)
    p = cb.pack(q, sc)
    assert p.nbytes == cb.packed_bytes(384, 384)
    q2, s2 = cb.unpack(p, 384, 384)
    assert np.array_equal(q2, q) and np.array_equal(s2.view(np.uint16), sc.view(np.uint16))


def test_pack_closed_form_positions():
    M, K = 384, 384
    NC = K // 128
    rng = np.random.default_rng(17)
    zero_q = np.zeros((M, K), dtype=np.int16)
    zero_s = np.zeros((M // 32, K), dtype=np.float16)
    base = cb.pack(zero_q, zero_s)
    assert np.all(base.reshape(-1, 17408)[:, 1024:] == 128) and np.all(base.reshape(-1, 17408)[:, :1024] == 0)
    for _ in range(40):
        m, k = int(rng.integers(0, M)), int(rng.integers(0, K))
        q = zero_q.copy()
        q[m, k] = -77
        p = cb.pack(q, zero_s)
        at = ((m // 128) * NC + k // 128) * 17408 + 1024 + (k % 128) * 128 + (m % 128)
        assert np.flatnonzero(p != base).tolist() == [at] and int(p[at]) == 128 - 77
        mb = int(rng.integers(0, M // 32))
        s = zero_s.copy()
        s.view(np.uint16)[mb, k] = 0xBEEF
        p = cb.pack(zero_q, s)
        at = ((mb // 4) * NC + k // 128) * 17408 + 8 * (k % 128) + 2 * (mb % 4)
        assert np.flatnonzero(p != base).tolist() == [at, at + 1]
        assert p[at] == 0xEF and p[at + 1] == 0xBE
    q = zero_q.copy()
    q[0, 0], q[1, 0] = -128, 127                    # the extreme codes
    p = cb.pack(q, zero_s)
    assert int(p[1024]) == 0 and int(p[1025]) == 255


@pytest.mark.parametrize("M,K", [(127, 128), (128, 100), (0, 128)])
def test_bad_shapes(M, K):
    with pytest.raises(ValueError):
        cb.packed_bytes(M, K)


def test_pad_rows():
    W = make_fp_weights(256, 128, 18)[:130]
    P = cb.pad_rows(W)
    assert P.shape == (256, 128) and np.array_equal(P[:130], W) and np.all(P[130:] == 0)
    assert cb.pad_rows(P) is P
