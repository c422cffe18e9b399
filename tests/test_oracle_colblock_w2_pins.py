"""Pins for the 2-bit column-block oracle (oracle/colblock_w2.py): each test checks it against
something other than its own formula - exactly representable inputs, error bounds, symmetries,
hand-made rounding cases, pure-Python brute force, independent NumPy expressions, closed-form byte
and bit positions, and the 4-bit oracle (a coarser grid must not be more accurate).  The paper (Section
4.1.3) only states that the layout carries over to other bit-widths, 2 to 8 bits; format and rule are
this build's reading, stated in the oracle's header."""
import numpy as np
import pytest

from oracle import colblock as cb4
from oracle import colblock_w2 as cb
from workloads import make_fp_weights, make_x, quantile_threshold


def representable(M, K, seed):
    """W = (c0 - 1.5) * s0 with both outer levels present in every block and power-of-two s0: exact."""
    rng = np.random.default_rng(seed)
    c0 = rng.integers(0, 4, size=(M, K)).astype(np.uint8)
    c0.reshape(M // 32, 32, K)[:, 0, :] = rng.choice([0, 3], size=(M // 32, K))
    s0 = (2.0 ** rng.integers(-12, -3, size=(M // 32, K))).astype(np.float16)
    W = ((c0.astype(np.float32) - np.float32(1.5)) * np.repeat(s0.astype(np.float32), 32, axis=0)).astype(np.float32)
    return W, c0, s0


def test_representable_matrix_quantizes_exactly():
    W, c0, s0 = representable(512, 256, 1)
    c, s = cb.quantize(W)
    assert np.array_equal(c, c0)
    assert np.array_equal(s.view(np.uint16), s0.view(np.uint16))
    assert np.array_equal(cb.dequant(c, s), W.astype(np.float64))


def test_error_bound_code_range_and_coarser_than_four_bits():
    W = make_fp_weights(1024, 384, 2)
    c, s = cb.quantize(W)
    assert c.min() >= 0 and c.max() <= 3
    sf = np.repeat(s.astype(np.float64), 32, axis=0)
    err = np.abs(cb.dequant(c, s) - W.astype(np.float64))
    # half a step (a step is one scale), plus what rounding the scale to fp16 (relative 2^-11) can push the largest weight
    assert np.all(err <= 0.5 * sf + 1.5 * sf * 2.0 ** -11 + 1e-12)
    # every block with a non-zero scale reaches an outer level
    outer = np.max(np.abs(c.reshape(-1, 32, 384).astype(np.int16) * 2 - 3), axis=1)
    assert np.all(outer[s.astype(np.float32) > 0] == 3)
    q4, s4 = cb4.quantize(W[:1024])
    err4 = np.abs(cb4.dequant(q4, s4) - W.astype(np.float64))
    assert np.sqrt(np.mean(err ** 2)) > 2 * np.sqrt(np.mean(err4 ** 2))     # 4 levels against 16


def test_zero_and_tiny_blocks():
    W = make_fp_weights(512, 128, 3)
    W[0:32, 5] = 0.0
    W[32:64, 9] = np.float32(1e-9)        # max/1.5 rounds to fp16 zero
    c, s = cb.quantize(W)
    assert s[0, 5] == 0 and np.all(c[0:32, 5] == 0)
    assert s[1, 9] == 0 and np.all(c[32:64, 9] == 0)
    d = cb.dequant(c, s)
    assert np.all(d[0:32, 5] == 0) and np.all(d[32:64, 9] == 0)


def test_scale_and_sign_symmetry():
    W = make_fp_weights(512, 256, 4)
    c, s = cb.quantize(W)
    c2, s2 = cb.quantize(W * np.float32(2.0))
    assert np.array_equal(c2, c) and np.array_equal(s2.astype(np.float32), s.astype(np.float32) * 2)
    cn, sn = cb.quantize(-W)
    assert np.array_equal(sn.view(np.uint16), s.view(np.uint16))
    # mirrored levels, except exactly on a decision boundary (w/s in {-1, 0, 1}), where half-to-even
    # rounding of w/s + 1.5 is not mirror-symmetric; random fp32 weights never sit there
    assert np.array_equal(cn, 3 - c)


def test_decision_boundaries_and_ties():
    W = np.zeros((512, 128), dtype=np.float32)
    vals = [1.5, -1.5, 0.25, -0.25, 0.75, 1.25, -0.75, -1.25, 0.0, 1.0, -1.0, 0.999, -0.999, 1.001, -1.001]
    W[: len(vals), 0] = vals                      # scale = 1.5 / 1.5 = 1 exactly
    c, s = cb.quantize(W)
    assert float(s[0, 0]) == 1.0
    # w + 1.5 = 3, 0, 1.75, 1.25, 2.25, 2.75, 0.75, 0.25, 1.5 (tie -> 2), 2.5 (tie -> 2), 0.5 (tie -> 0), ...
    assert c[: len(vals), 0].tolist() == [3, 0, 2, 1, 2, 3, 1, 0, 2, 2, 0, 2, 1, 3, 0]


def test_quantizer_against_pure_python():
    W = make_fp_weights(512, 128, 5)
    c, s = cb.quantize(W)
    rng = np.random.default_rng(6)
    for _ in range(300):
        b, k = int(rng.integers(0, 16)), int(rng.integers(0, 128))
        col = [float(v) for v in W[32 * b:32 * b + 32, k]]
        amax = max(abs(v) for v in col)
        sc = float(np.float16(np.float32(amax) / np.float32(1.5)))
        assert sc == float(s[b, k])
        for r, v in enumerate(col):
            pos = v / sc + 1.5
            if abs(abs(pos - np.floor(pos)) - 0.5) < 1e-3:
                continue                      # too close to a tie for a double-precision cross-check
            assert int(c[32 * b + r, k]) == max(0, min(3, int(round(pos))))


def case(M, K, seed, s=0.5):
    W = make_fp_weights(M, K, seed)
    c, sc = cb.quantize(W)
    x = make_x(K, "laplace", seed + 1)
    return c, sc, x, quantile_threshold(x, s)


def test_gemv_threshold_zero_is_dense_product():
    c, sc, x, _ = case(512, 256, 10)
    Wd = ((c.reshape(-1, 32, 256).astype(np.float64) - 1.5) * sc.astype(np.float64)[:, None, :]).reshape(512, 256)
    assert np.allclose(cb.gemv(c, sc, x, 0.0)[0], Wd @ x[0].astype(np.float64), rtol=1e-12, atol=1e-12)


def test_gemv_threshold_inf_is_zero_and_definition():
    c, sc, x, thr = case(512, 256, 11)
    assert np.all(cb.gemv(c, sc, x, float("inf")) == 0)
    xz = x.copy()
    xz[np.abs(xz.astype(np.float32)) < np.float32(thr)] = 0
    assert np.allclose(cb.gemv(c, sc, x, thr), cb.gemv(c, sc, xz, 0.0), rtol=1e-12, atol=1e-12)
    kept = np.flatnonzero(~(np.abs(x[0].astype(np.float32)) < np.float32(thr)))
    assert np.array_equal(np.flatnonzero(cb.keep_mask(x, thr)), kept) and 0 < kept.size < 256


def test_gemv_brute_force_pure_python():
    c, sc, x, thr = case(512, 128, 12)
    got = cb.gemv(c, sc, x, thr)[0]
    xs = [float(v) for v in x[0]]
    for m in range(0, 512, 37):
        acc = 0.0
        for k in range(128):
            if not (abs(float(np.float32(x[0, k]))) < float(np.float32(thr))):
                acc += (int(c[m, k]) - 1.5) * float(sc[m // 32, k]) * xs[k]
        assert abs(acc - got[m]) <= 1e-9 * max(1.0, abs(acc))


def test_gemv_column_probe_and_additivity():
    c, sc, x, _ = case(512, 128, 13)
    for k in range(128):
        e = np.zeros((1, 128), dtype=np.float16)
        e[0, k] = -1.5
        want = -1.5 * (c[:, k].astype(np.float64) - 1.5) * np.repeat(sc[:, k].astype(np.float64), 32)
        assert np.array_equal(cb.gemv(c, sc, e, 0.5)[0], want)
    a, b = x.copy(), x.copy()
    a[0, 64:] = 0
    b[0, :64] = 0
    assert np.allclose(cb.gemv(c, sc, a, 0.0) + cb.gemv(c, sc, b, 0.0), cb.gemv(c, sc, x, 0.0), rtol=1e-12, atol=1e-12)


def test_gemv_is_a_coarse_but_unbiased_image_of_the_unquantized_product():
    """Four levels reproduce W x far worse than sixteen, yet the error stays a fraction of the product."""
    W = make_fp_weights(512, 512, 14)
    x = make_x(512, "laplace", 15)
    exact = W.astype(np.float64) @ x[0].astype(np.float64)
    c, s = cb.quantize(W)
    q4, s4 = cb4.quantize(W)
    e2 = np.abs(cb.gemv(c, s, x, 0.0)[0] - exact)
    e4 = np.abs(cb4.gemv(q4, s4, x, 0.0)[0] - exact)
    assert np.sqrt(np.mean(e2 ** 2)) > 2 * np.sqrt(np.mean(e4 ** 2))
    assert np.sqrt(np.mean(e2 ** 2)) < 0.7 * np.sqrt(np.mean(exact ** 2))


def test_pack_size_and_round_trip():
    assert cb.packed_bytes(512, 128) == 20480
    assert cb.packed_bytes(4096, 4096) == 4096 * 4096 // 4 + (4096 // 32) * 4096 * 2
    c, sc, _, _ = case(1024, 384, 16)
    p = cb.pack(c, sc)
    assert p.nbytes == cb.packed_bytes(1024, 384)
    c2, s2 = cb.unpack(p, 1024, 384)
    assert np.array_equal(c2, c) and np.array_equal(s2.view(np.uint16), sc.view(np.uint16))


def test_pack_closed_form_positions():
    M, K = 1024, 384
    NC = K // 128
    rng = np.random.default_rng(17)
    zero_c = np.zeros((M, K), dtype=np.uint8)
    zero_s = np.zeros((M // 32, K), dtype=np.float16)
    base = cb.pack(zero_c, zero_s)
    assert np.all(base == 0)
    for _ in range(40):
        m, k = int(rng.integers(0, M)), int(rng.integers(0, K))
        code = int(rng.integers(1, 4))
        c = zero_c.copy()
        c[m, k] = code
        p = cb.pack(c, zero_s)
        at = ((m // 512) * NC + k // 128) * 20480 + 4096 + (k % 128) * 128 + (m % 512) // 4
        assert np.flatnonzero(p != base).tolist() == [at] and int(p[at]) == code << (2 * (m % 4))
        mb = int(rng.integers(0, M // 32))
        s = zero_s.copy()
        s.view(np.uint16)[mb, k] = 0xBEEF
        p = cb.pack(zero_c, s)
        at = ((mb // 16) * NC + k // 128) * 20480 + 32 * (k % 128) + 2 * (mb % 16)
        assert np.flatnonzero(p != base).tolist() == [at, at + 1]
        assert p[at] == 0xEF and p[at + 1] == 0xBE


@pytest.mark.parametrize("M,K", [(511, 128), (512, 100), (0, 128), (256, 128)])
def test_bad_shapes(M, K):
    with pytest.raises(ValueError):
        cb.packed_bytes(M, K)


def test_pad_rows():
    W = make_fp_weights(1024, 128, 18)[:530]
    P = cb.pad_rows(W)
    assert P.shape == (1024, 128) and np.array_equal(P[:530], W) and np.all(P[530:] == 0)
    assert cb.pad_rows(P) is P
