"""Pins for the CPU oracle: every check here compares oracle/ with something that is not
the oracle's own formula - a NumPy library routine, a closed form, brute force in pure
Python, an exact-arithmetic case, an invariant of the method, or the paper's worked
example.  CPU only."""
import itertools
import os

import numpy as np
import pytest

import oracle
from workloads import make_weights, make_x, quantile_threshold, seed_for

G = 128
R = 256
CH = 2 * R + G * R // 2   # 16896 bytes per (block-row, group) chunk


def small(M=512, K=1024, seed=1, dist="normal"):
    w = make_weights(M, K, seed)
    x = make_x(K, dist, seed + 50)
    return w, x


# ---------------------------------------------------------------- number formats / dequant

def test_half_to_double_all_bit_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)       # NumPy's own conversion
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_dequant_matches_independent_numpy_expression():
    w, _ = small()
    want = w["q"].astype(np.float64) * np.repeat(w["scales"].astype(np.float64), G, axis=1)
    got = oracle.dequant(w["q_rowmajor"], w["scales"])
    assert np.array_equal(got, want)


def test_dequant_sign_and_nibble_order_by_hand():
    # one row, K = 128: codes -8..7 repeated; byte b holds k=2b (low) and k=2b+1 (high)
    K = 128
    codes = np.array([(k % 16) - 8 for k in range(K)], dtype=np.int64)
    raw = np.zeros((256, K // 2), dtype=np.uint8)
    for k in range(K):
        nib = int(codes[k]) & 0xF
        raw[0, k // 2] |= nib << (4 * (k % 2))
    scales = np.full((256, 1), 0.5, dtype=np.float16)
    got = oracle.dequant(raw, scales)
    assert np.array_equal(got[0], 0.5 * codes)
    assert np.all(got[1:] == 0.0)


# ---------------------------------------------------------------- mask / gather

@pytest.mark.parametrize("sparsity", [0.0, 0.25, 0.5, 0.65, 0.9])
def test_gather_matches_flatnonzero(sparsity):
    x = make_x(4096, "laplace", 7)
    thr = quantile_threshold(x, sparsity)
    idx, n = oracle.gather(x, thr)
    want = np.flatnonzero(~(np.abs(x[0].astype(np.float32)) < np.float32(thr)))
    assert n == want.size
    assert np.array_equal(idx, want.astype(np.int32))
    assert np.all(np.diff(idx) > 0)
    assert np.array_equal(oracle.mask(x, thr), np.isin(np.arange(4096), want))


def test_gather_threshold_edge_cases():
    x = make_x(1024, "normal", 3)
    idx, n = oracle.gather(x, 0.0)
    assert n == 1024 and np.array_equal(idx, np.arange(1024))      # thr = 0 keeps all
    idx, n = oracle.gather(x, float("inf"))
    assert n == 0 and idx.size == 0                                # thr = inf keeps none
    # exact ties with the threshold are KEPT (sparse iff |x| < thr, strictly)
    xt = np.array([[0.5, -0.5, 0.25, 0.0, -0.0, 0.75, 0.4995]], dtype=np.float16)
    xt = np.ascontiguousarray(np.tile(xt, (1, 1)))
    idx, n = oracle.gather(xt, 0.5)
    assert list(idx) == [0, 1, 5]
    # exact zeros are kept at thr = 0
    idx, n = oracle.gather(xt, 0.0)
    assert n == xt.shape[1]
    # NaN is kept for every threshold, +-inf is kept even at thr = inf
    xn = np.array([[np.nan, 1.0, np.inf, -np.inf, 0.1]], dtype=np.float16)
    idx, n = oracle.gather(xn, float("inf"))
    assert list(idx) == [0, 2, 3]


def test_gather_count_is_monotone_in_threshold():
    x = make_x(4096, "laplace", 11)
    counts = [oracle.gather(x, t)[1] for t in np.linspace(0, 4, 33)]
    assert all(a >= b for a, b in zip(counts, counts[1:]))
    assert counts[0] == 4096


def test_gather_batch_union():
    x = make_x(2048, "laplace", 5, batch=4)
    thr = quantile_threshold(x, 0.5)
    idx, n = oracle.gather(x, thr)
    keep = np.zeros(2048, dtype=bool)
    for b in range(4):
        keep |= ~(np.abs(x[b].astype(np.float32)) < np.float32(thr))
    assert np.array_equal(idx, np.flatnonzero(keep).astype(np.int32))
    # four identical rows behave as batch 1
    x1 = x[:1]
    i1, n1 = oracle.gather(x1, thr)
    i4, n4 = oracle.gather(np.ascontiguousarray(np.repeat(x1, 4, axis=0)), thr)
    assert n1 == n4 and np.array_equal(i1, i4)


# ---------------------------------------------------------------- gemv values

def dense_numpy(w, x):
    Wd = w["q"].astype(np.float64) * np.repeat(w["scales"].astype(np.float64), G, axis=1)
    return Wd, Wd @ x.astype(np.float64).T        # [M, batch]


def test_gemv_threshold_zero_is_dense_quantized_gemv():
    w, x = small()
    _, want = dense_numpy(w, x)
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0)
    np.testing.assert_allclose(got[0], want[:, 0], rtol=1e-12, atol=1e-12)


def test_gemv_threshold_inf_is_zero_vector():
    w, x = small()
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, float("inf"))
    assert got.shape == (1, 512) and np.all(got == 0.0)


@pytest.mark.parametrize("sparsity", [0.25, 0.5, 0.65])
def test_gemv_equals_dense_on_zeroed_x(sparsity):
    """The definition itself: sparse result == dense GEMV fed x with dropped entries zeroed."""
    w, x = small(dist="laplace")
    thr = quantile_threshold(x, sparsity)
    Wd, _ = dense_numpy(w, x)
    xz = x[0].astype(np.float64).copy()
    xz[np.abs(x[0].astype(np.float32)) < np.float32(thr)] = 0.0
    want = Wd @ xz
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)[0]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_gemv_brute_force_tiny_pure_python():
    M, K = 256, 256
    w = make_weights(M, K, 21)
    x = make_x(K, "normal", 22)
    thr = quantile_threshold(x, 0.5)
    q, s = w["q"], w["scales"]
    xs = [float(v) for v in x[0]]
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)[0]
    for m in range(0, M, 17):
        acc = 0.0
        for k in range(K):
            if abs(xs[k]) < thr:
                continue
            acc += float(s[m, k // G]) * int(q[m, k]) * xs[k]
        assert abs(got[m] - acc) <= 1e-12 * max(1.0, abs(acc))


def test_gemv_exact_arithmetic_case_is_bit_exact():
    """Integer x and power-of-two scales: every product and partial sum is an exactly
    representable number, so any correct implementation gives exactly this."""
    M, K = 256, 512
    rng = np.random.default_rng(5)
    w = make_weights(M, K, 31)
    scales = (2.0 ** rng.integers(-6, -2, size=(M, K // G))).astype(np.float16)
    x = rng.integers(-4, 5, size=(1, K)).astype(np.float16)
    thr = 2.0
    keep = np.abs(x[0].astype(np.float64)) >= 2.0
    want = ((w["q"].astype(np.int64) * keep[None, :] * x[0].astype(np.int64)[None, :])
            .reshape(M, K // G, G).sum(axis=2) * scales.astype(np.float64)).sum(axis=1)
    got = oracle.gemv(w["q_rowmajor"], scales, x, thr)[0]
    assert np.array_equal(got, want)


def test_gemv_column_probe_every_column():
    """x = c * e_k  =>  y = c * Wd[:, k] exactly (catches any index / transpose mistake)."""
    M, K = 256, 256
    w = make_weights(M, K, 41)
    Wd = w["q"].astype(np.float64) * np.repeat(w["scales"].astype(np.float64), G, axis=1)
    for k in range(K):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, k] = -1.5
        got = oracle.gemv(w["q_rowmajor"], w["scales"], x, 1.0)[0]
        assert np.array_equal(got, -1.5 * Wd[:, k]), k


def test_gemv_additive_over_disjoint_kept_sets():
    w, x = small(dist="laplace")
    thr = quantile_threshold(x, 0.4)
    xa, xb = x.copy(), x.copy()
    xa[0, 0::2] = 0          # zeroed entries fall under the threshold -> dropped
    xb[0, 1::2] = 0
    ya = oracle.gemv(w["q_rowmajor"], w["scales"], xa, thr)[0]
    yb = oracle.gemv(w["q_rowmajor"], w["scales"], xb, thr)[0]
    y = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)[0]
    np.testing.assert_allclose(ya + yb, y, rtol=1e-12, atol=1e-12)


def test_gemv_error_to_dense_is_bounded_by_threshold():
    w, x = small(dist="laplace")
    thr = quantile_threshold(x, 0.5)
    Wd, dense = dense_numpy(w, x)
    dropped = np.abs(x[0].astype(np.float32)) < np.float32(thr)
    bound = thr * np.abs(Wd[:, dropped]).sum(axis=1)
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)[0]
    assert np.all(np.abs(got - dense[:, 0]) <= bound + 1e-9)


def test_gemv_batch_rows_use_own_values_on_union_set():
    M, K = 256, 512
    w = make_weights(M, K, 51)
    x = make_x(K, "laplace", 52, batch=4)
    thr = quantile_threshold(x, 0.5)
    keep = np.zeros(K, dtype=bool)
    for b in range(4):
        keep |= ~(np.abs(x[b].astype(np.float32)) < np.float32(thr))
    Wd = w["q"].astype(np.float64) * np.repeat(w["scales"].astype(np.float64), G, axis=1)
    want = (Wd[:, keep] @ x.astype(np.float64)[:, keep].T).T
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    # identical rows == batch 1; thr = 0 == four dense GEMVs
    x4 = np.ascontiguousarray(np.repeat(x[:1], 4, axis=0))
    y1 = oracle.gemv(w["q_rowmajor"], w["scales"], x[:1], thr)
    y4 = oracle.gemv(w["q_rowmajor"], w["scales"], x4, thr)
    assert all(np.array_equal(y4[b], y1[0]) for b in range(4))
    y0 = oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0)
    np.testing.assert_allclose(y0, (Wd @ x.astype(np.float64).T).T, rtol=1e-12, atol=1e-12)


def test_gemv_rows_agrees_with_full_gemv():
    w, x = small(dist="laplace")
    thr = quantile_threshold(x, 0.5)
    rows = [0, 1, 255, 256, 300, 511]
    full = oracle.gemv(w["q_rowmajor"], w["scales"], x, thr)
    part = oracle.gemv_rows(w["q_rowmajor"], w["scales"], x, thr, rows)
    assert np.array_equal(part[0], full[0, rows])


# ---------------------------------------------------------------- partition (Figure 6)

def test_partition_paper_worked_example(golden_dir):
    with open(os.path.join(golden_dir, "partition_fig6.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    for row in rows:
        n_ns, parts, sizes = int(row[0]), int(row[1]), [int(v) for v in row[2:]]
        got = oracle.partition(n_ns, parts)
        assert [e - b for b, e in got] == sizes


@pytest.mark.parametrize("n_ns,parts", [(0, 4), (1, 4), (9, 3), (10, 3), (2048, 32), (2047, 64),
                                        (5, 64), (28672, 112)])
def test_partition_is_disjoint_covering_and_even(n_ns, parts):
    sl = oracle.partition(n_ns, parts)
    assert sl[0][0] == 0 and sl[-1][1] == n_ns
    assert all(a[1] == b[0] for a, b in zip(sl, sl[1:]))
    sizes = [e - b for b, e in sl]
    assert min(sizes) >= 0 and max(sizes) - min(sizes) <= 1


# ---------------------------------------------------------------- reference packer

def closed_form_code_pos(m, k, NG):
    """(byte offset, high-nibble flag) of code (m, k) in the packed buffer."""
    return ((m // R) * NG + k // G) * CH + 512 + (k % G) * 128 + (m % R) // 2, m % 2


def closed_form_scale_pos(m, g, NG):
    return ((m // R) * NG + g) * CH + 2 * (m % R)


def test_pack_size_formula():
    for M, K in [(256, 128), (512, 1024), (4096, 4096), (11008, 4096), (28672, 8192)]:
        assert oracle.packed_bytes(M, K) == M * K // 2 + M * (K // G) * 2
        assert oracle.packed_bytes(M, K) % 128 == 0


def test_pack_roundtrip_bit_exact():
    w = make_weights(768, 640, 61)
    p = oracle.pack(w["q_rowmajor"], w["scales"])
    q2, s2 = oracle.unpack(p, 768, 640)
    assert np.array_equal(q2, w["q_rowmajor"])
    assert np.array_equal(s2.view(np.uint16), w["scales"].view(np.uint16))


def test_pack_one_hot_codes_land_at_closed_form_position():
    M, K = 512, 384
    NG = K // G
    scales = np.zeros((M, NG), dtype=np.float16)        # bits 0 -> scale bytes all zero
    for m, k in [(0, 0), (1, 0), (0, 1), (255, 127), (256, 128), (257, 129), (511, 383), (300, 200),
                 (13, 250)]:
        raw = np.zeros((M, K // 2), dtype=np.uint8)
        raw[m, k // 2] = (0x5 << (4 * (k % 2)))         # code +5 -> stored 13
        p = oracle.pack(raw, scales)
        off, high = closed_form_code_pos(m, k, NG)
        # every other code is 0 -> stored nibble 8 -> byte 0x88 in the code area
        expect_byte = (13 << 4 | 0x8) if high else (0x8 << 4 | 13)
        assert p[off] == expect_byte, (m, k)
        code_area = np.ones(p.size, dtype=bool)
        for t in range(M // R):
            for g in range(NG):
                base = (t * NG + g) * CH
                code_area[base:base + 512] = False
        others = code_area.copy()
        others[off] = False
        assert np.all(p[others] == 0x88)
        assert np.all(p[~code_area] == 0)


def test_pack_position_encoding_matrix():
    """Each code encodes its own coordinates; decode every packed nibble by the closed form."""
    M, K = 512, 256
    NG = K // G
    mm, kk = np.meshgrid(np.arange(M), np.arange(K), indexing="ij")
    code = ((3 * mm + 5 * kk + (mm // 7)) % 16) - 8
    lo = (code[:, 0::2] & 0xF).astype(np.uint8)
    hi = (code[:, 1::2] & 0xF).astype(np.uint8)
    raw = np.ascontiguousarray(lo | (hi << 4))
    sc = (np.arange(M * NG).reshape(M, NG) % 2048).astype(np.uint16)   # distinct bit patterns
    p = oracle.pack(raw, sc.view(np.float16))
    for m, k in itertools.product(range(0, M, 37), range(0, K, 11)):
        off, high = closed_form_code_pos(m, k, NG)
        nib = (p[off] >> 4) if high else (p[off] & 0xF)
        assert nib == (code[m, k] + 8), (m, k)
    for m, g in itertools.product(range(0, M, 29), range(NG)):
        off = closed_form_scale_pos(m, g, NG)
        assert int(p[off]) | (int(p[off + 1]) << 8) == int(sc[m, g])


def test_gemv_group_64_against_independent_expression():
    """Groups of 64 columns in the oracle's GEMV: threshold 0 equals (q * S repeated 64 times) @ x, and a
    threshold drops exactly the columns np.flatnonzero would."""
    w = make_weights(256, 512, 6464, group=64)
    x = make_x(512, "laplace", 6465)
    Wd = w["q"].astype(np.float64) * np.repeat(w["scales"].astype(np.float64), 64, axis=1)
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.0, group=64)[0]
    assert np.allclose(got, Wd @ x[0].astype(np.float64), rtol=1e-12, atol=1e-12)
    keep = ~(np.abs(x[0].astype(np.float32)) < np.float32(0.7))
    got = oracle.gemv(w["q_rowmajor"], w["scales"], x, 0.7, group=64)[0]
    assert np.allclose(got, Wd[:, keep] @ x[0, keep].astype(np.float64), rtol=1e-12, atol=1e-12)


def test_pack_group_64_closed_form_positions():
    """Groups of 64 columns: chunk (t, g) is 512 + 64 * 128 = 8704 bytes and holds columns 64 g .. 64 g + 63;
    every code and scale sits at its closed-form place, and the oracle's own dequantizer with group = 64
    reads the same source the packer was given."""
    M, K, Gq = 512, 384, 64
    NGq, CHq = K // Gq, 512 + Gq * 128
    rng = np.random.default_rng(64)
    code = rng.integers(-8, 8, size=(M, K))
    raw = ((code[:, 0::2] & 0xF) | ((code[:, 1::2] & 0xF) << 4)).astype(np.uint8)
    sc = rng.integers(1, 65536, size=(M, NGq), dtype=np.uint16)
    p = oracle.pack(raw, sc, group=Gq)
    assert p.size == (M // 256) * NGq * CHq == oracle.packed_bytes(M, K, Gq)
    for m, k in itertools.product(range(0, M, 13), range(0, K, 5)):
        off = ((m // 256) * NGq + k // Gq) * CHq + 512 + (k % Gq) * 128 + (m % 256) // 2
        nib = (p[off] >> 4) if m % 2 else (p[off] & 0xF)
        assert nib == code[m, k] + 8, (m, k)
    for m, g in itertools.product(range(0, M, 29), range(NGq)):
        off = ((m // 256) * NGq + g) * CHq + 2 * (m % 256)
        assert int(p[off]) | (int(p[off + 1]) << 8) == int(sc[m, g])
    q2, s2 = oracle.unpack(p, M, K, group=Gq)
    assert np.array_equal(q2, raw) and np.array_equal(s2.view(np.uint16), sc)
    with pytest.raises(ValueError):
        oracle.pack(raw, sc, group=32)


def test_pack_rejects_bad_shapes():
    raw = np.zeros((256, 50), dtype=np.uint8)          # K = 100 is not a multiple of the group
    with pytest.raises(ValueError):
        oracle.pack(raw, np.zeros((256, 1), dtype=np.float16))


@pytest.mark.parametrize("M", [1, 100, 257, 300])
def test_pack_ragged_rows_closed_form_and_padding(M):
    """A ragged M keeps the closed-form place of every real code and scale; every nibble of a
    missing row holds code 8 (weight 0) and every missing scale is 0 bits; size = ceil(M/256) tiles."""
    K, NG = 256, 2
    rng = np.random.default_rng(900 + M)
    code = rng.integers(-8, 8, size=(M, K))
    raw = ((code[:, 0::2] & 0xF) | ((code[:, 1::2] & 0xF) << 4)).astype(np.uint8)
    sc = rng.integers(1, 65536, size=(M, NG), dtype=np.uint16)
    p = oracle.pack(raw, sc)
    T = (M + 255) // 256
    assert p.size == T * NG * 16896 == oracle.packed_bytes(M, K)
    for m, k in itertools.product(range(256 * T), range(0, K, 7)):
        off, high = closed_form_code_pos(m, k, NG)
        nib = (p[off] >> 4) if high else (p[off] & 0xF)
        assert nib == (code[m, k] + 8 if m < M else 8), (m, k)
    for m, g in itertools.product(range(256 * T), range(NG)):
        off = closed_form_scale_pos(m, g, NG)
        assert int(p[off]) | (int(p[off + 1]) << 8) == (int(sc[m, g]) if m < M else 0)
    q2, s2 = oracle.unpack(p, M, K)
    assert np.array_equal(q2, raw) and np.array_equal(s2.view(np.uint16), sc)
