"""CPU-only checks of the library's host side: it loads, exports every symbol the header
declares, its packer matches the oracle's reference packer byte for byte, and argument
errors come back as status codes.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2511_04477_amd as spqt
from workloads import make_weights

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions(header="spqt.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spqt_[a-z_0-9]+)\s*\(", text)))


def test_calibration_library_exports_every_declared_symbol():
    L = ctypes.CDLL(os.path.join(ROOT, "paper_2511_04477_amd", "libspqt_calib.so"))
    names = declared_functions("spqt_calib.h")
    assert names == ["spqt_calib_copy", "spqt_calib_empty", "spqt_calib_read", "spqt_calib_read_blocked",
                     "spqt_calib_read_lines", "spqt_calib_rowmajor_gemv"]
    for n in names:
        assert getattr(L, n) is not None
    # argument checks happen before any launch
    L.spqt_calib_read.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    assert L.spqt_calib_read(None, 16, None, 0, 4, None) == -1
    L.spqt_calib_rowmajor_gemv.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_void_p, ctypes.c_float, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
    assert L.spqt_calib_rowmajor_gemv(None, 16, 256, 128, 16, 0.0, 0, 16, None) == -1
    assert L.spqt_calib_rowmajor_gemv(16, 16, 256, 100, 16, 0.0, 0, 16, None) == -1
    assert L.spqt_calib_rowmajor_gemv(16, 16, 256, 65536, 16, 0.0, 0, 16, None) == -1     # x would not fit LDS
    assert L.spqt_calib_rowmajor_gemv(8, 16, 256, 128, 16, 0.0, 0, 16, None) == -1        # misaligned codes
    assert L.spqt_calib_read(16, 24, 16, 0, 4, None) == -1


def test_library_exports_every_declared_symbol():
    L = spqt.lib()
    names = declared_functions()
    assert set(names) == set(spqt.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_colblock_header_symbols_are_exported():
    L = spqt.lib()
    names = [n for n in declared_functions("spqt_colblock.h") if n.startswith("spqt_cb")]
    assert set(names) == set(spqt.CB_EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


@pytest.mark.parametrize("M,K", [(256, 128), (512, 384), (1024, 1024)])
def test_colblock_quantizer_matches_oracle_bit_exact(M, K):
    """The library's offline quantizer and the oracle's (independent NumPy code, same fp32 rule)
    must agree on every scale bit and every code, and on the packed bytes."""
    from oracle import colblock as cb
    from workloads import make_fp_weights
    W = make_fp_weights(M, K, 500 + M + K)
    W[0:32, 3] = 0.0                      # an all-zero block
    W[32:64, 7] = np.float32(1e-9)        # a block whose scale underflows to zero
    W[64:96, 11] = [(-1) ** r * 0.5 * (r % 15) for r in range(32)]   # exact ties: amax = 7, scale = 1
    got = spqt.spqt_cb_quantize(W)
    q, s = cb.quantize(W)
    want = cb.pack(q, s)
    assert got.nbytes == want.nbytes == spqt.spqt_cb_packed_bytes(M, K) == cb.packed_bytes(M, K)
    assert np.array_equal(got, want)
    back = spqt.spqt_cb_dequantize(got, M, K)
    assert np.array_equal(back.astype(np.float64), cb.dequant(q, s))


@pytest.mark.parametrize("M,K", [(256, 128), (512, 384), (1024, 512)])
def test_kquant_quantizer_matches_oracle_bit_exact(M, K):
    """K-quant flavour: every header bit and every code of the library's quantizer equals the
    oracle's (independent NumPy code, same fp32 rule); the library's dequantizer gives the
    oracle's values rounded to fp32."""
    from oracle import colblock_k as ck
    from workloads import make_fp_weights
    W = make_fp_weights(M, K, 600 + M + K)
    W[:, 3] = 0.0                                          # a zero superblock
    W[0:32, 7] = np.abs(W[0:32, 7]) + 0.01                 # all-positive block
    W[32:64, 7] = -np.abs(W[32:64, 7]) - 0.01              # all-negative block
    W[64:96, 11] = np.float32(1e-9)                        # scale underflows to zero
    got = spqt.spqt_cbk_quantize(W)
    p = ck.quantize(W)
    want = ck.pack(p)
    assert got.nbytes == want.nbytes == spqt.spqt_cb_packed_bytes(M, K)
    assert np.array_equal(got, want)
    back = spqt.spqt_cbk_dequantize(got, M, K)
    assert np.array_equal(back, ck.dequant(p).astype(np.float32))


@pytest.mark.parametrize("M,K", [(128, 128), (384, 384), (1024, 512), (1, 128), (130, 256), (255, 128)])
def test_eight_bit_quantizer_matches_oracle_bit_exact(M, K):
    """8-bit flavour: every scale bit and every code of the library's quantizer equals the oracle's
    (independent NumPy code, same fp32 rule), also on a ragged M (missing rows count as zero weights);
    the library's dequantizer gives the oracle's values."""
    from oracle import colblock_w8 as c8
    from workloads import make_fp_weights
    W = make_fp_weights(128 * ((M + 127) // 128), K, 700 + M + K)[:M].copy()
    if M >= 96:
        W[0:32, 3] = 0.0                      # an all-zero block
        W[32:64, 7] = np.float32(1e-9)        # a block whose scale underflows to zero
        W[64:96, 11] = [(-1) ** r * 0.5 * (r % 255) for r in range(32)]   # exact ties under scale 2^-k
    got = spqt.spqt_cb8_quantize(W)
    q, s = c8.quantize(c8.pad_rows(W))
    want = c8.pack(q, s)
    assert got.nbytes == want.nbytes == spqt.spqt_cb8_packed_bytes(M, K) == ((M + 127) // 128) * (K // 128) * spqt.CB8_CHUNK_BYTES
    assert np.array_equal(got, want)
    back = spqt.spqt_cb8_dequantize(got, M, K)
    assert back.shape == (M, K) and np.array_equal(back.astype(np.float64), c8.dequant(q, s)[:M])


@pytest.mark.parametrize("M,K", [(512, 128), (1024, 384), (700, 256), (1, 128), (33, 128)])
def test_two_bit_quantizer_matches_oracle_bit_exact(M, K):
    """2-bit flavour: every scale bit and every code of the library's quantizer equals the oracle's
    (independent NumPy code, same fp32 rule), also on a ragged M (missing rows count as zero weights);
    the library's dequantizer gives the oracle's values."""
    from oracle import colblock_w2 as c2
    from workloads import make_fp_weights
    W = make_fp_weights(512 * ((M + 511) // 512), K, 720 + M + K)[:M].copy()
    if M >= 128:
        W[0:32, 3] = 0.0                      # an all-zero block
        W[32:64, 7] = np.float32(1e-9)        # a block whose scale underflows to zero
        W[64:96, 11] = [(-1) ** r * 0.25 * (r % 7) for r in range(32)]    # max 1.5 -> scale 1: exact ties at 0, +-1
        W[96:128, 13] = [1.5, -1.5] + [0.0, 1.0, -1.0, 0.5, -0.5] * 6     # every decision boundary of the four levels
    got = spqt.spqt_cb2_quantize(W)
    c, s = c2.quantize(c2.pad_rows(W))
    want = c2.pack(c, s)
    assert got.nbytes == want.nbytes == spqt.spqt_cb2_packed_bytes(M, K) == ((M + 511) // 512) * (K // 128) * spqt.CB2_CHUNK_BYTES
    assert np.array_equal(got, want)
    back = spqt.spqt_cb2_dequantize(got, M, K)
    assert back.shape == (M, K) and np.array_equal(back.astype(np.float64), c2.dequant(c, s)[:M])


def test_colblock_bad_arguments():
    L = spqt.lib()
    out = ctypes.c_size_t()
    assert L.spqt_cb_packed_bytes(256, 100, ctypes.byref(out)) == -2
    assert L.spqt_cb_packed_bytes(256, 128, None) == -1
    w = np.zeros((256, 128), dtype=np.float32)
    small = np.zeros(16, dtype=np.uint8)
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert L.spqt_cb_quantize(vp(w), 256, 128, vp(small), small.nbytes) == -4
    assert L.spqt_cb_quantize(None, 256, 128, vp(small), small.nbytes) == -1
    assert L.spqt_cb_gemv(None, 256, 128, 16, 1, None, None, 16, None, 0, None, None) == -1
    assert L.spqt_cb_gemv(128, 256, 100, 16, 1, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cb_gemv(64, 256, 128, 16, 1, None, None, 16, None, 0, None, None) == -3
    assert L.spqt_cb_gemv(128, 256, 128, 16, 1, 16, None, 16, None, 0, None, None) == -1
    assert L.spqt_cb_gemv(128, 256, 128, 16, 5, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cbk_quantize(None, 256, 128, vp(small), small.nbytes) == -1
    assert L.spqt_cbk_quantize(vp(w), 256, 128, vp(small), small.nbytes) == -4
    assert L.spqt_cbk_gemv(None, 256, 128, 16, 1, None, None, 16, None, 0, None, None) == -1
    assert L.spqt_cbk_gemv(128, 256, 100, 16, 1, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cbk_gemv(128, 256, 128, 16, 5, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cbk_gemv_fused(128, 256, 128, 16, ctypes.c_float(float("nan")), 16, None, 0, None, None) == -1
    assert L.spqt_cbk_gemv_fused(None, 256, 128, 16, ctypes.c_float(0.5), 16, None, 0, None, None) == -1
    assert L.spqt_cb8_packed_bytes(128, 100, ctypes.byref(out)) == -2
    assert L.spqt_cb8_quantize(vp(w), 256, 128, vp(small), small.nbytes) == -4
    assert L.spqt_cb8_quantize(None, 256, 128, vp(small), small.nbytes) == -1
    assert L.spqt_cb8_gemv(None, 256, 128, 16, None, None, 16, None, 0, None, None) == -1
    assert L.spqt_cb8_gemv(128, 256, 100, 16, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cb8_gemv(64, 256, 128, 16, None, None, 16, None, 0, None, None) == -3
    assert L.spqt_cb8_gemv(128, 256, 128, 16, 16, None, 16, None, 0, None, None) == -1   # idx without count
    assert L.spqt_cb2_packed_bytes(512, 100, ctypes.byref(out)) == -2
    assert L.spqt_cb2_packed_bytes(512, 128, None) == -1
    assert L.spqt_cb2_quantize(vp(w), 256, 128, vp(small), small.nbytes) == -4
    assert L.spqt_cb2_quantize(None, 256, 128, vp(small), small.nbytes) == -1
    assert L.spqt_cb2_dequantize(None, 256, 128, vp(w)) == -1
    assert L.spqt_cb2_gemv(None, 256, 128, 16, None, None, 16, None, 0, None, None) == -1
    assert L.spqt_cb2_gemv(128, 256, 100, 16, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cb2_gemv(64, 256, 128, 16, None, None, 16, None, 0, None, None) == -3
    assert L.spqt_cb2_gemv(128, 256, 128, 16, 16, None, 16, None, 0, None, None) == -1   # idx without count
    assert L.spqt_cb2_gemv_fused(128, 256, 128, 16, ctypes.c_float(float("nan")), 16, None, 0, None, None) == -1
    assert L.spqt_cb2_gemv_fused(None, 256, 128, 16, ctypes.c_float(0.5), 16, None, 0, None, None) == -1
    assert L.spqt_cb8_gemv_fused(128, 256, 128, 16, ctypes.c_float(float("nan")), 16, None, 0, None, None) == -1
    assert L.spqt_cb8_gemv_fused(128, 256, 100, 16, ctypes.c_float(0.5), 16, None, 0, None, None) == -2
    assert L.spqt_cb2_gemv_rows(128, 512, 128, 16, 4, None, None, 16, None, 0, None, None) == -2   # at most 3 rows at 2 bits
    assert L.spqt_cb2_gemv_rows(128, 512, 128, 16, 0, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cb8_gemv_rows(128, 512, 128, 16, 5, None, None, 16, None, 0, None, None) == -2
    assert L.spqt_cb8_gemv_rows(128, 512, 128, 16, 2, 16, None, 16, None, 0, None, None) == -1     # idx without count
    cfg = spqt.LaunchCfg(17, 4, 0)
    assert L.spqt_cb2_gemv(128, 256, 128, 16, None, None, 16, None, 0, None, ctypes.byref(cfg)) == -1   # more than 16 splits


def test_status_strings():
    assert spqt.spqt_status_str(0) == "SPQT_OK"
    for code in (-1, -2, -3, -4, -5):
        assert spqt.spqt_status_str(code).startswith("SPQT_E")


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (768, 640), (1024, 4096)])
def test_pack_matches_oracle_packer_bit_exact(M, K):
    w = make_weights(M, K, 1000 + M + K)
    got = spqt.spqt_pack(w["q_rowmajor"], w["scales"])
    want = oracle.pack(w["q_rowmajor"], w["scales"])
    assert got.nbytes == want.nbytes == spqt.spqt_packed_bytes(M, K)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("M,K", [(256, 128), (512, 1024), (300, 640)])
def test_pack_group_64_matches_oracle_and_round_trips(M, K):
    """Quantization groups of 64 columns: same layout with 64-column chunks."""
    w = make_weights(M, K, 1100 + M + K, group=64)
    got = spqt.spqt_pack(w["q_rowmajor"], w["scales"], group=64)
    assert got.nbytes == spqt.spqt_packed_bytes(M, K, 64) == ((M + 255) // 256) * (K // 64) * (512 + 64 * 128)
    assert np.array_equal(got, oracle.pack(w["q_rowmajor"], w["scales"], group=64))
    q2, s2 = spqt.spqt_unpack(got, M, K, group=64)
    assert np.array_equal(q2, w["q_rowmajor"]) and np.array_equal(s2.view(np.uint16), w["scales"].view(np.uint16))


def test_pack_extreme_codes_and_scale_bits():
    M, K = 256, 256
    raw = np.zeros((M, K // 2), dtype=np.uint8)
    raw[0::2] = 0x87      # codes +7 (low) and -8 (high)
    raw[1::2] = 0x78
    sc = np.arange(M * 2, dtype=np.uint16).reshape(M, 2) * 31 + 7   # arbitrary bit patterns
    got = spqt.spqt_pack(raw, sc)
    assert np.array_equal(got, oracle.pack(raw, sc))


def test_unpack_is_exact_inverse():
    w = make_weights(512, 384, 77)
    p = spqt.spqt_pack(w["q_rowmajor"], w["scales"])
    q2, s2 = spqt.spqt_unpack(p, 512, 384)
    assert np.array_equal(q2, w["q_rowmajor"])
    assert np.array_equal(s2.view(np.uint16), w["scales"].view(np.uint16))
    # and the library's unpack inverts the ORACLE's packer too
    q3, s3 = spqt.spqt_unpack(oracle.pack(w["q_rowmajor"], w["scales"]), 512, 384)
    assert np.array_equal(q3, w["q_rowmajor"]) and np.array_equal(s3.view(np.uint16), s2.view(np.uint16))


@pytest.mark.parametrize("M", [1, 2, 255, 257, 300, 701])
def test_ragged_row_count_is_zero_padded(M):
    """M need not be a multiple of the block height: the last block-row is stored with weight 0
    (code 8) and scale bits 0 in the missing rows.  Pinned three ways: library == oracle packer;
    both == the ordinary path fed the explicitly zero-padded matrix; unpack gives the M rows back."""
    K = 256
    w = make_weights(256 * ((M + 255) // 256), K, 4000 + M)
    q, sc = w["q_rowmajor"][:M].copy(), w["scales"][:M].copy()
    got = spqt.spqt_pack(q, sc)
    assert got.nbytes == spqt.spqt_packed_bytes(M, K) == ((M + 255) // 256) * 2 * spqt.CHUNK_BYTES
    assert np.array_equal(got, oracle.pack(q, sc))
    Mp = 256 * ((M + 255) // 256)
    qp = np.zeros((Mp, K // 2), dtype=np.uint8)
    sp = np.zeros((Mp, K // 128), dtype=np.float16)
    qp[:M], sp[:M] = q, sc
    assert np.array_equal(got, spqt.spqt_pack(qp, sp))
    q2, s2 = spqt.spqt_unpack(got, M, K)
    assert np.array_equal(q2, q) and np.array_equal(s2.view(np.uint16), sc.view(np.uint16))
    q3, s3 = oracle.unpack(got, M, K)
    assert np.array_equal(q3, q) and np.array_equal(s3.view(np.uint16), sc.view(np.uint16))


@pytest.mark.parametrize("M", [1, 31, 33, 255, 300, 513])
def test_ragged_row_count_column_block_quantizers(M):
    """Column-block quantizers on a ragged M: the missing rows of the last superblock-row count as
    zero weights (they cannot change a block's max |w|, nor a min/max that already includes 0), so the
    real rows' values equal those of quantizing the padded matrix, and library == oracle bytes."""
    from oracle import colblock as cb, colblock_k as ck
    from workloads import make_fp_weights
    K = 256
    W = make_fp_weights(256 * ((M + 255) // 256), K, 4100 + M)[:M].copy()
    got = spqt.spqt_cb_quantize(W)
    q, s = cb.quantize(cb.pad_rows(W))
    assert np.array_equal(got, cb.pack(q, s))
    back = spqt.spqt_cb_dequantize(got, M, K)
    assert back.shape == (M, K) and np.array_equal(back.astype(np.float64), cb.dequant(q, s)[:M])
    assert np.all(q[M:] == 0)
    gotk = spqt.spqt_cbk_quantize(W)
    p = ck.quantize(ck.pad_rows(W))
    assert np.array_equal(gotk, ck.pack(p))
    backk = spqt.spqt_cbk_dequantize(gotk, M, K)
    assert np.array_equal(backk, ck.dequant(p).astype(np.float32)[:M])


def test_sizes():
    assert spqt.spqt_packed_bytes(4096, 4096) == 4096 * 4096 // 2 + 4096 * 32 * 2
    assert spqt.spqt_packed_bytes(256, 128) == spqt.CHUNK_BYTES
    assert spqt.spqt_workspace_bytes(4096, 4096) >= 4096 * 4 * spqt.MAX_SPLITS


@pytest.mark.parametrize("M,K,group", [(256, 127, 128), (256, 128, 32), (256, 128, 256), (0, 128, 128), ((1 << 24) + 1, 128, 128),
                                       (256, 0, 128), (-256, 128, 128)])
def test_bad_shapes_are_rejected(M, K, group):
    out = ctypes.c_size_t()
    assert spqt.lib().spqt_packed_bytes(M, K, group, ctypes.byref(out)) == -2   # SPQT_ESHAPE


def test_null_and_small_buffers_are_rejected_on_the_host():
    L = spqt.lib()
    out = ctypes.c_size_t()
    assert L.spqt_packed_bytes(256, 128, 128, None) == -1
    raw = np.zeros((256, 64), dtype=np.uint8)
    sc = np.zeros((256, 1), dtype=np.uint16)
    small = np.zeros(100, dtype=np.uint8)
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert L.spqt_pack(vp(raw), vp(sc), 256, 128, 128, vp(small), small.nbytes) == -4
    assert L.spqt_pack(None, vp(sc), 256, 128, 128, vp(small), small.nbytes) == -1
    # device entry points validate before touching the GPU, so these run without one
    assert L.spqt_gather(None, 128, 1, ctypes.c_float(0.0), None, None, None) == -1
    assert L.spqt_gather(16, 100, 1, ctypes.c_float(0.0), 16, 16, None) == -2
    assert L.spqt_gather(16, 1 << 20, 1, ctypes.c_float(0.0), 16, 16, None) == -2
    assert L.spqt_gather(16, 128, 5, ctypes.c_float(0.0), 16, 16, None) == -2
    assert L.spqt_gather(16, 128, 1, ctypes.c_float(float("nan")), 16, 16, None) == -1
    assert L.spqt_gather(18, 128, 1, ctypes.c_float(0.0), 16, 16, None) == -3
    assert L.spqt_gather_rows(4096, 128, 2, ctypes.c_float(0.0), 16, 16, None, None) == -1     # no copy buffer
    assert L.spqt_gather_rows(4096, 128, 2, ctypes.c_float(0.0), 16, 16, 4096, None) == -1     # copy == x
    assert L.spqt_gather_rows(4096, 128, 2, ctypes.c_float(0.0), 16, 16, 4096 + 256, None) == -1  # overlaps row 1
    assert L.spqt_gather_rows(4096, 128, 2, ctypes.c_float(0.0), 16, 16, 8192 + 8, None) == -3  # misaligned copy
    assert L.spqt_gather_rows(4096, 100, 2, ctypes.c_float(0.0), 16, 16, 8192, None) == -2
    assert L.spqt_gemv(None, 256, 128, 128, 16, 1, None, None, 16, None, 0, None) == -1
    assert L.spqt_gemv(128, 256, 100, 128, 16, 1, None, None, 16, None, 0, None) == -2
    assert L.spqt_gemv(64, 256, 128, 128, 16, 1, None, None, 16, None, 0, None) == -3
    assert L.spqt_gemv(128, 256, 128, 128, 16, 1, 16, None, 16, None, 0, None) == -1  # idx without count
    assert L.spqt_gemv(128, 256, 128, 128, 16, 7, None, None, 16, None, 0, None) == -2
    # one launch for several rows: same checks, and 4 wavefronts per workgroup only
    fr = L.spqt_gemv_fused_rows
    assert fr(None, 256, 128, 128, 16, 2, ctypes.c_float(0.0), 0, 16, None, 0, None, None) == -1
    assert fr(128, 256, 100, 128, 16, 2, ctypes.c_float(0.0), 0, 16, None, 0, None, None) == -2
    assert fr(128, 256, 128, 128, 16, 5, ctypes.c_float(0.0), 0, 16, None, 0, None, None) == -2
    assert fr(128, 256, 128, 128, 16, 2, ctypes.c_float(float("nan")), 0, 16, None, 0, None, None) == -1
    assert fr(64, 256, 128, 128, 16, 2, ctypes.c_float(0.0), 0, 16, None, 0, None, None) == -3
    two_waves = spqt.binding.LaunchCfg(1, 2, 0)
    assert fr(128, 256, 128, 128, 16, 2, ctypes.c_float(0.0), 0, 16, None, 0, None, ctypes.byref(two_waves)) == -1
    no_ws = spqt.binding.LaunchCfg(4, 0, 0)
    assert fr(128, 1024, 1024, 128, 16, 2, ctypes.c_float(0.0), 0, 16, None, 0, None, ctypes.byref(no_ws)) == -1


@pytest.mark.parametrize("M,K", [(512, 1024), (4096, 4096), (1024, 4096), (11008, 4096), (4096, 11008),
                                 (14336, 4096), (4096, 14336), (28672, 8192), (8192, 28672)])
def test_default_launch_shape_is_valid(M, K):
    for sparse in (False, True):
        splits, waves = spqt.spqt_default_cfg(M, K, 1, sparse)
        assert 1 <= splits <= spqt.MAX_SPLITS and waves in (1, 2, 4)


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU measurement: --gpus N > 1 exits with a message before touching a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "one-GPU" in r.stderr


def test_product_package_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing under the product package may reference it."""
    pkg = os.path.join(ROOT, "paper_2511_04477_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f), encoding="utf-8", errors="ignore").read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)


def test_packers_agree_on_random_shapes_and_bytes():
    """Property check (hypothesis): for arbitrary code bytes and scale bit patterns the library's
    repacker equals the oracle's byte for byte and unpack inverts it; the column-block quantizer
    equals the oracle's on arbitrary finite weights with mixed magnitudes."""
    from hypothesis import given, settings, strategies as st
    from oracle import colblock as cb

    @settings(max_examples=25, deadline=None)
    @given(st.integers(1, 3), st.integers(1, 5), st.integers(0, 2 ** 32 - 1))
    def check(tm, kg, seed):
        M, K = 256 * tm, 128 * kg
        rng = np.random.default_rng(seed)
        raw = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
        sc = rng.integers(0, 65536, size=(M, K // 128), dtype=np.uint16)
        got = spqt.spqt_pack(raw, sc)
        assert np.array_equal(got, oracle.pack(raw, sc))
        q2, s2 = spqt.spqt_unpack(got, M, K)
        assert np.array_equal(q2, raw) and np.array_equal(s2.view(np.uint16), sc)
        W = (rng.standard_normal((M, K)) * 10.0 ** rng.integers(-6, 3, size=(1, K))).astype(np.float32)
        W[rng.random((M, K)) < 0.05] = 0.0
        q, s = cb.quantize(W)
        assert np.array_equal(spqt.spqt_cb_quantize(W), cb.pack(q, s))

    check()
