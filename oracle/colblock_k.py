"""CPU oracle for the K-quant flavour of the column-block zigzag layout.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this module;
the product package never does.  Plain NumPy, written from the paper and the format text below,
sharing nothing with the HIP path.

What the paper says of its format (Section 4.1.1): Q4_K - a superblock of 256 weights split into eight
blocks of 32, weights stored in 4 bits, "shared 6-bit block scales and a 16-bit superblock scale and min".
The paper gives no more than that.  THIS BUILD'S READING, taken from the public K-quant format and not
from the paper: besides its 6-bit scale every block also has a 6-bit MINIMUM; a superblock has one
16-bit scale d for the block scales and one, dmin, for the block minima; a weight is decoded as
(d * sc_b) * q - (dmin * m_b) with q in 0..15.  In the zigzag layout (Section 4.1.2) a
superblock is 256 consecutive rows of ONE column and superblocks are stored row-major by
superblock-row; the model is re-quantized offline into this form (Section 5).

The decode rule above is the format's; the quantizer below is this build's own (a plain min/max
rule, not llama.cpp's search), evaluated in fp32 exactly as written because its results decide
integers:

  block b of a superblock (rows 32b..32b+31 of the column):
      lo_b = min(min w, 0)     hi_b = max(max w, 0)
      scale_b = (hi_b - lo_b) / 15        min_b = 0 - lo_b                    (both >= 0; a zero minimum is +0)
  superblock:
      d    = fp16( max_b scale_b / 63 )   dmin = fp16( max_b min_b / 63 )     (round to nearest even)
      sc_b = d    > 0 ? clamp(rint(scale_b / float(d)),    0, 63) : 0
      m_b  = dmin > 0 ? clamp(rint(min_b   / float(dmin)), 0, 63) : 0
      se_b = float(d) * sc_b              me_b = float(dmin) * m_b
      q    = se_b > 0 ? clamp(rint((w + me_b) / se_b), 0, 15) : 0
  value = se_b * q - me_b

Packed form ("ZZ-CBK"): T = M/256 superblock-rows, NC = K/128 chunks of 128 columns; chunk (t, c)
at byte offset (t*NC + c) * 18432:
  bytes [16 j .. 16 j + 15], j = 0..127   the superblock header of column 128c + j:
        bytes 0-1 d (fp16, little endian), bytes 2-3 dmin (fp16), bytes 4-15 a 96-bit little-endian
        bit string: sc_0 .. sc_7 then m_0 .. m_7, 6 bits each, first value in the lowest bits
  bytes [2048 + 128 j + i], i = 0..127    codes of column 128c + j: low nibble = q of row 256t + 2i,
                                           high nibble = q of row 256t + 2i + 1 (plain 0..15)
"""
from __future__ import annotations

import numpy as np

TILE_ROWS = 256
BLOCK_ROWS = 32
CHUNK_COLS = 128
CHUNK_BYTES = CHUNK_COLS * 16 + CHUNK_COLS * 128   # 18432


def check_shape(M: int, K: int) -> None:
    if M <= 0 or K <= 0 or M % TILE_ROWS or K % CHUNK_COLS:
        raise ValueError("column-block layout needs M % 256 == 0 and K % 128 == 0")


def pad_rows(W: np.ndarray) -> np.ndarray:
    """A matrix whose M is not a multiple of 256 is handled as the same matrix with zero rows
    appended up to the next multiple (the paper states no rule for a ragged edge; this is the
    build's).  Everything below works on the padded matrix; outputs past row M are ignored."""
    W = np.asarray(W)
    extra = (-W.shape[0]) % TILE_ROWS
    if extra == 0:
        return W
    return np.concatenate([W, np.zeros((extra, W.shape[1]), dtype=W.dtype)], axis=0)


def packed_bytes(M: int, K: int) -> int:
    check_shape(M, K)
    return (M // TILE_ROWS) * (K // CHUNK_COLS) * CHUNK_BYTES


def quantize(W: np.ndarray):
    """fp32 [M, K] -> dict(q uint8 [M, K] in 0..15, sc uint8 [M/32, K], m uint8 [M/32, K],
    d fp16 [M/256, K], dmin fp16 [M/256, K]) by the rule in the header."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    M, K = W.shape
    check_shape(M, K)
    f32 = np.float32
    blocks = W.reshape(M // BLOCK_ROWS, BLOCK_ROWS, K)
    lo = np.minimum(blocks.min(axis=1), f32(0))
    hi = np.maximum(blocks.max(axis=1), f32(0))
    scale_b = ((hi - lo) / f32(15)).astype(np.float32)             # [M/32, K]
    min_b = (f32(0) - lo).astype(np.float32)
    sb = scale_b.reshape(M // TILE_ROWS, 8, K)
    mb = min_b.reshape(M // TILE_ROWS, 8, K)
    d = (sb.max(axis=1) / f32(63)).astype(np.float16)              # [M/256, K]
    dmin = (mb.max(axis=1) / f32(63)).astype(np.float16)
    df = d.astype(np.float32)[:, None, :]
    dmf = dmin.astype(np.float32)[:, None, :]
    with np.errstate(divide="ignore", invalid="ignore"):
        sc = np.where(df > 0, np.clip(np.rint(sb / df), 0, 63), 0).astype(np.uint8)
        m = np.where(dmf > 0, np.clip(np.rint(mb / dmf), 0, 63), 0).astype(np.uint8)
    se = (df * sc.astype(np.float32)).astype(np.float32).reshape(M // BLOCK_ROWS, 1, K)
    me = (dmf * m.astype(np.float32)).astype(np.float32).reshape(M // BLOCK_ROWS, 1, K)
    with np.errstate(divide="ignore", invalid="ignore"):
        r = np.clip(np.rint((blocks + me) / se), 0, 15)
    q = np.where(np.broadcast_to(se > 0, r.shape), r, 0).astype(np.uint8)
    return {"q": q.reshape(M, K), "sc": sc.reshape(M // BLOCK_ROWS, K), "m": m.reshape(M // BLOCK_ROWS, K),
            "d": d, "dmin": dmin}


def dequant(p: dict) -> np.ndarray:
    """fp64 [M, K]: (float(d) * sc) * q - float(dmin) * m."""
    q = p["q"]
    d = np.repeat(p["d"].astype(np.float64), 8, axis=0)            # per block
    dm = np.repeat(p["dmin"].astype(np.float64), 8, axis=0)
    se = np.repeat(d * p["sc"].astype(np.float64), BLOCK_ROWS, axis=0)
    me = np.repeat(dm * p["m"].astype(np.float64), BLOCK_ROWS, axis=0)
    return se * q.astype(np.float64) - me


def keep_mask(x: np.ndarray, threshold: float) -> np.ndarray:
    """Section 2: an entry is sparse iff |x| < threshold (compared in fp32)."""
    x = np.atleast_2d(x)
    a = np.abs(x.astype(np.float32))
    return np.any(~(a < np.float32(threshold)), axis=0)


def gemv(p: dict, x: np.ndarray, threshold: float) -> np.ndarray:
    """y[b, m] = sum over kept k of value[m, k] * x[b, k], in fp64."""
    x = np.atleast_2d(x)
    keep = keep_mask(x, threshold)
    Wd = dequant(p)
    out = np.empty((x.shape[0], Wd.shape[0]), dtype=np.float64)
    for b in range(x.shape[0]):
        out[b] = Wd[:, keep] @ x[b, keep].astype(np.float64)
    return out


def pack(p: dict) -> np.ndarray:
    """Quantized parts -> packed bytes, following the format text field by field."""
    q = p["q"]
    M, K = q.shape
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    out = np.zeros((T, NC, CHUNK_BYTES), dtype=np.uint8)
    d = np.ascontiguousarray(p["d"]).view(np.uint16).reshape(T, NC, CHUNK_COLS)
    dm = np.ascontiguousarray(p["dmin"]).view(np.uint16).reshape(T, NC, CHUNK_COLS)
    sc = p["sc"].reshape(T, 8, NC, CHUNK_COLS)
    m = p["m"].reshape(T, 8, NC, CHUNK_COLS)
    code = q.reshape(T, TILE_ROWS, NC, CHUNK_COLS)
    for j in range(CHUNK_COLS):
        out[:, :, 16 * j + 0] = (d[:, :, j] & 0xFF).astype(np.uint8)
        out[:, :, 16 * j + 1] = (d[:, :, j] >> 8).astype(np.uint8)
        out[:, :, 16 * j + 2] = (dm[:, :, j] & 0xFF).astype(np.uint8)
        out[:, :, 16 * j + 3] = (dm[:, :, j] >> 8).astype(np.uint8)
        bits = np.zeros((T, NC), dtype=object)
        for b in range(8):
            bits = bits + (sc[:, b, :, j].astype(object) << (6 * b))
            bits = bits + (m[:, b, :, j].astype(object) << (48 + 6 * b))
        for byte in range(12):
            out[:, :, 16 * j + 4 + byte] = ((bits >> (8 * byte)) & 0xFF).astype(np.uint8)
        for i in range(128):
            out[:, :, 2048 + 128 * j + i] = code[:, 2 * i, :, j] | (code[:, 2 * i + 1, :, j] << 4)
    return out.reshape(-1)


def unpack(packed: np.ndarray, M: int, K: int) -> dict:
    """Inverse of pack."""
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    pk = np.ascontiguousarray(packed, dtype=np.uint8).reshape(T, NC, CHUNK_BYTES)
    q = np.empty((T, TILE_ROWS, NC, CHUNK_COLS), dtype=np.uint8)
    sc = np.empty((T, 8, NC, CHUNK_COLS), dtype=np.uint8)
    m = np.empty((T, 8, NC, CHUNK_COLS), dtype=np.uint8)
    d = np.empty((T, NC, CHUNK_COLS), dtype=np.uint16)
    dm = np.empty((T, NC, CHUNK_COLS), dtype=np.uint16)
    for j in range(CHUNK_COLS):
        h = pk[:, :, 16 * j:16 * j + 16].astype(np.uint16)
        d[:, :, j] = h[:, :, 0] | (h[:, :, 1] << 8)
        dm[:, :, j] = h[:, :, 2] | (h[:, :, 3] << 8)
        bits = np.zeros((T, NC), dtype=object)
        for byte in range(12):
            bits = bits + (pk[:, :, 16 * j + 4 + byte].astype(object) << (8 * byte))
        for b in range(8):
            sc[:, b, :, j] = ((bits >> (6 * b)) & 63).astype(np.uint8)
            m[:, b, :, j] = ((bits >> (48 + 6 * b)) & 63).astype(np.uint8)
        for i in range(128):
            byte = pk[:, :, 2048 + 128 * j + i]
            q[:, 2 * i, :, j] = byte & 0x0F
            q[:, 2 * i + 1, :, j] = byte >> 4
    return {"q": q.reshape(M, K), "sc": sc.reshape(M // BLOCK_ROWS, K), "m": m.reshape(M // BLOCK_ROWS, K),
            "d": d.reshape(T, K).view(np.float16), "dmin": dm.reshape(T, K).view(np.float16)}
