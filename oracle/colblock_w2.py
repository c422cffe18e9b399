"""CPU oracle for the 2-bit flavour of the column-block zigzag layout.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this module;
the product package never does.  Plain NumPy, written from the paper and the format text below,
sharing nothing with the HIP path.

The paper states that the layout carries over to other bit-widths, "e.g., 2-8 bit" (Section 4.1.3),
without giving one.  This build's 2-bit reading keeps what the 4-bit layout is built around - one
activation column's weights of a block-row are ONE 128-byte run - so a block-row is 512 rows high
instead of 256, and keeps the 32-row blocks with one fp16 scale each (Section 4.1.1's block size).
Four levels leave no room for a zero level and a symmetric range at once; the rule is the plain
mid-rise one, the levels being -1.5 s, -0.5 s, +0.5 s, +1.5 s:

  block    = rows 32b .. 32b+31 of one column
  scale s  = fp16( max|w| / 1.5 )            fp32 divide, then round to nearest even
  code  c  = clamp( rint( w / float(s) + 1.5 ), 0, 3 )     fp32, round half to even;
             c = 0 for every weight of a block whose scale rounds to zero (its values are then -0.0 = 0)
  value    = (c - 1.5) * float(s)

The rule is evaluated in fp32 exactly as written because its results decide integers.

Packed form ("ZZ-CB32-W2"): T = M/512 block-rows, NC = K/128 chunks of 128 columns; chunk (t, c)
at byte offset (t*NC + c) * 20480:
  bytes [32 j + 2 b], j = 0..127, b = 0..15   fp16 scale (little endian) of rows 512t+32b .. +31 of
                                              column 128c + j
  bytes [4096 + 128 j + i], i = 0..127        codes of rows 512t + 4i + e, e = 0..3, of column 128c + j,
                                              row 4i + e in bits 2e, 2e + 1
"""
from __future__ import annotations

import numpy as np

TILE_ROWS = 512
BLOCK_ROWS = 32
CHUNK_COLS = 128
SCALE_BYTES = CHUNK_COLS * 32
CHUNK_BYTES = SCALE_BYTES + CHUNK_COLS * 128   # 20480


def check_shape(M: int, K: int) -> None:
    if M <= 0 or K <= 0 or M % TILE_ROWS or K % CHUNK_COLS:
        raise ValueError("2-bit column-block layout needs M % 512 == 0 and K % 128 == 0")


def pad_rows(W: np.ndarray) -> np.ndarray:
    """A matrix whose M is not a multiple of 512 is handled as the same matrix with zero rows
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
    """fp32 [M, K] -> (c uint8 [M, K] in 0..3, scales fp16 [M/32, K]) by the rule in the header."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    M, K = W.shape
    check_shape(M, K)
    blocks = W.reshape(M // BLOCK_ROWS, BLOCK_ROWS, K)
    amax = np.max(np.abs(blocks), axis=1)                           # fp32 [M/32, K]
    scales = (amax / np.float32(1.5)).astype(np.float16)            # fp32 divide, RNE to fp16
    sf = scales.astype(np.float32)
    c = np.zeros((M // BLOCK_ROWS, BLOCK_ROWS, K), dtype=np.uint8)
    with np.errstate(divide="ignore", invalid="ignore"):
        pos = blocks / sf[:, None, :] + np.float32(1.5)             # fp32 divide, fp32 add
    r = np.clip(np.rint(pos), 0, 3)                                 # rint: half to even
    live = np.broadcast_to((sf > 0)[:, None, :], r.shape)
    c[live] = r[live].astype(np.uint8)
    return c.reshape(M, K), scales


def dequant(c: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """fp64 [M, K] of (c - 1.5) * float(scale)."""
    s = np.repeat(scales.astype(np.float64), BLOCK_ROWS, axis=0)
    return (c.astype(np.float64) - 1.5) * s


def keep_mask(x: np.ndarray, threshold: float) -> np.ndarray:
    """Section 2: an entry is sparse iff |x| < threshold (compared in fp32)."""
    x = np.atleast_2d(x)
    a = np.abs(x.astype(np.float32))
    return np.any(~(a < np.float32(threshold)), axis=0)


def gemv(c: np.ndarray, scales: np.ndarray, x: np.ndarray, threshold: float) -> np.ndarray:
    """y[b, m] = sum over kept k of (c[m, k] - 1.5) * scale[m/32, k] * x[b, k], in fp64."""
    x = np.atleast_2d(x)
    keep = keep_mask(x, threshold)
    Wd = dequant(c, scales)
    out = np.empty((x.shape[0], c.shape[0]), dtype=np.float64)
    for b in range(x.shape[0]):
        out[b] = Wd[:, keep] @ x[b, keep].astype(np.float64)
    return out


def pack(c: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """(c, scales) -> packed bytes, field by field along the format text."""
    M, K = c.shape
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    out = np.zeros((T, NC, CHUNK_BYTES), dtype=np.uint8)
    sbits = np.ascontiguousarray(scales).view(np.uint16).reshape(T, 16, NC, CHUNK_COLS)     # [t, b, c, j]
    code = c.astype(np.uint8).reshape(T, TILE_ROWS, NC, CHUNK_COLS)                         # [t, row, c, j]
    for j in range(CHUNK_COLS):
        for b in range(16):
            v = sbits[:, b, :, j]
            out[:, :, 32 * j + 2 * b] = (v & 0xFF).astype(np.uint8)
            out[:, :, 32 * j + 2 * b + 1] = (v >> 8).astype(np.uint8)
        for i in range(128):
            byte = np.zeros((T, NC), dtype=np.uint8)
            for e in range(4):
                byte |= (code[:, 4 * i + e, :, j] & 3) << (2 * e)
            out[:, :, SCALE_BYTES + 128 * j + i] = byte
    return out.reshape(-1)


def unpack(packed: np.ndarray, M: int, K: int):
    """Inverse of pack."""
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    p = np.ascontiguousarray(packed, dtype=np.uint8).reshape(T, NC, CHUNK_BYTES)
    c = np.empty((T, TILE_ROWS, NC, CHUNK_COLS), dtype=np.uint8)
    sbits = np.empty((T, 16, NC, CHUNK_COLS), dtype=np.uint16)
    for j in range(CHUNK_COLS):
        for b in range(16):
            sbits[:, b, :, j] = p[:, :, 32 * j + 2 * b].astype(np.uint16) | (p[:, :, 32 * j + 2 * b + 1].astype(np.uint16) << 8)
        for i in range(128):
            byte = p[:, :, SCALE_BYTES + 128 * j + i]
            for e in range(4):
                c[:, 4 * i + e, :, j] = (byte >> (2 * e)) & 3
    return c.reshape(M, K), sbits.reshape(M // BLOCK_ROWS, K).view(np.float16)
