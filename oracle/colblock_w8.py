"""CPU oracle for the 8-bit flavour of the column-block zigzag layout.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may import this module;
the product package never does.  Plain NumPy, written from the paper and the format text below,
sharing nothing with the HIP path.

The paper states that the layout carries over to other bit-widths (Section 4.1.3) without
giving one.  This build's 8-bit reading keeps what the 4-bit layout is built around - one
activation column's weights of a block-row are ONE 128-byte run - so a block-row is 128 rows
high instead of 256, and keeps the 32-row blocks with one fp16 scale each (Section 4.1.1's block
size):

  block    = rows 32b .. 32b+31 of one column
  scale s  = fp16( max|w| / 127 )            fp32 divide, then round to nearest even
  code  q  = clamp( rint( w / float(s) ), -128, 127 )     fp32, round half to even;
             q = 0 for every weight of a block whose scale rounds to zero
  value    = q * float(s)

The rule is evaluated in fp32 exactly as written because its results decide integers.

Packed form ("ZZ-CB32-W8"): T = M/128 block-rows, NC = K/128 chunks of 128 columns; chunk (t, c)
at byte offset (t*NC + c) * 17408:
  bytes [8 j + 2 b], j = 0..127, b = 0..3    fp16 scale (little endian) of rows 128t+32b .. +31 of
                                             column 128c + j
  bytes [1024 + 128 j + i], i = 0..127       code of row 128t + i of column 128c + j, stored q + 128
"""
from __future__ import annotations

import numpy as np

TILE_ROWS = 128
BLOCK_ROWS = 32
CHUNK_COLS = 128
CHUNK_BYTES = CHUNK_COLS * 8 + CHUNK_COLS * 128   # 17408


def check_shape(M: int, K: int) -> None:
    if M <= 0 or K <= 0 or M % TILE_ROWS or K % CHUNK_COLS:
        raise ValueError("8-bit column-block layout needs M % 128 == 0 and K % 128 == 0")


def pad_rows(W: np.ndarray) -> np.ndarray:
    """A matrix whose M is not a multiple of 128 is handled as the same matrix with zero rows
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
    """fp32 [M, K] -> (q int16 [M, K] in -128..127, scales fp16 [M/32, K]) by the rule in the header."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    M, K = W.shape
    check_shape(M, K)
    blocks = W.reshape(M // BLOCK_ROWS, BLOCK_ROWS, K)
    amax = np.max(np.abs(blocks), axis=1)                           # fp32 [M/32, K]
    scales = (amax / np.float32(127.0)).astype(np.float16)          # fp32 divide, RNE to fp16
    sf = scales.astype(np.float32)
    q = np.zeros((M // BLOCK_ROWS, BLOCK_ROWS, K), dtype=np.int16)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = blocks / sf[:, None, :]                             # fp32 divide
    r = np.clip(np.rint(ratio), -128, 127)                          # rint: half to even
    live = np.broadcast_to((sf > 0)[:, None, :], r.shape)
    q[live] = r[live].astype(np.int16)
    return q.reshape(M, K), scales


def dequant(q: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """fp64 [M, K] of q * float(scale)."""
    s = np.repeat(scales.astype(np.float64), BLOCK_ROWS, axis=0)
    return q.astype(np.float64) * s


def keep_mask(x: np.ndarray, threshold: float) -> np.ndarray:
    """Section 2: an entry is sparse iff |x| < threshold (compared in fp32)."""
    x = np.atleast_2d(x)
    a = np.abs(x.astype(np.float32))
    return np.any(~(a < np.float32(threshold)), axis=0)


def gemv(q: np.ndarray, scales: np.ndarray, x: np.ndarray, threshold: float) -> np.ndarray:
    """y[b, m] = sum over kept k of q[m, k] * scale[m/32, k] * x[b, k], in fp64."""
    x = np.atleast_2d(x)
    keep = keep_mask(x, threshold)
    Wd = dequant(q, scales)
    out = np.empty((x.shape[0], q.shape[0]), dtype=np.float64)
    for b in range(x.shape[0]):
        out[b] = Wd[:, keep] @ x[b, keep].astype(np.float64)
    return out


def pack(q: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """(q, scales) -> packed bytes, field by field along the format text."""
    M, K = q.shape
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    out = np.zeros((T, NC, CHUNK_BYTES), dtype=np.uint8)
    sbits = np.ascontiguousarray(scales).view(np.uint16).reshape(T, 4, NC, CHUNK_COLS)    # [t, b, c, j]
    code = (q.astype(np.int32) + 128).astype(np.uint8).reshape(T, TILE_ROWS, NC, CHUNK_COLS)  # [t, i, c, j]
    for j in range(CHUNK_COLS):
        for b in range(4):
            v = sbits[:, b, :, j]
            out[:, :, 8 * j + 2 * b] = (v & 0xFF).astype(np.uint8)
            out[:, :, 8 * j + 2 * b + 1] = (v >> 8).astype(np.uint8)
        for i in range(TILE_ROWS):
            out[:, :, 1024 + 128 * j + i] = code[:, i, :, j]
    return out.reshape(-1)


def unpack(packed: np.ndarray, M: int, K: int):
    """Inverse of pack."""
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    p = np.ascontiguousarray(packed, dtype=np.uint8).reshape(T, NC, CHUNK_BYTES)
    q = np.empty((T, TILE_ROWS, NC, CHUNK_COLS), dtype=np.int16)
    sbits = np.empty((T, 4, NC, CHUNK_COLS), dtype=np.uint16)
    for j in range(CHUNK_COLS):
        for b in range(4):
            sbits[:, b, :, j] = p[:, :, 8 * j + 2 * b].astype(np.uint16) | (p[:, :, 8 * j + 2 * b + 1].astype(np.uint16) << 8)
        for i in range(TILE_ROWS):
            q[:, i, :, j] = p[:, :, 1024 + 128 * j + i].astype(np.int16) - 128
    return q.reshape(M, K), sbits.reshape(M // BLOCK_ROWS, K).view(np.float16)
