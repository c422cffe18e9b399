"""CPU oracle for the column-block variant of the zigzag layout.  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline / parity pre-checks may
import this module; the product package never does.  Plain NumPy, written from the paper
and the format text below, sharing nothing with the HIP path.

What the paper defines (Section 4.1.2, "Zigzag weight layout"): the quantization groups
themselves run along a column - one superblock is 256 consecutive rows of ONE column, split
like Q4_K into eight blocks of 32 weights (Section 4.1.1) - and superblocks are stored
row-major (all columns of superblock-row 0, then row 1, ...), so a sparse activation entry
skips whole superblocks together with their scales.  The model is re-quantized offline into
this form (Section 5).

What this build fixes where the paper leaves it open (symmetric int4 as everywhere else in
this build instead of Q4_K's 6-bit scales and mins; same 4.5 bits per weight):

  block      32 consecutive rows of one column: rows 32 b' .. 32 b' + 31, column k
  scale      one fp16 per block:   s = fp16( max|w| / 7 )            (fp32 arithmetic, RNE)
  code       q = clamp( rint( w / float(s) ), -8, 7 )  in fp32, round half to even;
             q = 0 for every weight of a block whose scale rounds to 0
  value      q * float(s)

Because a floating-point result decides an integer here, the rule is evaluated in fp32 as
written (the precision the library's quantizer uses), not in fp64.

Packed form ("ZZ-CB32"): T = M/256 superblock-rows, NC = K/128 chunks of 128 columns;
chunk (t, c) at byte offset (t*NC + c) * 18432:
  bytes [16 j + 2 b], j = 0..127, b = 0..7   fp16 scale of rows 256t+32b..+31 of column 128c+j
  bytes [2048 + 128 j + i], i = 0..127       column 128c+j: low nibble = code of row 256t+2i,
                                              high nibble = code of row 256t+2i+1, stored q+8
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
    """fp32 [M, K] -> (q int8 [M, K], scales fp16 [M/32, K]) by the rule in the header."""
    W = np.ascontiguousarray(W, dtype=np.float32)
    M, K = W.shape
    check_shape(M, K)
    blocks = W.reshape(M // BLOCK_ROWS, BLOCK_ROWS, K)
    amax = np.max(np.abs(blocks), axis=1)                           # fp32 [M/32, K]
    scales = (amax / np.float32(7.0)).astype(np.float16)            # fp32 divide, RNE to fp16
    sf = scales.astype(np.float32)
    q = np.zeros((M // BLOCK_ROWS, BLOCK_ROWS, K), dtype=np.int8)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = blocks / sf[:, None, :]                             # fp32 divide
    r = np.clip(np.rint(ratio), -8, 7)                              # rint: half to even
    live = np.broadcast_to((sf > 0)[:, None, :], r.shape)
    q[live] = r[live].astype(np.int8)
    return q.reshape(M, K), scales


def dequant(q: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """fp64 [M, K] of q * float(scale)."""
    M, K = q.shape
    s = np.repeat(scales.astype(np.float64), BLOCK_ROWS, axis=0)
    return q.astype(np.float64) * s


def keep_mask(x: np.ndarray, threshold: float) -> np.ndarray:
    """Section 2: an entry is sparse iff |x| < threshold (compared in fp32); batch rows are OR-ed."""
    x = np.atleast_2d(x)
    a = np.abs(x.astype(np.float32))
    return np.any(~(a < np.float32(threshold)), axis=0)


def gemv(q: np.ndarray, scales: np.ndarray, x: np.ndarray, threshold: float) -> np.ndarray:
    """y[b, m] = sum over kept k of q[m, k] * scale[m/32, k] * x[b, k], in fp64."""
    x = np.atleast_2d(x)
    keep = keep_mask(x, threshold)
    Wd = dequant(q, scales)
    xk = np.where(keep[None, :], x.astype(np.float64), 0.0)
    out = np.empty((x.shape[0], q.shape[0]), dtype=np.float64)
    for b in range(x.shape[0]):
        out[b] = Wd[:, keep] @ xk[b, keep]
    return out


def pack(q: np.ndarray, scales: np.ndarray) -> np.ndarray:
    """(q, scales) -> packed bytes, one element at a time along the format text (vectorised
    over superblock-rows and chunks only)."""
    M, K = q.shape
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    out = np.zeros((T, NC, CHUNK_BYTES), dtype=np.uint8)
    sbits = np.ascontiguousarray(scales).view(np.uint16).reshape(T, 8, NC, CHUNK_COLS)   # [t, b, c, j]
    code = (q.astype(np.int16) + 8).astype(np.uint8).reshape(T, TILE_ROWS, NC, CHUNK_COLS)  # [t, r, c, j]
    for j in range(CHUNK_COLS):
        for b in range(8):
            v = sbits[:, b, :, j]
            out[:, :, 16 * j + 2 * b] = (v & 0xFF).astype(np.uint8)
            out[:, :, 16 * j + 2 * b + 1] = (v >> 8).astype(np.uint8)
        for i in range(128):
            lo = code[:, 2 * i, :, j]
            hi = code[:, 2 * i + 1, :, j]
            out[:, :, 2048 + 128 * j + i] = lo | (hi << 4)
    return out.reshape(-1)


def unpack(packed: np.ndarray, M: int, K: int):
    """Inverse of pack."""
    check_shape(M, K)
    T, NC = M // TILE_ROWS, K // CHUNK_COLS
    p = np.ascontiguousarray(packed, dtype=np.uint8).reshape(T, NC, CHUNK_BYTES)
    q = np.empty((T, TILE_ROWS, NC, CHUNK_COLS), dtype=np.int8)
    sbits = np.empty((T, 8, NC, CHUNK_COLS), dtype=np.uint16)
    for j in range(CHUNK_COLS):
        for b in range(8):
            sbits[:, b, :, j] = p[:, :, 16 * j + 2 * b].astype(np.uint16) | (p[:, :, 16 * j + 2 * b + 1].astype(np.uint16) << 8)
        for i in range(128):
            byte = p[:, :, 2048 + 128 * j + i]
            q[:, 2 * i, :, j] = (byte & 0x0F).astype(np.int8) - 8
            q[:, 2 * i + 1, :, j] = (byte >> 4).astype(np.int8) - 8
    return q.reshape(M, K), sbits.reshape(M // BLOCK_ROWS, K).view(np.float16)
