"""Thin ctypes binding over libspqt.so: argument marshalling only.

Same names as the C ABI (include/spqt.h).  Host calls take NumPy arrays; device calls take
torch CUDA tensors (PyTorch supplies device memory and the stream, nothing else) and launch
on torch's current stream unless one is given.  There is no fallback of any kind: if the
shared library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libspqt.so")

SPQT_OK = 0
TILE_ROWS = 256
GROUP = 128
CHUNK_BYTES = 16896
MAX_SPLITS = 64
CFG_NO_COMPACTION = 1
CFG_Y_FP16 = 4
CFG_GROUP_PASSES = 8
CFG_EVEN_SHARES = 16

EXPORTS = [
    "spqt_status_str", "spqt_packed_bytes", "spqt_workspace_bytes", "spqt_workspace_init",
    "spqt_pack", "spqt_unpack", "spqt_gather", "spqt_gather_rows", "spqt_gemv", "spqt_gemv_ex", "spqt_gemv_static", "spqt_gemv_fused", "spqt_gemv_fused_rows",
    "spqt_default_cfg",
]


CB_EXPORTS = ["spqt_cb_packed_bytes", "spqt_cb_quantize", "spqt_cb_dequantize", "spqt_cb_gemv",
              "spqt_cb_gemv_fused", "spqt_cbk_quantize", "spqt_cbk_dequantize", "spqt_cbk_gemv", "spqt_cbk_gemv_fused",
              "spqt_cb8_packed_bytes", "spqt_cb8_quantize", "spqt_cb8_dequantize", "spqt_cb8_gemv", "spqt_cb8_gemv_fused", "spqt_cb8_gemv_rows",
              "spqt_cb2_packed_bytes", "spqt_cb2_quantize", "spqt_cb2_dequantize", "spqt_cb2_gemv", "spqt_cb2_gemv_fused", "spqt_cb2_gemv_rows"]
CB_CHUNK_BYTES = 18432
CB8_CHUNK_BYTES = 17408
CB2_CHUNK_BYTES = 20480


class SpqtError(RuntimeError):
    pass


class LaunchCfg(ctypes.Structure):
    _fields_ = [("splits", ctypes.c_int), ("waves", ctypes.c_int), ("flags", ctypes.c_int)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load libspqt.so (built in-tree by paper_2511_04477_amd.build); raise if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise SpqtError(f"{LIB_PATH} is not built; run `python -m paper_2511_04477_amd.build` "
                            "(there is no CPU or PyTorch fallback)")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        vp, i64, i32, sz = c.c_void_p, c.c_int64, c.c_int, c.c_size_t
        L.spqt_status_str.restype = c.c_char_p
        L.spqt_status_str.argtypes = [i32]
        L.spqt_packed_bytes.argtypes = [i64, i64, i32, c.POINTER(sz)]
        L.spqt_workspace_bytes.argtypes = [i64, i64, i32, c.POINTER(sz)]
        L.spqt_workspace_init.argtypes = [vp, sz, vp]
        L.spqt_pack.argtypes = [vp, vp, i64, i64, i32, vp, sz]
        L.spqt_unpack.argtypes = [vp, i64, i64, i32, vp, vp]
        L.spqt_gather.argtypes = [vp, i64, i32, c.c_float, vp, vp, vp]
        L.spqt_gather_rows.argtypes = [vp, i64, i32, c.c_float, vp, vp, vp, vp]
        L.spqt_gemv.argtypes = [vp, i64, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp]
        L.spqt_gemv_ex.argtypes = [vp, i64, i64, i32, vp, i32, vp, vp, vp, vp, sz, vp,
                                   c.POINTER(LaunchCfg)]
        L.spqt_gemv_static.argtypes = [vp, i64, i64, i32, vp, i32, vp, vp, vp, vp]
        L.spqt_gemv_fused.argtypes = [vp, i64, i64, i32, vp, c.c_float, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_gemv_fused_rows.argtypes = [vp, i64, i64, i32, vp, i32, c.c_float, i32, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_default_cfg.argtypes = [i64, i64, i32, i32, c.POINTER(LaunchCfg)]
        L.spqt_cb_packed_bytes.argtypes = [i64, i64, c.POINTER(sz)]
        L.spqt_cb_quantize.argtypes = [vp, i64, i64, vp, sz]
        L.spqt_cb_dequantize.argtypes = [vp, i64, i64, vp]
        L.spqt_cb_gemv.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cb_gemv_fused.argtypes = [vp, i64, i64, vp, c.c_float, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cbk_quantize.argtypes = [vp, i64, i64, vp, sz]
        L.spqt_cbk_dequantize.argtypes = [vp, i64, i64, vp]
        L.spqt_cbk_gemv.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cbk_gemv_fused.argtypes = [vp, i64, i64, vp, c.c_float, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cb8_packed_bytes.argtypes = [i64, i64, c.POINTER(sz)]
        L.spqt_cb8_quantize.argtypes = [vp, i64, i64, vp, sz]
        L.spqt_cb8_dequantize.argtypes = [vp, i64, i64, vp]
        L.spqt_cb8_gemv.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cb2_packed_bytes.argtypes = [i64, i64, c.POINTER(sz)]
        L.spqt_cb2_quantize.argtypes = [vp, i64, i64, vp, sz]
        L.spqt_cb2_dequantize.argtypes = [vp, i64, i64, vp]
        L.spqt_cb2_gemv.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cb8_gemv_rows.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cb2_gemv_rows.argtypes = [vp, i64, i64, vp, i32, vp, vp, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cb8_gemv_fused.argtypes = [vp, i64, i64, vp, c.c_float, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        L.spqt_cb2_gemv_fused.argtypes = [vp, i64, i64, vp, c.c_float, vp, vp, sz, vp, c.POINTER(LaunchCfg)]
        for name in EXPORTS[1:] + CB_EXPORTS:
            getattr(L, name).restype = i32
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != SPQT_OK:
        raise SpqtError(lib().spqt_status_str(rc).decode())


def spqt_status_str(status: int) -> str:
    return lib().spqt_status_str(int(status)).decode()


def spqt_packed_bytes(M: int, K: int, group: int = GROUP) -> int:
    out = ctypes.c_size_t()
    _check(lib().spqt_packed_bytes(M, K, group, ctypes.byref(out)))
    return out.value


def spqt_workspace_bytes(M: int, K: int, batch: int = 1) -> int:
    out = ctypes.c_size_t()
    _check(lib().spqt_workspace_bytes(M, K, batch, ctypes.byref(out)))
    return out.value


def spqt_default_cfg(M: int, K: int, batch: int = 1, sparse: bool = True):
    cfg = LaunchCfg()
    _check(lib().spqt_default_cfg(M, K, batch, int(sparse), ctypes.byref(cfg)))
    return cfg.splits, cfg.waves


# ----------------------------------------------------------------------------- host calls

def _np_ptr(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(ctypes.c_void_p)


def spqt_pack(q_rowmajor: np.ndarray, scales: np.ndarray, group: int = GROUP) -> np.ndarray:
    """uint8[M, K/2] codes + fp16 (or uint16 bits) [M, K/group] scales -> packed uint8 bytes."""
    q = np.ascontiguousarray(q_rowmajor, dtype=np.uint8)
    s = np.ascontiguousarray(scales)
    s = s.view(np.uint16) if s.dtype == np.float16 else s
    if s.dtype != np.uint16 or q.ndim != 2 or s.ndim != 2:
        raise SpqtError("spqt_pack: need uint8[M,K/2] codes and fp16/uint16[M,K/group] scales")
    M, K = q.shape[0], q.shape[1] * 2
    if s.shape != (M, K // group if group else 0):
        raise SpqtError("spqt_pack: scales shape does not match [M, K/group]")
    out = np.empty(spqt_packed_bytes(M, K, group), dtype=np.uint8)
    _check(lib().spqt_pack(_np_ptr(q), _np_ptr(s), M, K, group, _np_ptr(out), out.nbytes))
    return out


def spqt_unpack(packed: np.ndarray, M: int, K: int, group: int = GROUP):
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    if p.nbytes < spqt_packed_bytes(M, K, group):
        raise SpqtError("spqt_unpack: packed buffer too small")
    q = np.empty((M, K // 2), dtype=np.uint8)
    s = np.empty((M, K // group), dtype=np.uint16)
    _check(lib().spqt_unpack(_np_ptr(p), M, K, group, _np_ptr(q), _np_ptr(s)))
    return q, s.view(np.float16)


# --------------------------------------------------------------------------- device calls

def _stream_ptr(stream) -> int:
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _dev(t, dtype, what):
    import torch
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise SpqtError(f"{what}: need a contiguous CUDA tensor of dtype {dtype}")
    return t.data_ptr()


def _y_out(y):
    """(device pointer, flag bits) of an output tensor: fp32, or fp16 with SPQT_CFG_Y_FP16."""
    import torch
    if isinstance(y, torch.Tensor) and y.dtype == torch.float16:
        return _dev(y, torch.float16, "y"), CFG_Y_FP16
    return _dev(y, torch.float32, "y"), 0


def _cfg(splits, waves, flags) -> LaunchCfg:
    return LaunchCfg(int(splits), int(waves), int(flags))


def spqt_workspace_init(workspace, stream=None) -> None:
    import torch
    p = _dev(workspace, torch.uint8, "workspace")
    _check(lib().spqt_workspace_init(p, workspace.numel(), _stream_ptr(stream)))


def new_workspace(M: int, K: int, batch: int = 1, device="cuda"):
    """Allocate and prepare a workspace tensor for spqt_gemv on this shape."""
    import torch
    ws = torch.empty(spqt_workspace_bytes(M, K, batch), dtype=torch.uint8, device=device)
    spqt_workspace_init(ws)
    return ws


def spqt_gather(x, threshold: float, idx_out, count_out, stream=None) -> None:
    """x fp16[K] or [batch, K]; idx_out int32[>=K]; count_out int32[1] (all on the GPU)."""
    import torch
    xp = _dev(x, torch.float16, "x")
    batch, K = (1, x.shape[0]) if x.dim() == 1 else (x.shape[0], x.shape[1])
    ip = _dev(idx_out, torch.int32, "idx_out")
    cp = _dev(count_out, torch.int32, "count_out")
    if idx_out.numel() < K or count_out.numel() < 1:
        raise SpqtError("spqt_gather: idx_out needs K entries and count_out one")
    _check(lib().spqt_gather(xp, K, batch, float(threshold), ip, cp, _stream_ptr(stream)))


def spqt_gather_rows(x, threshold: float, idx_out, count_out, x_masked_out, stream=None) -> None:
    """spqt_gather plus x_masked_out (fp16, same shape as x): every row with its own dropped
    entries zeroed; feed it to a GEMV with idx_out / count_out for per-row kept sets."""
    import torch
    xp = _dev(x, torch.float16, "x")
    batch, K = (1, x.shape[0]) if x.dim() == 1 else (x.shape[0], x.shape[1])
    ip = _dev(idx_out, torch.int32, "idx_out")
    cp = _dev(count_out, torch.int32, "count_out")
    mp = _dev(x_masked_out, torch.float16, "x_masked_out")
    if idx_out.numel() < K or count_out.numel() < 1 or x_masked_out.numel() != x.numel():
        raise SpqtError("spqt_gather_rows: idx_out needs K entries, count_out one, x_masked_out the size of x")
    _check(lib().spqt_gather_rows(xp, K, batch, float(threshold), ip, cp, mp, _stream_ptr(stream)))


def spqt_gemv(packed, M: int, K: int, x, idx, count, y, workspace, stream=None, group: int = GROUP,
              splits: int = 0, waves: int = 0, flags: int = 0) -> None:
    """packed uint8 (device); x fp16[K] or [batch,K]; idx/count from spqt_gather or None/None
    for the dense kernel; y fp32 (or fp16) [M] or [batch,M]; workspace from new_workspace()."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    batch = 1 if x.dim() == 1 else x.shape[0]
    if x.shape[-1] != K or y.numel() != batch * M or packed.numel() < spqt_packed_bytes(M, K, group):
        raise SpqtError("spqt_gemv: x / y / packed sizes do not match M, K, batch")
    ip = cp = None
    if idx is not None:
        ip = _dev(idx, torch.int32, "idx")
        cp = _dev(count, torch.int32, "count")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    if splits or waves or yflags or flags:
        cfg = _cfg(splits, waves, int(flags) | yflags)
        rc = lib().spqt_gemv_ex(pp, M, K, group, xp, batch, ip, cp, yp, wp, wbytes,
                                _stream_ptr(stream), ctypes.byref(cfg))
    else:
        rc = lib().spqt_gemv(pp, M, K, group, xp, batch, ip, cp, yp, wp, wbytes, _stream_ptr(stream))
    _check(rc)


def spqt_gemv_static(packed, M: int, K: int, x, idx, count, y, stream=None, group: int = GROUP) -> None:
    """spqt_gemv without a workspace argument: the exchange words live in the library's own device array."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp = _dev(y, torch.float32, "y")
    batch = 1 if x.dim() == 1 else x.shape[0]
    if x.shape[-1] != K or y.numel() != batch * M or packed.numel() < spqt_packed_bytes(M, K, group):
        raise SpqtError("spqt_gemv_static: x / y / packed sizes do not match M, K, batch")
    ip = cp = None
    if idx is not None:
        ip = _dev(idx, torch.int32, "idx")
        cp = _dev(count, torch.int32, "count")
    _check(lib().spqt_gemv_static(pp, M, K, group, xp, batch, ip, cp, yp, _stream_ptr(stream)))


def spqt_gemv_fused(packed, M: int, K: int, x, threshold: float, y, workspace, stream=None,
                    group: int = GROUP, splits: int = 0, waves: int = 0, flags: int = 0) -> None:
    """Threshold + compaction + GEMV in one launch (batch 1): x fp16[K], y fp32 (or fp16) [M]."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    if x.numel() != K or y.numel() != M or packed.numel() < spqt_packed_bytes(M, K, group):
        raise SpqtError("spqt_gemv_fused: x / y / packed sizes do not match M, K (batch 1 only)")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, int(flags) | yflags)
    _check(lib().spqt_gemv_fused(pp, M, K, group, xp, float(threshold), yp, wp, wbytes,
                                 _stream_ptr(stream), ctypes.byref(cfg)))


def spqt_gemv_fused_rows(packed, M: int, K: int, x, threshold: float, y, workspace, own_sets: bool = False, stream=None,
                         group: int = GROUP, splits: int = 0) -> None:
    """Threshold + compaction + GEMV in one launch for x fp16[batch, K], batch 1..4; y fp32 (or fp16) [batch, M].
    own_sets: every row sums over its own kept columns instead of the union."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    batch = 1 if x.dim() == 1 else x.shape[0]
    if x.shape[-1] != K or y.numel() != batch * M or packed.numel() < spqt_packed_bytes(M, K, group):
        raise SpqtError("spqt_gemv_fused_rows: x / y / packed sizes do not match M, K, batch")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, 0, yflags)
    _check(lib().spqt_gemv_fused_rows(pp, M, K, group, xp, batch, float(threshold), int(bool(own_sets)), yp, wp, wbytes,
                                      _stream_ptr(stream), ctypes.byref(cfg)))


# ------------------------------------------------------------- column-block variant (spqt_colblock.h)

def spqt_cb_packed_bytes(M: int, K: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().spqt_cb_packed_bytes(M, K, ctypes.byref(out)))
    return out.value


def spqt_cb_quantize(w: np.ndarray) -> np.ndarray:
    """fp32 [M, K] -> packed column-block bytes (host)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim != 2:
        raise SpqtError("spqt_cb_quantize: need float32[M, K]")
    M, K = w.shape
    out = np.empty(spqt_cb_packed_bytes(M, K), dtype=np.uint8)
    _check(lib().spqt_cb_quantize(_np_ptr(w), M, K, _np_ptr(out), out.nbytes))
    return out


def spqt_cb_dequantize(packed: np.ndarray, M: int, K: int) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    if p.nbytes < spqt_cb_packed_bytes(M, K):
        raise SpqtError("spqt_cb_dequantize: packed buffer too small")
    out = np.empty((M, K), dtype=np.float32)
    _check(lib().spqt_cb_dequantize(_np_ptr(p), M, K, _np_ptr(out)))
    return out


def spqt_cb_gemv(packed, M: int, K: int, x, idx, count, y, workspace, stream=None, splits: int = 0,
                 waves: int = 0) -> None:
    """Column-block GEMV: packed uint8 (device), x fp16[K] or [batch, K], idx/count from spqt_gather
    or None/None for the dense kernel, y fp32 (or fp16) [M] or [batch, M], workspace from
    new_workspace()."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    batch = 1 if x.dim() == 1 else x.shape[0]
    if x.shape[-1] != K or y.numel() != batch * M or packed.numel() < spqt_cb_packed_bytes(M, K):
        raise SpqtError("spqt_cb_gemv: x / y / packed sizes do not match M, K, batch")
    ip = cp = None
    if idx is not None:
        ip = _dev(idx, torch.int32, "idx")
        cp = _dev(count, torch.int32, "count")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(lib().spqt_cb_gemv(pp, M, K, xp, batch, ip, cp, yp, wp, wbytes, _stream_ptr(stream), ctypes.byref(cfg)))


def spqt_cb_gemv_fused(packed, M: int, K: int, x, threshold: float, y, workspace, stream=None,
                       splits: int = 0, waves: int = 0) -> None:
    """Threshold + compaction + column-block GEMV in one launch (batch 1)."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    if x.numel() != K or y.numel() != M or packed.numel() < spqt_cb_packed_bytes(M, K):
        raise SpqtError("spqt_cb_gemv_fused: x / y / packed sizes do not match M, K (batch 1 only)")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(lib().spqt_cb_gemv_fused(pp, M, K, xp, float(threshold), yp, wp, wbytes, _stream_ptr(stream),
                                    ctypes.byref(cfg)))


# ---------------------------------------------------------------- K-quant flavour (spqt_colblock.h)

def spqt_cbk_quantize(w: np.ndarray) -> np.ndarray:
    """fp32 [M, K] -> packed K-quant column-block bytes (host)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim != 2:
        raise SpqtError("spqt_cbk_quantize: need float32[M, K]")
    M, K = w.shape
    out = np.empty(spqt_cb_packed_bytes(M, K), dtype=np.uint8)
    _check(lib().spqt_cbk_quantize(_np_ptr(w), M, K, _np_ptr(out), out.nbytes))
    return out


def spqt_cbk_dequantize(packed: np.ndarray, M: int, K: int) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    if p.nbytes < spqt_cb_packed_bytes(M, K):
        raise SpqtError("spqt_cbk_dequantize: packed buffer too small")
    out = np.empty((M, K), dtype=np.float32)
    _check(lib().spqt_cbk_dequantize(_np_ptr(p), M, K, _np_ptr(out)))
    return out


def spqt_cbk_gemv(packed, M: int, K: int, x, idx, count, y, workspace, stream=None, splits: int = 0,
                  waves: int = 0) -> None:
    """K-quant column-block GEMV: x fp16[K] or [batch, K] (idx/count None/None for the dense kernel)."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    batch = 1 if x.dim() == 1 else x.shape[0]
    if x.shape[-1] != K or y.numel() != batch * M or packed.numel() < spqt_cb_packed_bytes(M, K):
        raise SpqtError("spqt_cbk_gemv: x / y / packed sizes do not match M, K, batch")
    ip = cp = None
    if idx is not None:
        ip = _dev(idx, torch.int32, "idx")
        cp = _dev(count, torch.int32, "count")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(lib().spqt_cbk_gemv(pp, M, K, xp, batch, ip, cp, yp, wp, wbytes, _stream_ptr(stream), ctypes.byref(cfg)))


def spqt_cbk_gemv_fused(packed, M: int, K: int, x, threshold: float, y, workspace, stream=None,
                        splits: int = 0, waves: int = 0) -> None:
    """Threshold + compaction + K-quant column-block GEMV in one launch (batch 1)."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    if x.numel() != K or y.numel() != M or packed.numel() < spqt_cb_packed_bytes(M, K):
        raise SpqtError("spqt_cbk_gemv_fused: x / y / packed sizes do not match M, K (batch 1 only)")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(lib().spqt_cbk_gemv_fused(pp, M, K, xp, float(threshold), yp, wp, wbytes, _stream_ptr(stream),
                                     ctypes.byref(cfg)))


# ------------------------------------------------------------------ 8-bit flavour (spqt_colblock.h)

def spqt_cb8_packed_bytes(M: int, K: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().spqt_cb8_packed_bytes(M, K, ctypes.byref(out)))
    return out.value


def spqt_cb8_quantize(w: np.ndarray) -> np.ndarray:
    """fp32 [M, K] -> packed 8-bit column-block bytes (host)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim != 2:
        raise SpqtError("spqt_cb8_quantize: need float32[M, K]")
    M, K = w.shape
    out = np.empty(spqt_cb8_packed_bytes(M, K), dtype=np.uint8)
    _check(lib().spqt_cb8_quantize(_np_ptr(w), M, K, _np_ptr(out), out.nbytes))
    return out


def spqt_cb8_dequantize(packed: np.ndarray, M: int, K: int) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    if p.nbytes < spqt_cb8_packed_bytes(M, K):
        raise SpqtError("spqt_cb8_dequantize: packed buffer too small")
    out = np.empty((M, K), dtype=np.float32)
    _check(lib().spqt_cb8_dequantize(_np_ptr(p), M, K, _np_ptr(out)))
    return out


def spqt_cb8_gemv(packed, M: int, K: int, x, idx, count, y, workspace, stream=None, splits: int = 0,
                  waves: int = 0) -> None:
    """8-bit column-block GEMV, batch 1 (idx/count None/None for the dense kernel)."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    if x.numel() != K or y.numel() != M or packed.numel() < spqt_cb8_packed_bytes(M, K):
        raise SpqtError("spqt_cb8_gemv: x / y / packed sizes do not match M, K (batch 1 only)")
    ip = cp = None
    if idx is not None:
        ip = _dev(idx, torch.int32, "idx")
        cp = _dev(count, torch.int32, "count")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(lib().spqt_cb8_gemv(pp, M, K, xp, ip, cp, yp, wp, wbytes, _stream_ptr(stream), ctypes.byref(cfg)))


# ------------------------------------------------------------------ 2-bit flavour (spqt_colblock.h)

def spqt_cb2_packed_bytes(M: int, K: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().spqt_cb2_packed_bytes(M, K, ctypes.byref(out)))
    return out.value


def spqt_cb2_quantize(w: np.ndarray) -> np.ndarray:
    """fp32 [M, K] -> packed 2-bit column-block bytes (host)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    if w.ndim != 2:
        raise SpqtError("spqt_cb2_quantize: need float32[M, K]")
    M, K = w.shape
    out = np.empty(spqt_cb2_packed_bytes(M, K), dtype=np.uint8)
    _check(lib().spqt_cb2_quantize(_np_ptr(w), M, K, _np_ptr(out), out.nbytes))
    return out


def spqt_cb2_dequantize(packed: np.ndarray, M: int, K: int) -> np.ndarray:
    p = np.ascontiguousarray(packed, dtype=np.uint8)
    if p.nbytes < spqt_cb2_packed_bytes(M, K):
        raise SpqtError("spqt_cb2_dequantize: packed buffer too small")
    out = np.empty((M, K), dtype=np.float32)
    _check(lib().spqt_cb2_dequantize(_np_ptr(p), M, K, _np_ptr(out)))
    return out


def spqt_cb2_gemv(packed, M: int, K: int, x, idx, count, y, workspace, stream=None, splits: int = 0,
                  waves: int = 0) -> None:
    """2-bit column-block GEMV, batch 1 (idx/count None/None for the dense kernel)."""
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    if x.numel() != K or y.numel() != M or packed.numel() < spqt_cb2_packed_bytes(M, K):
        raise SpqtError("spqt_cb2_gemv: x / y / packed sizes do not match M, K (batch 1 only)")
    ip = cp = None
    if idx is not None:
        ip = _dev(idx, torch.int32, "idx")
        cp = _dev(count, torch.int32, "count")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(lib().spqt_cb2_gemv(pp, M, K, xp, ip, cp, yp, wp, wbytes, _stream_ptr(stream), ctypes.byref(cfg)))


def _width_fused(fn_name, bytes_fn, packed, M, K, x, threshold, y, workspace, stream, splits, waves):
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    if x.numel() != K or y.numel() != M or packed.numel() < bytes_fn(M, K):
        raise SpqtError(f"{fn_name}: x / y / packed sizes do not match M, K (batch 1 only)")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(getattr(lib(), fn_name)(pp, M, K, xp, float(threshold), yp, wp, wbytes, _stream_ptr(stream), ctypes.byref(cfg)))


def spqt_cb8_gemv_fused(packed, M: int, K: int, x, threshold: float, y, workspace, stream=None, splits: int = 0,
                        waves: int = 0) -> None:
    """8-bit column-block gather + GEMV in one launch, batch 1."""
    _width_fused("spqt_cb8_gemv_fused", spqt_cb8_packed_bytes, packed, M, K, x, threshold, y, workspace, stream, splits, waves)


def spqt_cb2_gemv_fused(packed, M: int, K: int, x, threshold: float, y, workspace, stream=None, splits: int = 0,
                        waves: int = 0) -> None:
    """2-bit column-block gather + GEMV in one launch, batch 1."""
    _width_fused("spqt_cb2_gemv_fused", spqt_cb2_packed_bytes, packed, M, K, x, threshold, y, workspace, stream, splits, waves)


def _width_rows(fn_name, bytes_fn, packed, M, K, x, idx, count, y, workspace, stream, splits, waves):
    import torch
    pp = _dev(packed, torch.uint8, "packed")
    xp = _dev(x, torch.float16, "x")
    yp, yflags = _y_out(y)
    batch = x.numel() // K
    if x.numel() != batch * K or y.numel() != batch * M or packed.numel() < bytes_fn(M, K):
        raise SpqtError(f"{fn_name}: x / y / packed sizes do not match M, K")
    ip = cp = None
    if idx is not None:
        ip = _dev(idx, torch.int32, "idx")
        cp = _dev(count, torch.int32, "count")
    wp, wbytes = None, 0
    if workspace is not None:
        wp, wbytes = _dev(workspace, torch.uint8, "workspace"), workspace.numel()
    cfg = _cfg(splits, waves, yflags)
    _check(getattr(lib(), fn_name)(pp, M, K, xp, batch, ip, cp, yp, wp, wbytes, _stream_ptr(stream), ctypes.byref(cfg)))


def spqt_cb8_gemv_rows(packed, M: int, K: int, x, idx, count, y, workspace, stream=None, splits: int = 0,
                       waves: int = 0) -> None:
    """8-bit column-block GEMV for x fp16[batch][K], batch 1..4, on the union list (or dense)."""
    _width_rows("spqt_cb8_gemv_rows", spqt_cb8_packed_bytes, packed, M, K, x, idx, count, y, workspace, stream, splits, waves)


def spqt_cb2_gemv_rows(packed, M: int, K: int, x, idx, count, y, workspace, stream=None, splits: int = 0,
                       waves: int = 0) -> None:
    """2-bit column-block GEMV for x fp16[batch][K], batch 1..3, on the union list (or dense)."""
    _width_rows("spqt_cb2_gemv_rows", spqt_cb2_packed_bytes, packed, M, K, x, idx, count, y, workspace, stream, splits, waves)
