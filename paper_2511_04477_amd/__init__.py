"""MI355X-native SpQt hot path: zigzag repack, sparse index gather, sparse int4 GEMV.

The work is done by hand-written HIP kernels in libspqt.so (C ABI in include/spqt.h); this
package only marshals arguments.  There is no CPU fallback.
"""
from .binding import (  # noqa: F401
    SpqtError,
    LaunchCfg,
    LIB_PATH,
    EXPORTS,
    CB_EXPORTS,
    CB_CHUNK_BYTES,
    TILE_ROWS,
    GROUP,
    CHUNK_BYTES,
    MAX_SPLITS,
    CFG_NO_COMPACTION,
    lib,
    new_workspace,
    spqt_default_cfg,
    spqt_gather,
    spqt_gemv,
    spqt_gemv_fused,
    spqt_pack,
    spqt_packed_bytes,
    spqt_status_str,
    spqt_unpack,
    spqt_workspace_bytes,
    spqt_workspace_init,
    spqt_cb_packed_bytes,
    spqt_cb_quantize,
    spqt_cb_dequantize,
    spqt_cb_gemv,
    spqt_cb_gemv_fused,
    spqt_cbk_quantize,
    spqt_cbk_dequantize,
    spqt_cbk_gemv,
)
