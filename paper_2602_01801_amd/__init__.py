"""FAST-AR attention hot path for one MI355X: TempCache, AnnSA / AnnCA selection, block-sparse attention.

The work is done by ``libfastar.so`` (hand-written HIP for gfx950, C ABI in ``include/fastar.h``);
this package only marshals PyTorch device tensors into that ABI.
"""
from .binding import (  # noqa: F401
    BF16,
    EXPORTS,
    F32,
    LIB_PATH,
    OP_COMPRESS,
    OP_SELECT_CROSS,
    OP_SELECT_LSH,
    REP_LAST,
    REP_MEAN,
    REP_MEDOID,
    OP_SELECT_SELF,
    Cache,
    Codec,
    FastarError,
    ann_cross_attn_fwd,
    ann_select_cross,
    ann_select_lsh,
    ann_select_self,
    ann_select_self_static,
    encode,
    encode_sign,
    init,
    kv8_empty,
    kv_to_fp8,
    lib,
    probe_copy,
    probe_mfma_bf16,
    sparse_attn_fwd,
    sparse_attn_fwd_fp8,
    tempcache_compress,
    workspace_bytes,
)
