"""MI355X-native SDVG hot path: block-causal attention over a KV cache, KV commit / rollback
and worst-frame routing, as hand-written HIP kernels behind a C ABI (include/sdvg.h).

This package is only the thin Python binding of libsdvg.so; every step runs in the HIP
kernels. It raises if the library has not been built (python -m paper_2604_17397_amd.build).
"""
from .binding import (  # noqa: F401
    SdvgError,
    KVCache,
    block_attn,
    block_attn_batch,
    block_attn_commit,
    kv_commit_mark,
    block_attn_batch_static,
    block_attn_workspace_bytes,
    kv_commit,
    kv_rollback,
    rope,
    kv_commit_rope,
    buffer_snapshot,
    worst_frame_route,
    worst_frame_route_batch,
    probe_mfma,
    lib,
    status_string,
    SDVG_BF16,
    SDVG_F32,
)
