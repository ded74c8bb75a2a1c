"""CPU fp64 oracle for the SDVG hot path. Test infrastructure, not the product.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this package.
"""
from .oracle import (  # noqa: F401
    block_attn,
    kv_commit,
    kv_rollback,
    buffer_copy,
    route,
    rope,
    num_threads,
    KVMirror,
)
