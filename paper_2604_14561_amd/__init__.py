"""MI355X-native per-rank Ulysses attention-input path (QKV projection, Q/K RMSNorm + RoPE,
all-to-all pack/unpack, V-Major tile selection) as hand-written HIP behind a C ABI.

``binding`` marshals arguments to ``libcocodiff.so``; ``build`` compiles it in-tree.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    RECV_MAJOR,
    SEND_MAJOR,
    CocodiffError,
    Rope,
    Shape,
    a2a_pack,
    a2a_pack_hs,
    a2a_unpack,
    a2a_unpack_norm_rope,
    a2a_unpack_select,
    a2a_unpack_seq,
    cache_active_count,
    qk_norm_rope,
    qk_norm_rope_pack,
    qkv_proj,
    qkv_proj_fused,
    qkv_proj_hs,
    qkv_proj_pack,
    qkv_proj_plan,
    rope_table,
    util_copy,
    util_mfma_rate,
    version,
    vmajor_gather,
    vmajor_scatter,
    vmajor_select,
    vmajor_select_static,
    vmajor_token_metric,
    vmajor_topk,
    vmajor_select_workspace_bytes,
)
