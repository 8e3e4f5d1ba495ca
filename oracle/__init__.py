"""CPU oracle for the Ulysses attention-input path (TEST INFRASTRUCTURE ONLY).

A plain, slow, obviously correct implementation of what the path computes,
written from the paper's definitions: fp64 projection, fp64 RMSNorm and rotary
embedding, explicit index loops for the all-to-all pack / exchange / unpack
and for the V-Major tile selection.  It shares no code with the HIP library and
never imports it.  Only the tests, the smoke run and the benchmark's CPU
baseline leg may call it; the product path never does.

Every function here is pinned by tests that do not go through this package's
own formulas (brute force on tiny inputs, closed forms, invariants, library
routines in special cases); no function is "parity unpinned".
"""
from . import ref  # noqa: F401
from .ref import (  # noqa: F401
    a2a_exchange,
    a2a_pack,
    a2a_pack_hs,
    a2a_unpack,
    a2a_unpack_seq,
    active_count,
    build_c,
    cache_ratio,
    omp_max_threads,
    qk_norm_rope,
    qkv_proj,
    rms_norm,
    rope_rotate,
    token_coords,
    token_l1_metric,
    topk_active,
    vmajor_gather,
    vmajor_scatter,
    vmajor_select,
    widen,
)
