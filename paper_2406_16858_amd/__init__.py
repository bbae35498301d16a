"""MI355X (gfx950) hot path of EAGLE-2's dynamic draft tree: thin Python binding.

The functions here only marshal torch tensors (device pointers, the current HIP
stream) into the C ABI declared in include/eagle2.h; every step of the method
runs in the HIP kernels of libeagle2_hip.so.  There is no CPU fallback: if the
library has not been built the import of `binding` raises.
"""
from .binding import (  # noqa: F401
    AttnCfg,
    DraftCfg,
    DraftWeights,
    draft_weights,
    eagle2_draft_forward,
    eagle2_draft_workspace_bytes,
    Eagle2Error,
    FLAG_NO_RERANK,
    FLAG_RANK_BY_CONFIDENCE,
    FLAG_STATIC_TREE,
    RoundCfg,
    eagle2_accept,
    eagle2_accept_noalloc,
    eagle2_accept_noalloc_scratch_bytes,
    eagle2_commit_kv,
    eagle2_commit_kv_fp8,
    eagle2_commit_round,
    eagle2_expand,
    eagle2_kernel_timing_enable,
    eagle2_kernel_timing_read,
    eagle2_rerank,
    eagle2_tree_attn,
    eagle2_tree_attn_fp8kv,
    eagle2_version,
    eagle2_workspace_bytes,
    lib_path,
    load_library,
)
from .round import DraftModel, DraftRound  # noqa: F401
