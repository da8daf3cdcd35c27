"""MI355X-native Star Attention hot path: Python binding of the C-ABI library.

The names mirror include/star_attn.h.  This layer only marshals arguments
(pointers of torch tensors, the shape struct, the current HIP stream); every
step of the computation runs in the HIP kernels of libstarattn.so.  There is no
CPU or PyTorch fallback: if the library is missing or fails, an error is raised.
"""
from .binding import (  # noqa: F401
    BF16, F32, ANCHOR_FIRST, ANCHOR_PREVIOUS, ANCHOR_EXTERNAL, ANCHOR_PER_BLOCK, ANCHOR_ALL_BLOCKS,
    StarAttnError, StarShape, lib_path, load_library, phase1, phase1_anchor, phase1_rope,
    phase1_workspace_bytes, phase2, phase2_partial, phase2_rope, merge, rope, status_string,
    workspace_bytes, kernel_path, alloc_cache, alloc_workspace, phase2_plan, PlanInfo, phase2_static, STATIC_SCRATCH_BYTES,
)
