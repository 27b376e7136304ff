"""MI355X-native MuLoCo optimizer hot path: thin Python binding over libmuloco.so.

Every step of the method runs in the HIP kernels of the C-ABI library; this package
only marshals arguments (device pointers, shapes, the current stream).  There is no
CPU or PyTorch fallback: if the library is missing, calls raise.
"""
from .binding import (  # noqa: F401
    MLC_F32, MLC_BF16, MulocoError, InnerGroup, OuterGroup, MuonHParams, OuterHParams,
    library, library_path, strerror,
    newton_schulz, newton_schulz_workspace_bytes, newton_schulz_workspace_min_bytes,
    newton_schulz_static_scratch, STATIC_SCRATCH_BYTES,
    muloco_inner_step, muloco_inner_workspace_bytes, muloco_inner_workspace_min_bytes,
    muloco_outer_step, muloco_quantize_delta, muloco_adamw_step, AdamWHParams,
    muloco_topk_outer_step, muloco_topk_workspace_bytes,
    muloco_timing_enable, muloco_timing_read, KERNEL_FAMILIES,
)
