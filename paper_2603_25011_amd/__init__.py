"""MI355X-native sparse-lexical (SPLADE-style) LM head: C-ABI HIP library + thin Python binding."""
from .binding import (  # noqa: F401
    LSR_BF16, LSR_F32, LsrError, library_path, load_library, lsr_head_backward, lsr_head_backward_ex, lsr_head_backward_ex_workspace_bytes,
    lsr_head_backward_profiled, lsr_head_forward_static, lsr_copy_probe, lsr_gather_probe, LSR_STATIC_SCRATCH_BYTES,
    lsr_head_forward, lsr_head_forward_profiled, lsr_head_plan, lsr_head_workspace_bytes, lsr_mfma_peak_probe, lsr_status_string,
)
