"""MI355X (gfx950) ReLU linear attention for long video token sequences.

Thin Python binding over libsvlinattn.so (hand-written HIP kernels behind a C
ABI, declared in include/sv_linattn.h, include/sv_tconv.h and include/sv_measure.h).  PyTorch is used by callers for device
memory and streams only; every step of the computation runs in the library.
"""
from .binding import (  # noqa: F401
    SV_BF16, SV_F32, SvError, TensorDesc, desc_of, library_path, load_library,
    sv_block_linattn_lookahead, sv_block_linattn_step, sv_linattn_apply, sv_linattn_state,
    sv_linattn_workspace_bytes, sv_status_string, sv_version, EXPORTS,
    sv_linattn_state_rope, sv_linattn_apply_rope, sv_block_linattn_step_rope, sv_block_linattn_lookahead_rope, sv_linattn_workspace_init,
    Rope3D, sv_linattn_state_rope3d, sv_linattn_apply_rope3d, sv_block_linattn_step_rope3d,
    sv_block_linattn_lookahead_rope3d, sv_tconv_block_step, sv_stream_read, sv_stream_copy,
    sv_linattn_workspace_status, sv_linattn_workspace_status_offset, sv_linattn_set_wait_limit, sv_block_linattn_step_static, sv_measure_apply_variant, sv_measure_assume_dies,
    sv_mfma_stream, sv_measure_tconv_variant,
)
