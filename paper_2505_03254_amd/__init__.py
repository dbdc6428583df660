"""MI355X-native ternary pointwise-convolution path of PROM (arXiv 2505.03254).

The product is libprom.so (HIP kernels for gfx950 behind the C ABI of include/prom.h).
This package is the thin Python binding: it marshals torch tensors (used only as device
memory and for the current stream) into the C calls.  Nothing is computed in Python and
there is no fallback: if the library has not been built, every call raises.
"""
from .binding import (  # noqa: F401
    PromError, Requant, PwPlan, library_path, load_library,
    prom_packed_size, prom_pack_ternary, prom_unpack_ternary,
    prom_pw_conv, prom_pw_conv_ex, prom_pw_conv_addsub, prom_pw_accum_i32, prom_dw_conv, prom_gconv3x3, prom_gconv_pack, prom_gconv_frag_size,
    prom_block, prom_block_workspace_size, prom_block_is_fused, prom_block_can_fuse, prom_strerror,
    BLOCK_AUTO, BLOCK_FUSED, BLOCK_UNFUSED, BLOCK_DWPROJ, BLOCK_PLANES, prom_block_planes_applies, prom_dw_pw_conv, prom_dw_pw_can_fuse, prom_block_noalloc, prom_block_noalloc_max_workspace,
    prom_quantize_pw_absmean, prom_quantize_dw_absmax, prom_quantize_gconv_absmax,
    prom_quantize_activation_absmax, prom_pw_conv_dynq,
    prom_pw_plan_query, prom_pw_batchable, prom_pw_batch_class, prom_pw_conv_sequence, PwSequence, prom_dw_conv_sequence, DwSequence, prom_gconv3x3_sequence, GconvSequence, prom_copy_bytes,
    prom_stream_read, prom_stream_write, prom_mfma_i8_loop, prom_requant_check,
)
