"""MI355X-native XFP fused decode (dequant-GEMV) library: Python binding.

The arithmetic lives in libxfp.so (hand-written HIP for gfx950, C ABI declared
in include/xfp.h).  This package only marshals arguments; PyTorch is used for
device memory and streams.  There is no CPU fallback: if the library cannot
be loaded, importing the binding's entry points raises.
"""
from .binding import (  # noqa: F401
    XFP_BF16, XFP_F16, XFP_ROUTE_BATCH, XFP_ROUTE_GENERAL, XFP_ROUTE_SPLIT_K, XFP_ROUTE_STREAM, XFP_ROUTE_TILE, XFP_ROUTE_WIDE, XFP_KERNEL_AUTO, XFP_KERNEL_STREAM, XFP_KERNEL_TILE, XFP_F32, XFP_X_BF16, XFP_MODE_V2, XFP_MODE_V2A, DeviceWeights, XfpError, library_path, load_library,
    upload, xfp_check_contents, xfp_convert_bf16_to_f16, xfp_dequant_bulk, xfp_gemv, xfp_gemv_noalloc, xfp_gemv_moe, xfp_gemv_moe_combine, xfp_gemv_moe_silu_mul, xfp_init, xfp_probe_copy, xfp_probe_read, xfp_repack_word10, xfp_repack_words, xfp_route, xfp_select_kernel, xfp_strerror,
    xfp_unpack_indices, xfp_version,
)
from .format import bytes_per_weight, load_xfp, save_xfp  # noqa: F401
