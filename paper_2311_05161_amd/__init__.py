"""MI355X (gfx950) W4A8 linear layer of arXiv 2311.05161: dINT4 weights x INT8 activations.

The product is the C-ABI shared library ``libw4a8.so`` (declared in ``include/w4a8.h``, built
from ``csrc/`` by ``python -m paper_2311_05161_amd.build``); this package is its thin binding.
"""
from .binding import (  # noqa: F401
    BF16, EXPORTS, F16, F32, LAYOUT_CANONICAL, LAYOUT_TILED, LIB_PATH, W4A8Error,
    gemm_workspace_bytes, load_library, pack_dint4, quantize_act_int8, quantize_weight_dint4,
    status_string, unpack_dint4, w4a8_gemm, w4a8_gemm_static, w4a8_linear,
    dint4_weight_sums, quantize_act_int8_asym, w4a8_gemm_asym, w4a8_gemm_batched,
    quantize_value_dint4,
    FMT_DINT3, FMT_DINT4, FMT_INT4, quantize_weight_format, w4a8_gemm_format, pack_dint3, unpack_dint3, pack_format, unpack_format,
    dint_error_terms,
    FMT_DINT4_C4, FMT_DINT4_C8, expand_special_value, w4a8_gemm_special,
    aqas_channel_absmax, aqas_scale, aqas_search, dint4_clipped_params, aqas_clip_search,
)
