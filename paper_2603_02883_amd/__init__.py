"""MI355X-native FB4 online quantizer: C-ABI library (libfb4.so) and its Python binding."""
from .binding import (DTYPE_BF16, DTYPE_F32, ERR_ALLOC, ERR_HIP, ERR_INVALID_ARG, ERR_UNSUPPORTED,  # noqa: F401
                      FLAG_TWO_STAGE, OK, SEL_LUT, SEL_SSE, Fb4Error, Luts, fb4_build_luts,
                      fb4_attention_scores, fb4_build_luts_host, fb4_decompose, fb4_dequantize, fb4_free_luts, fb4_opts,
                      fb4_gelu_quantize, fb4_gelu_table_host, fb4_layernorm_quantize, fb4_probe_mfma_rate, fb4_quantize, fb4_quantize_decompose, fb4_quantize_seda, fb4_repack_mxfp8, fb4_seda_assign, fb4_seda_main_anchor, fb4_seda_main_anchor_3d, fb4_seda_profile, fb4_select_salient_tokens, opts, strerror, version, workspace_bytes)
