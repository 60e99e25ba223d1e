"""MI355X-native implementation of MEDA's prefill-time KV-cache compression pass.

The work is done by libmeda.so (hand-written HIP for gfx950, C ABI declared in include/meda.h);
this package is the thin Python binding with the same names.  There is no CPU fallback: if the
library has not been built, every call raises.
"""
from ._lib import (MedaError, MedaParams, MedaDecodeParams, Decoder, make_decode_params, meda_decode_attention,
                   meda_decode_attention_noalloc, DECODE_NOALLOC_MAX_BYTES, meda_peak_stream_read, meda_peak_mfma_bf16, meda_peak_mfma_valu,
                   meda_decode_workspace_bytes, meda_quantize_fp8, meda_dequantize_fp8, Compressor, CompressedCache, load_library, library_path,
                   make_params, meda_compress, meda_workspace_bytes, meda_workspace_region,
                   meda_profile_enable, meda_profile_read, meda_phase_name, meda_status_string,
                   EXPORTED_SYMBOLS, REGIONS, N_PHASES, FLAG_UNIFORM_BUDGET, FLAG_NO_MERGE, FLAG_FULL_PROMPT)

__all__ = ["MedaError", "MedaParams", "MedaDecodeParams", "Decoder", "make_decode_params", "meda_decode_attention",
           "meda_decode_attention_noalloc", "DECODE_NOALLOC_MAX_BYTES", "meda_peak_stream_read", "meda_peak_mfma_bf16", "meda_peak_mfma_valu",
           "meda_decode_workspace_bytes", "meda_quantize_fp8", "meda_dequantize_fp8", "Compressor", "CompressedCache", "load_library", "library_path",
           "make_params", "meda_compress", "meda_workspace_bytes", "meda_workspace_region",
           "meda_profile_enable", "meda_profile_read", "meda_phase_name", "meda_status_string",
           "EXPORTED_SYMBOLS", "REGIONS", "N_PHASES", "FLAG_UNIFORM_BUDGET", "FLAG_NO_MERGE", "FLAG_FULL_PROMPT"]
