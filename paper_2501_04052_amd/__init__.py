"""MI355X-native RaZeR (arxiv 2501.04052) weight-only / weight-activation linear layer.

The product is the HIP shared library behind ``include/razer.h``; this package
is its thin Python binding (argument marshalling only) plus seeded synthetic
inputs.  There is no CPU fallback: without the built library every call raises.
"""
from .binding import (  # noqa: F401
    ACT, BF16, F32, WEIGHT, WEIGHT_F16, RazerError, RazerTensor, lib_path, load_library, razer_dequant,
    razer_linear, razer_linear_grouped, razer_linear_static, razer_prepack, razer_quantize, PreparedCall, prepare_linear, prepare_linear_grouped, razer_status_string, razer_workspace_bytes,
    razer_workspace_bytes_grouped, razer_probe_dispatch_events, razer_probe_stream_read, razer_probe_mfma_bf16, razer_probe_mfma_fp4,
    razer_tune_force, razer_tune_lookup, razer_tune_table_size,
)
