"""SQuant weight-quantization solver for MI355X (gfx950): HIP kernels behind a C ABI."""
from .binding import (OUT_INT8, OUT_INT4, OUT_F32, OUT_BF16, OUTPUTS, squant_quantize_ex,  # noqa: F401
                      squant_quantize_batched_ex, squant_output_bytes, squant_activation_ranges,
                      squant_quantize_network, MODE_E, MODE_EK, MODE_EKC, MODE_EC, MODES, BatchPlan, SQuantError,  # noqa: F401
                      squant_batched_workspace_bytes, squant_max_channel_elems, squant_quantize,
                      squant_quantize_batched, squant_status_string, squant_version)
