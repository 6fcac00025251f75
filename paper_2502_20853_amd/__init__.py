"""MI355X (gfx950) implementation of the MXFP4 quantized linear layer of TetraJet
(arxiv 2502.20853): HIP kernels behind a C ABI (include/mxfp4.h) and a thin
binding with the same names."""
from .binding import (  # noqa: F401
    DTYPE_BF16, DTYPE_F32, GEMM_BWD_DW, GEMM_BWD_DX, GEMM_FWD, ROUND_RTN, ROUND_SR,
    SCALE_FLOOR, SCALE_TRUNCFREE, MxError,
    mx_dequantize, mx_ema_weight_quant, mx_linear_bwd_dw, mx_linear_bwd_dx, mx_linear_fwd, mx_linear_fwd_bias,
    mx_linear_workspace_bytes, mx_quantize, mx_quantize_transposed, mx_quantize_transposed_batch, mx_version,
    OscillationState, mx_oscillation_accumulate, mx_ramping_factor,
    RateOfChangeState, mx_quant_confidence, mx_rate_of_change_step,
    RampingAdamwState, mx_ramping_adamw_step,
    CALIBRATION_MFMA_OPERAND_BYTES, NOALLOC_MAX_WORKSPACE_BYTES, mx_calibration_copy, mx_calibration_mfma,
    mx_linear_bwd_dw_noalloc, mx_quantize_e3m0, mx_dequantize_e3m0, mx_linear_fwd_gelu_quant,
)
from .layer import MxLinearStep  # noqa: F401
from .module import MxLinear  # noqa: F401
from .optim import QRampingAdamW  # noqa: F401
