"""AttentionPredictor decode hot path for AMD MI355X: HIP kernels behind a C ABI + this thin binding."""
from .binding import AP_OK, AP_ERR_ARG, AP_ERR_ALIGN, AP_ERR_RANGE, AP_ERR_HIP, AP_ERR_UNSUPPORTED, AP_ERR_STATE  # noqa: F401
from .binding import AP_BF16, AP_F32, AP_FLAG_PREDICTOR_FP32, AP_PRED_ADVANCE, AP_PRED_HOLD, AP_PRED_REBASE, AP_PRED_SKIP, AP_STEP_REUSE_SELECTION, ApError, Context, EXPORTS, load_library, stream_copy, stream_read  # noqa: F401
