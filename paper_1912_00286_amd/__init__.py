"""MI355X-native mixed-precision stacked-LSTM training step.

The work is done by hand-written gfx950 HIP kernels behind a C ABI
(include/lstm_mi355.h).  This package is the thin ctypes binding with the same
entry-point names plus buffer plumbing on torch device tensors.  There is no
CPU fallback: importing `binding` fails loudly when the library is missing.
"""
from .binding import (  # noqa: F401
    LstmConfig, OptimizerConfig, TrainingStep, load_library, library_path,
    lstm_abi_version, lstm_last_error, lstm_param_count, lstm_param_offset, lstm_workspace_bytes,
    lstm_forward, lstm_backward, lstm_forward_static_scratch, STATIC_SCRATCH_BYTES, lstm_cast_params, grad_average, grad_average_masked, master_update, lr_schedule,
    DTYPE_FP32, DTYPE_FP16, DTYPE_BF16, HEAD_STEP_BCE, HEAD_LAST_BCE, HEAD_STEP_MSE, HEAD_FC_HINGE, OPT_SGD_MOMENTUM, OPT_ADAM,
    LstmError, lstm_timing_enable, lstm_timing_read, KERNEL_CLASSES, lstm_debug_gemm, lstm_debug_gemm_stream, lstm_debug_pack_blocked, lstm_debug_mfma_rate, lstm_debug_plan_regions,
)
