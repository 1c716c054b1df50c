"""MI355X (gfx950) hot path of Early-exiting Speculative Decoding.

Every step of a decoding round runs in the HIP library `libeesd.so` (C ABI in
include/eesd.h); this package is a thin ctypes binding with the same names.
PyTorch is used by callers only to own device memory and streams.
"""
from .binding import (  # noqa: F401
    EESD, EesdError, Stats, calibration_copy, host_cali_decide, host_cali_update, host_draw_k, host_layout_offset, host_ts_update, host_uniform, lib, lib_path, op_accept, op_accept_logits, op_gemm, op_gemm_noalloc, op_softmax_sample, pack_calibration, pack_weight, pack_weights, set_tunable,
    DTYPE_F32, DTYPE_BF16, TS_BETA, TS_FIXED, TS_SCHEDULE, TS_CALI, WEIGHTS_ROW_MAJOR, WEIGHTS_TILED, PACK_PLAIN, PACK_GATE_UP, PACK_QKV, GEMM_AUTO, GEMM_VALU, GEMM_MFMA,
)
