"""MI355X-native round/log/replay hot path of optimistic verifiable training.

Thin Python access to the C-ABI library (include/vt.h).  Every step of the path runs in the
HIP kernels of libvt_hip.so; this package only marshals PyTorch device pointers and streams.
There is no CPU fallback: calling any entry point without the built library raises.
"""
from .binding import (  # noqa: F401
    VT_OP_GEMM_ROUND_LOG, VT_OP_GEMM_ROUND_LOG_BR, VT_OP_ROUND_LOG, VT_OP_ROUND_REPLAY, VT_OP_THRESHOLD_STATS,
    VT_CONV_FORWARD, VT_CONV_WEIGHT_GRAD, VT_CONV_DATA_GRAD, Conv2d, VT_OP_LAYER_ROUND_LOG, VT_LAYER_ADD, VT_LAYER_RELU,
    VT_LAYER_GELU_TANH, VT_LAYER_GELU_ERF, VT_LAYER_NORM, VT_LAYER_SOFTMAX, VT_LAYER_BATCHNORM,
    VT_LAYER_BATCHNORM_RELU, vt_layer_f64_round_log, vt_conv2d_f64_round_log, vt_conv2d_gemm_shape,
    VtError, VtLogAbandoned, check_count, VT_COUNT_ABANDONED, Log, alloc_log, alloc_dense_log, vt_round_replay_dense, alloc_workspace, library_path, load_library,
    vt_gemm_f64_round_log, vt_gemm_f64_round_log_nested, vt_gemm_plan, vt_gemm_tail_plan, vt_round_log, vt_round_log_static, VT_ROUND_LOG_STATIC_MAX_N, vt_round_replay, vt_set_kernel_events, vt_strerror, vt_thr_from_tau,
    vt_threshold_stats, vt_thr_layer_from_stats, VT_THR_LAYER_MAX, vt_workspace_bytes, vt_sha256_tree, vt_merkle_root, VT_OP_SHA256_TREE, VT_OP_MERKLE_ROOT, VT_OP_CONV_DGRAD_ROUND_LOG,
    VT_OP_CONV_DGRAD_ROUND_LOG_BR, VT_A_ROW_MAJOR, VT_A_TRANSPOSED, VT_A_IM2COL_T,
)
