"""MI355X-native Elman-RNN training path (forward recurrence, output layer + loss, BPTT).

Thin ctypes binding over the C ABI in include/rnn.h; every step of the path runs in the HIP
kernels of librnn_mi355x.so.  There is no CPU fallback: loading fails loudly if the library
is missing.
"""
from .binding import (  # noqa: F401
    ACT_SIGMOID, ACT_TANH, FLAG_ACCUMULATE, FLAG_BF16X3_OUTPUT, FLAG_COOPERATIVE, FLAG_BPTT_RECOMPUTE, FLAG_REFERENCE_KERNELS, FLAG_SYNC,
    INPUT_DENSE, INPUT_TOKENS, LOSS_LINEAR_MSE, LOSS_SOFTMAX_CE, Dims, Grads, Params, RnnError,
    exported_symbols, lib, lib_path, rnn_bptt, rnn_check_tokens, rnn_forward, rnn_loss, rnn_measure_ceilings,
    rnn_profile_begin, rnn_profile_end, rnn_recurrence_variant, rnn_recurrence_workgroups, rnn_strerror,
    rnn_workspace_bytes, rnn_workspace_init, rnn_workspace_status, rnn_set_wait_limit,
    rnn_train_stream, rnn_train_stream_status, rnn_train_stream_workspace_bytes,
    rnn_window, rnn_window_one_launch, rnn_window_workspace_bytes, rnn_window_workspace_init, rnn_window_static, WINDOW_STATIC_BYTES,
    GN_METRIC_IDENTITY, GN_METRIC_LOSS, rnn_gauss_newton_vec, rnn_gauss_newton_workspace_bytes,
    MlpDims, MlpParams, mlp_params, rnn_mlp_train, rnn_mlp_workspace_bytes,
)
