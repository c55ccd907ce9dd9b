// Optional per-kernel timing with HIP events, for roofline reports.  Off by default; when off a
// launch costs one predictable branch.  When on, every kernel launch of the library is
// bracketed by two events recorded on the launch stream; rnn_profile_read synchronises on
// them and returns per-kernel launch counts and total milliseconds.
#pragma once
#include <hip/hip_runtime.h>

namespace rnn {

enum KernelId : int {
    K_GEMM_LOGITS = 0, K_GEMM_DV, K_GEMM_G, K_GEMM_DWH, K_GEMM_U, K_GEMM_DWX, K_GEMM_DH0,
    K_SPLITK_REDUCE, K_TRANSPOSE,
    K_REC_FWD, K_REC_BWD, K_CE_ROW_STATS, K_MSE_ROW_LOSS, K_LOSS_REDUCE, K_DZ,
    K_COLSUM_PARTIAL, K_COLSUM_FINISH, K_DWX_TOKENS, K_CHECK_TOKENS,
    K_SKINNY_LOGITS, K_SKINNY_BACK, K_SKINNY_REVERSE, K_MISC, K_TRAIN_STREAM, K_WINDOW, K_GN_METRIC, K_SPLIT_BF16,
    K_MLP_FWD, K_MLP_CE, K_MLP_BWD, K_MLP_UPDATE,
    K_COUNT
};

extern int g_profile_on;
void profile_before(int kid, hipStream_t s);
void profile_after(int kid, hipStream_t s);

struct ProfileScope {
    int kid;
    hipStream_t s;
    ProfileScope(int k, hipStream_t st) : kid(k), s(st) { if (g_profile_on) profile_before(kid, s); }
    ~ProfileScope() { if (g_profile_on) profile_after(kid, s); }
};

}  // namespace rnn
