// Event-based per-kernel timing (see prof.hpp).  Host-only state, not thread-safe: meant for
// a single benchmarking thread.
#include "prof.hpp"

#include <vector>

#include "../../include/rnn.h"

namespace rnn {

int g_profile_on = 0;

namespace {
struct Rec { int kid; hipEvent_t a, b; };
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;
size_t g_cap = 0;
hipEvent_t g_pending = nullptr;

hipEvent_t take_event() {
    if (!g_pool.empty()) { hipEvent_t e = g_pool.back(); g_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
const char* const kNames[K_COUNT] = {
    "gemm_logits", "gemm_dV", "gemm_G", "gemm_dWh", "gemm_U", "gemm_dWx", "gemm_dh0",
    "splitk_reduce", "transpose",
    "rec_fwd", "rec_bwd", "ce_row_stats", "mse_row_loss", "loss_reduce", "dz",
    "colsum_partial", "colsum_finish", "dwx_tokens", "check_tokens",
    "skinny_logits", "skinny_back", "skinny_reverse", "misc", "train_stream", "window", "gn_metric", "split_bf16",
    "mlp_fwd", "mlp_ce", "mlp_bwd_data", "mlp_update"};
}  // namespace

void profile_before(int, hipStream_t s) {
    if (g_recs.size() >= g_cap) { g_pending = nullptr; return; }
    g_pending = take_event();
    if (g_pending) (void)hipEventRecord(g_pending, s);
}

void profile_after(int kid, hipStream_t s) {
    if (!g_pending) return;
    hipEvent_t b = take_event();
    if (!b) { g_pool.push_back(g_pending); g_pending = nullptr; return; }
    (void)hipEventRecord(b, s);
    g_recs.push_back({kid, g_pending, b});
    g_pending = nullptr;
}

}  // namespace rnn

extern "C" {

int rnn_profile_begin(int max_launches) {
    using namespace rnn;
    if (max_launches <= 0) return RNN_EINVAL;
    for (auto& r : g_recs) { g_pool.push_back(r.a); g_pool.push_back(r.b); }
    g_recs.clear();
    g_cap = (size_t)max_launches;
    g_profile_on = 1;
    return RNN_OK;
}

int rnn_profile_end(int n_kernels, int64_t* counts, double* total_ms) {
    using namespace rnn;
    g_profile_on = 0;
    if (n_kernels < K_COUNT || !counts || !total_ms) return RNN_EINVAL;
    for (int k = 0; k < n_kernels; ++k) { counts[k] = 0; total_ms[k] = 0.0; }
    int rc = RNN_OK;
    for (auto& r : g_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) {
            rc = RNN_EHIP;
        } else {
            counts[r.kid] += 1;
            total_ms[r.kid] += (double)ms;
        }
        g_pool.push_back(r.a);
        g_pool.push_back(r.b);
    }
    g_recs.clear();
    return rc;
}

int rnn_profile_kernel_count(void) { return rnn::K_COUNT; }

const char* rnn_profile_kernel_name(int kid) {
    return (kid >= 0 && kid < rnn::K_COUNT) ? rnn::kNames[kid] : "invalid";
}

}  // extern "C"
