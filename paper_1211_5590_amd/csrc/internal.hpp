// Host-side declarations of the kernel launchers behind the C ABI (one translation unit each).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace rnn {

// ---------------------------------------------------------------------------------------
// fp32 MFMA GEMM:  C[M,N] = (beta ? C : 0) + op(A) op(B) + bias_n[col]
//   a_t == false : A stored [M,K] (lda >= K)      a_t == true : A stored [K,M] (lda >= M)
//   b_t == false : B stored [K,N] (ldb >= N)      b_t == true : B stored [N,K] (ldb >= K)
// splitk_ws must hold gemm_splitk_floats(M,N,K) floats (0 => not needed).
struct GemmArgs {
    const float* A;
    const float* B;
    float* C;
    int M, N, K;
    int lda, ldb, ldc;
    bool a_t, b_t;
    const float* bias_n;  // nullable, length N
    int beta;             // 0 overwrite, 1 accumulate
    float* splitk_ws;     // nullable when gemm_splitk_floats == 0
    int prof_id;          // kernel id under which the profiler books this product (prof.hpp)
    // nullable: [M][gemm_stat_parts(N)][2] receives, per row and per 64-column part of the final
    // result, (max, sum of exp relative to that max); written only when gemm_fuses_stats(M,N,K)
    float* row_stats;
};
size_t gemm_splitk_floats(int M, int N, int K);
int gemm_stat_parts(int N);
bool gemm_fuses_stats(int M, int N, int K);
hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);

// C[m,n] = (beta ? C : 0) + sum over splits of part[s][m][n] + bias_n[n], fixed order
hipError_t launch_splitk_reduce(const float* part, float* C, const float* bias_n, int M, int N, int ldc,
                                int splits, int beta, hipStream_t s);

// ---------------------------------------------------------------------------------------
// bf16 hi/lo split products (gemm_bf16x3.hip): C[M,N] = A[M,K] B[N,K]^T + bias_n, float32 result,
// operands K-contiguous in "split form" (per row and slab of 32 k: 32 hi values, then 32 lo values;
// K padded with zeros to bf3_pad(K)) -- the form launch_split_bf16 writes; 4 bytes per padded element.
struct Bf3Args {
    const uint16_t* A;    // [M][2 lda]
    const uint16_t* B;    // [N][2 ldb]
    float* C;
    int M, N, K;
    int lda, ldb, ldc;
    const float* bias_n;  // nullable
    int beta;
    float* splitk_ws;     // bf3_splitk_floats(M,N,K) floats
    int prof_id;
    float* row_stats;     // [M][bf3_stat_parts(M,N,K)][2]; written only when bf3_fuses_stats(M,N,K)
};
int bf3_stat_parts(int M, int N, int K);
int bf3_pad(int k);
size_t bf3_splitk_floats(int M, int N, int K);
bool bf3_fuses_stats(int M, int N, int K);
// float32 [R,C] (leading dimension ld) -> split form, as it is [R][2 bf3_pad(C)] and/or transposed
// [C][2 bf3_pad(R)] (either may be NULL)
hipError_t launch_split_bf16(const float* src, int R, int C, int ld, uint16_t* rowmajor, uint16_t* transposed,
                             hipStream_t s);
hipError_t launch_gemm_bf16x3(const Bf3Args& g, hipStream_t s);
// logits -> d loss / d z directly in split form (both orientations) + per-chunk column sums for dc
hipError_t launch_dz_split(const float* Z, const float* lse, const int32_t* y, const float* Y, float* part, int N,
                           int O, int loss_kind, uint16_t* rowmajor, uint16_t* transposed, int* chunks_out,
                           hipStream_t s);

// ---------------------------------------------------------------------------------------
// Recurrence (forward and reverse-time loops)
struct RecFwdArgs {
    const float* Wh;   // [H,H]
    const float* Wx;   // token input: [NV,H]; unused for dense input
    const float* b;    // [H]
    const int32_t* x;  // token ids [T,B] or NULL
    const float* U;    // dense input: precomputed Wx x_t + b, [T,B,H]; NULL for token input
    const float* h0;   // nullable [B,H]
    float* hist;       // [T+1,B,H], or a 2-slot ring [2,B,H] when ring != 0
    float* h_last;     // nullable [B,H]
    int H, T, B, act, ring;
};
struct RecBwdArgs {
    const float* Wh;      // [H,H]
    const float* WhT;     // [H,H] transposed copy (reference and step-wise kernels)
    const float* G;       // [T,B,H] output-layer contribution to d loss / d h_t
    const float* h_all;   // [T+1,B,H]
    const float* dh_last; // nullable [B,H]
    float* Delta;         // [T,B,H] receives d loss / d a_t
    float* dh0;           // nullable [B,H]
    int H, T, B, act;
    float* splitk_ws;     // split-K scratch for the dh0 product (stepwise path)
};
// Resident-weight persistent loops (recurrence.hip).  One struct serves both directions.
struct RecResArgs {
    const float* Wh;
    int H, T, B, act;
    int P, R, L, ldw, w_floats;  // filled from the plan by the launcher
    int nq4, hpad;               // float4 per lane of a row, zero-padded row/vector length
    int32_t* flags;              // exchange boxes in the workspace (P > 1): [2][B][H] 64-bit words, 8-byte aligned
    int32_t* status;             // device status word: set to 1 when a bounded wait expires
    int spin_limit;              // <= 0: default
    int xcd_pack;                // set by the launcher: workgroup p of a sequence is blockIdx.x / 8 (see the kernel)
    int poll_sleep;              // role-split loop: pauses of 64 clocks between a workgroup's own stores and its first poll
    // forward
    const float* Wx; const float* b; const int32_t* x; const float* U; const float* h0;
    float* hist; float* h_last; int ring;
    // reverse
    const float* G; const float* h_all; const float* dh_last; float* Delta; float* dh0;
    // fused weight gradients of a short single sequence (reverse, P == 1, B == 1)
    int fuse_post; float* dWh; float* db; float* dWx; int beta;
    // Short single sequence (fuse_post): G is produced by the other workgroups of the launch
    // (gpart non-NULL marks this mode; otherwise G is given)
    const float* gpart; int gstrips; float* Gw;
    const unsigned long long* g_box; uint32_t epoch;   // G arrives as tagged words [T][H]; the fused
                                                       // launch fills epoch from the tag word
};
struct RecResPlan { int P, R, L, ldw, w_floats, nq4, hpad; size_t smem; };
// strips: column strips of the short-sequence output layer (fuse_post only, else 0)
bool rec_resident_plan(int H, int B, int T, bool bwd, bool fuse_post, int strips, RecResPlan* out);
hipError_t launch_rec_resident(RecResArgs a, const RecResPlan& pl, bool bwd, hipStream_t s);
// The same loop for sequences whose matrix needs several compute units, with the wavefronts of a
// workgroup split into computing and polling ones (recurrence_grid.hip).  Serves what the resident
// plan gives more than one workgroup, as long as the slice fits the registers of four wavefronts.
struct RecGridPlan { int P, R, OPW, hpad; size_t smem; };
bool rec_grid_plan(int H, int B, RecGridPlan* out);
hipError_t launch_rec_grid(RecResArgs a, const RecGridPlan& pl, bool bwd, hipStream_t s);
struct SkinnyArgs;
// reverse loop with fused weight gradients (workgroup 0) and the output layer's backward strips
// (one workgroup per strip) in one launch; a must have fuse_post set
hipError_t launch_rec_bwd_with_strips(RecResArgs a, const RecResPlan& pl, const SkinnyArgs& k, hipStream_t s);

// Batched recurrence run as one fused GEMM launch per time step (recurrence_step.hip); serves
// the shapes the resident-weight kernels do not cover (batch > 4).
hipError_t run_rec_fwd_stepwise(const RecFwdArgs& a, hipStream_t s);
hipError_t run_rec_bwd_stepwise(const RecBwdArgs& a, hipStream_t s);

// Persistent batched loop with register-resident weights (recurrence_mfma.hip), H <= 256, B > 4.
struct RecMfmaArgs {
    const float* Wh;
    int H, T, B, act;
    // forward
    const float* U;       // [T,B,H] input term including the bias (always materialised)
    const float* h0;      // nullable
    float* hist;          // [T+1,B,H] or 2-slot ring
    float* h_last;        // nullable
    int ring;
    // reverse
    const float* G; const float* h_all; const float* dh_last; float* Delta; float* dh0;
};
bool rec_batch_mfma_supported(int H, int B);
hipError_t launch_gather_input(const int32_t* x, const float* Wx, const float* b, float* U, int N,
                               int H, hipStream_t s);
hipError_t launch_rec_batch_mfma(const RecMfmaArgs& a, bool bwd, hipStream_t s);

// Persistent batched loop for 256 < H <= 1024 (recurrence_xcd.hip): one batch group per XCD, the state
// handed over through that XCD's L2.  Needs the full history (no ring) and the input term U.
struct RecXcdArgs {
    const float* Wh;
    int H, T, B, act;
    // forward
    const float* U;       // [T,B,H] input term including the bias
    const float* h0;      // nullable
    float* hist;          // [T+1,B,H]
    float* h_last;        // nullable
    // reverse
    const float* G; const float* h_all; const float* dh_last; float* Delta; float* dh0;
    int32_t* counters;    // 8 words of workspace (cleared by the launcher)
    int32_t* status;      // device status word: set to 1 when a bounded wait expires
    int spin_limit;       // <= 0: default
    int first_look_pause; // pauses of 64 clocks between the own tile's store and the first look (<= 0: default)
};
bool rec_xcd_supported(int H, int B, int T);                       // shape only (host)
bool rec_xcd_ready(int H, int act, bool bwd);               // and the current device can hold the grid at once
hipError_t launch_rec_xcd(const RecXcdArgs& a, bool bwd, hipStream_t s);

hipError_t launch_zero_words(int32_t* p, int n, hipStream_t s);
// polls a bounded wait between workgroups makes before it gives up (host state, rnn_set_wait_limit)
int wait_limit();
hipError_t launch_transpose(const float* src, float* dst, int rows, int cols, hipStream_t s);
hipError_t launch_rec_fwd_reference(const RecFwdArgs& a, hipStream_t s);
hipError_t launch_rec_bwd_reference(const RecBwdArgs& a, hipStream_t s);

// ---------------------------------------------------------------------------------------
// Output layer element-wise / row-wise kernels
hipError_t launch_ce_row_stats(const float* Z, const int32_t* y, float* lse, float* rowloss,
                               int N, int O, hipStream_t s);
// the same from the statistics the logits product left: stats [N][parts][2]
hipError_t launch_ce_merge_stats(const float* stats, int parts, const float* Z, const int32_t* y,
                                 float* lse, float* rowloss, int N, int O, hipStream_t s);
// squared-error partial sums over the flat [N*O] arrays: *n_partial (<= N) floats in `partial`
hipError_t launch_mse_partial(const float* Z, const float* Y, float* partial, int N, int O,
                              int* n_partial, hipStream_t s);
hipError_t launch_loss_reduce(const float* rowloss, int N, float scale, float* loss, hipStream_t s);
// Z -> dZ in place, plus per-row-chunk column sums into part[chunks][O]
int colsum_chunks(int N);
hipError_t launch_dz(float* Z, const float* lse, const int32_t* y, const float* Y, float* part,
                     int N, int O, int loss_kind, hipStream_t s);
hipError_t launch_colsum_partial(const float* M, float* part, int N, int C, hipStream_t s);
hipError_t launch_colsum_finish(const float* part, float* out, int chunks, int C, int beta,
                                hipStream_t s);

// ---------------------------------------------------------------------------------------
// Output layer of a short single sequence (skinny.hip): column-strip kernels, N <= 32 rows
struct SkinnyArgs {
    const float* Hs;      // [N,H] rows h_t
    const float* V;       // [H,O]
    const float* c;       // [O]
    const int32_t* y;     // [N]
    float* Z;             // [N,O] logits (workspace)
    unsigned long long* stat_box;  // tagged words: [N][strips][2] strip max / sum exp, then [N] target logits
    unsigned long long* g_box;     // tagged words: [N][H] G, from the backward strips to the reverse loop
    uint32_t epoch;       // tag of this launch's words (never 0): filled in by the kernel from *epoch_word
    uint32_t* epoch_word; // device word: tag of the last launch on these boxes (see next_tag)
    int spin_limit;       // polls a bounded wait makes before it gives up
    int32_t* status;      // device status word: set to 1 when a bounded wait expires
    float* loss;          // device scalar written by the merging workgroup (logits kernel)
    float* lse;           // [N]
    float* dV; float* dc; // gradients
    float* gpart;         // [strips][N][H]
    float* dWx_zero;      // token-gradient matrix to zero fill, or NULL
    const int32_t* xids;  // [N] input token ids (rows of dWx the reverse loop's workgroup writes itself)
    float* vy;            // [N][H] column y_n of V per row (workspace)
    int H, O, N, NV, beta;
};
int skinny_strips(int O);
bool skinny_supported(int N, int H, int O);
size_t skinny_stat_box_bytes(int N, int O);
hipError_t launch_skinny_logits(const SkinnyArgs& a, hipStream_t s);   // logits, statistics and loss

// ---------------------------------------------------------------------------------------
// Small kernels of the Gauss-Newton-vector product (gauss_newton.hip)
hipError_t launch_reverse_rows(const float* src, float* dst, int T, int row, hipStream_t s);   // dst[t] = src[T-1-t]
hipError_t launch_gather_add(const int32_t* x, const float* M, float* C, int N, int H, hipStream_t s);
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s);
hipError_t launch_scale(float* p, size_t n, float alpha, hipStream_t s);
// RZ_n <- (p * RZ_n - p (p . RZ_n)) * scale, p = softmax(Z_n)
hipError_t launch_gn_softmax_metric(const float* Z, float* RZ, int N, int O, float scale, hipStream_t s);

// ---------------------------------------------------------------------------------------
// Token-keyed gradient of the input matrix and id validation
// scratch (>= scratch_floats floats) and slot_table (>= dwx_table_ints(N, NV) ints) enable the grouped form
size_t dwx_table_ints(int N, int NV);
hipError_t launch_dwx_tokens(const int32_t* x, const float* Delta, float* dWx, int N, int NV,
                             int H, int beta, float* scratch, size_t scratch_floats,
                             int32_t* seen_flags, hipStream_t s);
hipError_t launch_check_tokens(const int32_t* ids, int64_t n, int32_t limit, int32_t* bad,
                               hipStream_t s);

}  // namespace rnn
