// Training step of a feed-forward classifier (the paper's neural-network training benchmark:
// 10-class classification of a 784-dimensional input by logistic regression, one hidden layer
// of 500 units or three of 1000, stochastic gradient descent on batches of 1, 10 or 60):
//
//     a_l = act(W_l a_{l-1} + b_l),  z = W_L a_{L-1} + b_L,  loss = mean(logsumexp(z) - z[y]),
//     W_l <- W_l - lr dloss/dW_l,  b_l <- b_l - lr dloss/db_l      after every batch.
//
// At these sizes a step moves a few megabytes of weights and computes almost nothing, so what it
// costs is launches and memory round trips.  A step is 2 L + 2 launches (L hidden layers: L + 1
// forward, the last of them with the loss in its epilogue when there are at most 16 classes, L
// backward, and ONE update of all layers, which also adds up the batch's loss), each
// built like the batched recurrence's step kernel to pay one round trip: a workgroup owns a
// 16 x 16 tile of the result, its 16 wavefronts split the contraction in slices of 64 and request
// their whole share of both operands at once, straight into the lane registers
// v_mfma_f32_16x16x4_f32 reads them from; the partial tiles meet in LDS once and the epilogue is
// fused (bias + activation forward, activation derivative backward).  The update kernel forms
// dW = dZ^T a in matrix-core tiles over the batch and applies it in place together with the
// bias update, so weight gradients never exist in memory; all layers share that launch, which
// is why every dZ_l is kept until the backward chain has ended.  No atomics: results are
// run-to-run identical.
#include "../../include/rnn.h"

#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <math.h>

namespace rnn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int MW = 16, MNT = MW * kWave, MKC = 64;

template <bool VEC>
__device__ __forceinline__ float4 ld_k4(const float* __restrict__ row, int k, int klim) {
    if (VEC && k + 3 < klim) return *reinterpret_cast<const float4*>(row + k);
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k + 0 < klim) t.x = row[k + 0];
    if (k + 1 < klim) t.y = row[k + 1];
    if (k + 2 < klim) t.z = row[k + 2];
    if (k + 3 < klim) t.w = row[k + 3];
    return t;
}

template <int ACT>
__device__ __forceinline__ float apply_act(float a) {
    return ACT == 0 ? sigmoidf_fast(a) : (ACT == 1 ? tanhf_fast(a) : a);
}

// C[M,N] = act(A[M,K] W[N,K]^T + bias[N]);  ACT 0 sigmoid, 1 tanh, 2 none.
// grid (ceil(N/16), ceil(M/16)), 1024 threads.  Lane (r = lane % 16, g = lane / 16) of a wavefront
// holds k = k0 + 16 s + 4 g + e of row r of A and of row r of W: the same permuted walk of K for both.
// CE (output layer with N <= 16, ACT 2): the tile holds whole rows of logits, so the epilogue goes on
// to the loss: C receives dZ = (softmax - onehot(y)) / M instead of the logits and losspart[blockIdx.y]
// the sum of the workgroup's row losses lse - z[y] (rows in order).
template <int ACT, bool VEC, bool CE = false>
__global__ __launch_bounds__(MNT) void mlp_fwd_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                      const float* __restrict__ bias, float* __restrict__ C,
                                                      int M, int N, int K, const int32_t* __restrict__ y,
                                                      float* __restrict__ losspart) {
    __shared__ float red[MW][4][kWave];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int g = lane / 16, nn = lane % 16;
    const int n0 = blockIdx.x * 16, m0 = blockIdx.y * 16;
    const int col = n0 + nn;
    const float bv = (wave < 4 && col < N) ? bias[col] : 0.f;   // requested before the product
    const bool a_ok = m0 + nn < M, b_ok = col < N;
    const float* arow = A + (size_t)min(m0 + nn, M - 1) * K;
    const float* brow = W + (size_t)min(col, N - 1) * K;
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    const int nchunks = (K + MKC - 1) / MKC;
    for (int kc = wave; kc < nchunks; kc += MW) {
        const int k0 = kc * MKC + 4 * g;
        float4 a[4], b[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            a[s] = a_ok ? ld_k4<VEC>(arow, k0 + 16 * s, K) : make_float4(0.f, 0.f, 0.f, 0.f);
            b[s] = b_ok ? ld_k4<VEC>(brow, k0 + 16 * s, K) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].x, b[s].x, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].y, b[s].y, acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].z, b[s].z, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].w, b[s].w, acc1, 0, 0, 0);
        }
    }
    // result layout of the 16x16 tile: lane -> column nn; register i -> row 4 g + i
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][i][lane] = acc0[i] + acc1[i];
    __syncthreads();
    if constexpr (!CE) {
        if (wave >= 4) return;
        const int row = m0 + 4 * g + wave;
        if (row >= M || col >= N) return;
        float v = bv;
#pragma unroll
        for (int w = 0; w < MW; ++w) v += red[w][wave][lane];
        C[(size_t)row * N + col] = apply_act<ACT>(v);
    } else {
        __shared__ float rowloss[16];
        if (wave < 4) {
            // the 16 lanes of a quarter-wave hold the 16 columns of row 4 g + wave
            const int row = m0 + 4 * g + wave;
            const bool ok = row < M && col < N;
            float v = bv;
#pragma unroll
            for (int w = 0; w < MW; ++w) v += red[w][wave][lane];
            const int yy = row < M ? y[row] : -1;
            const float m = max16(ok ? v : -INFINITY);
            const float se = sum16(ok ? __expf(v - m) : 0.f);
            const float lse = m + __logf(se);
            const float zy = sum16((ok && col == yy) ? v : 0.f);
            if (ok) C[(size_t)row * N + col] = (__expf(v - lse) - (col == yy ? 1.f : 0.f)) * (1.0f / (float)M);
            if (nn == 0) rowloss[4 * g + wave] = row < M ? lse - zy : 0.f;
        }
        __syncthreads();
        if (tid == 0) {
            float sum = 0.f;
            for (int r = 0; r < 16; ++r) sum += rowloss[r];
            losspart[blockIdx.y] = sum;
        }
    }
}

// dZprev[M,Kin] = (dZ[M,Nout] W[Nout,Kin]) * act'(Aprev[M,Kin]): the contraction runs over the rows
// of W, so W is the n-contiguous operand (one value per request, 16 lanes = 64 contiguous bytes).
// grid (ceil(Kin/16), ceil(M/16)), 1024 threads.
template <int ACT, bool VEC>
__global__ __launch_bounds__(MNT) void mlp_bwd_data_kernel(const float* __restrict__ dZ, const float* __restrict__ W,
                                                           const float* __restrict__ Aprev, float* __restrict__ dZprev,
                                                           int M, int Nout, int Kin) {
    __shared__ float red[MW][4][kWave];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int g = lane / 16, nn = lane % 16;
    const int n0 = blockIdx.x * 16, m0 = blockIdx.y * 16;
    const int col = n0 + nn;
    float hv = 0.f;
    if (wave < 4 && col < Kin && m0 + 4 * g + wave < M) hv = Aprev[(size_t)(m0 + 4 * g + wave) * Kin + col];
    const bool a_ok = m0 + nn < M, b_ok = col < Kin;
    const float* arow = dZ + (size_t)min(m0 + nn, M - 1) * Nout;
    const float* bcol = W + min(col, Kin - 1);
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    const int nchunks = (Nout + MKC - 1) / MKC;
    for (int kc = wave; kc < nchunks; kc += MW) {
        const int k0 = kc * MKC + 4 * g;
        float a[16], b[16];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const float4 av = a_ok ? ld_k4<VEC>(arow, k0 + 16 * s, Nout) : make_float4(0.f, 0.f, 0.f, 0.f);
            a[4 * s] = av.x; a[4 * s + 1] = av.y; a[4 * s + 2] = av.z; a[4 * s + 3] = av.w;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int k = k0 + 16 * s + e;
                b[4 * s + e] = (b_ok && k < Nout) ? bcol[(size_t)k * Kin] : 0.f;
            }
        }
#pragma unroll
        for (int q = 0; q < 16; q += 2) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[q], b[q], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[q + 1], b[q + 1], acc1, 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][i][lane] = acc0[i] + acc1[i];
    __syncthreads();
    if (wave >= 4) return;
    const int row = m0 + 4 * g + wave;
    if (row >= M || col >= Kin) return;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < MW; ++w) v += red[w][wave][lane];
    dZprev[(size_t)row * Kin + col] = v * (ACT == 0 ? act_grad<0>(hv) : act_grad<1>(hv));
}

// W[n,k] -= lr sum_m dZ[m,n] Aprev[m,k];  b[n] -= lr sum_m dZ[m,n].
// A wavefront owns 16 rows of W by 64 columns (four 16x16 tiles sharing the dZ operand) and walks
// the batch four rows per matrix instruction; per layer (ceil(Kin/256), ceil(Nout/16)) workgroups of 256 threads.
// MB > 0: the batch has at most 16 MB rows and every operand (and the tile of W itself) is
// requested before the first product, one memory round trip for the whole update; MB = 0: any batch.
struct UpdateLayers {
    const float* dZ[RNN_MLP_MAX_LAYERS];      // [M, Nout]
    const float* Aprev[RNN_MLP_MAX_LAYERS];   // [M, Kin]
    float* W[RNN_MLP_MAX_LAYERS];
    float* b[RNN_MLP_MAX_LAYERS];
    int Nout[RNN_MLP_MAX_LAYERS], Kin[RNN_MLP_MAX_LAYERS];
    int gx[RNN_MLP_MAX_LAYERS];               // workgroups along Kin
    int first[RNN_MLP_MAX_LAYERS + 1];        // first workgroup of the layer in the flat grid
    int layers;
    const float* losspart;                    // per 16-row group of the batch: sum of its row losses
    int nparts;                               // 0: the loss was written by its own kernel
    float* loss;
};

// One launch updates every layer: the flat grid is the layers' (ceil(Kin/256) x ceil(Nout/16)) grids
// one after another (all dZ_l are kept until the backward chain has ended).
template <int MB>
__global__ __launch_bounds__(256) void mlp_update_kernel(const UpdateLayers ul, int M, float lr) {
    int l = 0;
    while (l + 1 < ul.layers && (int)blockIdx.x >= ul.first[l + 1]) ++l;
    const int local = blockIdx.x - ul.first[l];
    const int bx = local % ul.gx[l], by = local / ul.gx[l];
    const float* __restrict__ dZ = ul.dZ[l];
    const float* __restrict__ Aprev = ul.Aprev[l];
    float* __restrict__ W = ul.W[l];
    float* __restrict__ b = ul.b[l];
    const int Nout = ul.Nout[l], Kin = ul.Kin[l];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int q = lane / 16, r = lane % 16;
    const int n0 = by * 16;
    const int k0 = (bx * 4 + wave) * 64;
    if (blockIdx.x == 0 && tid == 64 && ul.nparts > 0) {   // the batch's mean loss, groups in order
        float sum = 0.f;
        for (int g = 0; g < ul.nparts; ++g) sum += ul.losspart[g];
        *ul.loss = sum / (float)M;
    }
    if (bx == 0 && wave == 0) {
        // bias: lane (q, r) sums the rows m = q, q + 4, ... of column n0 + r; the four partial sums
        // of a column meet through lane exchanges in a fixed order
        float s = 0.f;
        if (n0 + r < Nout)
            for (int m = q; m < M; m += 4) s += dZ[(size_t)m * Nout + n0 + r];
        s += __shfl_xor(s, 16, kWave);
        s += __shfl_xor(s, 32, kWave);
        if (q == 0 && n0 + r < Nout) b[n0 + r] -= lr * s;
    }
    if (k0 >= Kin) return;
    const bool n_ok = n0 + r < Nout;
    const int ncol = min(n0 + r, Nout - 1);
    f32x4 acc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // tile layout: lane -> column r (k index); register i -> row 4 q + i (n index)
    float wv[4][4];
    if (MB > 0) {
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int k = k0 + 16 * t + r, n = n0 + 4 * q + i;
                wv[t][i] = (k < Kin && n < Nout) ? W[(size_t)n * Kin + k] : 0.f;
            }
    }
    constexpr int UB = MB > 0 ? MB : 1;
    const int mend = MB > 0 ? 16 * MB : M;
    for (int mb = 0; mb < mend; mb += 16 * UB) {
        float a[UB][4], x[UB][4][4];
#pragma unroll
        for (int v = 0; v < UB; ++v)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int m = mb + 16 * v + 4 * u + q;
                const bool m_ok = m < M;
                const int mm = min(m, M - 1);
                a[v][u] = (m_ok && n_ok) ? dZ[(size_t)mm * Nout + ncol] : 0.f;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int k = k0 + 16 * t + r;
                    x[v][u][t] = (m_ok && k < Kin) ? Aprev[(size_t)mm * Kin + k] : 0.f;
                }
            }
#pragma unroll
        for (int v = 0; v < UB; ++v)
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[v][u], x[v][u][t], acc[t], 0, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int k = k0 + 16 * t + r;
        if (k >= Kin) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = n0 + 4 * q + i;
            if (n >= Nout) continue;
            float* dst = W + (size_t)n * Kin + k;
            *dst = (MB > 0 ? wv[t][i] : *dst) - lr * acc[t][i];
        }
    }
}

// One workgroup of 16 wavefronts: per row log-sum-exp, the row's loss, dZ = (softmax - onehot) / M
// in place over the logits, and the batch's mean loss (rows summed in order).  M <= 1024.
__global__ __launch_bounds__(1024) void mlp_ce_kernel(float* __restrict__ Z, const int32_t* __restrict__ y,
                                                      float* __restrict__ loss, int M, int O) {
    __shared__ float rowloss[1024];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const float inv = 1.0f / (float)M;
    for (int row = wave; row < M; row += 16) {
        float* z = Z + (size_t)row * O;
        const int yy = y[row];
        float m = -INFINITY;
        for (int k = lane; k < O; k += kWave) m = fmaxf(m, z[k]);
        m = max64(m);
        float s = 0.f;
        for (int k = lane; k < O; k += kWave) s += __expf(z[k] - m);
        s = sum64(s);
        const float lse = m + __logf(s);
        if (lane == 0) rowloss[row] = lse - z[yy];
        for (int k = lane; k < O; k += kWave) {
            float d = __expf(z[k] - lse);
            if (k == yy) d -= 1.f;
            z[k] = d * inv;
        }
    }
    __syncthreads();
    if (wave == 0) {   // fixed order: lane l adds rows l, l + 64, ...; then the lanes in a fixed tree
        float s = 0.f;
        for (int r = lane; r < M; r += kWave) s += rowloss[r];
        s = sum64(s);
        if (lane == 0) *loss = s * inv;
    }
}

struct Widths { int w[RNN_MLP_MAX_LAYERS + 2]; int layers; };

bool mlp_dims_ok(const rnn_mlp_dims* d) {
    if (!d) return false;
    if (d->in_dim <= 0 || d->out_dim <= 0 || d->batch <= 0 || d->n_hidden < 0) return false;
    if (d->n_hidden + 1 > RNN_MLP_MAX_LAYERS) return false;
    if (d->n_hidden > 0 && d->hidden <= 0) return false;
    if (d->act != RNN_ACT_SIGMOID && d->act != RNN_ACT_TANH) return false;
    if (d->flags & ~RNN_FLAG_SYNC) return false;
    if (d->in_dim > (1 << 20) || d->hidden > (1 << 20) || d->out_dim > (1 << 20)) return false;
    return true;
}

Widths widths_of(const rnn_mlp_dims* d) {
    Widths w;
    w.layers = d->n_hidden + 1;
    w.w[0] = d->in_dim;
    for (int l = 1; l <= d->n_hidden; ++l) w.w[l] = d->hidden;
    w.w[w.layers] = d->out_dim;
    return w;
}

inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

// workspace: activations of the hidden layers, logits / dZ of the output layer, two dZ buffers of
// the hidden width
struct MlpPlan { size_t act[RNN_MLP_MAX_LAYERS + 1], Z, dz[RNN_MLP_MAX_LAYERS], losspart, total; };

MlpPlan mlp_plan(const rnn_mlp_dims* d) {
    const Widths w = widths_of(d);
    MlpPlan p{};
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += up256(bytes); return o; };
    for (int l = 1; l < w.layers; ++l) p.act[l] = take((size_t)d->batch * w.w[l] * 4);
    p.Z = take((size_t)d->batch * d->out_dim * 4);
    // dZ of layer l's outputs, l < layers - 1 (the last layer's is Z itself, in place)
    for (int l = 0; l + 1 < w.layers; ++l) p.dz[l] = take((size_t)d->batch * w.w[l + 1] * 4);
    p.losspart = take((size_t)((d->batch + 15) / 16 + 1) * 4);   // + one word that takes the loss when the caller wants none
    p.total = off;
    return p;
}

bool al16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

hipError_t launch_fwd(int act, const float* A, const float* W, const float* b, float* C, int M, int N, int K,
                      hipStream_t s) {
    dim3 grid((N + 15) / 16, (M + 15) / 16);
    const bool vec = K % 4 == 0 && al16(A) && al16(W);
    ProfileScope ps(K_MLP_FWD, s);
#define RNN_MLP_FWD(ACT)                                                                              \
    do {                                                                                              \
        if (vec) hipLaunchKernelGGL((mlp_fwd_kernel<ACT, true>), grid, dim3(MNT), 0, s, A, W, b, C, M, N, K, nullptr, nullptr);  \
        else hipLaunchKernelGGL((mlp_fwd_kernel<ACT, false>), grid, dim3(MNT), 0, s, A, W, b, C, M, N, K, nullptr, nullptr);     \
    } while (0)
    if (act == 0) RNN_MLP_FWD(0); else if (act == 1) RNN_MLP_FWD(1); else RNN_MLP_FWD(2);
#undef RNN_MLP_FWD
    return hipGetLastError();
}

// output layer of at most 16 classes with the loss in its epilogue
hipError_t launch_fwd_ce(const float* A, const float* W, const float* b, float* dZ, int M, int N, int K,
                         const int32_t* y, float* losspart, hipStream_t s) {
    dim3 grid(1, (M + 15) / 16);
    const bool vec = K % 4 == 0 && al16(A) && al16(W);
    ProfileScope ps(K_MLP_FWD, s);
    if (vec) hipLaunchKernelGGL((mlp_fwd_kernel<2, true, true>), grid, dim3(MNT), 0, s, A, W, b, dZ, M, N, K, y, losspart);
    else hipLaunchKernelGGL((mlp_fwd_kernel<2, false, true>), grid, dim3(MNT), 0, s, A, W, b, dZ, M, N, K, y, losspart);
    return hipGetLastError();
}

}  // namespace
}  // namespace rnn

extern "C" {

int rnn_mlp_workspace_bytes(const rnn_mlp_dims* dims, size_t* bytes) {
    if (!rnn::mlp_dims_ok(dims) || !bytes) return RNN_EINVAL;
    *bytes = rnn::mlp_plan(dims).total;
    return RNN_OK;
}

int rnn_mlp_train(const rnn_mlp_dims* dims, const rnn_mlp_params* params, const float* X, const int32_t* y,
                  int64_t n_batches, float lr, float* losses, void* workspace, size_t workspace_bytes,
                  void* hip_stream) {
    using namespace rnn;
    if (!mlp_dims_ok(dims) || !params || !X || !y || n_batches < 0) return RNN_EINVAL;
    if (dims->batch > 1024) return RNN_EUNSUPPORTED;
    const Widths w = widths_of(dims);
    for (int l = 0; l < w.layers; ++l)
        if (!params->W[l] || !params->b[l] || !al16(params->W[l]) || !al16(params->b[l])) return RNN_EINVAL;
    if ((reinterpret_cast<uintptr_t>(X) & 15u) || (reinterpret_cast<uintptr_t>(y) & 3u) ||
        (reinterpret_cast<uintptr_t>(losses) & 3u))
        return RNN_EINVAL;
    const MlpPlan pl = mlp_plan(dims);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < pl.total)
        return RNN_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const int B = dims->batch, L = w.layers;
    float* Z = reinterpret_cast<float*>(ws + pl.Z);
    // the one update launch of a batch: every layer's grid, one after another
    // at most 16 classes: the output layer's tile holds whole rows, its epilogue forms the loss and
    // dZ, and the update launch adds up the batch's loss
    const bool fused_ce = dims->out_dim <= 16;
    float* losspart = reinterpret_cast<float*>(ws + pl.losspart);
    float* scratch_loss = losspart + (B + 15) / 16;   // when the caller wants no losses
    UpdateLayers ul{};
    ul.layers = L;
    ul.losspart = losspart;
    ul.nparts = fused_ce ? (B + 15) / 16 : 0;
    int total_wgs = 0;
    for (int l = 0; l < L; ++l) {
        ul.dZ[l] = l + 1 < L ? reinterpret_cast<const float*>(ws + pl.dz[l]) : Z;
        ul.W[l] = params->W[l];
        ul.b[l] = params->b[l];
        ul.Nout[l] = w.w[l + 1];
        ul.Kin[l] = w.w[l];
        ul.gx[l] = (w.w[l] + 255) / 256;
        ul.first[l] = total_wgs;
        total_wgs += ul.gx[l] * ((w.w[l + 1] + 15) / 16);
    }
    ul.first[L] = total_wgs;
    for (int64_t i = 0; i < n_batches; ++i) {
        const float* x_in = X + (size_t)i * B * dims->in_dim;
        const float* a_prev = x_in;
        // forward
        float* loss_out = losses ? losses + i : scratch_loss;
        for (int l = 0; l < L; ++l) {
            float* out = l + 1 < L ? reinterpret_cast<float*>(ws + pl.act[l + 1]) : Z;
            hipError_t e;
            if (l + 1 == L && fused_ce)
                e = launch_fwd_ce(a_prev, params->W[l], params->b[l], Z, B, w.w[l + 1], w.w[l], y + (size_t)i * B,
                                  losspart, s);
            else
                e = launch_fwd(l + 1 < L ? dims->act : 2, a_prev, params->W[l], params->b[l], out, B, w.w[l + 1],
                               w.w[l], s);
            if (e != hipSuccess) return RNN_EHIP;
            a_prev = out;
        }
        if (!fused_ce) {
            ProfileScope ps(K_MLP_CE, s);
            hipLaunchKernelGGL(mlp_ce_kernel, dim3(1), dim3(1024), 0, s, Z, y + (size_t)i * B, loss_out, B,
                               dims->out_dim);
            if (hipGetLastError() != hipSuccess) return RNN_EHIP;
        }
        // backward: dZ_{l-1} from dZ_l and the weights as they were in the forward pass, layer by
        // layer; every dZ_l is kept, and one launch then updates all W_l and b_l in place
        const float* dz = Z;
        for (int l = L - 1; l > 0; --l) {
            const float* a_in = reinterpret_cast<const float*>(ws + pl.act[l]);
            float* dz_prev = reinterpret_cast<float*>(ws + pl.dz[l - 1]);
            dim3 grid((w.w[l] + 15) / 16, (B + 15) / 16);
            ProfileScope ps(K_MLP_BWD, s);
            const bool vec = w.w[l + 1] % 4 == 0;   // dZ rows stay 16-byte aligned (workspace regions are)
#define RNN_MLP_BWD(ACT, VEC)                                                                              \
    hipLaunchKernelGGL((mlp_bwd_data_kernel<ACT, VEC>), grid, dim3(MNT), 0, s, dz, params->W[l], a_in, dz_prev, \
                       B, w.w[l + 1], w.w[l])
            if (dims->act == 0) { if (vec) RNN_MLP_BWD(0, true); else RNN_MLP_BWD(0, false); }
            else { if (vec) RNN_MLP_BWD(1, true); else RNN_MLP_BWD(1, false); }
#undef RNN_MLP_BWD
            if (hipGetLastError() != hipSuccess) return RNN_EHIP;
            dz = dz_prev;
        }
        {
            for (int l = 0; l < L; ++l)
                ul.Aprev[l] = l > 0 ? reinterpret_cast<const float*>(ws + pl.act[l]) : x_in;
            ul.loss = loss_out;
            ProfileScope ps(K_MLP_UPDATE, s);
#define RNN_MLP_UPD(MB) hipLaunchKernelGGL(mlp_update_kernel<MB>, dim3(total_wgs), dim3(256), 0, s, ul, B, lr)
            if (B <= 16) RNN_MLP_UPD(1); else if (B <= 32) RNN_MLP_UPD(2); else if (B <= 64) RNN_MLP_UPD(4);
            else RNN_MLP_UPD(0);
#undef RNN_MLP_UPD
            if (hipGetLastError() != hipSuccess) return RNN_EHIP;
        }
    }
    if (dims->flags & RNN_FLAG_SYNC)
        if (hipStreamSynchronize(s) != hipSuccess) return RNN_EHIP;
    return RNN_OK;
}

}  // extern "C"
