// Row-wise and element-wise kernels of the output layer: log-sum-exp row statistics, the
// d loss / d logits producer fused with its column sums (element-wise chain fused into one
// pass, as the paper's loop-fusion rewrite does for scalar operations), and deterministic
// column-sum / scalar reductions.  All of these are HBM-bandwidth bound.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

// rows summed by one workgroup before the second stage: at least 64, and few enough chunks
// (<= 512) that the second stage stays short
__host__ __device__ inline int rows_per_chunk(int N) {
    const int r = (N + 511) / 512;
    return r < 64 ? 64 : r;
}

// One workgroup per row: lse = m + log(sum exp(z - m)), rowloss = lse - z[y].
__global__ __launch_bounds__(256) void ce_row_stats_kernel(const float* __restrict__ Z,
                                                           const int32_t* __restrict__ y,
                                                           float* __restrict__ lse,
                                                           float* __restrict__ rowloss, int O) {
    __shared__ float sm[4], ss[4];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const float* z = Z + (size_t)n * O;
    float m = -INFINITY, s = 0.f;
    for (int k = tid; k < O; k += blockDim.x) {
        const float v = z[k];
        if (v > m) {
            s = s * __expf(m - v) + 1.f;  // exp(-inf) = 0 on the first element
            m = v;
        } else {
            s += __expf(v - m);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off, kWave), s2 = __shfl_xor(s, off, kWave);
        lse_merge(m, s, m2, s2);
    }
    if (lane == 0) { sm[wave] = m; ss[wave] = s; }
    __syncthreads();
    if (tid == 0) {
        float M = sm[0], S = ss[0];
        for (int w = 1; w < 4; ++w) lse_merge(M, S, sm[w], ss[w]);
        const float l = M + logf(S);
        lse[n] = l;
        rowloss[n] = l - z[y[n]];
    }
}

__global__ __launch_bounds__(256) void mse_row_loss_kernel(const float* __restrict__ Z,
                                                           const float* __restrict__ Y,
                                                           float* __restrict__ rowloss, int O) {
    __shared__ float ss[4];
    const int n = blockIdx.x, tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    float s = 0.f;
    for (int k = tid; k < O; k += blockDim.x) {
        const float e = Z[(size_t)n * O + k] - Y[(size_t)n * O + k];
        s = fmaf(e, e, s);
    }
    s = wave_sum(s);
    if (lane == 0) ss[wave] = s;
    __syncthreads();
    if (tid == 0) rowloss[n] = (ss[0] + ss[1]) + (ss[2] + ss[3]);
}

// loss = scale * sum rowloss (single workgroup, fixed order)
__global__ __launch_bounds__(1024) void loss_reduce_kernel(const float* __restrict__ rowloss, int N,
                                                           float scale, float* __restrict__ loss) {
    __shared__ float ss[16];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    float s = 0.f;
    for (int n = tid; n < N; n += blockDim.x) s += rowloss[n];
    s = wave_sum(s);
    if (lane == 0) ss[wave] = s;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int w = 0; w < 16; ++w) t += ss[w];
        *loss = t * scale;
    }
}

// grid (column chunks of 256, row chunks of rows_per_chunk(N)).  Thread = one column; it walks
// the chunk's rows, turns z into d loss / d z in place, and keeps the column's partial sum.
template <int LOSS>
__global__ __launch_bounds__(256) void dz_kernel(float* __restrict__ Z, const float* __restrict__ lse,
                                                 const int32_t* __restrict__ y,
                                                 const float* __restrict__ Y,
                                                 float* __restrict__ part, int N, int O, float scale) {
    const int col = blockIdx.x * 256 + threadIdx.x;
    const int rpc = rows_per_chunk(N);
    const int r0 = blockIdx.y * rpc;
    const int r1 = min(N, r0 + rpc);
    if (col >= O) return;
    float cs = 0.f;
    for (int n = r0; n < r1; ++n) {
        const size_t idx = (size_t)n * O + col;
        float d;
        if (LOSS == 0) {
            d = __expf(Z[idx] - lse[n]);
            if (y[n] == col) d -= 1.f;
            d *= scale;
        } else {
            d = (Z[idx] - Y[idx]) * scale;
        }
        Z[idx] = d;
        cs += d;
    }
    part[(size_t)blockIdx.y * O + col] = cs;
}

__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* __restrict__ M,
                                                             float* __restrict__ part, int N, int C) {
    const int col = blockIdx.x * 256 + threadIdx.x;
    const int rpc = rows_per_chunk(N);
    const int r0 = blockIdx.y * rpc;
    const int r1 = min(N, r0 + rpc);
    if (col >= C) return;
    float cs = 0.f;
    for (int n = r0; n < r1; ++n) cs += M[(size_t)n * C + col];
    part[(size_t)blockIdx.y * C + col] = cs;
}

__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ part,
                                                            float* __restrict__ out, int chunks,
                                                            int C, int beta) {
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col >= C) return;
    float s = 0.f;
    for (int k = 0; k < chunks; ++k) s += part[(size_t)k * C + col];
    out[col] = beta ? out[col] + s : s;
}

}  // namespace

int colsum_chunks(int N) { const int r = rows_per_chunk(N); return (N + r - 1) / r; }

hipError_t launch_ce_row_stats(const float* Z, const int32_t* y, float* lse, float* rowloss, int N,
                               int O, hipStream_t s) {
    ProfileScope ps(K_CE_ROW_STATS, s);
    hipLaunchKernelGGL(ce_row_stats_kernel, dim3(N), dim3(256), 0, s, Z, y, lse, rowloss, O);
    return hipGetLastError();
}

hipError_t launch_mse_row_loss(const float* Z, const float* Y, float* rowloss, int N, int O,
                               hipStream_t s) {
    ProfileScope ps(K_MSE_ROW_LOSS, s);
    hipLaunchKernelGGL(mse_row_loss_kernel, dim3(N), dim3(256), 0, s, Z, Y, rowloss, O);
    return hipGetLastError();
}

hipError_t launch_loss_reduce(const float* rowloss, int N, float scale, float* loss, hipStream_t s) {
    ProfileScope ps(K_LOSS_REDUCE, s);
    hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, rowloss, N, scale, loss);
    return hipGetLastError();
}

hipError_t launch_dz(float* Z, const float* lse, const int32_t* y, const float* Y, float* part,
                     int N, int O, int loss_kind, hipStream_t s) {
    dim3 grid((O + 255) / 256, colsum_chunks(N));
    ProfileScope ps(K_DZ, s);
    if (loss_kind == 0) {
        const float scale = 1.0f / (float)N;
        hipLaunchKernelGGL(dz_kernel<0>, grid, dim3(256), 0, s, Z, lse, y, Y, part, N, O, scale);
    } else {
        const float scale = (float)(2.0 / ((double)N * (double)O));
        hipLaunchKernelGGL(dz_kernel<1>, grid, dim3(256), 0, s, Z, lse, y, Y, part, N, O, scale);
    }
    return hipGetLastError();
}

hipError_t launch_colsum_partial(const float* M, float* part, int N, int C, hipStream_t s) {
    dim3 grid((C + 255) / 256, colsum_chunks(N));
    ProfileScope ps(K_COLSUM_PARTIAL, s);
    hipLaunchKernelGGL(colsum_partial_kernel, grid, dim3(256), 0, s, M, part, N, C);
    return hipGetLastError();
}

hipError_t launch_colsum_finish(const float* part, float* out, int chunks, int C, int beta,
                                hipStream_t s) {
    ProfileScope ps(K_COLSUM_FINISH, s);
    hipLaunchKernelGGL(colsum_finish_kernel, dim3((C + 255) / 256), dim3(256), 0, s, part, out,
                       chunks, C, beta);
    return hipGetLastError();
}

}  // namespace rnn
