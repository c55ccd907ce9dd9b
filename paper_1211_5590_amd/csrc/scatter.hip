// Gradient of the token-indexed input matrix, dWx[v,:] = sum over the rows n with x_n = v of
// Delta[n,:], as an ownership scan: every wavefront owns one vocabulary row, scans the id
// list for its token and adds the matching rows in ascending n.  No floating-point atomics,
// so the result is run-to-run identical however skewed (Zipf) the ids are, and the same pass
// writes the zero rows of tokens that do not occur.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

constexpr int kQ = 16;                      // columns per lane per pass
constexpr int kColsPerPass = kQ * kWave;    // 1024: one pass for H <= 1024, many loads in flight

__global__ __launch_bounds__(256) void dwx_tokens_kernel(const int32_t* __restrict__ x,
                                                         const float* __restrict__ Delta,
                                                         float* __restrict__ dWx, int N, int NV,
                                                         int H, int beta) {
    const int lane = threadIdx.x % kWave;
    const int v = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (v >= NV) return;
    for (int c0 = 0; c0 < H; c0 += kColsPerPass) {
        float acc[kQ];
#pragma unroll
        for (int q = 0; q < kQ; ++q) acc[q] = 0.f;
        bool seen = false;
        for (int n0 = 0; n0 < N; n0 += kWave) {
            const int n = n0 + lane;
            const bool hit = n < N && x[n] == v;
            unsigned long long mask = __ballot(hit);
            while (mask) {
                const int src = __ffsll((long long)mask) - 1;
                mask &= mask - 1;
                seen = true;
                const float* row = Delta + (size_t)(n0 + src) * H;
#pragma unroll
                for (int q = 0; q < kQ; ++q) {
                    const int col = c0 + q * kWave + lane;
                    if (col < H) acc[q] += row[col];
                }
            }
        }
        if (beta && !seen) continue;  // accumulate mode leaves untouched rows alone
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            const int col = c0 + q * kWave + lane;
            if (col < H) {
                float* dst = dWx + (size_t)v * H + col;
                *dst = beta ? *dst + acc[q] : acc[q];
            }
        }
    }
}

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t* p) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = 0;
}

__global__ __launch_bounds__(256) void check_tokens_kernel(const int32_t* __restrict__ ids,
                                                           int64_t n, int32_t limit,
                                                           int32_t* __restrict__ bad) {
    int cnt = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const int32_t v = ids[i];
        cnt += (v < 0 || v >= limit) ? 1 : 0;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
    if (threadIdx.x % kWave == 0 && cnt) atomicAdd(bad, cnt);  // integer: order-independent
}

}  // namespace

hipError_t launch_dwx_tokens(const int32_t* x, const float* Delta, float* dWx, int N, int NV, int H,
                             int beta, hipStream_t s) {
    const int rows_per_block = 256 / kWave;
    ProfileScope ps(K_DWX_TOKENS, s);
    hipLaunchKernelGGL(dwx_tokens_kernel, dim3((NV + rows_per_block - 1) / rows_per_block),
                       dim3(256), 0, s, x, Delta, dWx, N, NV, H, beta);
    return hipGetLastError();
}

hipError_t launch_check_tokens(const int32_t* ids, int64_t n, int32_t limit, int32_t* bad,
                               hipStream_t s) {
    ProfileScope ps(K_CHECK_TOKENS, s);
    hipLaunchKernelGGL(zero_i32_kernel, dim3(1), dim3(64), 0, s, bad);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    int blocks = (int)((n + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(check_tokens_kernel, dim3(blocks), dim3(256), 0, s, ids, n, limit, bad);
    return hipGetLastError();
}

}  // namespace rnn
