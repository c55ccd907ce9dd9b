// Gradient of the token-indexed input matrix, dWx[v,:] = sum over the rows n with x_n = v of
// Delta[n,:], as an ownership scan: every wavefront owns one vocabulary row, scans the id
// list (or, for long lists, one of up to 32 ranges of it) for its token and adds the matching
// rows in ascending n; range partials are then added in ascending range order.  No floating-point atomics,
// so the result is run-to-run identical however skewed (Zipf) the ids are, and the same pass
// writes the zero rows of tokens that do not occur.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

constexpr int kQ = 16;                      // columns per lane per pass
constexpr int kColsPerPass = kQ * kWave;    // 1024: one pass for H <= 1024, many loads in flight

// Sum of the Delta rows whose id equals v among ids [n_begin, n_end), ascending n; 16 columns
// per lane starting at c0.  Returns whether any row matched.
__device__ __forceinline__ bool scan_token(const int32_t* __restrict__ x,
                                           const float* __restrict__ Delta, int v, int n_begin,
                                           int n_end, int H, int c0, int lane, float (&acc)[kQ]) {
#pragma unroll
    for (int q = 0; q < kQ; ++q) acc[q] = 0.f;
    bool seen = false;
    for (int n0 = n_begin; n0 < n_end; n0 += kWave) {
        const int n = n0 + lane;
        const bool hit = n < n_end && x[n] == v;
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
    return seen;
}

// Whole id list per wavefront (short lists).
__global__ __launch_bounds__(256) void dwx_tokens_kernel(const int32_t* __restrict__ x,
                                                         const float* __restrict__ Delta,
                                                         float* __restrict__ dWx, int N, int NV,
                                                         int H, int beta) {
    const int lane = threadIdx.x % kWave;
    const int v = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (v >= NV) return;
    for (int c0 = 0; c0 < H; c0 += kColsPerPass) {
        float acc[kQ];
        const bool seen = scan_token(x, Delta, v, 0, N, H, c0, lane, acc);
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

// Long id lists: the list is cut into `chunks` ranges (blockIdx.y); a frequent token's rows are
// then summed by `chunks` wavefronts in parallel instead of one.  Partial rows go to part
// [chunk][v][H] only where the token occurs in the chunk; seen[chunk][v] says where.
__global__ __launch_bounds__(256) void dwx_tokens_partial_kernel(const int32_t* __restrict__ x,
                                                                 const float* __restrict__ Delta,
                                                                 float* __restrict__ part,
                                                                 int32_t* __restrict__ seen_flags,
                                                                 int N, int NV, int H, int chunk_len) {
    const int lane = threadIdx.x % kWave;
    const int v = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (v >= NV) return;
    const int c = blockIdx.y;
    const int n_begin = c * chunk_len, n_end = min(N, n_begin + chunk_len);
    bool any = false;
    for (int c0 = 0; c0 < H; c0 += kColsPerPass) {
        float acc[kQ];
        const bool seen = scan_token(x, Delta, v, n_begin, n_end, H, c0, lane, acc);
        any = any || seen;
        if (!seen) continue;
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            const int col = c0 + q * kWave + lane;
            if (col < H) part[((size_t)c * NV + v) * H + col] = acc[q];
        }
    }
    if (lane == 0) seen_flags[(size_t)c * NV + v] = any ? 1 : 0;
}

// dWx[v] = sum over the chunks (ascending) in which the token occurs; zero row if none.
__global__ __launch_bounds__(256) void dwx_tokens_finish_kernel(const float* __restrict__ part,
                                                                const int32_t* __restrict__ seen_flags,
                                                                float* __restrict__ dWx, int NV, int H,
                                                                int chunks, int beta) {
    const int lane = threadIdx.x % kWave;
    const int v = blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (v >= NV) return;
    unsigned mask = 0;  // chunks <= 32
    for (int c = 0; c < chunks; ++c)
        if (seen_flags[(size_t)c * NV + v]) mask |= 1u << c;
    if (beta && mask == 0) return;
    for (int c0 = 0; c0 < H; c0 += kColsPerPass) {
        float acc[kQ];
#pragma unroll
        for (int q = 0; q < kQ; ++q) acc[q] = 0.f;
        for (unsigned m = mask; m; m &= m - 1) {
            const int c = __ffs((int)m) - 1;
            const float* row = part + ((size_t)c * NV + v) * H;
#pragma unroll
            for (int q = 0; q < kQ; ++q) {
                const int col = c0 + q * kWave + lane;
                if (col < H) acc[q] += row[col];
            }
        }
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

int dwx_token_chunks(int N, int NV, int H, size_t scratch_floats) {
    int chunks = N / 1024;                                  // at least 1024 ids per chunk
    const size_t fit = scratch_floats / ((size_t)NV * H);   // partial rows must fit the scratch
    if ((size_t)chunks > fit) chunks = (int)fit;
    if (chunks > 32) chunks = 32;
    return chunks < 2 ? 1 : chunks;
}

hipError_t launch_dwx_tokens(const int32_t* x, const float* Delta, float* dWx, int N, int NV, int H,
                             int beta, float* scratch, size_t scratch_floats, int32_t* seen_flags,
                             hipStream_t s) {
    const int rows_per_block = 256 / kWave;
    const int blocks = (NV + rows_per_block - 1) / rows_per_block;
    const int chunks = (scratch && seen_flags) ? dwx_token_chunks(N, NV, H, scratch_floats) : 1;
    if (chunks == 1) {
        ProfileScope ps(K_DWX_TOKENS, s);
        hipLaunchKernelGGL(dwx_tokens_kernel, dim3(blocks), dim3(256), 0, s, x, Delta, dWx, N, NV, H, beta);
        return hipGetLastError();
    }
    int chunk_len = (N + chunks - 1) / chunks;
    chunk_len = (chunk_len + kWave - 1) / kWave * kWave;
    {
        ProfileScope ps(K_DWX_TOKENS, s);
        hipLaunchKernelGGL(dwx_tokens_partial_kernel, dim3(blocks, chunks), dim3(256), 0, s, x, Delta,
                           scratch, seen_flags, N, NV, H, chunk_len);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    ProfileScope ps(K_DWX_TOKENS, s);
    hipLaunchKernelGGL(dwx_tokens_finish_kernel, dim3(blocks), dim3(256), 0, s, scratch, seen_flags, dWx,
                       NV, H, chunks, beta);
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
