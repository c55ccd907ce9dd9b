// Gradient of the token-indexed input matrix, dWx[v,:] = sum over the rows n with x_n = v of
// Delta[n,:], without floating-point atomics: results are run-to-run identical however skewed
// (Zipf) the ids are, and the same pass writes the zero rows of tokens that do not occur.
//
// Grouped form (the normal one): the id list is cut into ranges of CL ids.  One workgroup per
// range sorts its (id, position) pairs in LDS (bitonic, keys are unique), which groups equal ids
// with ascending positions, and sums the Delta rows of every group in that order into a compact
// partial row; a table [token][range] records which partial row, if any, belongs to a token
// (or, for a token that occurs once in the range, which row of Delta).
// A second kernel, one wavefront per vocabulary row, adds the token's partial rows in ascending
// range order.  Delta is read once and every sum has a fixed order.
//
// Scan form (fallback when the scratch space is too small): every wavefront owns one
// vocabulary row and scans the whole id list for its token.
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

constexpr int kGroupThreads = 512;
constexpr int kRowsInFlight = 8;

// One range of CL ids per workgroup: sort, group, sum.  part: compact partial rows
// [range*CL + group][H]; slot[token][range] = group + 1, or -(n + 1) for a single occurrence at
// row n, where the token occurs in the range (the table is zeroed before this kernel).
template <int CL>
__global__ __launch_bounds__(kGroupThreads) void dwx_group_kernel(const int32_t* __restrict__ x,
                                                                  const float* __restrict__ Delta,
                                                                  float* __restrict__ part,
                                                                  int32_t* __restrict__ slot,
                                                                  int N, int NV, int H) {
    __shared__ unsigned long long key[CL];   // (id << 32) | position in the range; padding = ~0
    __shared__ int seg_start[CL + 1];
    __shared__ int s_scan[kGroupThreads];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int base = blockIdx.x * CL;
    for (int i = tid; i < CL; i += kGroupThreads) {
        const int n = base + i;
        key[i] = n < N ? ((unsigned long long)(unsigned)x[n] << 32) | (unsigned)i : ~0ull;
    }
    __syncthreads();
    for (int k = 2; k <= CL; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < CL; i += kGroupThreads) {
                const int partner = i ^ j;
                if (partner > i) {
                    const unsigned long long a = key[i], b = key[partner];
                    const bool up = (i & k) == 0;
                    if ((a > b) == up) { key[i] = b; key[partner] = a; }
                }
            }
            __syncthreads();
        }
    // group heads -> group numbers (block prefix sum over CL flags)
    constexpr int PER = (CL + kGroupThreads - 1) / kGroupThreads;
    const int nvalid = min(CL, N - base);
    int heads = 0;
    for (int u = 0; u < PER; ++u) {
        const int i = tid * PER + u;
        heads += (i < nvalid && (i == 0 || (key[i] >> 32) != (key[i - 1] >> 32))) ? 1 : 0;
    }
    s_scan[tid] = heads;
    __syncthreads();
    for (int off = 1; off < kGroupThreads; off <<= 1) {
        const int v = tid >= off ? s_scan[tid - off] : 0;
        __syncthreads();
        s_scan[tid] += v;
        __syncthreads();
    }
    int g = s_scan[tid] - heads;             // groups before this thread's elements
    const int ngroups = s_scan[kGroupThreads - 1];
    for (int u = 0; u < PER; ++u) {
        const int i = tid * PER + u;
        if (i < nvalid && (i == 0 || (key[i] >> 32) != (key[i - 1] >> 32))) seg_start[g++] = i;
    }
    if (tid == 0) seg_start[ngroups] = nvalid;
    __syncthreads();
    // one wavefront per group: rows added in ascending position, 16 columns per lane per pass.
    // A token that occurs once in the range needs no partial row: the table points at its
    // Delta row instead (negative entry).
    const int ranges = gridDim.x;
    for (int grp = wave; grp < ngroups; grp += kGroupThreads / kWave) {
        const int i0 = seg_start[grp], i1 = seg_start[grp + 1];
        const int v = (int)(key[i0] >> 32);
        if (i1 - i0 == 1) {
            if (lane == 0) slot[(size_t)v * ranges + blockIdx.x] = -(base + (int)(unsigned)key[i0] + 1);
            continue;
        }
        if ((H & 3) == 0) {
            // 256 columns per pass as one float4 per lane, eight rows in flight, added in order
            for (int c0 = 4 * lane; c0 < H; c0 += 4 * kWave) {
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
                for (int i = i0; i < i1; i += kRowsInFlight) {
                    float4 r[kRowsInFlight];
#pragma unroll
                    for (int u = 0; u < kRowsInFlight; ++u) {
                        const int ii = min(i + u, i1 - 1);
                        r[u] = *reinterpret_cast<const float4*>(Delta + (size_t)(base + (int)(unsigned)key[ii]) * H + c0);
                    }
#pragma unroll
                    for (int u = 0; u < kRowsInFlight; ++u)
                        if (i + u < i1) { acc.x += r[u].x; acc.y += r[u].y; acc.z += r[u].z; acc.w += r[u].w; }
                }
                *reinterpret_cast<float4*>(part + ((size_t)base + grp) * H + c0) = acc;
            }
        } else {
            for (int c0 = 0; c0 < H; c0 += kColsPerPass) {
                float acc[kQ];
#pragma unroll
                for (int q = 0; q < kQ; ++q) acc[q] = 0.f;
                for (int i = i0; i < i1; ++i) {
                    const float* row = Delta + (size_t)(base + (int)(unsigned)key[i]) * H;
#pragma unroll
                    for (int q = 0; q < kQ; ++q) {
                        const int col = c0 + q * kWave + lane;
                        if (col < H) acc[q] += row[col];
                    }
                }
#pragma unroll
                for (int q = 0; q < kQ; ++q) {
                    const int col = c0 + q * kWave + lane;
                    if (col < H) part[((size_t)base + grp) * H + col] = acc[q];
                }
            }
        }
        if (lane == 0) slot[(size_t)v * ranges + blockIdx.x] = grp + 1;
    }
}

// dWx[v] = sum over the ranges (ascending) of the token's partial rows; zero row if none.
// One wavefront per (token, chunk of 256 columns) when rows are 16-byte aligned (VEC), else
// per token with scalar columns; eight rows in flight, added in range order.
template <bool VEC>
__global__ __launch_bounds__(256) void dwx_gather_kernel(const float* __restrict__ part,
                                                         const int32_t* __restrict__ slot,
                                                         const float* __restrict__ Delta,
                                                         float* __restrict__ dWx, int NV, int H,
                                                         int ranges, int CL, int beta, int col_chunks) {
    const int lane = threadIdx.x % kWave;
    const long long task = (long long)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    const int v = (int)(task / col_chunks), chunk = (int)(task % col_chunks);
    if (v >= NV) return;
    const int c0 = VEC ? chunk * 4 * kWave + 4 * lane : 0;
    float4 acc4 = make_float4(0.f, 0.f, 0.f, 0.f);
    float acc[kQ];
#pragma unroll
    for (int q = 0; q < kQ; ++q) acc[q] = 0.f;
    bool any = false;
    for (int pass0 = 0; pass0 < (VEC ? 1 : (H + kColsPerPass - 1) / kColsPerPass); ++pass0) {
        const int cs = pass0 * kColsPerPass;
        if (!VEC) {
#pragma unroll
            for (int q = 0; q < kQ; ++q) acc[q] = 0.f;
        }
        for (int r0 = 0; r0 < ranges; r0 += kWave) {     // 64 table entries per look
            const int r = r0 + lane;
            const int sl = r < ranges ? slot[(size_t)v * ranges + r] : 0;
            unsigned long long mask = __ballot(sl != 0);
            any = any || mask != 0;
            while (mask) {
                const float* rows[kRowsInFlight];
                int cnt = 0;
#pragma unroll
                for (int u = 0; u < kRowsInFlight; ++u) {
                    rows[u] = Delta;                       // placeholder, not added
                    if (mask) {
                        const int src = __ffsll((long long)mask) - 1;
                        mask &= mask - 1;
                        const int e = __shfl(sl, src, kWave);
                        rows[u] = e > 0 ? part + ((size_t)(r0 + src) * CL + (e - 1)) * H
                                        : Delta + (size_t)(-e - 1) * H;
                        cnt = u + 1;
                    }
                }
                if (VEC) {
                    float4 t[kRowsInFlight];
#pragma unroll
                    for (int u = 0; u < kRowsInFlight; ++u)
                        t[u] = c0 < H ? *reinterpret_cast<const float4*>(rows[u] + c0) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                    for (int u = 0; u < kRowsInFlight; ++u)
                        if (u < cnt) { acc4.x += t[u].x; acc4.y += t[u].y; acc4.z += t[u].z; acc4.w += t[u].w; }
                } else {
                    for (int u = 0; u < cnt; ++u) {
#pragma unroll
                        for (int q = 0; q < kQ; ++q) {
                            const int col = cs + q * kWave + lane;
                            if (col < H) acc[q] += rows[u][col];
                        }
                    }
                }
            }
        }
        if (beta && !any) return;         // accumulate mode leaves untouched rows alone
        if (VEC) {
            if (c0 < H) {
                float4* dst = reinterpret_cast<float4*>(dWx + (size_t)v * H + c0);
                if (beta) { const float4 o = *dst; acc4.x += o.x; acc4.y += o.y; acc4.z += o.z; acc4.w += o.w; }
                *dst = acc4;
            }
        } else {
#pragma unroll
            for (int q = 0; q < kQ; ++q) {
                const int col = cs + q * kWave + lane;
                if (col < H) {
                    float* dst = dWx + (size_t)v * H + col;
                    *dst = beta ? *dst + acc[q] : acc[q];
                }
            }
        }
    }
}

__global__ void zero_table_kernel(int32_t* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
        p[i] = 0;
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

// ids per range of the grouped form: 256 while that gives at most 256 ranges, then larger
int dwx_range_len(int N) {
    int cl = 256;
    while (cl < 4096 && (N + cl - 1) / cl > 256) cl *= 2;
    return cl;
}
int dwx_ranges(int N) { const int cl = dwx_range_len(N); return (N + cl - 1) / cl; }
size_t dwx_table_ints(int N, int NV) { return (size_t)dwx_ranges(N) * NV; }

hipError_t launch_dwx_tokens(const int32_t* x, const float* Delta, float* dWx, int N, int NV, int H,
                             int beta, float* scratch, size_t scratch_floats, int32_t* slot_table,
                             hipStream_t s) {
    const int rows_per_block = 256 / kWave;
    const int blocks = (NV + rows_per_block - 1) / rows_per_block;
    const int cl = dwx_range_len(N), ranges = dwx_ranges(N);
    const bool grouped = scratch && slot_table && (size_t)ranges * cl * H <= scratch_floats;
    if (!grouped) {
        ProfileScope ps(K_DWX_TOKENS, s);
        hipLaunchKernelGGL(dwx_tokens_kernel, dim3(blocks), dim3(256), 0, s, x, Delta, dWx, N, NV, H, beta);
        return hipGetLastError();
    }
    {
        ProfileScope ps(K_DWX_TOKENS, s);
        const size_t n = dwx_table_ints(N, NV);
        size_t zb = (n + 2047) / 2048;
        if (zb > 1024) zb = 1024;
        hipLaunchKernelGGL(zero_table_kernel, dim3((unsigned)zb), dim3(256), 0, s, slot_table, n);
        switch (cl) {
            case 256: hipLaunchKernelGGL(dwx_group_kernel<256>, dim3(ranges), dim3(kGroupThreads), 0, s, x, Delta, scratch, slot_table, N, NV, H); break;
            case 512: hipLaunchKernelGGL(dwx_group_kernel<512>, dim3(ranges), dim3(kGroupThreads), 0, s, x, Delta, scratch, slot_table, N, NV, H); break;
            case 1024: hipLaunchKernelGGL(dwx_group_kernel<1024>, dim3(ranges), dim3(kGroupThreads), 0, s, x, Delta, scratch, slot_table, N, NV, H); break;
            case 2048: hipLaunchKernelGGL(dwx_group_kernel<2048>, dim3(ranges), dim3(kGroupThreads), 0, s, x, Delta, scratch, slot_table, N, NV, H); break;
            default: hipLaunchKernelGGL(dwx_group_kernel<4096>, dim3(ranges), dim3(kGroupThreads), 0, s, x, Delta, scratch, slot_table, N, NV, H); break;
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    ProfileScope ps(K_DWX_TOKENS, s);
    const bool vec = H % 4 == 0 && (reinterpret_cast<uintptr_t>(dWx) & 15u) == 0 &&
                     (reinterpret_cast<uintptr_t>(Delta) & 15u) == 0 && (reinterpret_cast<uintptr_t>(scratch) & 15u) == 0;
    if (vec) {
        const int col_chunks = (H + 4 * kWave - 1) / (4 * kWave);
        const long long tasks = (long long)NV * col_chunks;
        const unsigned gb = (unsigned)((tasks + rows_per_block - 1) / rows_per_block);
        hipLaunchKernelGGL(dwx_gather_kernel<true>, dim3(gb), dim3(256), 0, s, scratch, slot_table, Delta, dWx,
                           NV, H, ranges, cl, beta, col_chunks);
    } else {
        hipLaunchKernelGGL(dwx_gather_kernel<false>, dim3(blocks), dim3(256), 0, s, scratch, slot_table, Delta,
                           dWx, NV, H, ranges, cl, beta, 1);
    }
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
