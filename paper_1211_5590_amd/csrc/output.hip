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

// One wavefront per row: merges the (max, sum exp) pairs the logits product left per 64-column
// part, in a fixed order, into lse; rowloss = lse - z[y].
__global__ __launch_bounds__(256) void ce_merge_stats_kernel(const float* __restrict__ stats, int parts,
                                                             const float* __restrict__ Z,
                                                             const int32_t* __restrict__ y,
                                                             float* __restrict__ lse,
                                                             float* __restrict__ rowloss, int N, int O) {
    const int lane = threadIdx.x % kWave;
    const int n = blockIdx.x * 4 + threadIdx.x / kWave;
    if (n >= N) return;
    const float2* st = reinterpret_cast<const float2*>(stats) + (size_t)n * parts;
    float m = -INFINITY, s = 0.f;
    for (int q = lane; q < parts; q += kWave) {
        const float2 t = st[q];
        lse_merge(m, s, t.x, t.y);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float m2 = __shfl_xor(m, off, kWave), s2 = __shfl_xor(s, off, kWave);
        lse_merge(m, s, m2, s2);
    }
    if (lane == 0) {
        const float l = m + logf(s);
        lse[n] = l;
        rowloss[n] = l - Z[(size_t)n * O + y[n]];
    }
}

// Mean-squared error is a sum over the flat [N*O] array: workgroup b sums the squared errors of
// elements [b*per_block, (b+1)*per_block) in a fixed order and leaves one partial.
template <int VEC>
__global__ __launch_bounds__(256) void mse_partial_kernel(const float* __restrict__ Z,
                                                          const float* __restrict__ Y,
                                                          float* __restrict__ partial,
                                                          size_t total, size_t per_block) {
    __shared__ float ss[4];
    constexpr int U = 4;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const size_t begin = (size_t)blockIdx.x * per_block;
    const size_t end = begin + per_block < total ? begin + per_block : total;
    float s = 0.f;
    for (size_t i0 = begin + (size_t)tid * VEC; i0 < end; i0 += (size_t)256 * VEC * U) {
        float z[U][VEC], t[U][VEC];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t i = i0 + (size_t)u * 256 * VEC;
#pragma unroll
            for (int v = 0; v < VEC; ++v) { z[u][v] = 0.f; t[u][v] = 0.f; }
            if (i < end) {
                if (VEC == 4) {
                    const float4 a = *reinterpret_cast<const float4*>(Z + i);
                    const float4 c = *reinterpret_cast<const float4*>(Y + i);
                    z[u][0] = a.x; z[u][1 % VEC] = a.y; z[u][2 % VEC] = a.z; z[u][3 % VEC] = a.w;
                    t[u][0] = c.x; t[u][1 % VEC] = c.y; t[u][2 % VEC] = c.z; t[u][3 % VEC] = c.w;
                } else {
                    z[u][0] = Z[i]; t[u][0] = Y[i];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const float e = z[u][v] - t[u][v];
                s = fmaf(e, e, s);
            }
    }
    s = wave_sum(s);
    if (lane == 0) ss[wave] = s;
    __syncthreads();
    if (tid == 0) partial[blockIdx.x] = (ss[0] + ss[1]) + (ss[2] + ss[3]);
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

// Thread layout shared by the column-sum kernels.  The 256 threads of a workgroup form
// 2^txs column lanes (VEC adjacent columns each) times 256 >> txs row lanes, so that a narrow
// matrix still keeps every lane busy; row lanes walk the chunk's rows interleaved, U rows in
// flight per thread, and their partial sums are added through LDS in a fixed order.
struct ColLayout {
    int tx, ty, cx, ry;
    __device__ explicit ColLayout(int txs)
        : tx(1 << txs), ty(256 >> txs), cx(threadIdx.x & ((1 << txs) - 1)), ry(threadIdx.x >> txs) {}
};

template <int VEC>
__device__ __forceinline__ void load_vec(const float* p, float (&v)[VEC]) {
    if (VEC == 4) {
        const float4 a = *reinterpret_cast<const float4*>(p);
        v[0] = a.x; v[1 % VEC] = a.y; v[2 % VEC] = a.z; v[3 % VEC] = a.w;
    } else {
        v[0] = *p;
    }
}
template <int VEC>
__device__ __forceinline__ void store_vec(float* p, const float (&v)[VEC]) {
    if (VEC == 4) *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1 % VEC], v[2 % VEC], v[3 % VEC]);
    else *p = v[0];
}

// sums cs[] over the row lanes; the row-lane-0 threads write VEC columns of out_row
template <int VEC>
__device__ __forceinline__ void fold_row_lanes(const ColLayout& L, float (&cs)[VEC], float* red,
                                               float* out_row, int col, int C) {
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[threadIdx.x * VEC + v] = cs[v];
    __syncthreads();
    if (L.ry == 0 && col < C) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float s = 0.f;
            for (int r = 0; r < L.ty; ++r) s += red[(r * L.tx + L.cx) * VEC + v];
            out_row[col + v] = s;
        }
    }
}

// grid (column blocks, row chunks of rows_per_chunk(N)): turns z into d loss / d z in place and
// keeps per-chunk column sums in part[chunk][O].
template <int LOSS, int VEC>
__global__ __launch_bounds__(256) void dz_kernel(float* __restrict__ Z, const float* __restrict__ lse,
                                                 const int32_t* __restrict__ y,
                                                 const float* __restrict__ Y,
                                                 float* __restrict__ part, int N, int O, float scale,
                                                 int txs) {
    __shared__ float red[256 * VEC];
    constexpr int U = 4;
    const ColLayout L(txs);
    const int col = (blockIdx.x * L.tx + L.cx) * VEC;
    const int rpc = rows_per_chunk(N);
    const int r0 = blockIdx.y * rpc;
    const int r1 = min(N, r0 + rpc);
    float cs[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) cs[v] = 0.f;
    if (col < O) {
        for (int n0 = r0 + L.ry; n0 < r1; n0 += L.ty * U) {
            float z[U][VEC], t[U][VEC];
            float l[U];
            int yy[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int n = min(n0 + u * L.ty, r1 - 1);
                const size_t idx = (size_t)n * O + col;
                load_vec<VEC>(Z + idx, z[u]);
                if (LOSS == 0) { l[u] = lse[n]; yy[u] = y[n]; }
                else load_vec<VEC>(Y + idx, t[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int n = n0 + u * L.ty;
                if (n >= r1) continue;
                float d[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    if (LOSS == 0) {
                        d[v] = __expf(z[u][v] - l[u]);
                        if (yy[u] == col + v) d[v] -= 1.f;
                        d[v] *= scale;
                    } else {
                        d[v] = (z[u][v] - t[u][v]) * scale;
                    }
                    cs[v] += d[v];
                }
                store_vec<VEC>(Z + (size_t)n * O + col, d);
            }
        }
    }
    fold_row_lanes<VEC>(L, cs, red, part + (size_t)blockIdx.y * O, col, O);
}

template <int VEC>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float* __restrict__ M,
                                                             float* __restrict__ part, int N, int C,
                                                             int txs) {
    __shared__ float red[256 * VEC];
    constexpr int U = 8;
    const ColLayout L(txs);
    const int col = (blockIdx.x * L.tx + L.cx) * VEC;
    const int rpc = rows_per_chunk(N);
    const int r0 = blockIdx.y * rpc;
    const int r1 = min(N, r0 + rpc);
    float cs[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) cs[v] = 0.f;
    if (col < C) {
        for (int n0 = r0 + L.ry; n0 < r1; n0 += L.ty * U) {
            float m[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u)
                load_vec<VEC>(M + (size_t)min(n0 + u * L.ty, r1 - 1) * C + col, m[u]);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (n0 + u * L.ty < r1)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) cs[v] += m[u][v];
        }
    }
    fold_row_lanes<VEC>(L, cs, red, part + (size_t)blockIdx.y * C, col, C);
}

// out[col] = (beta ? out[col] : 0) + sum over chunks of part[chunk][col]; scalar columns, the
// chunks spread over the row lanes
__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ part,
                                                            float* __restrict__ out, int chunks,
                                                            int C, int beta, int txs) {
    __shared__ float red[256];
    constexpr int U = 8;
    const ColLayout L(txs);
    const int col = blockIdx.x * L.tx + L.cx;
    float cs[1] = {0.f};
    if (col < C) {
        for (int k0 = L.ry; k0 < chunks; k0 += L.ty * U) {
            float m[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                m[u] = part[(size_t)min(k0 + u * L.ty, chunks - 1) * C + col];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (k0 + u * L.ty < chunks) cs[0] += m[u];
        }
    }
    red[threadIdx.x] = cs[0];
    __syncthreads();
    if (L.ry == 0 && col < C) {
        float s = 0.f;
        for (int r = 0; r < L.ty; ++r) s += red[r * L.tx + L.cx];
        out[col] = beta ? out[col] + s : s;
    }
}

// log2 of the column lanes for a matrix of `cols` column groups: the smallest power of two
// that covers them, at most 256
int col_lane_shift(int cols) {
    int txs = 0;
    while ((1 << txs) < cols && txs < 8) ++txs;
    return txs;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

int colsum_chunks(int N) { const int r = rows_per_chunk(N); return (N + r - 1) / r; }

hipError_t launch_ce_row_stats(const float* Z, const int32_t* y, float* lse, float* rowloss, int N,
                               int O, hipStream_t s) {
    ProfileScope ps(K_CE_ROW_STATS, s);
    hipLaunchKernelGGL(ce_row_stats_kernel, dim3(N), dim3(256), 0, s, Z, y, lse, rowloss, O);
    return hipGetLastError();
}

hipError_t launch_ce_merge_stats(const float* stats, int parts, const float* Z, const int32_t* y,
                                 float* lse, float* rowloss, int N, int O, hipStream_t s) {
    ProfileScope ps(K_CE_ROW_STATS, s);
    hipLaunchKernelGGL(ce_merge_stats_kernel, dim3((N + 3) / 4), dim3(256), 0, s, stats, parts, Z, y, lse,
                       rowloss, N, O);
    return hipGetLastError();
}

hipError_t launch_mse_partial(const float* Z, const float* Y, float* partial, int N, int O,
                              int* n_partial, hipStream_t s) {
    const size_t total = (size_t)N * O;
    const bool vec = total % 4 == 0 && aligned16(Z) && aligned16(Y);
    const size_t quantum = 256 * 4 * 4;  // elements one workgroup covers per loop trip (vector form)
    size_t nb = (total + quantum - 1) / quantum;
    if (nb > 1024) nb = 1024;
    if (nb > (size_t)N) nb = (size_t)N;  // the partials live in the per-row loss buffer
    if (nb < 1) nb = 1;
    size_t per_block = (total + nb - 1) / nb;
    per_block = (per_block + 1023) / 1024 * 1024;
    nb = (total + per_block - 1) / per_block;
    *n_partial = (int)nb;
    ProfileScope ps(K_MSE_ROW_LOSS, s);
    if (vec) hipLaunchKernelGGL(mse_partial_kernel<4>, dim3((unsigned)nb), dim3(256), 0, s, Z, Y, partial, total, per_block);
    else hipLaunchKernelGGL(mse_partial_kernel<1>, dim3((unsigned)nb), dim3(256), 0, s, Z, Y, partial, total, per_block);
    return hipGetLastError();
}

hipError_t launch_loss_reduce(const float* rowloss, int N, float scale, float* loss, hipStream_t s) {
    ProfileScope ps(K_LOSS_REDUCE, s);
    hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(1024), 0, s, rowloss, N, scale, loss);
    return hipGetLastError();
}

hipError_t launch_dz(float* Z, const float* lse, const int32_t* y, const float* Y, float* part,
                     int N, int O, int loss_kind, hipStream_t s) {
    const bool vec = O % 4 == 0 && aligned16(Z) && (loss_kind == 0 || aligned16(Y));
    const int groups = vec ? O / 4 : O;
    const int txs = col_lane_shift(groups);
    dim3 grid((groups + (1 << txs) - 1) >> txs, colsum_chunks(N));
    ProfileScope ps(K_DZ, s);
    const float scale = loss_kind == 0 ? 1.0f / (float)N : (float)(2.0 / ((double)N * (double)O));
#define RNN_DZ(LOSS, VEC) \
    hipLaunchKernelGGL((dz_kernel<LOSS, VEC>), grid, dim3(256), 0, s, Z, lse, y, Y, part, N, O, scale, txs)
    if (loss_kind == 0) { if (vec) RNN_DZ(0, 4); else RNN_DZ(0, 1); }
    else { if (vec) RNN_DZ(1, 4); else RNN_DZ(1, 1); }
#undef RNN_DZ
    return hipGetLastError();
}

hipError_t launch_colsum_partial(const float* M, float* part, int N, int C, hipStream_t s) {
    const bool vec = C % 4 == 0 && aligned16(M);
    const int groups = vec ? C / 4 : C;
    const int txs = col_lane_shift(groups);
    dim3 grid((groups + (1 << txs) - 1) >> txs, colsum_chunks(N));
    ProfileScope ps(K_COLSUM_PARTIAL, s);
    if (vec) hipLaunchKernelGGL(colsum_partial_kernel<4>, grid, dim3(256), 0, s, M, part, N, C, txs);
    else hipLaunchKernelGGL(colsum_partial_kernel<1>, grid, dim3(256), 0, s, M, part, N, C, txs);
    return hipGetLastError();
}

hipError_t launch_colsum_finish(const float* part, float* out, int chunks, int C, int beta,
                                hipStream_t s) {
    // few column lanes per workgroup so that the chunks spread over many row lanes and many
    // workgroups share the columns
    const int txs = col_lane_shift(C < 16 ? C : 16);
    ProfileScope ps(K_COLSUM_FINISH, s);
    hipLaunchKernelGGL(colsum_finish_kernel, dim3((C + (1 << txs) - 1) >> txs), dim3(256), 0, s, part,
                       out, chunks, C, beta, txs);
    return hipGetLastError();
}

}  // namespace rnn
