// Opt-in reduced-precision form of the output layer's three large products (Z = H V + c,
// dV = H^T dZ, G = dZ V^T) on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, 16 times the
// fp32 matrix rate of this chip) with float32 accumulation.  Every float32 operand x is split
// once into two bf16 numbers, hi = bf16(x) and lo = bf16(x - hi), and a product a b is taken as
// hi_a hi_b + hi_a lo_b + lo_a hi_b (three matrix instructions; the dropped lo_a lo_b term and
// the rounding of lo are each below 2^-17 |a b|), so results stay within the float32 path's
// tolerances at a fifth of its matrix time.
//
// One kernel form serves all three products: C[M,N] = A[M,K] B[N,K]^T with both operands stored
// K-contiguous as bf16 planes (hi plane, lo plane), which is the layout a matrix instruction
// wants in its lanes (8 consecutive k of one row per lane).  The operands are brought into that
// form by split_kernel, one pass that writes the row-major and/or the transposed planes of a
// float32 matrix, zero-padded to multiples of 32 in K so that the product needs no K tail.
//
// Tiling of the product: 256 threads (4 wavefronts as 2x2) own a 128x128 tile, each wavefront
// 64x64 as 2x2 blocks of 32x32; K advances in slabs of 32 through two LDS buffers (next slab
// global -> registers while the current one feeds the matrix cores).  LDS rows are 64 bytes
// (four 16-byte chunks) without padding; chunk c of row r sits at position c ^ ((r >> 2) & 3),
// which makes both the 16-byte writes (4 lanes per row) and the fragment reads (32 rows, one
// chunk) conflict-free.  64 KB of LDS per workgroup: two workgroups per compute unit.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <math.h>

namespace rnn {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int TB = 128;        // tile edge (rows of A and rows of B per workgroup)
constexpr int KS = 32;         // K per slab
constexpr int NT = 256;
constexpr int PLANE = TB * KS * 2;   // bytes of one operand plane of one slab in LDS (8 KB)

// hi/lo split of 8 floats into two packed bf16x8 (round to nearest even both times)
__device__ __forceinline__ void split8(const float (&x)[8], uint4& hi, uint4& lo) {
    unsigned h[4], l[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const f32x2 v = {x[2 * p], x[2 * p + 1]};
        h[p] = __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
        const f32x2 r = {x[2 * p] - __uint_as_float(h[p] << 16), x[2 * p + 1] - __uint_as_float(h[p] & 0xffff0000u)};
        l[p] = __builtin_bit_cast(unsigned, __builtin_convertvector(r, bf16x2));
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
}

// src float32 [R,C] (leading dimension ld) -> bf16 hi/lo planes, row-major [R][Cp] (rm, nullable)
// and/or transposed [C][Rp] (tr, nullable); Cp, Rp = C, R rounded up to 32, pads written as 0.
// A plane pair is hi followed by lo.  One 64x64 tile per workgroup, through LDS.
__global__ __launch_bounds__(256) void split_kernel(const float* __restrict__ src, int R, int C, int ld,
                                                    uint16_t* __restrict__ rm, uint16_t* __restrict__ tr,
                                                    int Cp, int Rp, int vec) {
    constexpr int TS = 65;
    __shared__ float tile[64 * TS];
    const int tid = threadIdx.x;
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = tid / 16 + 16 * i, c4 = (tid % 16) * 4;
        const int gr = r0 + row, gc = c0 + c4;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (gr < R) {
            const float* p = src + (size_t)gr * ld + gc;
            if (vec && gc + 3 < C) {
                t = *reinterpret_cast<const float4*>(p);
            } else {
                if (gc + 0 < C) t.x = p[0];
                if (gc + 1 < C) t.y = p[1];
                if (gc + 2 < C) t.z = p[2];
                if (gc + 3 < C) t.w = p[3];
            }
        }
        float* d = tile + row * TS + c4;
        d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w;
    }
    __syncthreads();
    if (rm) {
        uint16_t* lo_plane = rm + (size_t)R * Cp;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = tid / 8 + 32 * i, c8 = (tid % 8) * 8;
            if (r0 + row < R && c0 + c8 < Cp) {
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = tile[row * TS + c8 + j];
                uint4 hi, lo;
                split8(x, hi, lo);
                const size_t at = (size_t)(r0 + row) * Cp + c0 + c8;
                *reinterpret_cast<uint4*>(rm + at) = hi;
                *reinterpret_cast<uint4*>(lo_plane + at) = lo;
            }
        }
    }
    if (tr) {
        uint16_t* lo_plane = tr + (size_t)C * Rp;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int col = tid / 8 + 32 * i, r8 = (tid % 8) * 8;
            if (c0 + col < C && r0 + r8 < Rp) {
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = tile[(r8 + j) * TS + col];
                uint4 hi, lo;
                split8(x, hi, lo);
                const size_t at = (size_t)(c0 + col) * Rp + r0 + r8;
                *reinterpret_cast<uint4*>(tr + at) = hi;
                *reinterpret_cast<uint4*>(lo_plane + at) = lo;
            }
        }
    }
}

struct Bf3Params {
    const uint16_t* A;   // hi plane [M][lda], lo plane follows at A + M*lda
    const uint16_t* B;   // hi plane [N][ldb], lo plane follows at B + N*ldb
    float* C;            // final output, or split-K partials [splits][M][N]
    const float* bias_n;
    float* stats;        // as in the float32 product: (max, sum exp) per row and 64-column part
    int M, N;
    int lda, ldb, ldc;   // lda, ldb in elements, multiples of 32
    int slabs;           // K slabs of 32 in total
    int slabs_per_split;
    int splits, beta;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ void tile_coords_bf3(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
    // each XCD (round-robin over 8 dies) gets a contiguous band of tiles; inside a band walk down M
    // within a narrow group of N tiles so that co-resident workgroups share operand slabs in L2
    const int total = tiles_m * tiles_n;
    int id = bid;
    const int per = total / 8;
    if (per > 0 && bid < per * 8) id = (bid % 8) * per + bid / 8;
    constexpr int GROUP_N = 4;
    const int group = id / (GROUP_N * tiles_m);
    const int first_n = group * GROUP_N;
    const int gsz = min(GROUP_N, tiles_n - first_n);
    const int in_group = id - group * GROUP_N * tiles_m;
    tn = first_n + in_group % gsz;
    tm = in_group / gsz;
}

// byte offset of chunk c (16 bytes = 8 bf16 of k) of row r inside one LDS plane
__device__ __forceinline__ int lds_chunk(int r, int c) { return r * 64 + ((c ^ ((r >> 2) & 3)) << 4); }

template <bool STATS>
__global__ __launch_bounds__(NT) void gemm_bf16x3_kernel(Bf3Params p) {
    // [buffer][A hi, A lo, B hi, B lo]
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][4][PLANE];

    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wm = wave / 2, wn = wave % 2;

    int tile_m, tile_n;
    tile_coords_bf3(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int m0 = tile_m * TB, n0 = tile_n * TB;
    const int sbeg = blockIdx.z * p.slabs_per_split;
    const int send = min(p.slabs, sbeg + p.slabs_per_split);
    const int nk = send - sbeg;

    // global -> LDS staging: per plane 128 rows x 4 chunks = 512 chunks, two per thread
    const int srow = tid / 4, schunk = tid % 4;
    // rows past the end repeat the last one (their results are never stored)
    const int ra0 = min(m0 + srow, p.M - 1), ra1 = min(m0 + srow + 64, p.M - 1);
    const int rb0 = min(n0 + srow, p.N - 1), rb1 = min(n0 + srow + 64, p.N - 1);
    const size_t kofs = (size_t)sbeg * KS + schunk * 8;
    const uint16_t* ga00 = p.A + (size_t)ra0 * p.lda + kofs;        // [row half][hi, lo]
    const uint16_t* ga10 = p.A + (size_t)ra1 * p.lda + kofs;
    const uint16_t* ga01 = ga00 + (size_t)p.M * p.lda;
    const uint16_t* ga11 = ga10 + (size_t)p.M * p.lda;
    const uint16_t* gb00 = p.B + (size_t)rb0 * p.ldb + kofs;
    const uint16_t* gb10 = p.B + (size_t)rb1 * p.ldb + kofs;
    const uint16_t* gb01 = gb00 + (size_t)p.N * p.ldb;
    const uint16_t* gb11 = gb10 + (size_t)p.N * p.ldb;
    const int soff0 = lds_chunk(srow, schunk), soff1 = lds_chunk(srow + 64, schunk);

    u32x4 st0, st1, st2, st3, st4, st5, st6, st7;
#define BF3_FETCH(slab)                                                              \
    do {                                                                             \
        const size_t k_ = (size_t)(slab) * KS;                                       \
        st0 = *reinterpret_cast<const u32x4*>(ga00 + k_);                          \
        st1 = *reinterpret_cast<const u32x4*>(ga10 + k_);                          \
        st2 = *reinterpret_cast<const u32x4*>(ga01 + k_);                          \
        st3 = *reinterpret_cast<const u32x4*>(ga11 + k_);                          \
        st4 = *reinterpret_cast<const u32x4*>(gb00 + k_);                          \
        st5 = *reinterpret_cast<const u32x4*>(gb10 + k_);                          \
        st6 = *reinterpret_cast<const u32x4*>(gb01 + k_);                          \
        st7 = *reinterpret_cast<const u32x4*>(gb11 + k_);                          \
    } while (0)
#define BF3_PARK(buf)                                                                \
    do {                                                                             \
        *reinterpret_cast<u32x4*>(&lds[buf][0][soff0]) = st0;                      \
        *reinterpret_cast<u32x4*>(&lds[buf][0][soff1]) = st1;                      \
        *reinterpret_cast<u32x4*>(&lds[buf][1][soff0]) = st2;                      \
        *reinterpret_cast<u32x4*>(&lds[buf][1][soff1]) = st3;                      \
        *reinterpret_cast<u32x4*>(&lds[buf][2][soff0]) = st4;                      \
        *reinterpret_cast<u32x4*>(&lds[buf][2][soff1]) = st5;                      \
        *reinterpret_cast<u32x4*>(&lds[buf][3][soff0]) = st6;                      \
        *reinterpret_cast<u32x4*>(&lds[buf][3][soff1]) = st7;                      \
    } while (0)

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    if (nk > 0) {
        BF3_FETCH(sbeg * 0);
        BF3_PARK(0);
    }
    __syncthreads();

    // fragment addresses: row = wave block + 32 i + lane % 32, chunk = 2 s + lane / 32
    int foff_a[2][2], foff_b[2][2];   // [i or j][k step]
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            foff_a[i][s] = lds_chunk(wm * 64 + 32 * i + lane % 32, 2 * s + lane / 32);
            foff_b[i][s] = lds_chunk(wn * 64 + 32 * i + lane % 32, 2 * s + lane / 32);
        }

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) BF3_FETCH(kt + 1);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 ah[2], al[2], bh[2], bl[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                ah[i] = *reinterpret_cast<const bf16x8*>(&lds[cur][0][foff_a[i][s]]);
                al[i] = *reinterpret_cast<const bf16x8*>(&lds[cur][1][foff_a[i][s]]);
                bh[i] = *reinterpret_cast<const bf16x8*>(&lds[cur][2][foff_b[i][s]]);
                bl[i] = *reinterpret_cast<const bf16x8*>(&lds[cur][3][foff_b[i][s]]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0);
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0);
                }
        }
        if (more) BF3_PARK(cur ^ 1);
        __syncthreads();
    }

    // Accumulator layout of a 32x32 block: lane -> column lane%32; register e -> row
    // 8*(e/4) + 4*(lane/32) + e%4.
    float* Cout = p.C + (p.splits > 1 ? (size_t)blockIdx.z * p.M * p.ldc : 0);
    const bool final_out = p.splits == 1;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + 32 * j + lane % 32;
            if (col >= p.N) continue;
            const float bias = (final_out && p.bias_n) ? p.bias_n[col] : 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm * 64 + 32 * i + 8 * (e / 4) + 4 * (lane / 32) + e % 4;
                if (row < p.M) {
                    float* dst = Cout + (size_t)row * p.ldc + col;
                    float v = acc[i][j][e] + bias;
                    if (final_out && p.beta) v += *dst;
                    *dst = v;
                }
            }
        }

    if (STATS && final_out) {
        const int nparts = p.tiles_n * 2;
        const int part = tile_n * 2 + wn;
        int col[2];
        float bias[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            col[j] = n0 + wn * 64 + 32 * j + lane % 32;
            bias[j] = (p.bias_n && col[j] < p.N) ? p.bias_n[col[j]] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float v[2];
                float m = -INFINITY;
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    v[j] = acc[i][j][e] + bias[j];
                    if (col[j] < p.N) m = fmaxf(m, v[j]);
                }
                m = max32(m);
                float sum = 0.f;
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    if (col[j] < p.N) sum += __expf(v[j] - m);
                sum = sum32(sum);
                const int row = m0 + wm * 64 + 32 * i + 8 * (e / 4) + 4 * (lane / 32) + e % 4;
                if (lane % 32 == 0 && row < p.M)
                    *reinterpret_cast<float2*>(p.stats + ((size_t)row * nparts + part) * 2) = make_float2(m, sum);
            }
    }
}

struct Bf3Split { int splits, slabs_per_split; };

// Two workgroups per compute unit: 512 resident tiles.  A product whose tiles do not fill whole
// rounds of them cuts K (deterministic partials, summed by the float32 path's reduce kernel).
Bf3Split plan_bf3(int M, int N, int K) {
    const int tiles = ((M + TB - 1) / TB) * ((N + TB - 1) / TB);
    const int slabs = (K + KS - 1) / KS;
    int splits = 1;
    if (slabs >= 64) {
        const double slots = 512.0, out_bytes = 4.0 * M * (double)N;
        const double t_full = 6.0 * M * N * (double)K / 800e12;   // three products at a typical rate
        double best = 1e30;
        const int cap = slabs / 32 < 16 ? slabs / 32 : 16;
        for (int sp = 1; sp <= cap; ++sp) {
            const double rounds = ceil(tiles * sp / slots) / sp;
            const double t = t_full * rounds * slots / tiles + (sp > 1 ? 2.0 * sp * out_bytes / 3e12 : 0.0);
            if (t < best * 0.97) { best = t; splits = sp; }
        }
    }
    int per = (slabs + splits - 1) / splits;
    splits = (slabs + per - 1) / per;
    return {splits, per};
}

}  // namespace

int bf3_pad(int k) { return (k + KS - 1) / KS * KS; }

size_t bf3_splitk_floats(int M, int N, int K) {
    const Bf3Split sp = plan_bf3(M, N, K);
    return sp.splits > 1 ? (size_t)sp.splits * M * N : 0;
}

bool bf3_fuses_stats(int M, int N, int K) { return plan_bf3(M, N, K).splits == 1; }

hipError_t launch_split_bf16(const float* src, int R, int C, int ld, uint16_t* rowmajor, uint16_t* transposed,
                             hipStream_t s) {
    if (R <= 0 || C <= 0) return hipErrorInvalidValue;
    const int vec = ((reinterpret_cast<uintptr_t>(src) & 15u) == 0 && ld % 4 == 0) ? 1 : 0;
    // tiles also cover the zero pads of both outputs
    const int Cp = bf3_pad(C), Rp = bf3_pad(R);
    dim3 grid((Rp + 63) / 64, (Cp + 63) / 64);   // the long dimension of this path's matrices is R
    if (grid.y > 65535u) return hipErrorInvalidValue;
    ProfileScope ps(K_SPLIT_BF16, s);
    hipLaunchKernelGGL(split_kernel, grid, dim3(256), 0, s, src, R, C, ld, rowmajor, transposed, Cp, Rp, vec);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16x3(const Bf3Args& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.lda % KS || g.ldb % KS || g.lda < g.K || g.ldb < g.K)
        return hipErrorInvalidValue;
    const Bf3Split sp = plan_bf3(g.M, g.N, g.K);
    if (sp.splits > 1 && !g.splitk_ws) return hipErrorInvalidValue;
    Bf3Params p;
    p.A = g.A; p.B = g.B; p.bias_n = g.bias_n;
    p.M = g.M; p.N = g.N; p.lda = g.lda; p.ldb = g.ldb;
    p.slabs = (g.K + KS - 1) / KS;
    p.slabs_per_split = sp.slabs_per_split; p.splits = sp.splits; p.beta = g.beta;
    p.tiles_m = (g.M + TB - 1) / TB;
    p.tiles_n = (g.N + TB - 1) / TB;
    p.stats = sp.splits == 1 ? g.row_stats : nullptr;
    if (sp.splits > 1) { p.C = g.splitk_ws; p.ldc = g.N; } else { p.C = g.C; p.ldc = g.ldc; }
    dim3 grid(p.tiles_m * p.tiles_n, 1, sp.splits);
    {
        ProfileScope ps(g.prof_id, s);
        if (p.stats) hipLaunchKernelGGL(gemm_bf16x3_kernel<true>, grid, dim3(NT), 0, s, p);
        else hipLaunchKernelGGL(gemm_bf16x3_kernel<false>, grid, dim3(NT), 0, s, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (sp.splits > 1)
        return launch_splitk_reduce(g.splitk_ws, g.C, g.bias_n, g.M, g.N, g.ldc, sp.splits, g.beta, s);
    return hipSuccess;
}

}  // namespace rnn
