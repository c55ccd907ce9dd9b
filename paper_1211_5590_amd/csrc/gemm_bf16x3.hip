// Opt-in reduced-precision form of the output layer's three large products (Z = H V + c,
// dV = H^T dZ, G = dZ V^T) on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, 16 times the
// fp32 matrix rate of this chip) with float32 accumulation.  Every float32 operand x is split
// once into two bf16 numbers, hi = bf16(x) and lo = bf16(x - hi), and a product a b is taken as
// hi_a hi_b + hi_a lo_b + lo_a hi_b (three matrix instructions; the dropped lo_a lo_b term and
// the rounding of lo are each below 2^-17 |a b|), so results stay within the float32 path's
// tolerances at a fraction of its matrix time.
//
// One kernel form serves all three products: C[M,N] = A[M,K] B[N,K]^T with both operands stored
// K-contiguous in bf16, which is the layout a matrix instruction wants in its lanes (8
// consecutive k of one row per lane).  Storage of an operand ("split form"): row r holds, for
// every slab of 32 k, the 32 hi values followed by the 32 lo values -- one 128-byte line per row
// and slab, so that the product's requests are whole cache lines; K is zero-padded to a multiple
// of 32 so that the product needs no K tail.  split_kernel brings a float32 matrix into that
// form in one pass, as it is and/or transposed.
//
// Tiling of the product (measured on this chip: the matrix and LDS part of a 128x128 tile runs
// at 70 % of the bf16 peak, but its operand requests, 32 KB per slab and workgroup, saturate
// the 64 bytes per clock of the compute unit's vector memory path and halve that): large
// products run 256x256 tiles (8 wavefronts as 2x4, each 128x64 as 4x2 blocks of 32x32; one
// workgroup per compute unit, half the request bytes per matrix instruction), small ones
// 128x128 tiles (4 wavefronts as 2x2, each 64x64; two workgroups per compute unit).  K advances
// in slabs of 32 through two LDS buffers (next slab global -> registers while the current one
// feeds the matrix cores; the barrier in the loop waits for LDS traffic only).  LDS rows are 64
// bytes per plane (four 16-byte chunks) without padding; chunk c of row r sits at position
// c ^ ((r >> 2) & 3), which makes both the 16-byte writes and the fragment reads (32 rows, one
// chunk) conflict-free.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <math.h>

#include <atomic>

namespace rnn {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int KS = 32;         // K per slab

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

// position (in bf16 elements) of k inside a split-form row: slab * 64 + (k % 32), lo at + 32
__host__ __device__ inline size_t split_pos(int k) { return (size_t)(k / KS) * (2 * KS) + (size_t)(k % KS); }

// A 64x64 float32 tile in LDS (row stride 65) -> its part of the split forms (see split_kernel).
__device__ __forceinline__ void write_split_tile(const float* __restrict__ tile, int r0, int c0, int R, int C,
                                                 uint16_t* __restrict__ rm, uint16_t* __restrict__ tr, int Cp,
                                                 int Rp) {
    constexpr int TS = 65;
    const int tid = threadIdx.x;
    if (rm) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = tid / 8 + 32 * i, c8 = (tid % 8) * 8;
            if (r0 + row < R && c0 + c8 < Cp) {
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = tile[row * TS + c8 + j];
                uint4 hi, lo;
                split8(x, hi, lo);
                uint16_t* at = rm + (size_t)(r0 + row) * (2 * Cp) + split_pos(c0 + c8);
                *reinterpret_cast<uint4*>(at) = hi;
                *reinterpret_cast<uint4*>(at + KS) = lo;
            }
        }
    }
    if (tr) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int col = tid / 8 + 32 * i, r8 = (tid % 8) * 8;
            if (c0 + col < C && r0 + r8 < Rp) {
                float x[8];
#pragma unroll
                for (int j = 0; j < 8; ++j) x[j] = tile[(r8 + j) * TS + col];
                uint4 hi, lo;
                split8(x, hi, lo);
                uint16_t* at = tr + (size_t)(c0 + col) * (2 * Rp) + split_pos(r0 + r8);
                *reinterpret_cast<uint4*>(at) = hi;
                *reinterpret_cast<uint4*>(at + KS) = lo;
            }
        }
    }
}

// src float32 [R,C] (leading dimension ld) -> split form, as it is [R][2 Cp] (rm, nullable) and/or
// transposed [C][2 Rp] (tr, nullable); Cp, Rp = C, R rounded up to 32, pads written as 0.
// One 64x64 tile per workgroup, through LDS.
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
    write_split_tile(tile, r0, c0, R, C, rm, tr, Cp, Rp);
}

// d loss / d z straight into split form: what dz + split_kernel do in two passes over [N,O], in one
// (the float32 dZ is never written: with the split products nothing reads it).  LOSS 0:
// (exp(z - lse) - onehot(y)) * scale; LOSS 1: (z - Y) * scale.  A workgroup walks the 64-row tiles
// of rows [blockIdx.x * rpg, + rpg) of one 64-column strip and leaves the column sums of its rows
// in part[blockIdx.x][O] (for dc; summed in a fixed order).  rpg is a multiple of 64.
template <int LOSS>
__global__ __launch_bounds__(256) void dz_split_kernel(const float* __restrict__ Z, const float* __restrict__ lse,
                                                       const int32_t* __restrict__ y, const float* __restrict__ Y,
                                                       float* __restrict__ part, int N, int O, float scale,
                                                       uint16_t* __restrict__ rm, uint16_t* __restrict__ tr, int Op,
                                                       int Np, int rpg, int vec) {
    constexpr int TS = 65;
    __shared__ float tile[64 * TS];
    const int tid = threadIdx.x;
    const int c0 = blockIdx.y * 64;
    const int r_begin = blockIdx.x * rpg, r_end = min(r_begin + rpg, Np);
    const int c4 = (tid % 16) * 4, gc = c0 + c4;
    float cs[4] = {0.f, 0.f, 0.f, 0.f};
    for (int r0 = r_begin; r0 < r_end; r0 += 64) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = tid / 16 + 16 * i, gr = r0 + row;
            float d[4] = {0.f, 0.f, 0.f, 0.f};
            if (gr < N) {
                const float* p = Z + (size_t)gr * O + gc;
                float zv[4] = {0.f, 0.f, 0.f, 0.f}, tv[4] = {0.f, 0.f, 0.f, 0.f};
                if (vec && gc + 3 < O) {
                    const float4 a = *reinterpret_cast<const float4*>(p);
                    zv[0] = a.x; zv[1] = a.y; zv[2] = a.z; zv[3] = a.w;
                    if (LOSS == 1) {
                        const float4 b = *reinterpret_cast<const float4*>(Y + (size_t)gr * O + gc);
                        tv[0] = b.x; tv[1] = b.y; tv[2] = b.z; tv[3] = b.w;
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (gc + e < O) {
                            zv[e] = p[e];
                            if (LOSS == 1) tv[e] = Y[(size_t)gr * O + gc + e];
                        }
                }
                if (LOSS == 0) {
                    const float l = lse[gr];
                    const int yy = y[gr];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (gc + e < O) d[e] = (__expf(zv[e] - l) - (yy == gc + e ? 1.f : 0.f)) * scale;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (gc + e < O) d[e] = (zv[e] - tv[e]) * scale;
                }
            }
            float* dst = tile + row * TS + c4;
#pragma unroll
            for (int e = 0; e < 4; ++e) { dst[e] = d[e]; cs[e] += d[e]; }
        }
        __syncthreads();
        write_split_tile(tile, r0, c0, N, O, rm, tr, Op, Np);
        __syncthreads();
    }
    // column sums: the 16 row lanes of a column meet in LDS, added in lane order
    float* red = tile;
#pragma unroll
    for (int e = 0; e < 4; ++e) red[(tid / 16) * 64 + c4 + e] = cs[e];
    __syncthreads();
    if (tid < 64 && c0 + tid < O) {
        float sum = 0.f;
        for (int r = 0; r < 16; ++r) sum += red[r * 64 + tid];
        part[(size_t)blockIdx.x * O + c0 + tid] = sum;
    }
}

struct Bf3Params {
    const uint16_t* A;   // split form [M][2 lda]
    const uint16_t* B;   // split form [N][2 ldb]
    float* C;            // final output, or split-K partials [splits][M][N]
    const float* bias_n;
    float* stats;        // as in the float32 product: (max, sum exp) per row and 64-column part
    int M, N;
    int lda, ldb, ldc;   // lda, ldb: padded K in elements (multiples of 32)
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

// WGM x WGN wavefronts, each TM x TN blocks of 32x32
template <int WGM, int WGN, int TM, int TN, bool STATS>
__global__ __launch_bounds__(WGM* WGN * 64) void gemm_bf16x3_kernel(Bf3Params p) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32, NTH = WGM * WGN * 64;
    constexpr int APLANE = BM * 64, BPLANE = BN * 64;       // bytes of one plane of one slab
    constexpr int STAGE = 2 * APLANE + 2 * BPLANE;           // A hi, A lo, B hi, B lo
    constexpr int NA = BM * 8 / NTH, NB = BN * 8 / NTH;      // 16-byte chunks per thread and slab
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];   // [2][STAGE]

    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wm = wave / WGN, wn = wave % WGN;

    int tile_m, tile_n;
    tile_coords_bf3(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int sbeg = blockIdx.z * p.slabs_per_split;
    const int send = min(p.slabs, sbeg + p.slabs_per_split);
    const int nk = send - sbeg;     // every split has at least one slab

    // global -> LDS staging: a row of a slab is 8 chunks (4 hi, 4 lo) = one 128-byte line; rows
    // past the end repeat the last one (their results are never stored)
    const uint16_t* ga[NA];
    const uint16_t* gb[NB];
    int sa_off[NA], sb_off[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int c = tid + NTH * i, row = c / 8, cc = c % 8;
        ga[i] = p.A + (size_t)min(m0 + row, p.M - 1) * (2 * p.lda) + (size_t)sbeg * (2 * KS) + cc * 8;
        sa_off[i] = (cc / 4) * APLANE + lds_chunk(row, cc % 4);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int c = tid + NTH * i, row = c / 8, cc = c % 8;
        gb[i] = p.B + (size_t)min(n0 + row, p.N - 1) * (2 * p.ldb) + (size_t)sbeg * (2 * KS) + cc * 8;
        sb_off[i] = 2 * APLANE + (cc / 4) * BPLANE + lds_chunk(row, cc % 4);
    }
    u32x4 ra[NA], rb[NB];
#define BF3_FETCH(slab)                                                                         \
    do {                                                                                        \
        const size_t k_ = (size_t)(slab) * (2 * KS);                                            \
        _Pragma("unroll") for (int i = 0; i < NA; ++i) ra[i] = *reinterpret_cast<const u32x4*>(ga[i] + k_); \
        _Pragma("unroll") for (int i = 0; i < NB; ++i) rb[i] = *reinterpret_cast<const u32x4*>(gb[i] + k_); \
    } while (0)
#define BF3_PARK(buf)                                                                           \
    do {                                                                                        \
        _Pragma("unroll") for (int i = 0; i < NA; ++i)                                          \
            *reinterpret_cast<u32x4*>(lds + (buf) * STAGE + sa_off[i]) = ra[i];                 \
        _Pragma("unroll") for (int i = 0; i < NB; ++i)                                          \
            *reinterpret_cast<u32x4*>(lds + (buf) * STAGE + sb_off[i]) = rb[i];                 \
    } while (0)

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    BF3_FETCH(0);
    BF3_PARK(0);
    __syncthreads();

    // fragment addresses: row = wave block + 32 i + lane % 32, chunk = 2 s + lane / 32
    int foff_a[TM][2], foff_b[TN][2];   // [block][k step]
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < TM; ++i) foff_a[i][s] = lds_chunk(wm * TM * 32 + 32 * i + lane % 32, 2 * s + lane / 32);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            foff_b[j][s] = 2 * APLANE + lds_chunk(wn * TN * 32 + 32 * j + lane % 32, 2 * s + lane / 32);
    }

    // products of one slab out of LDS buffer `cur` (a literal, so that every offset is an immediate)
#define BF3_COMPUTE(cur)                                                                              \
    _Pragma("unroll") for (int s = 0; s < 2; ++s) {                                                   \
        bf16x8 ah[TM], al[TM], bh[TN], bl[TN];                                                        \
        _Pragma("unroll") for (int i = 0; i < TM; ++i) {                                              \
            ah[i] = *reinterpret_cast<const bf16x8*>(lds + (cur) * STAGE + foff_a[i][s]);             \
            al[i] = *reinterpret_cast<const bf16x8*>(lds + (cur) * STAGE + APLANE + foff_a[i][s]);    \
        }                                                                                             \
        _Pragma("unroll") for (int j = 0; j < TN; ++j) {                                              \
            bh[j] = *reinterpret_cast<const bf16x8*>(lds + (cur) * STAGE + foff_b[j][s]);             \
            bl[j] = *reinterpret_cast<const bf16x8*>(lds + (cur) * STAGE + BPLANE + foff_b[j][s]);    \
        }                                                                                             \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al[i], bh[j], acc[i][j], 0, 0, 0); \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bl[j], acc[i][j], 0, 0, 0); \
        _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                \
            _Pragma("unroll") for (int j = 0; j < TN; ++j)                                            \
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah[i], bh[j], acc[i][j], 0, 0, 0); \
    }

    // A double iteration computes slabs kt and kt + 1 out of LDS buffers 0 and 1.  Requests and
    // parks are unconditional (past the end they repeat the last slab, which nobody reads).
    int kt = 0;
    for (; kt + 1 < nk; kt += 2) {
        BF3_FETCH(kt + 1);
        __builtin_amdgcn_sched_barrier(0);   // keep the requests ahead of the matrix work
        BF3_COMPUTE(0)
        __builtin_amdgcn_sched_barrier(0);
        BF3_PARK(1);
        lds_barrier();
        BF3_FETCH(min(kt + 2, nk - 1));
        __builtin_amdgcn_sched_barrier(0);
        BF3_COMPUTE(1)
        __builtin_amdgcn_sched_barrier(0);
        BF3_PARK(0);
        lds_barrier();
    }
    if (kt < nk) { BF3_COMPUTE(0) }   // odd count: the last slab sits in buffer 0
#undef BF3_COMPUTE
#undef BF3_FETCH
#undef BF3_PARK

    // Accumulator layout of a 32x32 block: lane -> column lane%32; register e -> row
    // 8*(e/4) + 4*(lane/32) + e%4.
    float* Cout = p.C + (p.splits > 1 ? (size_t)blockIdx.z * p.M * p.ldc : 0);
    const bool final_out = p.splits == 1;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * TN * 32 + 32 * j + lane % 32;
            if (col >= p.N) continue;
            const float bias = (final_out && p.bias_n) ? p.bias_n[col] : 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + wm * TM * 32 + 32 * i + 8 * (e / 4) + 4 * (lane / 32) + e % 4;
                if (row < p.M) {
                    float* dst = Cout + (size_t)row * p.ldc + col;
                    float v = acc[i][j][e] + bias;
                    if (final_out && p.beta) v += *dst;
                    *dst = v;
                }
            }
        }

    if constexpr (STATS) if (final_out) {
        static_assert(TN == 2, "a part of the row statistics is 64 columns");
        const int nparts = p.tiles_n * WGN;
        const int part = tile_n * WGN + wn;
        int col[TN];
        float bias[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            col[j] = n0 + wn * TN * 32 + 32 * j + lane % 32;
            bias[j] = (p.bias_n && col[j] < p.N) ? p.bias_n[col[j]] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float v[TN];
                float m = -INFINITY;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    v[j] = acc[i][j][e] + bias[j];
                    if (col[j] < p.N) m = fmaxf(m, v[j]);
                }
                m = max32(m);
                float sum = 0.f;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (col[j] < p.N) sum += __expf(v[j] - m);
                sum = sum32(sum);
                const int row = m0 + wm * TM * 32 + 32 * i + 8 * (e / 4) + 4 * (lane / 32) + e % 4;
                if (lane % 32 == 0 && row < p.M)
                    *reinterpret_cast<float2*>(p.stats + ((size_t)row * nparts + part) * 2) = make_float2(m, sum);
            }
    }
}

// Tile configuration and K cut of a product.
struct Bf3Plan { bool big; int tile, slots, splits, slabs_per_split; };

// Large products: 256x256 tiles, one workgroup per compute unit (256 resident tiles); small ones:
// 128x128 tiles, two per compute unit (512).  A product whose tiles do not fill whole rounds of
// the resident workgroups cuts K (deterministic partials, summed by the float32 path's reduce
// kernel).
Bf3Plan plan_bf3(int M, int N, int K) {
    Bf3Plan pl;
    pl.big = M >= 512 && N >= 512;
    pl.tile = pl.big ? 256 : 128;
    pl.slots = pl.big ? 256 : 512;
    const int tiles = ((M + pl.tile - 1) / pl.tile) * ((N + pl.tile - 1) / pl.tile);
    const int slabs = (K + KS - 1) / KS;
    int splits = 1;
    if (slabs >= 64) {
        const double slots = pl.slots, out_bytes = 4.0 * M * (double)N;
        const double t_full = 6.0 * M * N * (double)K / 1000e12;   // three products at a typical rate
        double best = 1e30;
        const int cap = slabs / 8 < 512 ? slabs / 8 : 512;   // at least 8 slabs (256 of K) per cut
        for (int sp = 1; sp <= cap; ++sp) {
            const double rounds = ceil(tiles * sp / slots) / sp;
            const double t = t_full * rounds * slots / tiles + (sp > 1 ? 2.0 * sp * out_bytes / 3e12 : 0.0);
            if (t < best * 0.97) { best = t; splits = sp; }
        }
    }
    pl.slabs_per_split = (slabs + splits - 1) / splits;
    pl.splits = (slabs + pl.slabs_per_split - 1) / pl.slabs_per_split;
    return pl;
}

template <int WGM, int WGN, int TM, int TN>
hipError_t launch_bf3(const Bf3Params& p, hipStream_t s) {
    constexpr int NTH = WGM * WGN * 64;
    constexpr size_t smem = 2 * (size_t)(2 * WGM * TM * 32 * 64 + 2 * WGN * TN * 32 * 64);
    dim3 grid(p.tiles_m * p.tiles_n, 1, p.splits);
    // per kernel form, once per process (one GPU): allow more than 64 KB of dynamic LDS
    static std::atomic<bool> raised[2];
    if (!raised[p.stats ? 1 : 0].load(std::memory_order_acquire)) {
        hipError_t e = p.stats
            ? hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16x3_kernel<WGM, WGN, TM, TN, true>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)
            : hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16x3_kernel<WGM, WGN, TM, TN, false>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        raised[p.stats ? 1 : 0].store(true, std::memory_order_release);
    }
    if (p.stats) hipLaunchKernelGGL((gemm_bf16x3_kernel<WGM, WGN, TM, TN, true>), grid, dim3(NTH), smem, s, p);
    else hipLaunchKernelGGL((gemm_bf16x3_kernel<WGM, WGN, TM, TN, false>), grid, dim3(NTH), smem, s, p);
    return hipGetLastError();
}



}  // namespace

int bf3_pad(int k) { return (k + KS - 1) / KS * KS; }

size_t bf3_splitk_floats(int M, int N, int K) {
    const Bf3Plan pl = plan_bf3(M, N, K);
    return pl.splits > 1 ? (size_t)pl.splits * M * N : 0;
}

bool bf3_fuses_stats(int M, int N, int K) { return plan_bf3(M, N, K).splits == 1; }

// 64-column parts per row the statistics of an M x N x K product come in
int bf3_stat_parts(int M, int N, int K) {
    const int tile = plan_bf3(M, N, K).tile;
    return (N + tile - 1) / tile * (tile / 64);
}

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

// Z [N,O] -> d loss / d z in split form (as it is and transposed) plus per-chunk column sums in
// part[chunks][O]; *chunks_out (<= colsum_chunks(N)) chunks are written.
hipError_t launch_dz_split(const float* Z, const float* lse, const int32_t* y, const float* Y, float* part, int N,
                           int O, int loss_kind, uint16_t* rowmajor, uint16_t* transposed, int* chunks_out,
                           hipStream_t s) {
    const int Op = bf3_pad(O), Np = bf3_pad(N);
    const int chunks = colsum_chunks(N);
    int rpg = (N + chunks - 1) / chunks;
    rpg = (rpg + 63) / 64 * 64;
    const int used = (Np + rpg - 1) / rpg;          // covers the zero pad rows of the transposed form too
    *chunks_out = used;
    const int vec = (O % 4 == 0 && (reinterpret_cast<uintptr_t>(Z) & 15u) == 0 &&
                     (loss_kind == 0 || (reinterpret_cast<uintptr_t>(Y) & 15u) == 0)) ? 1 : 0;
    dim3 grid(used, (Op + 63) / 64);
    if (grid.y > 65535u) return hipErrorInvalidValue;
    const float scale = loss_kind == 0 ? 1.0f / (float)N : (float)(2.0 / ((double)N * (double)O));
    ProfileScope ps(K_DZ, s);
    if (loss_kind == 0)
        hipLaunchKernelGGL(dz_split_kernel<0>, grid, dim3(256), 0, s, Z, lse, y, Y, part, N, O, scale, rowmajor,
                           transposed, Op, Np, rpg, vec);
    else
        hipLaunchKernelGGL(dz_split_kernel<1>, grid, dim3(256), 0, s, Z, lse, y, Y, part, N, O, scale, rowmajor,
                           transposed, Op, Np, rpg, vec);
    return hipGetLastError();
}

hipError_t launch_gemm_bf16x3(const Bf3Args& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.lda % KS || g.ldb % KS || g.lda < g.K || g.ldb < g.K)
        return hipErrorInvalidValue;
    const Bf3Plan pl = plan_bf3(g.M, g.N, g.K);
    if (pl.splits > 1 && !g.splitk_ws) return hipErrorInvalidValue;
    Bf3Params p;
    p.A = g.A; p.B = g.B; p.bias_n = g.bias_n;
    p.M = g.M; p.N = g.N; p.lda = g.lda; p.ldb = g.ldb;
    p.slabs = (g.K + KS - 1) / KS;
    p.slabs_per_split = pl.slabs_per_split; p.splits = pl.splits; p.beta = g.beta;
    p.tiles_m = (g.M + pl.tile - 1) / pl.tile;
    p.tiles_n = (g.N + pl.tile - 1) / pl.tile;
    p.stats = pl.splits == 1 ? g.row_stats : nullptr;
    if (pl.splits > 1) { p.C = g.splitk_ws; p.ldc = g.N; } else { p.C = g.C; p.ldc = g.ldc; }
    {
        ProfileScope ps(g.prof_id, s);
        const hipError_t e = pl.big ? launch_bf3<2, 4, 4, 2>(p, s) : launch_bf3<2, 2, 2, 2>(p, s);
        if (e != hipSuccess) return e;
    }
    if (pl.splits > 1)
        return launch_splitk_reduce(g.splitk_ws, g.C, g.bias_n, g.M, g.N, g.ldc, pl.splits, g.beta, s);
    return hipSuccess;
}

}  // namespace rnn
