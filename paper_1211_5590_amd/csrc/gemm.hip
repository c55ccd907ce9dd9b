// fp32 GEMM on the CDNA4 matrix cores (v_mfma_f32_16x16x4_f32), used for every product that
// the path batches over time outside the loop (the paper's Scan property 8: per-step
// vector-matrix products become one matrix-matrix product): the output projection Z = H V + c,
// its two backward products dV = H^T dZ and G = dZ V^T, the recurrent weight gradient
// dWh = Delta^T H_prev, and the dense-input projections.
//
// Tiling: a 256-thread workgroup (4 wavefronts as 2x2) owns a BM x BN tile of C; each
// wavefront owns (BM/2) x (BN/2) as 16x16 MFMA blocks held in accumulation registers.
// K advances in slabs of 16 through two LDS buffers: the next slab is fetched from global
// memory into registers while the current one feeds the MFMAs, then parked in the other
// buffer (one barrier per slab).  An operand whose K runs along memory keeps that order in LDS
// ([row][16 k], 16-byte chunks XOR-swizzled by row so that both the 16-byte stores and the 16-byte
// fragment reads are conflict-free); an operand stored K-major stays K-major ([k][row], scalar
// fragment reads of 16 consecutive words per quarter-wave).  A wavefront walks the 16 k of a slab
// in the order k = 4(lane/16) + e, the same for both operands, so that one 16-byte read feeds
// four matrix instructions.  Interior tiles
// fetch whole slabs with one uniform base per slab and loop-invariant per-lane offsets; only edge
// tiles and a ragged last slab take the checked path.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <math.h>

namespace rnn {
namespace {

typedef float f32x4v __attribute__((ext_vector_type(4)));

constexpr int BK = 16;
constexpr int PAD = 4;
constexpr int NT = 256;

struct GemmParams {
    const float* A;
    const float* B;
    float* C;          // final output, or split-K partials [splits][M][N]
    const float* bias_n;
    int M, N, K;
    int lda, ldb, ldc;
    int kchunk;        // K range per blockIdx.z (multiple of BK)
    int beta;
    int splits;
    int tiles_m, tiles_n;
    int prof_id;
    float* stats;      // nullable: per row and per 64-column part (max, sum of exp relative to it)
};

// One operand tile of R rows (R = BM or BN) by BK columns of K, fetched into registers.
// KCONTIG: element (r,k) lives at src[r*ld + k]   (A not transposed, or B given as [N,K])
// else   : element (r,k) lives at src[k*ld + r]   (A given as [K,M], or B given as [K,N])
template <int R, bool KCONTIG, bool VEC>
struct TileLoader {
    static constexpr int NV4 = R * BK / 4 / NT;  // float4 per thread
    float4 v[NV4];
    unsigned off[NV4];   // interior tiles: element offset of this lane's float4 from the slab's base
    bool interior;       // uniform over the workgroup: every row of the tile exists, 16-byte loads legal

    __device__ __forceinline__ static void coords(int i, int tid, int& r, int& k) {
        if (KCONTIG) {
            r = tid / 4 + (NT / 4) * i;
            k = (tid % 4) * 4;
        } else {
            constexpr int Q = R / 4;  // float4 per k-row
            const int idx = tid + NT * i;
            k = idx / Q;
            r = (idx % Q) * 4;
        }
    }

    __device__ __forceinline__ void init(int ld, int r0, int rlim, int tid) {
        interior = VEC && r0 + R <= rlim;
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            int r, k;
            coords(i, tid, r, k);
            off[i] = KCONTIG ? (unsigned)r * (unsigned)ld + (unsigned)k : (unsigned)k * (unsigned)ld + (unsigned)r;
        }
    }

    // One slab into registers, to be parked by store().  Interior tiles and whole slabs: one
    // uniform base per slab, loop-invariant lane offsets, no checks; otherwise every limit checked.
    __device__ __forceinline__ void load(const float* __restrict__ src, int ld, int r0, int k0,
                                         int rlim, int klim, int tid) {
        if (interior && k0 + BK <= klim) {
            const float* base = KCONTIG ? src + (size_t)r0 * ld + k0 : src + (size_t)k0 * ld + r0;
#pragma unroll
            for (int i = 0; i < NV4; ++i) v[i] = *reinterpret_cast<const float4*>(base + off[i]);
            return;
        }
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            int r, k;
            coords(i, tid, r, k);
            const int gr = r0 + r, gk = k0 + k;
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
            if (KCONTIG) {
                if (gr < rlim) {
                    const float* p = src + (size_t)gr * ld + gk;
                    if (VEC && gk + 3 < klim) {
                        t = *reinterpret_cast<const float4*>(p);
                    } else {
                        if (gk + 0 < klim) t.x = p[0];
                        if (gk + 1 < klim) t.y = p[1];
                        if (gk + 2 < klim) t.z = p[2];
                        if (gk + 3 < klim) t.w = p[3];
                    }
                }
            } else {
                if (gk < klim) {
                    const float* p = src + (size_t)gk * ld + gr;
                    if (VEC && gr + 3 < rlim) {
                        t = *reinterpret_cast<const float4*>(p);
                    } else {
                        if (gr + 0 < rlim) t.x = p[0];
                        if (gr + 1 < rlim) t.y = p[1];
                        if (gr + 2 < rlim) t.z = p[2];
                        if (gr + 3 < rlim) t.w = p[3];
                    }
                }
            }
            v[i] = t;
        }
    }

    // LDS tile layout: KCONTIG S[r][16] with the 4-float chunk c of row r at position
    // c ^ ((r >> 2) & 3); otherwise S[k][r] with row stride R + PAD
    __device__ __forceinline__ void store(float* __restrict__ S, int tid) const {
#pragma unroll
        for (int i = 0; i < NV4; ++i) {
            int r, k;
            coords(i, tid, r, k);
            if (KCONTIG) *reinterpret_cast<float4*>(&S[r * BK + 4 * ((k / 4) ^ ((r >> 2) & 3))]) = v[i];
            else *reinterpret_cast<float4*>(&S[k * (R + PAD) + r]) = v[i];
        }
    }

    // the four values k = 4g + e (e = 0..3) of tile row `row`
    __device__ __forceinline__ static float4 fragment(const float* __restrict__ S, int row, int g) {
        if (KCONTIG) return *reinterpret_cast<const float4*>(&S[row * BK + 4 * (g ^ ((row >> 2) & 3))]);
        const float* q = S + 4 * g * (R + PAD) + row;
        return make_float4(q[0], q[R + PAD], q[2 * (R + PAD)], q[3 * (R + PAD)]);
    }
};

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (round-robin
// dispatch over 8 dies, each with its own L2), so give every XCD a contiguous band of
// tiles, and inside a band walk down M within a narrow group of N tiles so that the
// workgroups resident together share operand slabs in that die's L2.
__device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
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

template <int BM, int BN, bool AT, bool BT, bool VEC, bool STATS>
__global__ __launch_bounds__(NT) void gemm_f32_kernel(GemmParams p) {
    constexpr int TM = BM / 32, TN = BN / 32;  // 16x16 MFMA blocks per wavefront, per dim
    __shared__ __attribute__((aligned(16))) float As[2][BK * (BM + PAD)];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK * (BN + PAD)];

    const int tid = threadIdx.x;
    const int lane = tid % 64, wave = tid / 64;
    const int wm = wave / 2, wn = wave % 2;

    int tile_m, tile_n;
    tile_coords(blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int kbeg = blockIdx.z * p.kchunk;
    const int kend = min(p.K, kbeg + p.kchunk);
    const int nk = (kend - kbeg + BK - 1) / BK;

    TileLoader<BM, !AT, VEC> la;
    TileLoader<BN, BT, VEC> lb;

    f32x4v acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = (f32x4v){0.f, 0.f, 0.f, 0.f};

    // v_mfma_f32_16x16x4_f32: lane l supplies A[row l%16][k l/16] and B[k l/16][col l%16] and
    // receives C[row 4(l/16) + e][col l%16] in register e.  The 16 k of a slab are walked as
    // k = 4(l/16) + e over four instructions e = 0..3, the same for both operands, so one
    // 16-byte read of a K-ordered tile row feeds all four.
    const int arow = wm * (BM / 2) + lane % 16;
    const int brow = wn * (BN / 2) + lane % 16;
    const int g = lane / 16;

    la.init(p.lda, m0, p.M, tid);
    lb.init(p.ldb, n0, p.N, tid);
    if (nk > 0) {
        la.load(p.A, p.lda, m0, kbeg, p.M, kend, tid);
        lb.load(p.B, p.ldb, n0, kbeg, p.N, kend, tid);
        la.store(As[0], tid);
        lb.store(Bs[0], tid);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) {
            la.load(p.A, p.lda, m0, kbeg + (kt + 1) * BK, p.M, kend, tid);
            lb.load(p.B, p.ldb, n0, kbeg + (kt + 1) * BK, p.N, kend, tid);
        }
        const float* as = As[cur];
        const float* bs = Bs[cur];
        float4 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = TileLoader<BM, !AT, VEC>::fragment(as, arow + 16 * i, g);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = TileLoader<BN, BT, VEC>::fragment(bs, brow + 16 * j, g);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const float av = e == 0 ? fa[i].x : e == 1 ? fa[i].y : e == 2 ? fa[i].z : fa[i].w;
                    const float bv = e == 0 ? fb[j].x : e == 1 ? fb[j].y : e == 2 ? fb[j].z : fb[j].w;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bv, acc[i][j], 0, 0, 0);
                }
        if (more) {
            la.store(As[cur ^ 1], tid);
            lb.store(Bs[cur ^ 1], tid);
        }
        __syncthreads();
    }

    float* Cout = p.C + (p.splits > 1 ? (size_t)blockIdx.z * p.M * p.ldc : 0);
    const bool final_out = p.splits == 1;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = n0 + wn * (BN / 2) + 16 * j + lane % 16;
            if (col >= p.N) continue;
            const float bias = (final_out && p.bias_n) ? p.bias_n[col] : 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int row = m0 + wm * (BM / 2) + 16 * i + 4 * g + e;
                if (row < p.M) {
                    float* dst = Cout + (size_t)row * p.ldc + col;
                    float v = acc[i][j][e] + bias;
                    if (final_out && p.beta) v += *dst;
                    *dst = v;
                }
            }
        }

    // Fused row statistics of a log-sum-exp over the columns: every wavefront leaves, for each of
    // its rows, the maximum of its 64 columns and the sum of exponentials relative to it (the 16
    // lanes of a quarter-wave hold 16 columns of the same row in register e of every block j).
    if (STATS && final_out) {
        const int nparts = p.tiles_n * 2;
        const int part = tile_n * 2 + wn;
        int col[TN];
        float bias[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            col[j] = n0 + wn * (BN / 2) + 16 * j + lane % 16;
            bias[j] = (p.bias_n && col[j] < p.N) ? p.bias_n[col[j]] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v[TN];
                float m = -INFINITY;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    v[j] = acc[i][j][e] + bias[j];
                    if (col[j] < p.N) m = fmaxf(m, v[j]);
                }
                m = max16(m);   // register-to-register lane exchanges: no LDS round trips in the chain
                float sum = 0.f;
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    if (col[j] < p.N) sum += __expf(v[j] - m);
                sum = sum16(sum);
                const int row = m0 + wm * (BM / 2) + 16 * i + 4 * g + e;
                if (lane % 16 == 0 && row < p.M)
                    *reinterpret_cast<float2*>(p.stats + ((size_t)row * nparts + part) * 2) = make_float2(m, sum);
            }
    }
}

// C[m,n] = (beta ? C : 0) + sum_s part[s][m][n] + bias[n], fixed summation order.
// A workgroup owns 16*VEC consecutive outputs; its 256 threads are 16 output lanes times 16
// split lanes, every split lane adds the splits s = lane, lane+16, ... (8 loads in flight) and
// the 16 partial sums are folded through LDS in lane order.
template <int VEC>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part,
                                                            float* __restrict__ C,
                                                            const float* __restrict__ bias, int M,
                                                            int N, int ldc, int splits, int beta) {
    __shared__ float red[256 * VEC];
    constexpr int U = 8;
    const size_t total = (size_t)M * N;
    const int ox = threadIdx.x & 15, sy = threadIdx.x >> 4;
    const size_t idx = ((size_t)blockIdx.x * 16 + ox) * VEC;
    float acc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
    if (idx < total) {
        for (int k0 = sy; k0 < splits; k0 += 16 * U) {
            float m[U][VEC];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float* src = part + (size_t)min(k0 + 16 * u, splits - 1) * total + idx;
                if (VEC == 4) {
                    const float4 a = *reinterpret_cast<const float4*>(src);
                    m[u][0] = a.x; m[u][1 % VEC] = a.y; m[u][2 % VEC] = a.z; m[u][3 % VEC] = a.w;
                } else {
                    m[u][0] = *src;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (k0 + 16 * u < splits)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[v] += m[u][v];
        }
    }
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[threadIdx.x * VEC + v] = acc[v];
    __syncthreads();
    if (sy == 0 && idx < total) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            float s = 0.f;
            for (int r = 0; r < 16; ++r) s += red[(r * 16 + ox) * VEC + v];
            const size_t e = idx + v;
            const int m = (int)(e / N), n = (int)(e % N);
            if (bias) s += bias[n];
            float* dst = C + (size_t)m * ldc + n;
            if (beta) s += *dst;
            *dst = s;
        }
    }
}

constexpr int BM_ = 128, BN_ = 128;

struct SplitPlan {
    int splits, kchunk;
};

// Row tile of a product: 128, or 64 where 128-row tiles would leave most compute units without a
// workgroup (few rows, no K to cut): twice the workgroups keep twice the requests in flight.
int pick_bm(int M, int N, int K) {
    const int tiles = ((M + BM_ - 1) / BM_) * ((N + BN_ - 1) / BN_);
    return (tiles < 128 && K <= 512 && M > 64) ? 64 : 128;
}

SplitPlan plan_split(int M, int N, int K) {
    const int bm_ = pick_bm(M, N, K);
    const int tiles = ((M + bm_ - 1) / bm_) * ((N + BN_ - 1) / BN_);
    int splits = 1;
    if (tiles < 256 && K > 512) {
        const int by_k = (K + 255) / 256;          // at least 256 of K per split
        const int by_fill = (1024 + tiles - 1) / tiles;  // aim at ~4 workgroups per CU
        splits = by_k < by_fill ? by_k : by_fill;
        if (splits < 1) splits = 1;
    } else if (K >= 2048) {
        // Enough tiles to fill the chip, but a whole number of tiles rarely fills whole rounds
        // of the 256 x 3 resident workgroups: 632 tiles leave 18 % of the slots idle.  Cutting K
        // evens the rounds out; the price is the partial-sum traffic and the reduction launch.
        // Pick the cut with the least estimated time.  Without a cut, a last round that leaves
        // every compute unit at most one workgroup is cheap, since a workgroup alone on its unit
        // runs about 2.5 times faster (measured: 1024 tiles take 1.4 rounds, not 2).
        const double slots = 768.0, flops = 2.0 * M * N * (double)K, out_bytes = 4.0 * M * (double)N;
        const double t_full = flops / 100e12;                      // at a typical achieved rate
        double best = 1e30, t_of[9];
        for (int sp = 1; sp <= 8; ++sp) {
            const long units = (long)tiles * sp, whole = units / 768, rem = units % 768;
            const double last = rem == 0 ? 0.0 : (sp == 1 && rem <= 256) ? 0.4 : 1.0;
            const double rounds = ((double)whole + last) / sp;      // in units of one full-K round
            // the slices' partial results are written once more than an uncut result and read back
            // by the reduction, which streams them at about the rate of a copy
            t_of[sp] = t_full * rounds * slots / tiles + (sp > 1 ? (2.0 * sp + 1.0) * out_bytes / 4.5e12 : 0.0);
            if (t_of[sp] < best * 0.97) { best = t_of[sp]; splits = sp; }   // a cut has to pay for itself
        }
        // Among near-equal plans prefer a cut that fills whole rounds exactly.  Measured on the
        // largest such product (16384 x 1024 x 10000): uncut it has two states, 2.64 and 3.17 ms,
        // which differ in how often the workgroups of an XCD share their operand panels through its
        // L2 and which a launch falls into by chance; cut three ways (exactly four rounds) it takes
        // 2.61 ms + 0.04 ms of reduction in either, also under a probe that forces the slow state.
        if (splits == 1)
            for (int sp = 2; sp <= 8; ++sp)
                if ((long)tiles * sp % 768 == 0 && t_of[sp] <= 1.03 * t_of[1]) { splits = sp; break; }
    }
    int kchunk = (K + splits - 1) / splits;
    kchunk = (kchunk + BK - 1) / BK * BK;
    if (kchunk < BK) kchunk = BK;
    splits = (K + kchunk - 1) / kchunk;
    if (splits < 1) splits = 1;
    return {splits, kchunk};
}

template <int BM, int BN, bool AT, bool BT, bool VEC, bool STATS = false>
hipError_t launch_variant(const GemmParams& p, hipStream_t s) {
    dim3 grid(p.tiles_m * p.tiles_n, 1, p.splits);
    ProfileScope ps(p.prof_id, s);
    hipLaunchKernelGGL((gemm_f32_kernel<BM, BN, AT, BT, VEC, STATS>), grid, dim3(NT), 0, s, p);
    return hipGetLastError();
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

int gemm_stat_parts(int N) { return 2 * ((N + BN_ - 1) / BN_); }
bool gemm_fuses_stats(int M, int N, int K) { return plan_split(M, N, K).splits == 1; }

size_t gemm_splitk_floats(int M, int N, int K) {
    const SplitPlan sp = plan_split(M, N, K);
    return sp.splits > 1 ? (size_t)sp.splits * M * N : 0;
}

// The same sum for rows of whole float4 groups: one thread per four consecutive outputs, the
// partials of the K slices added in slice order (eight 16-byte requests in flight per thread), one
// pass over the partial buffer at the rate memory delivers it.
__global__ __launch_bounds__(256) void splitk_reduce_rows4_kernel(const float4* __restrict__ part, float* __restrict__ C,
                                                                  const float* __restrict__ bias, size_t total4,
                                                                  int N4, int ldc, int splits, int beta) {
    constexpr int U = 8;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total4; i += (size_t)gridDim.x * blockDim.x) {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int s0 = 0; s0 < splits; s0 += U) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = part[(size_t)min(s0 + u, splits - 1) * total4 + i];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (s0 + u < splits) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
        }
        const size_t m = i / N4;
        const int n = (int)(i - m * N4) * 4;
        if (bias) {
            const float4 b = *reinterpret_cast<const float4*>(bias + n);
            acc.x += b.x; acc.y += b.y; acc.z += b.z; acc.w += b.w;
        }
        float4* dst = reinterpret_cast<float4*>(C + m * (size_t)ldc + n);
        if (beta) {
            const float4 c = *dst;
            acc.x += c.x; acc.y += c.y; acc.z += c.z; acc.w += c.w;
        }
        *dst = acc;
    }
}

hipError_t launch_splitk_reduce(const float* part, float* C, const float* bias_n, int M, int N, int ldc,
                                int splits, int beta, hipStream_t s) {
    const size_t total = (size_t)M * N;
    ProfileScope ps(K_SPLITK_REDUCE, s);
    // few slices of a large result: stream them; many slices of a small one: the kernel that also
    // spreads the slices over lanes
    if (splits <= 32 && total >= ((size_t)1 << 20) && N % 4 == 0 && ldc % 4 == 0 && aligned16(part) && aligned16(C) &&
        (!bias_n || aligned16(bias_n))) {
        const size_t total4 = total / 4;
        const unsigned blocks = (unsigned)((total4 + 255) / 256 < 4096 ? (total4 + 255) / 256 : 4096);
        hipLaunchKernelGGL(splitk_reduce_rows4_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<const float4*>(part),
                           C, bias_n, total4, N / 4, ldc, splits, beta);
        return hipGetLastError();
    }
    if (total % 4 == 0) {  // the partial buffer is 16-byte aligned workspace
        const unsigned blocks = (unsigned)((total / 4 + 15) / 16);
        hipLaunchKernelGGL(splitk_reduce_kernel<4>, dim3(blocks), dim3(256), 0, s, part, C, bias_n, M, N, ldc,
                           splits, beta);
    } else {
        const unsigned blocks = (unsigned)((total + 15) / 16);
        hipLaunchKernelGGL(splitk_reduce_kernel<1>, dim3(blocks), dim3(256), 0, s, part, C, bias_n, M, N, ldc,
                           splits, beta);
    }
    return hipGetLastError();
}

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
    const SplitPlan sp = plan_split(g.M, g.N, g.K);
    if (sp.splits > 1 && !g.splitk_ws) return hipErrorInvalidValue;
    const int bm = pick_bm(g.M, g.N, g.K), bn = BN_;

    GemmParams p;
    p.A = g.A; p.B = g.B; p.bias_n = g.bias_n;
    p.M = g.M; p.N = g.N; p.K = g.K;
    p.lda = g.lda; p.ldb = g.ldb;
    p.stats = sp.splits == 1 ? g.row_stats : nullptr;
    p.kchunk = sp.kchunk; p.beta = g.beta; p.splits = sp.splits; p.prof_id = g.prof_id;
    p.tiles_m = (g.M + bm - 1) / bm;
    p.tiles_n = (g.N + bn - 1) / bn;
    if (sp.splits > 1) { p.C = g.splitk_ws; p.ldc = g.N; } else { p.C = g.C; p.ldc = g.ldc; }

    // float4 global loads need 16-byte aligned bases, leading dimensions that are multiples
    // of 4, and split boundaries that keep every 4-group inside the valid range (kchunk is a
    // multiple of 16).  The loaders check the per-element limits themselves.
    const bool vec = aligned16(g.A) && aligned16(g.B) && g.lda % 4 == 0 && g.ldb % 4 == 0;

    hipError_t e;
#define RNN_GEMM_DISPATCH(AT, BT)                                                                \
    do {                                                                                         \
        if (bm == 64) e = vec ? launch_variant<64, BN_, AT, BT, true>(p, s) : launch_variant<64, BN_, AT, BT, false>(p, s); \
        else e = vec ? launch_variant<BM_, BN_, AT, BT, true>(p, s) : launch_variant<BM_, BN_, AT, BT, false>(p, s);      \
    } while (0)
    if (p.stats) {   // only the plain-layout product (the output projection) carries the statistics
        if (g.a_t || g.b_t) return hipErrorInvalidValue;
        if (bm == 64) e = vec ? launch_variant<64, BN_, false, false, true, true>(p, s)
                              : launch_variant<64, BN_, false, false, false, true>(p, s);
        else e = vec ? launch_variant<BM_, BN_, false, false, true, true>(p, s)
                     : launch_variant<BM_, BN_, false, false, false, true>(p, s);
    } else if (!g.a_t && !g.b_t) RNN_GEMM_DISPATCH(false, false);
    else if (g.a_t && !g.b_t) RNN_GEMM_DISPATCH(true, false);
    else if (!g.a_t && g.b_t) RNN_GEMM_DISPATCH(false, true);
    else RNN_GEMM_DISPATCH(true, true);
#undef RNN_GEMM_DISPATCH
    if (e != hipSuccess) return e;

    if (sp.splits > 1) e = launch_splitk_reduce(g.splitk_ws, g.C, g.bias_n, g.M, g.N, g.ldc, sp.splits, g.beta, s);
    return e;
}

}  // namespace rnn
