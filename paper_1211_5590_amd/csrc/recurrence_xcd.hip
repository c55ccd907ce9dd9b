// Persistent batched time loop for hidden sizes whose matrix needs many compute units (batch > 4,
// 256 < hidden <= 1024): ONE launch for all steps instead of one launch per step.
//
// The paper's Scan keeps the loop inside one graph node so that nothing per step happens outside
// compiled code (properties 4 and 5) and keeps every state (property 1); the per-step kernel
// boundary of recurrence_step.hip costs more than the step's arithmetic.  Here the chip's layout
// does the work instead: batch rows are independent, so the batch is cut into 8 groups of up to 8
// rows, one group per XCD, and the 32 compute units of an XCD share that group's recurrence.  Every
// workgroup holds 32 output columns of the matrix (all K) in registers for the whole launch and
// produces, per step, the 8 x 32 tile of the new state on the matrix cores (v_mfma_f32_4x4x1 with
// the state broadcast over the column blocks, as in recurrence_mfma.hip; the eight wavefronts split
// K and meet in LDS).  Groups never talk to each other.
//
// Inside a group the new state travels through the L2 cache the 32 compute units share, with no
// flags, fences of the whole cache or kernel boundaries:
//   * the state IS the history: a workgroup stores its tile of h_all[t+1] (forward) or Delta[t]
//     (reverse) with ordinary stores; the first-level cache writes through, so the tile reaches the
//     XCD's L2;
//   * the rows a step will produce were filled with a sentinel (a NaN pattern arithmetic never
//     produces) before the launch; the polling wavefronts of every workgroup invalidate their
//     first-level cache (the acquire half of a device-scope fence), read the group's rows with
//     ordinary loads that hit in the L2, and repeat until no sentinel is left.  Every 4-byte value
//     validates itself, so no ordering between the stores is needed.
// This relies on two properties of the part that the launch checks or that were measured: all
// workgroups of a group run on one XCD (a workgroup takes its group from the XCD it finds itself
// on and its column slice from a per-XCD counter, so the assignment holds by construction whenever
// the 256 workgroups are co-resident: cooperative launch, one workgroup per compute unit), and an
// ordinary store is visible to an invalidate + load of another compute unit of the same XCD
// (measured: 2 M words handed over without a stale one; across XCDs every word was stale, which is
// why groups do not span XCDs).  Every wait is bounded and an expired wait sets the status word.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <stdlib.h>

#include <mutex>
#include <type_traits>

namespace rnn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int XT = 512;            // threads: 8 wavefronts
constexpr int RB = 8;              // batch rows per group
constexpr int CWD = 32;            // output columns per workgroup
constexpr int NGRP = 8;            // groups = XCDs
constexpr int NSLOT = 32;          // workgroups per group
constexpr unsigned kSentinel = 0xFFFFFFFFu;

#ifdef RNN_REC_TRACE
__device__ long long g_xcd_trace[4 * 8];
#define XT_DECL long long xt_prev = clock64(); long long xt_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define XTM(k) do { const long long xt_n = clock64(); xt_acc[k] += xt_n - xt_prev; xt_prev = xt_n; } while (0)
#define XT_COUNT(k, n) do { xt_acc[k] += (n); } while (0)
#define XT_FLUSH(bwd) do { if (grp == 0 && slot == 0 && (tid == 0 || tid == 256)) \
        for (int k_ = 0; k_ < 8; ++k_) g_xcd_trace[((bwd ? 2 : 0) + (tid == 0 ? 0 : 1)) * 8 + k_] = xt_acc[k_]; } while (0)
#else
#define XT_DECL
#define XTM(k)
#define XT_COUNT(k, n)
#define XT_FLUSH(bwd)
#endif

__device__ __forceinline__ void xcd_lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
__device__ __forceinline__ bool fresh(float4 v) {
    return __float_as_uint(v.x) != kSentinel && __float_as_uint(v.y) != kSentinel &&
           __float_as_uint(v.z) != kSentinel && __float_as_uint(v.w) != kSentinel;
}

// Lane layout of the product as in recurrence_mfma.hip: lane l = 32 hf + 4 blk + ri; blocks blk and
// 8 + blk produce columns 4 blk .. 4 blk + 3 of the workgroup's 32 for two different k; the lane
// supplies the B value M[k][c0 + l % 32] and receives rows 0..3 of a row group at that column; the
// state value is broadcast from block abid of each half (cbsz = 3).  KW = k per wavefront.
template <int ACT, bool BWD, int KW>
__global__ __launch_bounds__(XT) void rec_xcd_kernel(RecXcdArgs a) {
    constexpr int NQ = KW / 64;            // 16-byte state reads per lane, row group and step
    constexpr int KP = 8 * KW;             // padded K
    constexpr int LDH = KP + 16;           // LDS row stride: the 4 rows of a read land 16 banks apart
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ int s_abort, s_grp, s_slot;
    __shared__ __attribute__((aligned(16))) int s_stored[4];
    float* hs = smem;                      // [RB][LDH] state, zero padded; columns KW w .. belong to wavefront w alone
    float* part = smem + RB * LDH;         // [2][8 wavefronts][RB][CWD] partial tiles, by step parity

    const int H = a.H, B = a.B, T = a.T;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int hf = lane / 32, blk = (lane % 32) / 4, ri = lane % 4;
    const size_t bh = (size_t)B * H;

    // ---- which group and which column slice: by the XCD this workgroup runs on ------------------
    if (tid == 0) {
        unsigned id;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
        const int xcc = (int)(id & 0xf);
        s_grp = xcc;
        s_slot = xcc < NGRP ? atomicAdd(a.counters + xcc, 1) : NSLOT;
        s_abort = 0;
    }
    if (tid < 4) s_stored[tid] = 0;
    __syncthreads();
    const int grp = s_grp, slot = s_slot;
    const int b0 = grp * RB, c0 = slot * CWD;
    if (grp >= NGRP || slot >= NSLOT) {          // not the layout this kernel is built on
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }
    if (b0 >= B || c0 >= H) return;              // nothing to do here, and nobody waits for this workgroup
    const int nrows = min(RB, B - b0);
    const int col = c0 + lane % 32, colc = min(col, H - 1);

    // ---- resident weights: wreg[j] = M[k][col], k = KW wave + 64 (j / 32) + 32 hf + j % 32,
    //      M = Wh^T (forward) or Wh (reverse); zero outside the matrix ------------------------------
    const int kb = KW * wave;
    float wreg[KW / 2];
#pragma unroll
    for (int j = 0; j < KW / 2; ++j) {
        const int k = kb + 64 * (j / 32) + 32 * hf + (j % 32);
        const int kc = min(k, H - 1);
        wreg[j] = BWD ? a.Wh[(size_t)kc * H + colc] : a.Wh[(size_t)colc * H + kc];
    }
    const float colmask = col < H ? 1.f : 0.f;
#pragma unroll
    for (int j = 0; j < KW / 2; ++j) {
        const int k = kb + 64 * (j / 32) + 32 * hf + (j % 32);
        wreg[j] *= k < H ? colmask : 0.f;
    }

    // ---- initial state of the group's rows (every workgroup of the group computes all of it;
    //      the owner of a column stores it) ----------------------------------------------------------
    for (int i = tid; i < RB * LDH; i += XT) hs[i] = 0.f;
    __syncthreads();
    for (int i = tid; i < RB * H; i += XT) {
        const int m = i / H, j = i - m * H, row = b0 + m;
        if (row >= B) continue;
        float v;
        if (!BWD) {
            v = a.h0 ? a.h0[(size_t)row * H + j] : 0.f;
            if (j >= c0 && j < c0 + CWD) a.hist[(size_t)row * H + j] = v;                  // slot 0
        } else {
            const size_t e = (size_t)(T - 1) * bh + (size_t)row * H + j;
            const float c = a.dh_last ? a.dh_last[(size_t)row * H + j] : 0.f;
            const float h = a.h_all[(size_t)T * bh + (size_t)row * H + j];
            v = (a.G[e] + c) * act_grad<ACT>(h);
            if (j >= c0 && j < c0 + CWD) a.Delta[e] = v;
        }
        hs[m * LDH + j] = v;
    }
    __syncthreads();

    const int nsteps = BWD ? T - 1 : T;

    // ---- epilogue lanes (wavefronts 0..3): lane e finishes row e / 32, column c0 + e % 32 ---------
    const int em = tid / CWD, ec = c0 + tid % CWD;
    const bool e_on = tid < RB * CWD && em < nrows && ec < H;
    const size_t e_off = (size_t)min(b0 + em, B - 1) * H + min(ec, H - 1);
    auto load_epi = [&](int s, float& x0, float& x1) {     // requested two steps ahead, clamped: always valid
        const int sc = max(min(s, nsteps - 1), 0);
        const int t = BWD ? max(T - 2 - sc, 0) : sc;
        const size_t base = (size_t)t * bh;
        if (!BWD) {
            x0 = a.U[base + e_off];
        } else {
            x0 = a.G[base + e_off];
            x1 = a.h_all[base + bh + e_off];
        }
    };
    float n0[2] = {0.f, 0.f}, n1[2] = {0.f, 0.f};
    if (wave < 4) {
        load_epi(0, n0[0], n1[0]);
        load_epi(1, n0[1], n1[1]);
    }

    // ---- polling lanes (wavefronts 4..7): lane pl collects the 16-byte pieces pl + 256 u of the
    //      group's RB x H rows ---------------------------------------------------------------------
    // ---- every wavefront collects the K slice of the state its own product needs (RB rows x KW
    //      columns, produced by KW / 32 workgroups of the group): lane l takes the 16-byte pieces
    //      l + 64 u, piece = (row, 4 columns) ------------------------------------------------------
    constexpr int NP = KW / 32;            // pieces per lane
    int p_goff[NP], p_loff[NP];
    unsigned p_need = 0;
#pragma unroll
    for (int u = 0; u < NP; ++u) {
        const int idx = lane + 64 * u;
        const int m = idx / (KW / 4), c4 = idx - m * (KW / 4);
        const int k = kb + 4 * c4;
        const bool on = m < nrows && k < H;
        p_goff[u] = on ? (b0 + m) * H + k : b0 * H;           // clamped duplicates outside the matrix
        p_loff[u] = m * LDH + k;
        if (on) p_need |= 1u << u;
    }

    XT_DECL;
    // partial tile of this wavefront's K slice: out[rg][i] = rows 4 rg + 2 hf + i
    auto product = [&](float (&out)[2][2]) {
        const float* hc = hs;
#pragma unroll
        for (int rg = 0; rg < 2; ++rg) {
            float areg[4 * NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const float4 v = *reinterpret_cast<const float4*>(hc + (4 * rg + ri) * LDH + kb + 64 * q + 32 * hf + 4 * blk);
                areg[4 * q] = v.x; areg[4 * q + 1] = v.y; areg[4 * q + 2] = v.z; areg[4 * q + 3] = v.w;
            }
            f32x4 acc[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int ab = 0; ab < 8; ++ab)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        // cbsz = 3: each half takes the state value from its block ab
                        switch (ab) {
                            case 0: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 0) * 4 + e], acc[e], 3, 0, 0); break;
                            case 1: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 1) * 4 + e], acc[e], 3, 1, 0); break;
                            case 2: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 2) * 4 + e], acc[e], 3, 2, 0); break;
                            case 3: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 3) * 4 + e], acc[e], 3, 3, 0); break;
                            case 4: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 4) * 4 + e], acc[e], 3, 4, 0); break;
                            case 5: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 5) * 4 + e], acc[e], 3, 5, 0); break;
                            case 6: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 6) * 4 + e], acc[e], 3, 6, 0); break;
                            default: acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * q + e], wreg[(8 * q + 7) * 4 + e], acc[e], 3, 7, 0); break;
                        }
                    }
            const f32x4 p4 = (acc[0] + acc[1]) + (acc[2] + acc[3]);
#pragma unroll
            for (int i = 0; i < 2; ++i) {     // add the two k halves: rows 0,2 in one swap, rows 1,3 in the other
                const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(p4[i]), __float_as_uint(p4[i + 2]), false, false);
                out[rg][i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
            }
        }
    };
    auto park_partial = [&](int par, const float (&out)[2][2]) {
        float* pp = part + par * 8 * RB * CWD;
#pragma unroll
        for (int rg = 0; rg < 2; ++rg)
#pragma unroll
            for (int i = 0; i < 2; ++i) pp[(wave * RB + 4 * rg + 2 * hf + i) * CWD + lane % 32] = out[rg][i];
    };
    auto tile_sum = [&](int par) {            // epilogue lanes: the eight wavefronts' partial sums
        const float* pp = part + par * 8 * RB * CWD;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) v += pp[(w * RB + em) * CWD + tid % CWD];
        return v;
    };
    // This wavefront's K slice of the rows at `src` into its columns of the LDS state, waiting until
    // no sentinel is left.  The first look uses ordinary loads: these rows have never been read by
    // this compute unit, so they miss in its first-level cache and are served by the L2 the group
    // shares (measured: a compute unit takes 32 KB out of the L2 in 1550 clocks at best, which is
    // why every wavefront fetches only what its own product needs and starts that product without
    // waiting for the others).  A piece that was looked at too early holds sentinels and is now cached
    // here; every further look uses device-scope loads, which pass both caches (the tiles are stored
    // with device-scope stores, so they are in memory as well as in the L2).
    auto collect = [&](const float* src) {
        float4 v[NP];
        unsigned need = p_need;
        for (int spins = 0; need != 0; ++spins) {
            XT_COUNT(6, 1);
            if (spins > a.spin_limit) { s_abort = 1; break; }
            if (spins > 0) __builtin_amdgcn_s_sleep(2);
#define RNN_XCD_LOOK4(MOD)                                                                            \
            asm volatile("global_load_dwordx4 %0, %4, off" MOD "\n\t"                                 \
                         "global_load_dwordx4 %1, %5, off" MOD "\n\t"                                 \
                         "global_load_dwordx4 %2, %6, off" MOD "\n\t"                                 \
                         "global_load_dwordx4 %3, %7, off" MOD "\n\t"                                 \
                         "s_waitcnt vmcnt(0)"                                                         \
                         : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3])                         \
                         : "v"(src + p_goff[0]), "v"(src + p_goff[1]), "v"(src + p_goff[2]), "v"(src + p_goff[3]) \
                         : "memory")
#define RNN_XCD_LOOK2(MOD)                                                                            \
            asm volatile("global_load_dwordx4 %0, %2, off" MOD "\n\t"                                 \
                         "global_load_dwordx4 %1, %3, off" MOD "\n\t"                                 \
                         "s_waitcnt vmcnt(0)"                                                         \
                         : "=&v"(v[0]), "=&v"(v[1])                                                   \
                         : "v"(src + p_goff[0]), "v"(src + p_goff[1])                                 \
                         : "memory")
            if constexpr (NP == 4) {
                if (spins == 0) RNN_XCD_LOOK4(""); else RNN_XCD_LOOK4(" sc1");
            } else {
                if (spins == 0) RNN_XCD_LOOK2(""); else RNN_XCD_LOOK2(" sc1");
            }
#undef RNN_XCD_LOOK4
#undef RNN_XCD_LOOK2
#pragma unroll
            for (int u = 0; u < NP; ++u)
                if (fresh(v[u])) need &= ~(1u << u);
        }
#pragma unroll
        for (int u = 0; u < NP; ++u)
            if (p_need & (1u << u)) *reinterpret_cast<float4*>(hs + p_loff[u]) = v[u];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");    // the slice is read back by this wavefront alone
    };

    float last_v = 0.f;
    // One workgroup barrier per step (the partial tiles are complete); the partial buffers alternate by
    // step parity, and no wavefront can be more than one step ahead of the epilogue of its own
    // workgroup, because every later tile of the group needs that epilogue's output.
    auto step = [&](int s, auto slot_c, bool fetch_next) {
        constexpr int SLOT = decltype(slot_c)::value;   // s & 1: partial buffer and operand slot
        float out[2][2];
        XTM(0);
        product(out);
        park_partial(SLOT, out);
        XTM(1);
        xcd_lds_barrier();
        XTM(2);
        const int t = BWD ? T - 2 - s : s;
        float* dst = BWD ? a.Delta + (size_t)t * bh : a.hist + (size_t)(s + 1) * bh;
        if (wave < 4) {
            const float sum = tile_sum(SLOT);
            const float v = BWD ? (sum + n0[SLOT]) * act_grad<ACT>(n1[SLOT]) : activate<ACT>(sum + n0[SLOT]);
            if (e_on) __hip_atomic_store(dst + e_off, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            last_v = v;
            if (lane == 0) s_stored[wave] = s + 1;      // the tile is on its way
            load_epi(s + 2, n0[SLOT], n1[SLOT]);        // the slot is free again (unconditional: exact wait counts)
        }
        XTM(3);
        if (fetch_next) {
            // The other workgroups are in step with this one: look for their tiles a short pause after
            // this workgroup's own tile has been stored.
                        for (int spins = 0; spins < (1 << 16); ++spins) {
                const int4 f = lds_peek4(s_stored);
                if (f.x == s + 1 && f.y == s + 1 && f.z == s + 1 && f.w == s + 1) break;
                __builtin_amdgcn_s_sleep(1);
            }
            for (int k = 0; k < a.first_look_pause; ++k) __builtin_amdgcn_s_sleep(1);
            XTM(4);
            collect(dst);
        }
        XTM(5);
    };

    const bool final_state = BWD && a.dh0 != nullptr;   // delta_0 is needed once more, for dh0
    int s2 = 0;
    bool left = false;
    for (; s2 + 1 < nsteps; s2 += 2) {
        step(s2, std::integral_constant<int, 0>{}, true);
        step(s2 + 1, std::integral_constant<int, 1>{}, s2 + 2 < nsteps || final_state);
        if (s_abort) { left = true; break; }
    }
    if (!left && s2 < nsteps) step(s2, std::integral_constant<int, 0>{}, final_state);
    XT_FLUSH(BWD);
    __syncthreads();
    if (left || s_abort) {
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }
    if (!BWD) {
        if (a.h_last && wave < 4 && e_on) a.h_last[e_off] = nsteps > 0 ? last_v : hs[em * LDH + min(ec, H - 1)];
        return;
    }
    if (a.dh0) {   // dh0 = delta_0 Wh: one more product, no epilogue
        float out[2][2];
        product(out);
        park_partial(0, out);
        __syncthreads();
        if (wave < 4) {
            const float sum = tile_sum(0);
            if (e_on) a.dh0[e_off] = sum;
        }
    }
}

__global__ __launch_bounds__(256) void fill_sentinel_kernel(uint4* __restrict__ p, size_t n16) {
    const uint4 s = make_uint4(kSentinel, kSentinel, kSentinel, kSentinel);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) p[i] = s;
}

template <int ACT, bool BWD>
const void* pick_xcd_kernel(int kw) {
    return kw == 64 ? (const void*)rec_xcd_kernel<ACT, BWD, 64> : (const void*)rec_xcd_kernel<ACT, BWD, 128>;
}

size_t xcd_lds_bytes(int kw) { return ((size_t)RB * (8 * kw + 16) + (size_t)2 * 8 * RB * CWD) * 4; }

}  // namespace

bool rec_xcd_supported(int H, int B) {
    return B > 4 && B <= NGRP * RB && H > 256 && H <= NSLOT * CWD && H % 4 == 0;
}

template <bool BWD>
const void* xcd_kernel_for(int H, int act) {
    const int kw = H <= 512 ? 64 : 128;
    return act == 0 ? pick_xcd_kernel<0, BWD>(kw) : pick_xcd_kernel<1, BWD>(kw);
}

// Can all 256 workgroups be resident at once on the current device (one per compute unit)?  Asked
// once per kernel and device; also raises the kernel's LDS limit.
bool rec_xcd_ready(int H, int act, bool bwd) {
    const void* fn = bwd ? xcd_kernel_for<true>(H, act) : xcd_kernel_for<false>(H, act);
    const size_t lds = xcd_lds_bytes(H <= 512 ? 64 : 128);
    struct Seen { const void* fn; int dev; bool ok; };
    static Seen seen[16];
    static int n_seen = 0;
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < n_seen; ++i)
        if (seen[i].fn == fn && seen[i].dev == dev) return seen[i].ok;
    int per_cu = 0, cus = 0;
    const bool ok = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
                    hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, XT, lds) == hipSuccess &&
                    hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
                    per_cu >= 1 && cus == NGRP * NSLOT;
    if (n_seen < 16) seen[n_seen++] = Seen{fn, dev, ok};
    return ok;
}

hipError_t launch_rec_xcd(const RecXcdArgs& a, bool bwd, hipStream_t s) {
    if (!rec_xcd_supported(a.H, a.B) || a.T < 1) return hipErrorInvalidValue;
    if (!rec_xcd_ready(a.H, a.act, bwd)) return hipErrorNotSupported;
    const int kw = a.H <= 512 ? 64 : 128;
    const void* fn = bwd ? xcd_kernel_for<true>(a.H, a.act) : xcd_kernel_for<false>(a.H, a.act);
    const size_t lds = xcd_lds_bytes(kw);

    // the rows the loop will produce start as sentinels; the slice counters start at zero
    const size_t bh = (size_t)a.B * a.H;
    {
        ProfileScope ps(K_MISC, s);
        hipError_t e = launch_zero_words(a.counters, NGRP, s);
        if (e != hipSuccess) return e;
        float* first = bwd ? a.Delta : a.hist + bh;
        const size_t rows = bwd ? (size_t)(a.T - 1) : (size_t)a.T;
        const size_t n16 = rows * bh / 4;         // H % 4 == 0
        if (n16 > 0) {
            const unsigned blocks = (unsigned)((n16 + 255) / 256 < 2048 ? (n16 + 255) / 256 : 2048);
            hipLaunchKernelGGL(fill_sentinel_kernel, dim3(blocks), dim3(256), 0, s, reinterpret_cast<uint4*>(first), n16);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    ProfileScope ps(bwd ? K_REC_BWD : K_REC_FWD, s);
    RecXcdArgs args = a;
    if (args.spin_limit <= 0) args.spin_limit = wait_limit();
    if (args.first_look_pause <= 0) args.first_look_pause = 6;
#ifdef RNN_REC_TRACE
    if (const char* env = getenv("RNN_XCD_PAUSE")) args.first_look_pause = atoi(env);
#endif
    void* kargs[] = {&args};
    return hipLaunchCooperativeKernel(fn, dim3(NGRP * NSLOT), dim3(XT), kargs, (unsigned)lds, s);
}

}  // namespace rnn

#ifdef RNN_REC_TRACE
extern "C" int rnn_xcd_trace(long long* host_out, int n) {
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(rnn::g_xcd_trace), (size_t)n * 8) == hipSuccess ? 0 : -4;
}
#endif
