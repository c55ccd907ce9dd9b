// Persistent batched time loop for hidden sizes whose matrix needs many compute units (batch > 4,
// 256 < hidden <= 1024): ONE launch for all steps instead of one launch per step.
//
// The paper's Scan keeps the loop inside one graph node so that nothing per step happens outside
// compiled code (properties 4 and 5) and keeps every state (property 1); the per-step kernel
// boundary of recurrence_step.hip costs more than the step's arithmetic.  Here the chip's layout
// does the work instead: batch rows are independent, so the batch is cut into 16 groups of up to 4
// rows, two groups per XCD (groups x and x + 8 on XCD x), and 16 of the 32 compute units of an XCD
// share one group's recurrence.  Every workgroup holds 64 output columns of the matrix (all K) in
// registers for the whole launch and produces, per step, the 4 x 64 tile of the new state on the
// matrix cores; the eight wavefronts split K and meet in LDS.  Groups never talk to each other.
//
// Matrix instruction: v_mfma_f32_4x4x1 with the state broadcast over all 16 column blocks
// (cbsz = 4): lane l supplies the matrix value M[k][c0 + l] of one k per instruction and the state
// value of row l % 4 for the 16 k of its block l / 4, and receives rows 0..3 at column c0 + l.  The
// 16-byte piece of the state a lane fetches from memory (row l % 4, four consecutive k) is exactly
// what it feeds the instruction, so the state goes from the cache into the operand registers
// without passing LDS.
//
// Inside a group the new state travels through the L2 cache its compute units share, with no flags,
// no fences and no kernel boundaries:
//   * the state IS the history: a workgroup stores its tile of h_all[t+1] (forward) or Delta[t]
//     (reverse) with device-scope stores;
//   * the rows a step will produce were filled with a bit pattern arithmetic never produces (an
//     all-ones NaN) before the launch; every wavefront fetches the K slice its own product needs and
//     repeats until no such word is left.  Every 4-byte value validates itself, so no ordering between
//     the stores is needed.  The first look uses ordinary loads (lines this compute unit has never
//     cached: they are served by the XCD's L2); a look that came too early has left stale lines in the
//     first-level cache, so later looks use device-scope loads, which pass it.
// A workgroup takes its group from the XCD it finds itself on and its column slice from a per-XCD
// counter, so all workgroups of a group share one L2 by construction whenever the 256 workgroups are
// co-resident (cooperative launch, one workgroup per compute unit: checked before the launch).
// Every wait is bounded, and an expired wait sets the status word.
//
// Measured (H = 1024, batch 64, in-kernel clock): a step takes about 5300 clocks: 1150 for a
// wavefront's 128 matrix instructions, 400 for the epilogue, and about 2000 between the request
// for the new state and its arrival, which neither the bytes (4 or 8 rows per group), nor the scope
// of the store, nor how long the request waits after the store, nor having the lines in the L2
// before they are written changes; a request for rows written one step earlier returns in 400.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <stdlib.h>

#include <mutex>
#include <type_traits>
#include <utility>

namespace rnn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int XT = 512;            // threads: 8 wavefronts
constexpr int RB = 4;              // batch rows per group
constexpr int CWD = 64;            // output columns per workgroup
constexpr int NXCD = 8;            // XCDs: the layout this loop is built on
constexpr int WG_PER_XCD = 32;     // compute units per XCD = workgroups per XCD
constexpr int NSLOT = 16;          // workgroups per group
constexpr int NGRP = 16;           // groups: x and x + 8 on XCD x
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

// 64 matrix instructions: the four values of one state piece against 64 k of the matrix, block AB
// of the lanes supplying the state (abid) for k = 4 AB + e
template <int... AB>
__device__ __forceinline__ void mfma_blocks(const float4 st, const float* __restrict__ w, f32x4 (&acc)[4],
                                            std::integer_sequence<int, AB...>) {
    ((acc[0] = __builtin_amdgcn_mfma_f32_4x4x1f32(st.x, w[4 * AB + 0], acc[0], 4, AB, 0),
      acc[1] = __builtin_amdgcn_mfma_f32_4x4x1f32(st.y, w[4 * AB + 1], acc[1], 4, AB, 0),
      acc[2] = __builtin_amdgcn_mfma_f32_4x4x1f32(st.z, w[4 * AB + 2], acc[2], 4, AB, 0),
      acc[3] = __builtin_amdgcn_mfma_f32_4x4x1f32(st.w, w[4 * AB + 3], acc[3], 4, AB, 0)),
     ...);
}

// KW = k per wavefront (8 KW >= H)
template <int ACT, bool BWD, int KW>
__global__ __launch_bounds__(XT) void rec_xcd_kernel(RecXcdArgs a) {
    constexpr int NQ = KW / 64;            // 16-byte state pieces per lane and step
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ int s_abort, s_grp, s_slot;
    __shared__ __attribute__((aligned(16))) int s_stored[4];
    float* part = smem;                    // [2][8 wavefronts][RB][CWD] partial tiles, by step parity

    const int H = a.H, B = a.B, T = a.T;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int ri = lane % 4, kg = lane / 4;
    const size_t bh = (size_t)B * H;

    // ---- which group and which column slice: by the XCD this workgroup runs on ------------------
    if (tid == 0) {
        unsigned id;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
        const int xcc = (int)(id & 0xf);
        const int n = xcc < NXCD ? atomicAdd(a.counters + xcc, 1) : WG_PER_XCD;
        s_grp = n < WG_PER_XCD ? xcc + NXCD * (n / NSLOT) : NGRP;
        s_slot = n % NSLOT;
        s_abort = 0;
    }
    if (tid < 4) s_stored[tid] = 0;
    __syncthreads();
    const int grp = s_grp, slot = s_slot;
    const int b0 = grp * RB, c0 = slot * CWD;
    if (grp >= NGRP) {                           // not the layout this kernel is built on
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }
    if (b0 >= B || c0 >= H) return;              // nothing to do here, and nobody waits for this workgroup
    const int nrows = min(RB, B - b0);
    const int col = c0 + lane, colc = min(col, H - 1);

    // ---- resident weights: wreg[j] = M[kb + j][col], M = Wh^T (forward) or Wh (reverse); zero
    //      outside the matrix ----------------------------------------------------------------------
    const int kb = KW * wave;
    float wreg[KW];
    if (BWD) {
        // M[k][col] = Wh[k][col]: a lane's values lie along a column of Wh.  Fetched as 16-byte pieces
        // along the rows (a request covers four k of 256 bytes) into a wavefront-private LDS tile
        // [64 k][64 columns], 64 k at a time, from which every lane takes its column.
        float* stg = smem + wave * 64 * 65;
        const int r4 = lane >> 4, c4 = 4 * (lane & 15);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            float4 v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int k = kb + 64 * q + r4 + 4 * i, cc = c0 + c4;
                const bool on = k < H && cc < H;                     // H % 4 == 0: a piece is inside or outside
                v[i] = on ? *reinterpret_cast<const float4*>(a.Wh + (size_t)k * H + cc) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) *reinterpret_cast<float4*>(stg + (r4 + 4 * i) * 64 + c4) = v[i];
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the tile is this wavefront's own
#pragma unroll
            for (int j = 0; j < 64; ++j) wreg[64 * q + j] = stg[j * 64 + lane];
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __syncthreads();                                             // the partial tiles reuse this memory
    } else {
        // M[k][col] = Wh[col][k]: a lane's values lie along a row of Wh.  Fetched as 16-byte pieces
        // along the rows (a request covers four rows of 256 bytes) and turned through a
        // wavefront-private LDS tile [64 columns][64 k], 64 k at a time.
        constexpr int PITCH = 65;                 // odd: the transposed reads fall into distinct banks
        float* stg = smem + wave * 64 * PITCH;
        const int r4 = lane >> 4, k4 = 4 * (lane & 15);
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            float4 v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = c0 + r4 + 4 * i, k = kb + 64 * q + k4;
                const bool on = row < H && k < H;                    // H % 4 == 0: a piece is inside or outside
                v[i] = on ? *reinterpret_cast<const float4*>(a.Wh + (size_t)row * H + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                float* d = stg + (r4 + 4 * i) * PITCH + k4;
                d[0] = v[i].x; d[1] = v[i].y; d[2] = v[i].z; d[3] = v[i].w;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the tile is this wavefront's own
#pragma unroll
            for (int j = 0; j < 64; ++j) wreg[64 * q + j] = stg[lane * PITCH + j];
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        __syncthreads();                                             // the partial tiles reuse this memory
    }

    // ---- the state pieces of this lane: row ri, columns kb + 64 q + 4 kg .. + 3; pieces outside
    //      the matrix (rows past the batch, columns past H) stay zero ---------------------------------
    int p_off[NQ];
    bool p_on[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int k = kb + 64 * q + 4 * kg;
        p_on[q] = ri < nrows && k < H;
        p_off[q] = p_on[q] ? (b0 + ri) * H + k : b0 * H;       // clamped duplicates outside the matrix
    }
    float4 st[NQ];                         // the state of the coming step
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (p_on[q]) {
            if (!BWD) {
                if (a.h0) v = *reinterpret_cast<const float4*>(a.h0 + p_off[q]);
            } else {
                const float4 g = *reinterpret_cast<const float4*>(a.G + (size_t)(T - 1) * bh + p_off[q]);
                const float4 h = *reinterpret_cast<const float4*>(a.h_all + (size_t)T * bh + p_off[q]);
                float4 c = make_float4(0.f, 0.f, 0.f, 0.f);
                if (a.dh_last) c = *reinterpret_cast<const float4*>(a.dh_last + p_off[q]);
                v.x = (g.x + c.x) * act_grad<ACT>(h.x); v.y = (g.y + c.y) * act_grad<ACT>(h.y);
                v.z = (g.z + c.z) * act_grad<ACT>(h.z); v.w = (g.w + c.w) * act_grad<ACT>(h.w);
            }
        }
        st[q] = v;
    }

    const int nsteps = BWD ? T - 1 : T;

    // ---- epilogue lanes (wavefronts 0..3): wavefront w finishes row w, lane l column c0 + l ---------
    const int em = wave, ec = c0 + lane;
    const bool e_on = wave < RB && em < nrows && ec < H;
    const size_t e_off = (size_t)min(b0 + em, B - 1) * H + min(ec, H - 1);
    if (e_on) {    // slot 0 of the history (forward) / Delta[T-1] (reverse): the owner of a column stores it
        if (!BWD) {
            a.hist[e_off] = a.h0 ? a.h0[e_off] : 0.f;
        } else {
            const size_t e = (size_t)(T - 1) * bh + e_off;
            const float c = a.dh_last ? a.dh_last[e_off] : 0.f;
            a.Delta[e] = (a.G[e] + c) * act_grad<ACT>(a.h_all[(size_t)T * bh + e_off]);
        }
    }
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

    XT_DECL;
    // partial tile of this wavefront's K slice: element i = row i at column c0 + lane
    auto product = [&]() {
        f32x4 acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
        mfma_blocks(st[0], wreg, acc, std::make_integer_sequence<int, 16>{});
        if constexpr (NQ > 1) mfma_blocks(st[NQ - 1], wreg + 64 * (NQ - 1), acc, std::make_integer_sequence<int, 16>{});
        return (acc[0] + acc[1]) + (acc[2] + acc[3]);
    };
    auto park_partial = [&](int par, const f32x4 p4) {
        float* pp = part + (par * 8 + wave) * RB * CWD;
#pragma unroll
        for (int i = 0; i < 4; ++i) pp[i * CWD + lane] = p4[i];
    };
    auto tile_sum = [&](int par) {            // epilogue lanes: the eight wavefronts' partial sums
        const float* pp = part + par * 8 * RB * CWD + em * CWD + lane;
        float v = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) v += pp[w * RB * CWD];
        return v;
    };
    // The lane's pieces of the rows at `src`, waiting until no "not written yet" word is left.
    auto collect = [&](const float* src) {
        float4 v[NQ];
        unsigned need = 0;
#pragma unroll
        for (int q = 0; q < NQ; ++q) need |= p_on[q] ? 1u << q : 0u;
        const unsigned wanted = need;
        for (int spins = 0; need != 0; ++spins) {
            XT_COUNT(6, 1);
            if (spins > a.spin_limit) { s_abort = 1; break; }
            if (spins > 0) __builtin_amdgcn_s_sleep(2);
            if constexpr (NQ == 2) {
                if (spins == 0)
                    asm volatile("global_load_dwordx4 %0, %2, off\n\tglobal_load_dwordx4 %1, %3, off\n\ts_waitcnt vmcnt(0)"
                                 : "=&v"(v[0]), "=&v"(v[1]) : "v"(src + p_off[0]), "v"(src + p_off[1]) : "memory");
                else
                    asm volatile("global_load_dwordx4 %0, %2, off sc1\n\tglobal_load_dwordx4 %1, %3, off sc1\n\ts_waitcnt vmcnt(0)"
                                 : "=&v"(v[0]), "=&v"(v[1]) : "v"(src + p_off[0]), "v"(src + p_off[1]) : "memory");
            } else {
                if (spins == 0)
                    asm volatile("global_load_dwordx4 %0, %1, off\n\ts_waitcnt vmcnt(0)" : "=&v"(v[0]) : "v"(src + p_off[0]) : "memory");
                else
                    asm volatile("global_load_dwordx4 %0, %1, off sc1\n\ts_waitcnt vmcnt(0)" : "=&v"(v[0]) : "v"(src + p_off[0]) : "memory");
            }
#pragma unroll
            for (int q = 0; q < NQ; ++q)
                if (fresh(v[q])) need &= ~(1u << q);
        }
#pragma unroll
        for (int q = 0; q < NQ; ++q) st[q] = (wanted & (1u << q)) ? v[q] : make_float4(0.f, 0.f, 0.f, 0.f);
    };

    float last_v = 0.f;
    // One workgroup barrier per step (the partial tiles are complete); the partial buffers alternate by
    // step parity, and no wavefront can be more than one step ahead of the epilogue of its own
    // workgroup, because every later tile of the group needs that epilogue's output.
    auto step = [&](int s, auto slot_c, bool fetch_next) {
        constexpr int SLOT = decltype(slot_c)::value;   // s & 1: partial buffer and operand slot
        XTM(0);
        park_partial(SLOT, product());
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
            // this workgroup's own tile has been stored (a look that comes before its data costs a
            // second, slower one).
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
        if (a.h_last && e_on) a.h_last[e_off] = last_v;     // T >= 1: the last step's value
        return;
    }
    if (a.dh0) {   // dh0 = delta_0 Wh: one more product, no epilogue
        park_partial(0, product());
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

// partial tiles of a step; the forward kernel first stages its matrix slice there
size_t xcd_lds_bytes() { return (size_t)8 * 64 * 65 * 4; }

}  // namespace

// Shapes the one-launch loop serves and is the faster choice for.  The launch has a fixed cost (a
// cooperative launch, every workgroup loading its 256 KB of the matrix: about 28 us) and then takes
// 2.1 us per step, against 5.5 us per step for a launch per step, so the shortest sequences stay with
// the latter (cross-over at H = 1024, batch 64: 8 to 10 steps).
bool rec_xcd_supported(int H, int B, int T) {
    return T >= 10 && B > 4 && B <= NGRP * RB && H > 256 && H <= NSLOT * CWD && H % 4 == 0;
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
    const size_t lds = xcd_lds_bytes();
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
                    per_cu >= 1 && cus == NXCD * WG_PER_XCD;
    if (n_seen < 16) seen[n_seen++] = Seen{fn, dev, ok};
    return ok;
}

hipError_t launch_rec_xcd(const RecXcdArgs& a, bool bwd, hipStream_t s) {
    if (!rec_xcd_supported(a.H, a.B, a.T)) return hipErrorInvalidValue;
    if (!rec_xcd_ready(a.H, a.act, bwd)) return hipErrorNotSupported;
    const void* fn = bwd ? xcd_kernel_for<true>(a.H, a.act) : xcd_kernel_for<false>(a.H, a.act);
    const size_t lds = xcd_lds_bytes();

    // the rows the loop will produce start as sentinels; the slice counters start at zero
    const size_t bh = (size_t)a.B * a.H;
    {
        ProfileScope ps(K_MISC, s);
        hipError_t e = launch_zero_words(a.counters, NXCD, s);
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
    return hipLaunchCooperativeKernel(fn, dim3(NXCD * WG_PER_XCD), dim3(XT), kargs, (unsigned)lds, s);
}

}  // namespace rnn

#ifdef RNN_REC_TRACE
extern "C" int rnn_xcd_trace(long long* host_out, int n) {
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(rnn::g_xcd_trace), (size_t)n * 8) == hipSuccess ? 0 : -4;
}
#endif
