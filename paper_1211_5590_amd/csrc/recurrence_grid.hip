// Persistent time loop of ONE sequence spread over several compute units (batch 1 .. 4, hidden
// sizes whose recurrent matrix does not fit one unit: the "bigger sizes" of the paper's
// recurrent-network benchmark).  Same loop as recurrence.hip (Scan properties 1, 4, 5, 8: all
// steps in one launch, every state kept, only the product with the previous state inside the
// loop), with the work inside a workgroup split by ROLE so that nothing on the step's critical
// path waits for a store to be acknowledged:
//
//   wavefronts 0..3 ("compute")  hold the slice of Wh in registers: a wavefront owns OPW outputs,
//       lane l the columns k = 4(l + 64c) + e of them (c < 16/OPW), so a step reads the state from
//       LDS once per wavefront (16 bytes per lane and c) whatever the number of outputs.  The OPW
//       partial sums of a lane are folded across the 64 lanes by a transposing reduction (row and
//       half swaps between register pairs, then lane permutations inside groups of 8): 20
//       instructions, after which lane 8o holds output o.  That lane applies the epilogue, stores
//       the value as a self-validating word {step tag, value} for the other workgroups, stores the
//       history row, and writes the value to LDS.  These wavefronts never wait for memory inside
//       the loop (their epilogue operands are fetched a chunk of steps ahead).
//   wavefronts 4..7 ("poll")     collect the other workgroups' words of the step (all words of a
//       lane requested together, stale ones requested again together) and write them to LDS.
//   One LDS-only barrier per step joins the two.
//
// The words are written and polled with relaxed device-scope atomics (one memory round trip, no
// fences; measured: 0.29 us from store to a successful poll between two compute units of one XCD,
// 0.37 us across XCDs).  Two sets of boxes alternate by step parity; the launch is cooperative
// and every wait is bounded (a wait that expires sets the status word and the workgroup leaves).
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <stdlib.h>

namespace rnn {
namespace {

constexpr int kThreads = 512;
constexpr int kCompute = 256;   // threads of the compute wavefronts
constexpr int TC = 8;           // steps per prefetch chunk of the epilogue operands

#ifdef RNN_REC_TRACE
__device__ long long g_grid_trace[4 * 8];
#define GT_DECL long long gt_prev = clock64(); long long gt_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define GT(k) do { const long long gt_n = clock64(); gt_acc[k] += gt_n - gt_prev; gt_prev = gt_n; } while (0)
#define GT_COUNT(k, n) do { gt_acc[k] += (n); } while (0)
#define GT_FLUSH(bwd) do { if (p == 0 && bb == 0 && (tid == 0 || tid == kCompute)) \
        for (int k_ = 0; k_ < 8; ++k_) g_grid_trace[((bwd ? 2 : 0) + (tid == 0 ? 0 : 1)) * 8 + k_] = gt_acc[k_]; } while (0)
#else
#define GT_DECL
#define GT(k)
#define GT_COUNT(k, n)
#define GT_FLUSH(bwd)
#endif

// v0 <- rows/halves folded so that every lane keeps one of the two inputs' sums (see the header)
__device__ __forceinline__ float fold32(float x, float y) {   // lanes < 32: x total, lanes >= 32: y total
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float fold16(float x, float y) {   // even rows of 16 lanes: x, odd rows: y
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(y), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float fold8(float x, float y, bool upper) {   // lanes with bit 3 clear: x, set: y
    const float keep = upper ? y : x, send = upper ? x : y;
    return keep + dpp<0x128>(send);                           // row_ror:8 swaps the halves of a 16-lane row
}

// Sum of acc[o] over the 64 lanes; returns, in every lane, the total of output (lane >> 3) % OPW.
template <int OPW>
__device__ __forceinline__ float reduce_transposed(const float (&acc)[OPW], int lane) {
    const bool up8 = (lane & 8) != 0;
    float v;
    if (OPW == 8) {
        const float a0 = fold32(acc[0], acc[4]), a1 = fold32(acc[1], acc[5]);
        const float a2 = fold32(acc[2], acc[6]), a3 = fold32(acc[3], acc[7]);
        const float b0 = fold16(a0, a2), b1 = fold16(a1, a3);
        v = fold8(b0, b1, up8);
    } else if (OPW == 4) {
        const float b0 = fold16(acc[0], acc[2]), b1 = fold16(acc[1], acc[3]);
        v = swap32_sum(fold8(b0, b1, up8));
    } else if (OPW == 2) {
        v = swap32_sum(swap16_sum(fold8(acc[0], acc[1], up8)));
    } else {
        v = acc[0];
        v += dpp<0x128>(v);
        v = swap32_sum(swap16_sum(v));
    }
    v += dpp<0xB1>(v);      // lanes differing in bits 0..2 hold partial sums of the same output
    v += dpp<0x4E>(v);
    v += dpp<0x141>(v);     // mirror within 8 lanes: an exchange across bit 2 once bits 0 and 1 agree
    return v;
}

template <int ACT, bool BWD, int OPW>
__global__ __launch_bounds__(kThreads) void rec_grid_kernel(RecResArgs a) {
    constexpr int NC = 16 / OPW;          // float4 per lane and output: lane l holds k = 4(l + 64c) + e
    constexpr int HP = 256 * NC;          // padded state length (64 lanes x NC float4)
    constexpr int R = 4 * OPW;            // outputs per workgroup
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ int s_abort;
    __shared__ __attribute__((aligned(16))) int s_stored[4];   // per compute wavefront: tag of the last step it has stored
    int p = blockIdx.x;
    if (a.xcd_pack) {
        // Workgroups are dealt to the 8 XCDs in turn; with 8 times the workgroups launched and only
        // every eighth working, the P workgroups of a sequence share one die, which shortens the
        // exchange.  The others leave at once.
        if (blockIdx.x & 7) return;
        p = blockIdx.x >> 3;
    }
    const int bb = blockIdx.y;
    const int H = a.H, B = a.B, T = a.T;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool computing = tid < kCompute;
    const int r0 = p * R;
    const int rows = max(0, min(R, H - r0));
    const int o_lane = (lane >> 3) % OPW;                 // output of the wavefront this lane ends up with
    const int j_own = r0 + wave * OPW + o_lane;           // its hidden unit (compute wavefronts)
    const bool lead = computing && (lane & 7) == 0 && (lane >> 3) < OPW && j_own < H;
    const int nsteps = BWD ? T - 1 : T;

    float* vbuf = smem;                       // [2][HP] state, zero padded
    float* stash = vbuf + 2 * HP;             // [2][TC][2][R] epilogue operands of the lead lanes

    // ---- epilogue operands (forward: the hoisted input term; reverse: G_t and h_t) are fetched by the
    //      POLLING wavefronts, a chunk of TC steps ahead, into an LDS stash; the compute wavefronts issue
    //      no load inside the loop, so nothing there ever waits for memory (a wait for a load would
    //      also wait for the previous step's store to be acknowledged).  Polling lane pt serves step
    //      pt / R of the chunk and output pt % R; token ids are read one chunk earlier than the rows.
    const int pt = tid - kCompute;
    const int pf_u = pt / R, pf_o = pt % R;
    const bool pf_on = !computing && pf_u < TC && r0 + pf_o < H;
    const int pf_j = min(r0 + pf_o, H - 1);
    const float pf_bias = (!BWD && pf_on && !a.U) ? a.b[pf_j] : 0.f;
    int pf_id = 0;                               // token of this lane's step of the NEXT chunk to fetch
    auto pf_step = [&](int chunk) { return min(chunk * TC + pf_u, max(nsteps - 1, 0)); };
    auto pf_load_id = [&](int chunk) {
        if (!BWD && !a.U && pf_on) pf_id = a.x[(size_t)pf_step(chunk) * B + bb];
    };
    auto pf_issue = [&](int chunk, float& v0, float& v1) {     // requests only
        if (!pf_on) return;
        const int sidx = pf_step(chunk);
        if (!BWD) {
            v0 = a.U ? a.U[((size_t)sidx * B + bb) * H + pf_j] : a.Wx[(size_t)pf_id * H + pf_j];
        } else {
            const int t = T - 2 - sidx;
            v1 = a.h_all[((size_t)(t + 1) * B + bb) * H + pf_j];
            v0 = a.G[((size_t)t * B + bb) * H + pf_j];
        }
    };
    auto pf_park = [&](int chunk, float v0, float v1) {       // into the stash of that chunk
        if (!pf_on) return;
        float* st = stash + (size_t)(chunk & 1) * TC * 2 * R;
        st[(pf_u * 2) * R + pf_o] = v0 + pf_bias;
        if (BWD) st[(pf_u * 2 + 1) * R + pf_o] = v1;
    };
    if (nsteps > 0) {
        float v0 = 0.f, v1 = 0.f;
        pf_load_id(0);
        pf_issue(0, v0, v1);
        pf_load_id(1);
        pf_park(0, v0, v1);
    }
    if (tid == 0) s_abort = 0;
    if (tid < 4) s_stored[tid] = 0;

    // ---- the slice of Wh: wavefront w, output o, lane l: Wh[j][4(l + 64c) + e] (forward) or
    //      Wh[4(l + 64c) + e][j] (reverse: the transposed matrix), zeros outside the matrix -------
    float4 w[OPW][NC];
#pragma unroll
    for (int o = 0; o < OPW; ++o)
#pragma unroll
        for (int c = 0; c < NC; ++c) w[o][c] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (computing) {
#pragma unroll
        for (int o = 0; o < OPW; ++o) {
            const int j = r0 + wave * OPW + o;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int k = 4 * (lane + 64 * c);
                if (j < H && k < H) {
                    if (!BWD) {
                        const float* src = a.Wh + (size_t)j * H + k;
                        if ((H & 3) == 0) {
                            w[o][c] = *reinterpret_cast<const float4*>(src);
                        } else {
                            w[o][c].x = src[0];
                            if (k + 1 < H) w[o][c].y = src[1];
                            if (k + 2 < H) w[o][c].z = src[2];
                            if (k + 3 < H) w[o][c].w = src[3];
                        }
                    } else {
                        const float* src = a.Wh + (size_t)k * H + j;
                        w[o][c].x = src[0];
                        if (k + 1 < H) w[o][c].y = src[(size_t)H];
                        if (k + 2 < H) w[o][c].z = src[(size_t)2 * H];
                        if (k + 3 < H) w[o][c].w = src[(size_t)3 * H];
                    }
                }
            }
        }
    }
    for (int i = tid; i < 2 * HP; i += kThreads) vbuf[i] = 0.f;
    __syncthreads();

    // ---- initial vector: forward h_{-1} = h0 (also slot 0 of the history); reverse
    //      delta_{T-1} = (G_{T-1} + dh_last) * act'(h_{T-1}) (also Delta[T-1]) -------------------
    if (!BWD) {
        for (int j = tid; j < H; j += kThreads) {
            const float v = a.h0 ? a.h0[(size_t)bb * H + j] : 0.f;
            vbuf[j] = v;
            if (j >= r0 && j < r0 + rows) a.hist[(size_t)bb * H + j] = v;
        }
    } else {
        const size_t row = ((size_t)(T - 1) * B + bb) * H;
        const float* ht = a.h_all + ((size_t)T * B + bb) * H;
        for (int j = tid; j < H; j += kThreads) {
            const float c = a.dh_last ? a.dh_last[(size_t)bb * H + j] : 0.f;
            const float d = (a.G[row + j] + c) * act_grad<ACT>(ht[j]);
            vbuf[j] = d;
            if (j >= r0 && j < r0 + rows) a.Delta[row + j] = d;
        }
    }
    __syncthreads();

    // product of the wavefront's OPW rows with the vector v; every lane of group (lane >> 3) % OPW
    // gets that output's sum
    auto slice_dot = [&](const float* v) -> float {
        const float4* v4 = reinterpret_cast<const float4*>(v) + lane;
        float4 x[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) x[c] = v4[64 * c];
        float acc[OPW];
#pragma unroll
        for (int o = 0; o < OPW; ++o) {
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                s0 = fmaf(w[o][c].x, x[c].x, s0);
                s1 = fmaf(w[o][c].y, x[c].y, s1);
                s0 = fmaf(w[o][c].z, x[c].z, s0);
                s1 = fmaf(w[o][c].w, x[c].w, s1);
            }
            acc[o] = s0 + s1;
        }
        return reduce_transposed<OPW>(acc, lane);
    };

    int cur = 0;
    const ptrdiff_t out_stride = BWD ? -(ptrdiff_t)B * H : (ptrdiff_t)B * H;
    float* out_ptr = BWD ? a.Delta + ((size_t)max(T - 2, 0) * B + bb) * H
                         : a.hist + ((size_t)B + bb) * H;          // slot 1 = result of step 0
    float* const out_even = BWD ? nullptr : a.hist + (size_t)bb * H;               // ring slot 0
    float* const out_odd = BWD ? nullptr : a.hist + ((size_t)B + bb) * H;          // ring slot 1
    float* prev_row = nullptr;                // history row of the step before
    const int so = wave * OPW + o_lane;       // stash column of a lead lane
    GT_DECL;
    // The two roles run separate loops (one barrier per step in each): in a shared loop the compiler's
    // bookkeeping of outstanding memory operations would carry the polling wavefronts' loads into the
    // compute wavefronts' path and make every step wait for the previous step's store.
    // An expired wait is acted on every eighth step and after the loop: reading the flag would
    // otherwise sit on every step's critical path.  Until then the steps run on with whatever the
    // expired wait left, each wait bounded as before.
    auto box_of = [&](int s) {
        return reinterpret_cast<unsigned long long*>(a.flags) + ((size_t)(s & 1) * B + bb) * H;
    };
    bool left = false;
    if (computing) {
        for (int s = 0; s < nsteps; ++s) {
            GT(0);
            const unsigned tag = (unsigned)(s + 1);
            unsigned long long* box = box_of(s);
            float* vnext = vbuf + (cur ^ 1) * HP;
            const int chunk = s / TC, su = s - chunk * TC;
            const float* st = stash + (size_t)(chunk & 1) * TC * 2 * R;
            float x0 = 0.f, x1 = 0.f;
            if (lead) {
                x0 = st[(su * 2) * R + so];
                if (BWD) x1 = st[(su * 2 + 1) * R + so];
            }
            const float acc = slice_dot(vbuf + cur * HP);
            GT(1);
            if (lead) {
                const float val = BWD ? (x0 + acc) * act_grad<ACT>(x1) : activate<ACT>(acc + x0);
                tagged_store(box + j_own, tag, val);     // the other workgroups wait for it
                vnext[j_own] = val;
            }
            if (lane == 0) s_stored[wave] = (int)tag;    // tells this workgroup's polling wavefronts when to start
            GT(2);
            lds_barrier();
            GT(3);
            if ((s & 7) == 7 && s_abort) { left = true; break; }
            cur ^= 1;
        }
    } else {
        for (int s = 0; s < nsteps; ++s) {
            GT(0);
            const unsigned tag = (unsigned)(s + 1);
            unsigned long long* box = box_of(s);
            float* vnext = vbuf + (cur ^ 1) * HP;
            // While the compute wavefronts work: the previous step's slice goes to the history (a second
            // store in the compute wavefronts' epilogue would delay the one the others wait for) ...
            if (s > 0 && wave == 4 && lane < rows) prev_row[r0 + lane] = vbuf[cur * HP + r0 + lane];
            // ... and, at the first step of a chunk, the requests for the next chunk's epilogue operands.
            const int chunk = s / TC;
            const bool fetch_now = s - chunk * TC == 0 && (chunk + 1) * TC < nsteps;
            float pv0 = 0.f, pv1 = 0.f;
            if (fetch_now) {
                pf_issue(chunk + 1, pv0, pv1);
                pf_load_id(chunk + 2);
            }
            // Words of the other workgroups' slices.  A poll that arrives before its word costs more
            // than a whole extra round trip (measured on the exchange alone: 1.17 us per step when the
            // polls start at once, 0.68 us when they start as the words land), and all workgroups run
            // in step, so the polling starts once this workgroup's own compute wavefronts have issued
            // their stores, which they signal through LDS (a pause between looks: a tight spin of four
            // wavefronts would crowd the compute wavefronts' own LDS traffic).
            {
                                for (int spins = 0; spins < (1 << 16); ++spins) {
                    const int4 f = lds_peek4(s_stored);
                    if (f.x == (int)tag && f.y == (int)tag && f.z == (int)tag && f.w == (int)tag) break;
                    __builtin_amdgcn_s_sleep(1);
                }
                for (int k = 0; k < a.poll_sleep; ++k) __builtin_amdgcn_s_sleep(1);
            }
            GT(1);
            for (int j0 = pt; j0 < H; j0 += 4 * (kThreads - kCompute)) {
                long long idx[4];
                unsigned long long wd[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int j = j0 + u * (kThreads - kCompute);
                    idx[u] = (j < H && (j < r0 || j >= r0 + rows)) ? j : -1;   // own slice: written by the lead lanes
                }
                if (!wait4(box, idx, tag, a.spin_limit, wd)) s_abort = 1;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (idx[u] >= 0) vnext[idx[u]] = tagged_value(wd[u]);
            }
            if (fetch_now) pf_park(chunk + 1, pv0, pv1);
            GT(2);
            prev_row = (!BWD && a.ring) ? ((s & 1) ? out_even : out_odd) : out_ptr;
            out_ptr += out_stride;
            lds_barrier();
            GT(3);
            if ((s & 7) == 7 && s_abort) { left = true; break; }
            cur ^= 1;
        }
    }
    if (left) {      // uniform: every wavefront saw the flag at the same step
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }
    GT_FLUSH(BWD);
    __syncthreads();
    if (s_abort) {
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }

    const float* vfin = vbuf + cur * HP;
    if (nsteps > 0 && wave == 4 && lane < rows) prev_row[r0 + lane] = vfin[r0 + lane];   // the last step's slice
    if (!BWD) {
        if (a.h_last)
            for (int j = r0 + tid; j < r0 + rows; j += kThreads) a.h_last[(size_t)bb * H + j] = vfin[j];
        return;
    }
    if (a.dh0 && computing) {  // dh0 = Wh^T delta_0
        const float acc = slice_dot(vfin);
        if (lead) a.dh0[(size_t)bb * H + j_own] = acc;
    }
}

template <int ACT, bool BWD>
const void* pick_grid_kernel(int opw) {
    switch (opw) {
        case 8: return (const void*)rec_grid_kernel<ACT, BWD, 8>;
        case 4: return (const void*)rec_grid_kernel<ACT, BWD, 4>;
        case 2: return (const void*)rec_grid_kernel<ACT, BWD, 2>;
        default: return (const void*)rec_grid_kernel<ACT, BWD, 1>;
    }
}

}  // namespace

bool rec_grid_plan(int H, int B, RecGridPlan* out) {
    if (B < 1 || B > 4 || H < 1 || H > 4096) return false;
    const int opw = H <= 512 ? 8 : H <= 1024 ? 4 : H <= 2048 ? 2 : 1;
    RecGridPlan pl{};
    pl.OPW = opw;
    pl.R = 4 * opw;
    pl.P = (H + pl.R - 1) / pl.R;
    if (pl.P < 2 || pl.P * B > 128) return false;
    pl.hpad = 256 * (16 / opw);
    pl.smem = ((size_t)2 * pl.hpad + (size_t)2 * TC * 2 * pl.R) * 4;
    *out = pl;
    return true;
}

hipError_t launch_rec_grid(RecResArgs a, const RecGridPlan& pl, bool bwd, hipStream_t s) {
    a.P = pl.P; a.R = pl.R; a.hpad = pl.hpad;
    if (a.spin_limit <= 0) a.spin_limit = wait_limit();
    // a.poll_sleep: further pauses of 64 clocks between the own stores and the first poll (measured: none is best)
#ifdef RNN_REC_TRACE
    if (const char* env = getenv("RNN_POLL_SLEEP")) a.poll_sleep = atoi(env);
#endif
    // exchange boxes: 2 parities x B rows x H words of 64 bits, cleared in-stream (tags are step numbers)
    hipError_t e = launch_zero_words(a.flags, 4 * a.B * a.H, s);
    if (e != hipSuccess) return e;
    const void* fn;
    if (!bwd) fn = a.act == 0 ? pick_grid_kernel<0, false>(pl.OPW) : pick_grid_kernel<1, false>(pl.OPW);
    else fn = a.act == 0 ? pick_grid_kernel<0, true>(pl.OPW) : pick_grid_kernel<1, true>(pl.OPW);
    ProfileScope ps(bwd ? K_REC_BWD : K_REC_FWD, s);
    dim3 grid(pl.P, a.B), block(kThreads);
    a.xcd_pack = 0;
    if (pl.P <= 32 && pl.P * 8 * a.B <= 256) {   // the padded grid still fits the chip
        a.xcd_pack = 1;
        grid.x = pl.P * 8;
    }
    void* args[] = {&a};
    return hipLaunchCooperativeKernel(fn, grid, block, args, (unsigned)pl.smem, s);
}

}  // namespace rnn

#ifdef RNN_REC_TRACE
extern "C" int rnn_grid_trace(long long* host_out, int n) {
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(rnn::g_grid_trace), (size_t)n * 8) == hipSuccess ? 0 : -4;
}
#endif
