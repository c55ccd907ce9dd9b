// Persistent time-loop kernels with the recurrent matrix resident on chip (batch 1 .. 4).
//
// The paper's Scan runs its loop as one graph node whose per-step bookkeeping is done in
// compiled code, keeps every state for the gradient loop, and hoists everything that does not
// depend on the previous state out of the loop (Scan properties 1, 5, 8).  Here one launch
// runs all T steps; what stays inside the loop is only the product of Wh (forward) or Wh^T
// (reverse) with the previous state, a fused bias/activation (or activation-derivative)
// epilogue, and the store of the new state.
//
// Work split: P workgroups per batch row, each owning R = ceil(H/P) outputs and holding the
// matching slice of Wh (forward: rows; reverse: columns, transposed while loading) in LDS for
// the whole launch as zero-padded rows [output][k].  An output's dot product is shared by L
// adjacent lanes that read row and state as float4 (all reads in flight before the first
// multiply-add) and combine with DPP lane permutations.
// P = 1: the state lives in LDS and a step costs workgroup barriers that order LDS only.
// P > 1: every workgroup publishes its slice of the new state as self-validating 64-bit words
// {step tag, value} (relaxed device-scope atomic stores) and polls the other slices the same
// way: one memory round trip per step, no fences.  The launch is cooperative, so all P*B
// workgroups are co-resident; a wait that exceeds its spin limit sets the status word and
// makes the whole workgroup leave, so every wavefront terminates whatever happens.
//
// Global-memory latency is kept off the dependent chain: everything the setup needs is
// requested before anything is waited for, and the per-step epilogue operands (forward: the
// hoisted input term; reverse: G_t and h_t) are fetched a chunk of steps ahead.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"
#include "skinny_dev.hpp"

#include <type_traits>

namespace rnn {
namespace {

constexpr int kThreads = 512;
constexpr int kFuseMaxT = 32;  // longest sequence the fused weight-gradient tail accepts
constexpr int TC = 8;          // steps per prefetch chunk of the epilogue operands
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int NL = 20;         // independent global loads in flight per thread during setup

// Optional phase timing for tuning (-DRNN_REC_TRACE): two threads of the first workgroup (a polling
// one and a publishing one) sum the shader-clock cycles between consecutive marks over all steps.
#ifdef RNN_REC_TRACE
__device__ long long g_rec_trace[4 * 8];
#define RT_DECL long long rt_prev = clock64(); long long rt_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}
#define RT(k) do { const long long rt_n = clock64(); rt_acc[k] += rt_n - rt_prev; rt_prev = rt_n; } while (0)
#define RT_FLUSH(bwd) do { if (p == 0 && bb == 0 && (tid == 0 || tid == kThreads - kWave)) \
        for (int k_ = 0; k_ < 8; ++k_) g_rec_trace[((bwd ? 2 : 0) + (tid == 0 ? 0 : 1)) * 8 + k_] = rt_acc[k_]; } while (0)
#else
#define RT_DECL
#define RT(k)
#define RT_FLUSH(bwd)
#endif

// The time loops use lds_barrier() (common.hpp): __syncthreads() also waits for every outstanding
// global load and store, which would put a DRAM round trip on each step; the steps exchange the
// state vector through LDS, so LDS ordering is enough.

// i / d for 0 <= i < 2^24 and d > 0 without the integer-division expansion
__device__ __forceinline__ int fast_div(int i, int d, float inv) {
    int qn = (int)((float)i * inv);
    const int r = i - qn * d;
    if (r < 0) --qn;
    else if (r >= d) ++qn;
    return qn;
}

// Sum over groups of L adjacent lanes (L a power of two), result in every lane of the group.
// The first four stages use DPP lane permutations (a few cycles each, no LDS round trip):
// quad_perm xor 1, quad_perm xor 2, mirror within 8 lanes, mirror within 16 lanes; mirrors
// work because after the earlier stages all lanes of a half already hold the same sum.
__device__ __forceinline__ float group_sum(float v, int L) {
    if (L >= 2) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, false));
    if (L >= 4) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, false));
    if (L >= 8) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, false));
    if (L >= 16) v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, false));
    if (L >= 32) v = swap16_sum(v);     // rows of 16 lanes swapped between two registers: no LDS trip
    if (L >= 64) v = swap32_sum(v);
    return v;
}

template <int ACT, bool BWD>
__device__ __forceinline__ void rec_resident_body(const RecResArgs& a, const int p, const int bb,
                                                  float* smem) {
    __shared__ int s_abort;
    __shared__ int s_ids[kFuseMaxT];
    __shared__ int s_first[kFuseMaxT];
    const int H = a.H, P = a.P, R = a.R, ldw = a.ldw, L = a.L, B = a.B, T = a.T;
    const int tid = threadIdx.x;
    const int r0 = p * R;
    const int rows = max(0, min(R, H - r0));
    const int Hp = a.hpad;                    // padded vector length: 4 * L * nq4 >= H
    const float invH = 1.0f / (float)H;
    // LDS carve-up
    float* W = smem;                          // forward [R][ldw]; reverse [H][ldw]
    float* vbuf = smem + a.w_floats;          // [2][Hp], zero padded
    float* stash = vbuf + 2 * Hp;             // [2][TC][2][R] epilogue operands, private per lane
    float* Gl = stash + 2 * TC * 2 * R;       // fused tail only: [T][H] G, delta, h_{t-1}
    float* Dl = Gl + T * H;
    float* Hl = Dl + T * H;

    // thread roles
    const int q = tid % L;                               // which share of the k range
    const int own = tid / L;                             // which output of the slice
    const bool lead = (q == 0) && own < rows;            // finishes output r0 + own
    const int nsteps = BWD ? T - 1 : T;

    // Epilogue operands of TC consecutive steps starting at s0, for output j (lead lanes only).
    // Branch-free and in two phases (all ids first, then all rows), so that the requests
    // overlap instead of waiting for each other; steps past the end re-read the last one.
    const float bj = (!BWD && lead && !a.U) ? a.b[r0 + own] : 0.f;
    auto fetch_chunk = [&](int s0, int j, float (&x0)[TC], float (&x1)[TC]) {
        if (!BWD) {
            if (a.U) {
#pragma unroll
                for (int u = 0; u < TC; ++u) {
                    const size_t n = (size_t)min(s0 + u, nsteps - 1) * B + bb;
                    x0[u] = a.U[n * H + j];
                }
            } else {
                int ids[TC];
#pragma unroll
                for (int u = 0; u < TC; ++u) ids[u] = a.x[(size_t)min(s0 + u, nsteps - 1) * B + bb];
#pragma unroll
                for (int u = 0; u < TC; ++u) x0[u] = a.Wx[(size_t)ids[u] * H + j];
            }
        } else {
#pragma unroll
            for (int u = 0; u < TC; ++u) {
                const int t = T - 2 - min(s0 + u, nsteps - 1);
                x1[u] = a.h_all[((size_t)(t + 1) * B + bb) * H + j];
                if (!a.gpart) x0[u] = a.G[((size_t)t * B + bb) * H + j];
            }
        }
    };

    // ---- requests first: epilogue operands of the first chunk ------------------------------
    float nx0[TC], nx1[TC];
#pragma unroll
    for (int u = 0; u < TC; ++u) { nx0[u] = 0.f; nx1[u] = 0.f; }
    if (lead && nsteps > 0) fetch_chunk(0, r0 + own, nx0, nx1);
    if (tid == 0) s_abort = 0;
    if (BWD && a.fuse_post && tid < T) s_ids[tid] = a.x[tid];

    // ---- weight slice: registers when a lane's share is at most 8 float4, else LDS -------------
    // Weights never change during the launch, so the small-slice case keeps each lane's strip
    // of its row in 32 VGPRs, loaded straight from global memory (no staging, no LDS traffic
    // per step); larger slices stay in LDS as zero-padded rows.
    const bool wreg_mode = a.nq4 <= 8;
    float4 wreg[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) wreg[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (wreg_mode) {
        if (own < rows) {
            const int j = r0 + own;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int k = 4 * (q + u * L);
                if (u < a.nq4 && k < H) {
                    if (!BWD) {
                        const float* src = a.Wh + (size_t)j * H + k;
                        if ((H & 3) == 0) {
                            wreg[u] = *reinterpret_cast<const float4*>(src);
                        } else {
                            wreg[u].x = src[0];
                            if (k + 1 < H) wreg[u].y = src[1];
                            if (k + 2 < H) wreg[u].z = src[2];
                            if (k + 3 < H) wreg[u].w = src[3];
                        }
                    } else {  // column j of Wh
                        const float* src = a.Wh + (size_t)k * H + j;
                        wreg[u].x = src[0];
                        if (k + 1 < H) wreg[u].y = src[(size_t)H];
                        if (k + 2 < H) wreg[u].z = src[(size_t)2 * H];
                        if (k + 3 < H) wreg[u].w = src[(size_t)3 * H];
                    }
                }
            }
        }
    } else if (!BWD) {
        const int n = rows * H;  // rows r0.. are one contiguous block of Wh
        for (int base = tid; base < n; base += NL * kThreads) {
            float t[NL];
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                const int i = base + u * kThreads;
                t[u] = i < n ? a.Wh[(size_t)r0 * H + i] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                const int i = base + u * kThreads;
                if (i < n) {
                    const int r = fast_div(i, H, invH);
                    W[r * ldw + (i - r * H)] = t[u];
                }
            }
        }
        const int padw = ldw - H;
        if (padw > 0)
            for (int i = tid; i < rows * padw; i += kThreads) {  // zero the row padding
                const int r = i / padw;
                W[r * ldw + H + (i - r * padw)] = 0.f;
            }
    } else {
        const int n = H * rows;  // W[c][k] = Wh[k][r0 + c]: coalesced reads, transposing LDS writes
        const float invR = 1.0f / (float)(rows > 0 ? rows : 1);
        for (int base = tid; base < n; base += NL * kThreads) {
            float t[NL];
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                const int i = base + u * kThreads;
                t[u] = 0.f;
                if (i < n) {
                    const int k = fast_div(i, rows, invR);
                    t[u] = a.Wh[(size_t)k * H + r0 + (i - k * rows)];
                }
            }
#pragma unroll
            for (int u = 0; u < NL; ++u) {
                const int i = base + u * kThreads;
                if (i < n) {
                    const int k = fast_div(i, rows, invR);
                    W[(i - k * rows) * ldw + k] = t[u];
                }
            }
        }
        const int padw = ldw - H;
        if (padw > 0)
            for (int i = tid; i < rows * padw; i += kThreads) {
                const int r = i / padw;
                W[r * ldw + H + (i - r * padw)] = 0.f;
            }
    }
    for (int i = tid; i < 2 * Hp; i += kThreads) vbuf[i] = 0.f;

    // ---- fused tail inputs (short single sequence): h_{t-1} rows and the summed partial G -----
    if (BWD && a.fuse_post) {
        const int n = T * H;
        for (int base = tid; base < n; base += 8 * kThreads) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = (base + u * kThreads < n) ? a.h_all[base + u * kThreads] : 0.f;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (base + u * kThreads < n) Hl[base + u * kThreads] = t[u];
        }
    }
    if (BWD && a.gpart) {
        // G comes from the backward-strip workgroups of this launch as tagged words: all of a
        // thread's words are requested before the first one is examined.  Only used with the
        // fused tail (B == 1).
        const int n = T * H;
        for (int e0 = tid; e0 < n; e0 += 4 * kThreads) {
            unsigned long long w[4];
            long long idx[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) idx[u] = e0 + u * kThreads < n ? e0 + u * kThreads : -1;
            if (!wait4(a.g_box, idx, a.epoch, a.spin_limit, w)) s_abort = 1;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (idx[u] >= 0) Gl[idx[u]] = tagged_value(w[u]);
        }
    }
    __syncthreads();
    if (BWD && a.gpart && s_abort) {   // uniform: a bounded wait expired
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }

    // ---- initial vector ------------------------------------------------------------------
    // forward: h_{-1} = h0 (or zeros), also stored as slot 0 of the history.
    // reverse: delta_{T-1} = (G_{T-1} + dh_last) * act'(h_{T-1}), stored as Delta[T-1].
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
            const float g = a.gpart ? Gl[(T - 1) * H + j] : a.G[row + j];
            const float d = (g + c) * act_grad<ACT>(ht[j]);
            vbuf[j] = d;
            if (j >= r0 && j < r0 + rows) a.Delta[row + j] = d;
            if (a.fuse_post) Dl[(T - 1) * H + j] = d;
        }
    }
    __syncthreads();

    // One product of the resident slice with the vector v: every lane of an output's group gets
    // the full sum.  Rows and vector are zero padded to nq4 float4 per lane, so the common sizes
    // (nq4 <= 8, weights in registers) run fully unrolled without predicates: all LDS reads of the
    // state are issued before the first multiply-add, and a step pays for one LDS round trip.
    const float4* w4 = reinterpret_cast<const float4*>(W + min(own, R - 1) * ldw) + q;
    auto dot_fixed = [&](const float4* v4, auto count) -> float {
        constexpr int U = decltype(count)::value;
        float4 x[U];
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = v4[u * L];
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float& acc = (u & 1) ? acc1 : acc0;
            acc = fmaf(wreg[u].x, x[u].x, acc);
            acc = fmaf(wreg[u].y, x[u].y, acc);
            acc = fmaf(wreg[u].z, x[u].z, acc);
            acc = fmaf(wreg[u].w, x[u].w, acc);
        }
        return acc0 + acc1;
    };
    auto slice_dot = [&](const float* v) -> float {
        const float4* v4 = reinterpret_cast<const float4*>(v) + q;
        float acc;
        switch (a.nq4) {
            case 1: acc = dot_fixed(v4, std::integral_constant<int, 1>{}); break;
            case 2: acc = dot_fixed(v4, std::integral_constant<int, 2>{}); break;
            case 3: acc = dot_fixed(v4, std::integral_constant<int, 3>{}); break;
            case 4: acc = dot_fixed(v4, std::integral_constant<int, 4>{}); break;
            case 5: acc = dot_fixed(v4, std::integral_constant<int, 5>{}); break;
            case 6: acc = dot_fixed(v4, std::integral_constant<int, 6>{}); break;
            case 7: acc = dot_fixed(v4, std::integral_constant<int, 7>{}); break;
            case 8: acc = dot_fixed(v4, std::integral_constant<int, 8>{}); break;
            default: {  // long rows: batches of eight
                acc = 0.f;
                for (int u0 = 0; u0 < a.nq4; u0 += 8) {
                    float4 w[8], x[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const int uu = min(u0 + u, a.nq4 - 1);  // clamp: duplicates are masked below
                        w[u] = w4[uu * L];
                        x[u] = v4[uu * L];
                    }
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        if (u0 + u < a.nq4) {
                            acc = fmaf(w[u].x, x[u].x, acc);
                            acc = fmaf(w[u].y, x[u].y, acc);
                            acc = fmaf(w[u].z, x[u].z, acc);
                            acc = fmaf(w[u].w, x[u].w, acc);
                        }
                    }
                }
            }
        }
        return group_sum(acc, L);
    };

    // Steps.  forward: s = 0..T-1 computes h_s from h_{s-1}.  reverse: s = 0..T-2 computes
    // delta_t for t = T-2-s from delta_{t+1}.
    int cur = 0;
    // destination row of the step's result: a pointer that is bumped, not recomputed
    const ptrdiff_t out_stride = BWD ? -(ptrdiff_t)B * H : (ptrdiff_t)B * H;
    float* out_ptr = BWD ? a.Delta + ((size_t)max(T - 2, 0) * B + bb) * H
                         : a.hist + ((size_t)B + bb) * H;          // slot 1 = result of step 0
    float* const out_even = BWD ? nullptr : a.hist + (size_t)bb * H;               // ring slot 0
    float* const out_odd = BWD ? nullptr : a.hist + ((size_t)B + bb) * H;          // ring slot 1
    RT_DECL;
    for (int s = 0; s < nsteps; ++s) {
        RT(0);
        const int chunk = s / TC, su = s - chunk * TC;
        float* st = stash + (size_t)(chunk & 1) * TC * 2 * R;
        if (su == 0 && lead) {
#pragma unroll
            for (int u = 0; u < TC; ++u) {
                st[(u * 2) * R + own] = nx0[u] + bj;
                if (BWD) st[(u * 2 + 1) * R + own] = nx1[u];
            }
            if (s + TC < nsteps) fetch_chunk(s + TC, r0 + own, nx0, nx1);
        }
        const float* v = vbuf + cur * Hp;
        float* vnext = vbuf + (cur ^ 1) * Hp;
        const int t = BWD ? T - 2 - s : s;
        float* out_row = (!BWD && a.ring) ? ((s & 1) ? out_even : out_odd) : out_ptr;
        out_ptr += out_stride;
        // one pass covers every output of the slice: each output has its own lane group
        float val = 0.f;
        {
            const int j = r0 + own;
            float x0 = 0.f, x1 = 0.f;
            if (lead) {  // operands of the epilogue, requested before the product is waited for
                x0 = (BWD && a.gpart) ? Gl[t * H + j] : st[(su * 2) * R + own];
                if (BWD) x1 = st[(su * 2 + 1) * R + own];
            }
            RT(5);
            const float acc = slice_dot(v);
            RT(6);
            if (lead) {
                val = BWD ? (x0 + acc) * act_grad<ACT>(x1) : activate<ACT>(acc + x0);
                if (P == 1) out_row[j] = val;   // P > 1: after the exchange, off its critical path
                vnext[j] = val;
                if (BWD && a.fuse_post) Dl[t * H + j] = val;
            }
        }
        if (P > 1) {
            // Exchange of the new state between the P workgroups of this sequence.  Every value
            // travels as one 64-bit word {step tag, value}, written and polled with relaxed
            // device-scope atomics: the tag makes each word self-validating, so there is no
            // separate flag, no fence and a single memory round trip per step.  Two sets of boxes
            // alternate by step parity; a box is overwritten two steps later, and by then its
            // reader has read it (nobody publishes step s+1 before its own barrier below,
            // and step s+2 needs everybody's step s+1).  The boxes start zeroed: tags are >= 1.
            const unsigned tag = (unsigned)(s + 1);
            unsigned long long* box = reinterpret_cast<unsigned long long*>(a.flags) +
                                      ((size_t)(s & 1) * B + bb) * H;
            RT(1);
            // The last wavefront publishes the slice (and writes the history row); the others
            // poll.  A wavefront that polls right after storing would first wait for its own
            // stores to be acknowledged, once per step.
            lds_barrier();                        // the slice's new values are in vnext
            RT(2);
            if (tid >= kThreads - kWave) {
                for (int o = tid - (kThreads - kWave); o < rows; o += kWave) {
                    const float v = vnext[r0 + o];
                    tagged_store(box + r0 + o, tag, v);
                    out_row[r0 + o] = v;
                }
            } else {
                // all of a thread's words are requested before the first one is examined, and the
                // stale ones are requested again together: one memory round trip however many
                // words a thread collects (one poll after the other would cost a round trip each)
                for (int j0 = tid; j0 < H; j0 += 4 * (kThreads - kWave)) {
                    long long idx[4];
                    unsigned long long w[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int j = j0 + u * (kThreads - kWave);
                        idx[u] = (j < H && (j < r0 || j >= r0 + rows)) ? j : -1;   // own slice: already in LDS
                    }
                    if (!wait4(box, idx, tag, a.spin_limit, w)) s_abort = 1;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (idx[u] >= 0) vnext[idx[u]] = tagged_value(w[u]);
                }
            }
            RT(3);
            lds_barrier();
            RT(4);
            if (s_abort) {
                if (tid == 0) atomicExch(a.status, 1);
                return;  // uniform: the whole workgroup leaves
            }
        } else {
            lds_barrier();
        }
        cur ^= 1;
    }
    RT_FLUSH(BWD);
    __syncthreads();

    const float* vfin = vbuf + cur * Hp;
    if (!BWD) {
        if (a.h_last)
            for (int j = r0 + tid; j < r0 + rows; j += kThreads) a.h_last[(size_t)bb * H + j] = vfin[j];
        return;
    }
    if (a.dh0) {  // dh0 = Wh^T delta_0
        const float acc = slice_dot(vfin);
        if (lead) a.dh0[(size_t)bb * H + r0 + own] = acc;
    }
    if (!a.fuse_post) return;

    // ---- fused weight gradients for a short single sequence (P == 1, B == 1) -----------------
    // dWh = sum_t delta_t (x) h_{t-1},  db = sum_t delta_t,  dWx rows by token id; delta and
    // h_{t-1} rows are already in LDS.
    __syncthreads();
    // Overwrite and accumulate run as separate loops: a load inside a storing loop would make
    // every iteration wait for the previous store to be acknowledged.
    if (tid < T) {  // first step at which each step's token occurs
        int f = tid;
        for (int u = tid - 1; u >= 0; --u)
            if (s_ids[u] == s_ids[tid]) f = u;
        s_first[tid] = f;
    }
    auto tail = [&](auto accumulate) {
        constexpr bool ACC = decltype(accumulate)::value;
        for (int j = tid; j < H; j += kThreads) {
            float sum = 0.f;
            for (int t0 = 0; t0 < T; t0 += 8) {
                float d[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) d[u] = (t0 + u < T) ? Dl[(t0 + u) * H + j] : 0.f;
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += d[u];
            }
            a.db[j] = ACC ? a.db[j] + sum : sum;
        }
        // dWh = Delta^T Hprev on the matrix cores: both operands already sit K-major in LDS
        // ([t][.]), which is the order the 32x32x2 MFMA wants its lanes to fetch them in.
        const int lane = tid % kWave, wave = tid / kWave;
        const int nt = (H + 31) / 32;
        for (int tile = wave; tile < nt * nt; tile += kThreads / kWave) {
            const int m0 = (tile / nt) * 32, n0 = (tile % nt) * 32;
            const int m = m0 + lane % 32, n = n0 + lane % 32, ks = lane / 32;
            f32x16 acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
            for (int kk = 0; kk < T; kk += 2) {
                const int k = kk + ks;
                const float av = (k < T && m < H) ? Dl[k * H + m] : 0.f;
                const float bv = (k < T && n < H) ? Hl[k * H + n] : 0.f;
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc, 0, 0, 0);
            }
            if (n < H) {
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + 8 * (e / 4) + 4 * (lane / 32) + e % 4;
                    if (row < H) {
                        float* dst = a.dWh + (size_t)row * H + n;
                        *dst = ACC ? *dst + acc[e] : acc[e];
                    }
                }
            }
        }
        __syncthreads();  // Delta rows are folded in place below
        // Token rows: fold every repeated step into the row of its token's first step (ascending
        // step order, each lane only touches its own column), then write the first-step rows.
        for (int j = tid; j < H; j += kThreads) {
            for (int u = 1; u < T; ++u) {
                const int f = s_first[u];
                if (f != u) Dl[f * H + j] += Dl[u * H + j];
            }
            for (int t = 0; t < T; ++t) {
                if (s_first[t] != t) continue;
                float* dst = a.dWx + (size_t)s_ids[t] * H + j;
                *dst = ACC ? *dst + Dl[t * H + j] : Dl[t * H + j];
            }
        }
    };
    if (a.beta) tail(std::true_type{}); else tail(std::false_type{});
}

template <int ACT, bool BWD>
__global__ __launch_bounds__(kThreads) void rec_resident_kernel(RecResArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    if (a.xcd_pack) {
        // Workgroups are dealt to the 8 XCDs in turn; with 8 times the workgroups launched and
        // only every eighth working, the P workgroups of a sequence share one die (and its L2),
        // which shortens the state exchange.  The others leave at once.
        if (blockIdx.x & 7) return;
        rec_resident_body<ACT, BWD>(a, blockIdx.x >> 3, blockIdx.y, smem);
        return;
    }
    rec_resident_body<ACT, BWD>(a, blockIdx.x, blockIdx.y, smem);
}

// Backward pass of a short single sequence in one launch: workgroup 0 runs the reverse time loop
// with the fused weight gradients, workgroups 1.. run the backward strips of the output layer
// (their slices of G first, then dV, dc, zero fill of dWx).  Workgroup 0 waits, with a bounded
// spin, for the slices of G the strip workgroups of this same launch publish as tagged words; it
// therefore ends after every strip that publishes anything has read the launch's tag, and records
// that tag for the next launch on these boxes.
template <int ACT>
__global__ __launch_bounds__(kThreads) void rec_bwd_with_strips_kernel(RecResArgs a, SkinnyArgs k) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    static_assert(skinny::NTH == kThreads, "both parts use the same workgroup size");
    const unsigned tag = next_tag(tag_word_load(k.epoch_word));
    a.epoch = tag;
    k.epoch = tag;
    if (blockIdx.x == 0) {
        rec_resident_body<ACT, true>(a, 0, 0, smem);
        if (threadIdx.x == 0) tag_word_store(k.epoch_word, tag);
    } else {
        skinny::back_body(k, (int)blockIdx.x - 1, (int)gridDim.x - 1, smem);
    }
}

__global__ void zero_words_kernel(int32_t* p, int n) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0;
}

int pow2_floor(int v) {
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

}  // namespace

hipError_t launch_rec_bwd_with_strips(RecResArgs a, const RecResPlan& pl, const SkinnyArgs& k, hipStream_t s) {
    if (pl.P != 1 || a.B != 1 || !a.fuse_post) return hipErrorInvalidValue;
    a.P = pl.P; a.R = pl.R; a.L = pl.L; a.ldw = pl.ldw; a.w_floats = pl.w_floats;
    a.nq4 = pl.nq4; a.hpad = pl.hpad;
    if (a.spin_limit <= 0) a.spin_limit = wait_limit();
    const void* fn = a.act == 0 ? (const void*)rec_bwd_with_strips_kernel<0>
                                : (const void*)rec_bwd_with_strips_kernel<1>;
    size_t smem = pl.smem;
    if (skinny::back_smem(a.H) > smem) smem = skinny::back_smem(a.H);
    static size_t allowed[2] = {0, 0};
    const int slot = a.act == 0 ? 0 : 1;
    if (smem > 64 * 1024 && smem > allowed[slot]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        allowed[slot] = smem;
    }
    ProfileScope ps(K_REC_BWD, s);
    const dim3 grid(1 + skinny_strips(k.O)), block(kThreads);
    if (a.act == 0) hipLaunchKernelGGL((rec_bwd_with_strips_kernel<0>), grid, block, smem, s, a, k);
    else hipLaunchKernelGGL((rec_bwd_with_strips_kernel<1>), grid, block, smem, s, a, k);
    return hipGetLastError();
}

hipError_t launch_zero_words(int32_t* p, int n, hipStream_t s) {
    ProfileScope ps(K_MISC, s);
    const int blocks = n <= 4096 ? 1 : (n + 4095) / 4096 < 256 ? (n + 4095) / 4096 : 256;
    hipLaunchKernelGGL(zero_words_kernel, dim3(blocks), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

bool rec_resident_plan(int H, int B, int T, bool bwd, bool fuse_post, int strips, RecResPlan* out) {
    if (B > 4 || H > 4096) return false;
    if (fuse_post && (B != 1 || T > kFuseMaxT || !bwd)) return false;
    constexpr size_t kLdsBudget = 150 * 1024;  // of 160 KB per CU
    bool found = false;
    for (int P = 1; P <= 128; P *= 2) {
        if (P * B > 128) break;
        const int R = (H + P - 1) / P;
        if (R > kThreads) continue;  // one output per lane group
        RecResPlan pl{};
        pl.P = P; pl.R = R;
        int L = pow2_floor(kThreads / R);  // lanes sharing one output; R * L <= kThreads
        if (L > 64) L = 64;
        pl.L = L;
        const int H4 = (H + 3) / 4;
        pl.nq4 = (H4 + L - 1) / L;         // float4 per lane
        pl.hpad = 4 * L * pl.nq4;          // zero-padded row / vector length
        // lanes of a group read 4L consecutive words, so groups should start 4L banks apart
        int ldw = pl.hpad;
        if (L < 8) while (ldw % 32 != (4 * L) % 32) ldw += 4;
        pl.ldw = ldw;
        size_t w_floats = pl.nq4 <= 8 ? 0 : (size_t)R * ldw;   // small slices live in registers
        size_t floats = w_floats + 2 * (size_t)pl.hpad + (size_t)2 * TC * 2 * R;
        if (fuse_post) floats += (size_t)3 * T * H;
        if (floats * 4 <= kLdsBudget) {
            pl.w_floats = (int)w_floats; pl.smem = floats * 4;
            *out = pl;
            found = true;
            // A single workgroup pays no exchange; once the state is exchanged anyway, more
            // workgroups are cheap, so keep splitting until the slice fits in registers.
            if (P == 1 || pl.nq4 <= 8) return true;
            continue;
        }
        if (fuse_post) return false;  // the fused tail needs the single-workgroup form
    }
    return found;
}

hipError_t launch_rec_resident(RecResArgs a, const RecResPlan& pl, bool bwd, hipStream_t s) {
    a.P = pl.P; a.R = pl.R; a.L = pl.L; a.ldw = pl.ldw; a.w_floats = pl.w_floats;
    a.nq4 = pl.nq4; a.hpad = pl.hpad;
    if (a.spin_limit <= 0) a.spin_limit = wait_limit();
    if (pl.P > 1) {
        // exchange boxes: 2 parities x B rows x H words of 64 bits
        hipError_t e = launch_zero_words(a.flags, 4 * a.B * a.H, s);
        if (e != hipSuccess) return e;
    }
    const void* fn;
    if (!bwd) fn = a.act == 0 ? (const void*)rec_resident_kernel<0, false> : (const void*)rec_resident_kernel<1, false>;
    else fn = a.act == 0 ? (const void*)rec_resident_kernel<0, true> : (const void*)rec_resident_kernel<1, true>;
    static size_t allowed[4] = {0, 0, 0, 0};
    const int slot = (bwd ? 2 : 0) + (a.act == 0 ? 0 : 1);
    if (pl.smem > 64 * 1024 && pl.smem > allowed[slot]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.smem);
        if (e != hipSuccess) return e;
        allowed[slot] = pl.smem;
    }
    ProfileScope ps(bwd ? K_REC_BWD : K_REC_FWD, s);
    dim3 grid(pl.P, a.B), block(kThreads);
    a.xcd_pack = 0;
    if (pl.P > 1 && pl.P <= 32 && pl.P * 8 * a.B <= 256) {   // the padded grid still fits the chip
        a.xcd_pack = 1;
        grid.x = pl.P * 8;
    }
    if (pl.P > 1) {
        void* args[] = {&a};
        return hipLaunchCooperativeKernel(fn, grid, block, args, (unsigned)pl.smem, s);
    }
    if (!bwd) {
        if (a.act == 0) hipLaunchKernelGGL((rec_resident_kernel<0, false>), grid, block, pl.smem, s, a);
        else hipLaunchKernelGGL((rec_resident_kernel<1, false>), grid, block, pl.smem, s, a);
    } else {
        if (a.act == 0) hipLaunchKernelGGL((rec_resident_kernel<0, true>), grid, block, pl.smem, s, a);
        else hipLaunchKernelGGL((rec_resident_kernel<1, true>), grid, block, pl.smem, s, a);
    }
    return hipGetLastError();
}

}  // namespace rnn

#ifdef RNN_REC_TRACE
extern "C" int rnn_rec_trace(long long* host_out, int n) {
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(rnn::g_rec_trace), (size_t)n * 8) == hipSuccess ? 0 : -4;
}
#endif
