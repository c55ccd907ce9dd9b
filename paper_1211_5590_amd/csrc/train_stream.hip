// Many truncated-BPTT windows of a token stream with a fused SGD update in ONE persistent launch.
//
// The paper's function objects can repeat a compiled training function N times inside the
// runtime and hand back only the last result (its section on calling a function repeatedly),
// because at small model sizes the per-call overhead dominates.  Here the whole stream is one
// cooperative launch in which the model never leaves the chip:
//
//   workgroup 0 ("loop")    keeps Wh in registers twice (by rows for the forward loop, by columns
//                           for the reverse loop), the bias, and the states of the window in LDS;
//                           it runs the forward steps, the reverse steps and the updates of Wh, b
//                           and the touched rows of Wx
//   workgroups 1..S ("strips") each keep 128 vocabulary columns of V and c in LDS for the whole
//                           stream; per window they form the logits of their columns row by row as
//                           the hidden states arrive, the strip statistics of the log-sum-exp,
//                           their share of G = dZ V^T, and then update their columns in place
//
// Workgroups talk through self-validating 64-bit words {window tag, value} (relaxed device-scope
// atomics; one memory round trip, no fences).  Every box is single-buffered: a word of window
// w+1 is written only after the loop workgroup has started that window, which it does only after
// every strip has published its slice of G for window w, which a strip does only after it has
// read everything it needs from the boxes of window w.
//
// dV and dWx are never materialised: V <- V - lr Hs^T dZ is applied to the resident columns, and
// only the rows of Wx whose tokens occur in the window are rewritten.  The rank-T update of Wh is
// applied one rank-1 term at a time: to the row copy during the reverse loop, where it fills issue
// slots the latency-bound steps leave idle, and to the column copy while the loop workgroup waits
// for the next window's G (same order and same operands, so both copies stay bit-identical).
//
// Every wait is bounded; a wait that expires sets the status word and makes its workgroup leave,
// after which the others run into their own limits, so the grid always drains.
#include "../../include/rnn.h"

#include <stdlib.h>

#include <atomic>
#include <mutex>
#include <type_traits>

#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

// Exchange boxes of rnn_window_static, the form of the one-window call for callers that cannot
// allocate: a fixed array in the code object instead of a caller-provided workspace.  Every GPU
// the library runs on holds its own copy until the process ends.
constexpr size_t kStaticScratchBytes = RNN_WINDOW_STATIC_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace rnn {
int32_t* three_call_status_word(const rnn_dims* dims, void* workspace);   // api.hip
namespace {

constexpr int NT = 512;          // threads per workgroup (both roles)
constexpr int MAXH = NT / 4;     // four lanes share one hidden unit in the loop workgroup
constexpr int MAXT = 32;         // longest window
constexpr int CW = 128;          // vocabulary columns per strip
constexpr int ES = CW + 4;       // LDS row stride of the strip of V: the 16 rows of a 16-byte operand read
                                 // fall into distinct banks
constexpr int HT = 36;           // LDS row stride of the transposed hidden rows kept by a strip (>= MAXT + 4)
constexpr int MAX_TS = 2048;     // T * strips the strip statistics stage in LDS holds

struct StreamArgs {
    float *Wx, *Wh, *b, *V, *c;          // parameters (stream mode: updated in place)
    const int32_t* ids;                   // inputs: [n_windows*T (+ 1)]
    const int32_t* ys;                    // targets, same stride (stream mode: ids + 1)
    long long n_windows;
    unsigned tag0;                        // tag of the first window's words (never 0); the one-window
                                          // kernel takes it from *tagword instead
    unsigned* tagword;                    // device word: tag of the last window run on these boxes
    // gradient mode (one window, parameters untouched)
    float *dWx, *dWh, *db, *dV, *dc;
    int beta, NVin;                       // beta: add to the gradient buffers; NVin: rows of Wx
    const float* dh_last;                 // nullable [H]
    float *dh0, *h_all;                   // nullable [H], [T+1][H]
    float lr;
    const float* h0;                      // nullable [H]
    float* h_last;                        // nullable [H]
    float* losses;                        // nullable [n_windows]
    int H, NV, T, S;
    unsigned long long *hbox, *gbox, *vybox, *zybox, *statbox, *pbox;
    int32_t* status;
    int spin_limit;
};

// Optional phase timing for tuning (-DRNN_STREAM_TRACE): every workgroup sums the time between
// consecutive marks over all windows (100 MHz clock) and leaves the sums in g_trace.
#ifdef RNN_STREAM_TRACE
__device__ long long g_trace[257 * 16];
#define TS_DECL long long ts_prev = wall_clock64(); const long long ts_c0 = clock64(), ts_w0 = ts_prev; long long ts_acc[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}
#define TS(k) do { const long long ts_n = wall_clock64(); ts_acc[k] += ts_n - ts_prev; ts_prev = ts_n; } while (0)
#define TS_FLUSH do { ts_acc[14] = clock64() - ts_c0; ts_acc[15] = wall_clock64() - ts_w0; if (threadIdx.x == 0) for (int k_ = 0; k_ < 16; ++k_) g_trace[blockIdx.x * 16 + k_] = ts_acc[k_]; } while (0)
#else
#define TS_DECL
#define TS(k)
#define TS_FLUSH
#endif

// merge of (max, sum of exponentials) pairs over the 64 lanes, result in every lane
__device__ __forceinline__ void lse_merge64(float& m, float& s) {
    { const float m2 = dpp<0xB1>(m), s2 = dpp<0xB1>(s); lse_merge(m, s, m2, s2); }
    { const float m2 = dpp<0x4E>(m), s2 = dpp<0x4E>(s); lse_merge(m, s, m2, s2); }
    { const float m2 = dpp<0x141>(m), s2 = dpp<0x141>(s); lse_merge(m, s, m2, s2); }
    { const float m2 = dpp<0x140>(m), s2 = dpp<0x140>(s); lse_merge(m, s, m2, s2); }
    {
        const auto rm = __builtin_amdgcn_permlane16_swap(__float_as_uint(m), __float_as_uint(m), false, false);
        const auto rs = __builtin_amdgcn_permlane16_swap(__float_as_uint(s), __float_as_uint(s), false, false);
        m = __uint_as_float(rm[0]); s = __uint_as_float(rs[0]);
        lse_merge(m, s, __uint_as_float(rm[1]), __uint_as_float(rs[1]));
    }
    {
        const auto rm = __builtin_amdgcn_permlane32_swap(__float_as_uint(m), __float_as_uint(m), false, false);
        const auto rs = __builtin_amdgcn_permlane32_swap(__float_as_uint(s), __float_as_uint(s), false, false);
        m = __uint_as_float(rm[0]); s = __uint_as_float(rs[0]);
        lse_merge(m, s, __uint_as_float(rm[1]), __uint_as_float(rs[1]));
    }
}

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ __forceinline__ float dot4(float4 a, float4 b, float acc) {
    acc = fmaf(a.x, b.x, acc); acc = fmaf(a.y, b.y, acc);
    acc = fmaf(a.z, b.z, acc); acc = fmaf(a.w, b.w, acc);
    return acc;
}
// w <- w - s * h, element-wise
__device__ __forceinline__ void rank1(float4& w, float s, float4 h) {
    w.x = fmaf(-s, h.x, w.x); w.y = fmaf(-s, h.y, w.y); w.z = fmaf(-s, h.z, w.z); w.w = fmaf(-s, h.w, w.w);
}
__device__ __forceinline__ void rank1v(float4& w, float4 s, float h) {
    w.x = fmaf(-s.x, h, w.x); w.y = fmaf(-s.y, h, w.y); w.z = fmaf(-s.z, h, w.z); w.w = fmaf(-s.w, h, w.w);
}
// rows of Wx are re-read after they were rewritten by the same lane; device-scope accesses keep
// the first-level cache out of the question
__device__ __forceinline__ float dev_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void dev_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

size_t loop_lds_floats(int T, int NQ) { return (size_t)(2 * (T + 1) + 5 * T) * 16 * NQ; }
size_t strip_lds_floats(int NQ, int T, int S) {
    const int HR = 16 * NQ;
    return (size_t)HR * ES + CW + (size_t)32 * (HR + 4) + (size_t)HR * HT + (size_t)16 * (CW + 4) + (size_t)3 * T * S;
}

// ---------------------------------------------------------------------------------------
// Workgroup 0: time loops and the recurrent-layer updates.  NQ = float4 per lane of a row of Wh.
//
// Nothing but the two loops is on the critical path of a window:
//  * the rank-1 terms of the Wh update ride along with the steps (see the file header);
//  * the rows of Wx for window w+1 are requested while the strips work on window w, i.e. before
//    window w's update exists; the forward loop of w+1 subtracts, from the row of a token that
//    also occurred in window w, lr * delta of those steps (their numbers come from a table built
//    with the request); window w's own rows go to memory in the idle time of window w+1;
//  * the per-window step tables are built in the same idle time, one window ahead.
template <int ACT, int NQ>
__device__ __forceinline__ void loop_body(const StreamArgs& a, float* smem) {
    constexpr int HP = 16 * NQ;      // padded vector length
    __shared__ int s_ids[2][MAXT + 1];   // by window parity: token of each step
    __shared__ int s_first[2][MAXT];     // first step of the window with the same token
    __shared__ int4 s_ch[2][MAXT];       // the next four steps of the window with the same token (-1: none)
    __shared__ int4 s_pm[2][MAXT];       // the first four steps of the window whose token is the token of the
                                         // same-numbered step of the FOLLOWING window (-1: none)
    __shared__ int s_idf[MAXT + 1];      // tokens of the following window (scratch for the tables)
    __shared__ int s_abort;
    const int H = a.H, T = a.T, tid = threadIdx.x;
    const int own = tid >> 2, q = tid & 3;
    const int ownc = min(own, HP - 1);
    const bool live = own < H, lead = live && q == 0;
    float* Hl = smem;                        // [2][T+1][HP]  h_{-1} .. h_{T-1}, by window parity
    float* Dl = Hl + 2 * (T + 1) * HP;       // [T][HP] delta_t
    float* Sl = Dl + T * HP;                 // [T][HP] lr * delta_t
    float* Ul = Sl + T * HP;                 // [2][T][HP] rows of Wx of the window's tokens, by window parity
    float* Gl = Ul + 2 * T * HP;             // [T][HP] G_t
    const int lds_floats = (2 * (T + 1) + 5 * T) * HP;
    for (int i = tid; i < lds_floats; i += NT) smem[i] = 0.f;   // padding must read as zero

    float4 wf[NQ], wb[NQ];                   // Wh[own][k..k+3] and Wh[k..k+3][own], k = 4(q+4u)
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int k = 4 * (q + 4 * u);
        float f[4] = {0.f, 0.f, 0.f, 0.f}, g[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (live && k + e < H) {
                f[e] = a.Wh[(size_t)own * H + k + e];
                g[e] = a.Wh[(size_t)(k + e) * H + own];
            }
        wf[u] = make_float4(f[0], f[1], f[2], f[3]);
        wb[u] = make_float4(g[0], g[1], g[2], g[3]);
    }
    float bj = lead ? a.b[own] : 0.f;
    // ids of the windows w+1 and w+2 travel in registers of the threads tid <= T
    const int r0 = tid <= T ? a.ids[tid] : 0;
    int r1 = (tid <= T && a.n_windows > 1) ? a.ids[(size_t)T + tid] : 0;
    int r2 = (tid <= T && a.n_windows > 2) ? a.ids[(size_t)2 * T + tid] : 0;
    if (tid == 0) s_abort = 0;

    // step tables of the window whose tokens are in s_ids[p]; s_idf: tokens of the window after it
    auto make_tables = [&](int p, bool has_fol) {
        if (tid < T) {
            const int mine = s_ids[p][tid], theirs = has_fol ? s_idf[tid] : -1;
            int f = tid, nc = 0, np = 0;
            int4 ch = make_int4(-1, -1, -1, -1), pm = make_int4(-1, -1, -1, -1);
            for (int u0 = 0; u0 < T; u0 += 8) {
                int iv[8];
#pragma unroll
                for (int k = 0; k < 8; ++k) iv[k] = s_ids[p][min(u0 + k, T - 1)];
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    const int idx = u0 + k;
                    if (idx < T && iv[k] == mine) {
                        if (idx < f) f = idx;
                        if (idx > tid) {
                            if (nc == 0) ch.x = idx; else if (nc == 1) ch.y = idx;
                            else if (nc == 2) ch.z = idx; else if (nc == 3) ch.w = idx;
                            ++nc;
                        }
                    }
                    if (idx < T && iv[k] == theirs) {
                        if (np == 0) pm.x = idx; else if (np == 1) pm.y = idx;
                        else if (np == 2) pm.z = idx; else if (np == 3) pm.w = idx;
                        ++np;
                    }
                }
            }
            s_first[p][tid] = f;
            s_ch[p][tid] = ch;
            s_pm[p][tid] = pm;
        }
    };
    // sum over a token's steps of lr * delta for hidden unit `col`, steps given four at a time
    // (wave-uniform control flow: the tables do not depend on the lane)
    auto class_sum = [&](int4 c, int p, int col) -> float {
        float sum = 0.f;
        while (c.x >= 0) {
            const float v0 = Sl[c.x * HP + col], v1 = Sl[max(c.y, 0) * HP + col];
            const float v2 = Sl[max(c.z, 0) * HP + col], v3 = Sl[max(c.w, 0) * HP + col];
            const int4 more = s_ch[p][max(c.w, 0)];
            sum += v0;
            if (c.y >= 0) sum += v1;
            if (c.z >= 0) sum += v2;
            if (c.w >= 0) sum += v3;
            c = c.w >= 0 ? more : make_int4(-1, -1, -1, -1);
        }
        return sum;
    };

    __syncthreads();
    if (tid <= T) { s_ids[0][tid] = r0; s_idf[tid] = r1; }
    if (lead) Hl[own] = a.h0 ? a.h0[own] : 0.f;
    __syncthreads();
    make_tables(0, a.n_windows > 1);
    if (lead) {              // rows of Wx for window 0, eight requests in flight
        for (int t0 = 0; t0 < T; t0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = dev_load(a.Wx + (size_t)s_ids[0][min(t0 + u, T - 1)] * H + own);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (t0 + u < T) Ul[(t0 + u) * HP + own] = v[u];
        }
    }
    __syncthreads();

    TS_DECL;
    for (long long w = 0; w < a.n_windows; ++w) {
        TS(0);
        const int pw = (int)(w & 1), pn = pw ^ 1;
        const unsigned tag = a.tag0 + (unsigned)w;
        float* Hc = Hl + pw * (T + 1) * HP;           // this window's states
        const float* Ho = Hl + pn * (T + 1) * HP;     // the previous window's
        float* Uc = Ul + pw * T * HP;                  // this window's rows of Wx
        float* Uo = Ul + pn * T * HP;                  // the previous window's, then the next window's
        const bool prev = w > 0, have_next = w + 1 < a.n_windows;

        // ---- forward steps ----
        int4 pm_cur = prev ? s_pm[pn][0] : make_int4(-1, -1, -1, -1);
        for (int s = 0; s < T; ++s) {
            const float4* v4 = reinterpret_cast<const float4*>(Hc + s * HP) + q;
            float4 x[NQ];
#pragma unroll
            for (int u = 0; u < NQ; ++u) x[u] = v4[4 * u];
            float uin = Uc[s * HP + ownc];
            int4 pm_nx = make_int4(-1, -1, -1, -1);
            if (prev) {
                pm_nx = s_pm[pn][min(s + 1, T - 1)];
                if (pm_cur.x >= 0) {   // this step's token occurred in the previous window
                    uin -= class_sum(pm_cur, pn, ownc);
                    if (lead) Uc[s * HP + own] = uin;
                }
            }
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                if (u & 1) acc1 = dot4(wf[u], x[u], acc1); else acc0 = dot4(wf[u], x[u], acc0);
            }
            const float acc = sum4(acc0 + acc1);
            if (lead) {
                const float hv = activate<ACT>(acc + uin + bj);
                Hc[(s + 1) * HP + own] = hv;
                tagged_store(a.hbox + (size_t)s * H + own, tag, hv);
            }
            pm_cur = pm_nx;
            lds_barrier();
        }

        TS(1);
        // ---- while the strips work: the previous window's rows of Wx go to memory, then the
        //      tables and the rows of Wx for the next window are fetched ----
        if (prev) {   // column copy of Wh: the previous window's update, same terms in the same order
            for (int tt = T - 1; tt >= 0; --tt) {
                const float4* s4 = reinterpret_cast<const float4*>(Sl + tt * HP) + q;
                float4 sd[NQ];
#pragma unroll
                for (int u = 0; u < NQ; ++u) sd[u] = s4[4 * u];
                const float ho = Ho[tt * HP + ownc];
#pragma unroll
                for (int u = 0; u < NQ; ++u) rank1v(wb[u], sd[u], ho);
            }
        }
        if (prev && lead) {
            for (int t = 0; t < T; ++t) {
                if (s_first[pn][t] != t) continue;
                const int4 c = s_ch[pn][t];
                const float sum = Sl[t * HP + own] + class_sum(c, pn, own);
                dev_store(a.Wx + (size_t)s_ids[pn][t] * H + own, Uo[t * HP + own] - sum);
            }
        }
        lds_barrier();
        if (have_next) {
            if (tid <= T) { s_ids[pn][tid] = r1; s_idf[tid] = r2; }
            lds_barrier();
            make_tables(pn, w + 2 < a.n_windows);
            if (lead) {
                for (int t0 = 0; t0 < T; t0 += 8) {
                    float v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        v[u] = dev_load(a.Wx + (size_t)s_ids[pn][min(t0 + u, T - 1)] * H + own);
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        consume(v[u]);
                        if (t0 + u < T) Uo[(t0 + u) * HP + own] = v[u];
                    }
                }
            }
            if (tid <= T) {
                r1 = r2;
                if (w + 3 < a.n_windows) r2 = a.ids[(size_t)(w + 3) * T + tid];
            }
        }
        TS(2);
        // ---- G from the strips -------------------------------------------------------------
        {
            const int n = T * H;
            for (int e0 = tid; e0 < n; e0 += 4 * NT) {
                unsigned long long wd[4];
                long long idx[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) idx[u] = e0 + u * NT < n ? e0 + u * NT : -1;
                if (!wait4(a.gbox, idx, tag, a.spin_limit, wd)) s_abort = 1;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = e0 + u * NT;
                    if (e >= n) continue;
                    const int t = e / H;
                    Gl[t * HP + (e - t * H)] = tagged_value(wd[u]);
                }
            }
        }
        __syncthreads();
        if (s_abort) {
            if (tid == 0) atomicExch(a.status, 1);
            return;
        }

        TS(3);
        // ---- reverse steps; the row copy of Wh receives this window's update ------------------
        float bsum = 0.f;
        if (lead) {
            const float h = Hc[T * HP + own];
            const float d = Gl[(T - 1) * HP + own] * act_grad<ACT>(h);
            const float sl = a.lr * d;
            Dl[(T - 1) * HP + own] = d;
            Sl[(T - 1) * HP + own] = sl;
            bsum = d;
        }
        lds_barrier();
        for (int t = T - 2; t >= 0; --t) {
            const float4* d4 = reinterpret_cast<const float4*>(Dl + (t + 1) * HP) + q;
            const float4* h4 = reinterpret_cast<const float4*>(Hc + (t + 1) * HP) + q;
            float4 x[NQ], hh[NQ];
#pragma unroll
            for (int u = 0; u < NQ; ++u) { x[u] = d4[4 * u]; hh[u] = h4[4 * u]; }
            const float sj = Sl[(t + 1) * HP + ownc];
            const float g = Gl[t * HP + ownc], h = Hc[(t + 1) * HP + ownc];
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                if (u & 1) acc1 = dot4(wb[u], x[u], acc1); else acc0 = dot4(wb[u], x[u], acc0);
            }
            const float acc = sum4(acc0 + acc1);
            if (lead) {
                const float d = (g + acc) * act_grad<ACT>(h);
                const float sl = a.lr * d;
                Dl[t * HP + own] = d;
                Sl[t * HP + own] = sl;
                bsum += d;
            }
#pragma unroll
            for (int u = 0; u < NQ; ++u) rank1(wf[u], sj, hh[u]);   // term t+1: delta_{t+1} (x) h_t
            lds_barrier();
        }
        {   // term 0: delta_0 (x) h_{-1}
            const float4* h4 = reinterpret_cast<const float4*>(Hc) + q;
            float4 hh[NQ];
#pragma unroll
            for (int u = 0; u < NQ; ++u) hh[u] = h4[4 * u];
            const float sj = Sl[ownc];
#pragma unroll
            for (int u = 0; u < NQ; ++u) rank1(wf[u], sj, hh[u]);
        }
        TS(4);
        if (lead) {
            bj = fmaf(-a.lr, bsum, bj);
            Hl[pn * (T + 1) * HP + own] = Hc[T * HP + own];   // carried state
        }
        lds_barrier();
        TS(5);
    }
    TS_FLUSH;

    // ---- write the recurrent layer back: rows of Wx of the last window, Wh, b, the state --------
    const int pl = (int)((a.n_windows - 1) & 1);
    if (lead) {
        const float* Uc = Ul + pl * T * HP;
        for (int t = 0; t < T; ++t) {
            if (s_first[pl][t] != t) continue;
            const float sum = Sl[t * HP + own] + class_sum(s_ch[pl][t], pl, own);
            dev_store(a.Wx + (size_t)s_ids[pl][t] * H + own, Uc[t * HP + own] - sum);
        }
    }
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int k = 4 * (q + 4 * u);
        const float f[4] = {wf[u].x, wf[u].y, wf[u].z, wf[u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (live && k + e < H) a.Wh[(size_t)own * H + k + e] = f[e];
    }
    if (lead) {
        a.b[own] = bj;
        if (a.h_last) a.h_last[own] = Hl[pl * (T + 1) * HP + T * HP + own];
    }
}


// ---------------------------------------------------------------------------------------
// Workgroups 1..S: one strip of CW = 128 vocabulary columns each; wavefront w owns the 16 columns
// 16w.. of the strip.  All three products with the strip of V run on the matrix cores
// (v_mfma_f32_16x16x4: lane l supplies A[l%16][l/16] and B[l/16][l%16] and receives
// D[4(l/16)+r][l%16], r = 0..3), on up to 16 rows of the window per pass:
//   logits   Z[n][c]  = sum_i h[n][i] V[i][c]      M = rows, N = own 16 columns, K = hidden
//   share    P[n][i]  = sum_c e[n][c] V[i][c]      M = rows, N = 16 hidden rows per wavefront, K = columns
//   update   D[i][c]  = sum_n h[n][i] dZ[n][c]     M = hidden, N = own 16 columns, K = rows
// The logits of a wavefront's columns stay in its registers from the first product to the update
// (D's layout of Z is exactly the B operand the update wants).  NQ: the hidden dimension is padded
// to HR = 16*NQ rows of zeros; lane group kg = l/16 walks the hidden rows kg*4NQ.. in the first
// product.  Every phase issues all its LDS reads before it computes.
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int ESE = CW + 4;      // LDS row stride of the exponentials

template <int NQ, int MODE>   // MODE 0: SGD over a stream, 1: gradients of one window
__device__ __forceinline__ void strip_body(const StreamArgs& a, const int g, float* smem) {
    constexpr int HR = 16 * NQ, HPP = HR + 4, KC = 4 * NQ;
    __shared__ int s_y[MAXT];
    __shared__ float lse_s[MAXT];
    __shared__ float zy_s[MAXT];
    __shared__ float tmax[8 * 16], tsum[8 * 16];
    __shared__ int s_abort;
    const int H = a.H, T = a.T, S = a.S, NV = a.NV, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, m = lane & 15, kg = lane >> 4;
    const int k0 = g * CW, ncols = min(CW, NV - k0);
    const int cown = 16 * wave + m;                  // this lane's column of the strip
    const float invN = 1.0f / (float)T;
    const int npass = (T + 15) / 16;
    TS_DECL;
    float* Vs = smem;                     // [HR][ES]
    float* cs = Vs + HR * ES;             // [CW]
    float* hs = cs + CW;                  // [32][HPP] hidden rows of the window (rows past T: zeros)
    float* hsT = hs + 32 * HPP;           // [HR][HT]  the same, transposed
    float* es = hsT + HR * HT;            // [16][ESE] exp(z - strip max) of the current pass
    float* stage = es + 16 * ESE;         // [T][S][2]
    float* wts = stage + 2 * T * S;       // [T][S]

    // The strip of V: every element of the HR x 128 block is written (zeros outside the matrix);
    // 16-byte loads, all of a thread's requests in flight, when the rows allow it.
    if ((NV & 3) == 0) {
        const int c4 = tid & 31, ig = tid >> 5;
        float4 v[NQ];
#pragma unroll
        for (int u = 0; u < NQ; ++u) {
            const int i = ig + 16 * u;
            v[u] = (i < H && 4 * c4 < ncols) ? ld4(a.V + (size_t)i * NV + k0 + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < NQ; ++u) st4(Vs + (ig + 16 * u) * ES + 4 * c4, v[u]);
    } else {
        for (int e = tid; e < HR * CW; e += NT) {
            const int i = e / CW, cc = e - i * CW;
            Vs[i * ES + cc] = (i < H && cc < ncols) ? a.V[(size_t)i * NV + k0 + cc] : 0.f;
        }
    }
    if (tid < CW) cs[tid] = tid < ncols ? a.c[k0 + tid] : 0.f;
    for (int e = tid; e < 32 * HPP; e += NT) hs[e] = 0.f;
    for (int e = tid; e < HR * HT; e += NT) hsT[e] = 0.f;
    if (MODE == 1 && !a.beta) {
        // Gradient mode: zero fill of the token-gradient matrix, an even share of its rows per
        // strip, done now, while the forward loop runs.  The rows of the tokens that occur in the
        // window are left alone: the loop workgroup writes those in full, and nothing orders the
        // two workgroups.
        __shared__ int s_x[MAXT];
        __shared__ unsigned char s_skip[512];
        const int per = (a.NVin + S - 1) / S;
        const int r_lo = min(a.NVin, g * per), r_hi = min(a.NVin, r_lo + per);
        if (tid < T) s_x[tid] = a.ids[tid];
        for (int r0 = r_lo; r0 < r_hi; r0 += 512) {      // 512 rows at a time
            __syncthreads();
            {
                bool hit = false;
                for (int u = 0; u < T; ++u) hit = hit || s_x[u] == r0 + tid;
                s_skip[tid] = hit ? 1 : 0;
            }
            __syncthreads();
            const int rows = min(512, r_hi - r0);
            if ((H & 3) == 0) {
                const int H4 = H / 4, total = rows * H4;
                const float invH4 = 1.0f / (float)H4;
                for (int e = tid; e < total; e += NT) {
                    int row = (int)((float)e * invH4);
                    if (row * H4 > e) --row; else if ((row + 1) * H4 <= e) ++row;
                    if (!s_skip[row])
                        reinterpret_cast<float4*>(a.dWx + (size_t)r0 * H)[e] = make_float4(0.f, 0.f, 0.f, 0.f);
                }
            } else {
                const int total = rows * H;
                for (int e = tid; e < total; e += NT)
                    if (!s_skip[e / H]) a.dWx[(size_t)r0 * H + e] = 0.f;
            }
        }
    }
    int ny = tid < T ? a.ys[tid] : 0;               // targets of window 0
    if (tid == 0) s_abort = 0;
    __syncthreads();
    TS(11);

    for (long long w = 0; w < a.n_windows; ++w) {
        TS(0);
        const unsigned tag = a.tag0 + (unsigned)w;
        if (tid < T) {
            s_y[tid] = ny;
            if (w + 1 < a.n_windows) ny = a.ys[(size_t)(w + 1) * T + tid];
        }
        // ---- all hidden rows of the window ---------------------------------------------------
        {
            const int n = T * H;
            for (int e0 = tid; e0 < n; e0 += 4 * NT) {
                unsigned long long wd[4];
                long long idx[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) idx[u] = e0 + u * NT < n ? e0 + u * NT : -1;
                if (!wait4(a.hbox, idx, tag, a.spin_limit, wd)) s_abort = 1;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = e0 + u * NT;
                    if (e >= n) continue;
                    const int r = e / H, i = e - r * H;
                    const float v = tagged_value(wd[u]);
                    hs[r * HPP + i] = v;
                    hsT[i * HT + r] = v;
                }
            }
        }
        __syncthreads();
        if (s_abort) {
            if (tid == 0) atomicExch(a.status, 1);
            return;
        }
        TS(1);

        f32x4 zreg[2];                    // logits of this lane's column, rows 4kg.. of each pass
#pragma unroll
        for (int ps = 0; ps < 2; ++ps) {
            zreg[ps] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (ps >= npass) continue;
            const int n0 = 16 * ps;
            // ---- logits of the wavefront's 16 columns for 16 rows ---------------------------
            {
                float4 ha[NQ];
                float vb[KC];
#pragma unroll
                for (int u = 0; u < NQ; ++u) ha[u] = ld4(hs + (n0 + m) * HPP + kg * KC + 4 * u);
#pragma unroll
                for (int j = 0; j < KC; ++j) vb[j] = Vs[(kg * KC + j) * ES + cown];
                const float cb = cs[cown];
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u = 0; u < NQ; ++u) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ha[u].x, vb[4 * u], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ha[u].y, vb[4 * u + 1], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ha[u].z, vb[4 * u + 2], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ha[u].w, vb[4 * u + 3], acc, 0, 0, 0);
                }
                const bool cin = cown < ncols;
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = cin ? acc[r] + cb : -INFINITY;
                zreg[ps] = acc;
            }
            // ---- maximum per row over the strip: 16 columns in the wavefront, 8 wavefronts via LDS ----
            {
                float4 tm;
                float* tp = &tm.x;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float v = zreg[ps][r];
                    v = fmaxf(v, dpp<0xB1>(v)); v = fmaxf(v, dpp<0x4E>(v));
                    v = fmaxf(v, dpp<0x141>(v)); v = fmaxf(v, dpp<0x140>(v));
                    tp[r] = v;
                }
                if (m == 0) st4(tmax + wave * 16 + 4 * kg, tm);
            }
            lds_barrier();
            TS(9);
            float mx[4];
            {
                float4 t8[8];
                int yv[4];
#pragma unroll
                for (int wv = 0; wv < 8; ++wv) t8[wv] = ld4(tmax + wv * 16 + 4 * kg);
#pragma unroll
                for (int r = 0; r < 4; ++r) yv[r] = s_y[min(n0 + 4 * kg + r, T - 1)];
                float4 mm = t8[0];
#pragma unroll
                for (int wv = 1; wv < 8; ++wv) {
                    mm.x = fmaxf(mm.x, t8[wv].x); mm.y = fmaxf(mm.y, t8[wv].y);
                    mm.z = fmaxf(mm.z, t8[wv].z); mm.w = fmaxf(mm.w, t8[wv].w);
                }
                mx[0] = mm.x; mx[1] = mm.y; mx[2] = mm.z; mx[3] = mm.w;
                float4 sm;
                float* sp = &sm.x;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float e = __expf(zreg[ps][r] - mx[r]);
                    es[(4 * kg + r) * ESE + cown] = e;
                    sp[r] = sum16(e);
                    const int n = n0 + 4 * kg + r;
                    if (n < T && yv[r] - k0 == cown) tagged_store(a.zybox + n, tag, zreg[ps][r]);
                }
                if (m == 0) st4(tsum + wave * 16 + 4 * kg, sm);
            }
            lds_barrier();
            TS(10);
            if (tid < 16 && n0 + tid < T) {   // strip statistics of row n0 + tid
                float tm8[8], ts8[8];
#pragma unroll
                for (int wv = 0; wv < 8; ++wv) { tm8[wv] = tmax[wv * 16 + tid]; ts8[wv] = tsum[wv * 16 + tid]; }
                float mmx = tm8[0], ss = ts8[0];
#pragma unroll
                for (int wv = 1; wv < 8; ++wv) { mmx = fmaxf(mmx, tm8[wv]); ss += ts8[wv]; }
                unsigned long long* st = a.statbox + ((size_t)(n0 + tid) * S + g) * 2;
                tagged_store(st, tag, mmx);
                tagged_store(st + 1, tag, ss);
            }
            // ---- share of the softmax part of G relative to the strip maximum -------------------
            if (wave < NQ) {
                float4 ea[8], vb4[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    ea[u] = ld4(es + m * ESE + 32 * kg + 4 * u);
                    vb4[u] = ld4(Vs + (16 * wave + m) * ES + 32 * kg + 4 * u);
                }
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ea[u].x, vb4[u].x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ea[u].y, vb4[u].y, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ea[u].z, vb4[u].z, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ea[u].w, vb4[u].w, acc, 0, 0, 0);
                }
                const int i = 16 * wave + m;
                if (i < H) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int n = n0 + 4 * kg + r;
                        if (n < T) tagged_store(a.pbox + ((size_t)g * T + n) * H + i, tag, acc[r]);
                    }
                }
            }
            if (ps + 1 < npass) lds_barrier();   // the next pass overwrites tmax, tsum and es
        }
        // column y_n of V for the rows whose target lies in this strip
        for (int e = tid; e < T * H; e += NT) {
            const int n = e / H, i = e - n * H;
            const int yl = s_y[n] - k0;
            if (yl >= 0 && yl < CW) tagged_store(a.vybox + e, tag, Vs[i * ES + yl]);
        }

        TS(4);
        // ---- statistics of all strips -> lse per row and the strips' weights -----------------
        {
            const int cnt = T * S * 2;
            for (int w0 = tid; w0 < cnt; w0 += 4 * NT) {
                unsigned long long wd[4];
                long long idx[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) idx[u] = w0 + u * NT < cnt ? w0 + u * NT : -1;
                if (!wait4(a.statbox, idx, tag, a.spin_limit, wd)) s_abort = 1;
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (w0 + u * NT < cnt) stage[w0 + u * NT] = tagged_value(wd[u]);
            }
            if (g == S - 1 && tid < T) {   // target logits, for the loss (read before G is published)
                float v = 0.f;
                if (!tagged_wait(a.zybox + tid, tag, a.spin_limit, v)) s_abort = 1;
                zy_s[tid] = v;
            }
        }
        __syncthreads();
        if (s_abort) {
            if (tid == 0) atomicExch(a.status, 1);
            return;
        }
        TS(5);
        // The first batch of this strip's slice of G is requested before the row statistics are
        // merged (the shares were published a moment ago; the merge hides the round trip).
        const int gn = T * H, gper = (gn + S - 1) / S;
        const int o_lo = min(gn, g * gper), o_hi = min(gn, o_lo + gper);
        const int gj = tid & 31, gslot = tid >> 5;
        unsigned long long pw4[4] = {0ull, 0ull, 0ull, 0ull}, vy0 = 0ull;
        if (o_lo < o_hi) {
            const int oc = min(o_lo + gslot, o_hi - 1);
#pragma unroll
            for (int u = 0; u < 4; ++u) pw4[u] = tagged_load(a.pbox + (size_t)min(gj + 32 * u, S - 1) * gn + oc);
            vy0 = tagged_load(a.vybox + oc);
        }
        // lse_t = M + log(sum_g s_g exp(m_g - M)), M = max_g m_g; weight of strip g:
        // exp(m_g - lse_t) = exp(m_g - M) / sum.  32 lanes per row, strips in lane-strided order.
        auto merge = [&](auto per_lane) {
            constexpr int NP = decltype(per_lane)::value;     // strips per lane: S <= 32 * NP
            for (int t = tid >> 5; t < T; t += NT / 32) {
                const int j = tid & 31;
                float2 ms[NP];
#pragma unroll
                for (int u = 0; u < NP; ++u)
                    ms[u] = *reinterpret_cast<const float2*>(stage + (t * S + min(j + 32 * u, S - 1)) * 2);
                __builtin_amdgcn_sched_barrier(0);            // all reads in flight before the first use
                float mg[NP], sg[NP];
                float M = -INFINITY;
#pragma unroll
                for (int u = 0; u < NP; ++u) {
                    const bool in = j + 32 * u < S;
                    mg[u] = in ? ms[u].x : -INFINITY;
                    sg[u] = in ? ms[u].y : 0.f;
                    M = fmaxf(M, mg[u]);
                }
                M = fmaxf(M, dpp<0xB1>(M)); M = fmaxf(M, dpp<0x4E>(M));
                M = fmaxf(M, dpp<0x141>(M)); M = fmaxf(M, dpp<0x140>(M));
                {
                    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(M), __float_as_uint(M), false, false);
                    M = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
                }
                float sum = 0.f;
#pragma unroll
                for (int u = 0; u < NP; ++u) { mg[u] = __expf(mg[u] - M); sum = fmaf(sg[u], mg[u], sum); }
                sum = sum32(sum);
                const float rs = fast_rcp(sum);
#pragma unroll
                for (int u = 0; u < NP; ++u)
                    if (j + 32 * u < S) wts[t * S + j + 32 * u] = mg[u] * rs;
                if (j == 0) lse_s[t] = M + __logf(sum);
            }
        };
        if (S <= 96) merge(std::integral_constant<int, 3>{});
        else if (S <= 160) merge(std::integral_constant<int, 5>{});
        else merge(std::integral_constant<int, 8>{});
        lds_barrier();

        TS(6);
        // ---- this strip's slice of G: 32 lanes per output walk the strips in a fixed order ------
#pragma unroll
        for (int u = 0; u < 4; ++u) consume(pw4[u]);
        consume(vy0);
        {
            const int n = gn, j = gj, slot = gslot;
            for (int o0 = o_lo; o0 < o_hi; o0 += NT / 32) {
                const int o = o0 + slot;
                const bool have = o < o_hi;
                const int oc = have ? o : o_hi - 1;
                const int t = oc / H;
                float sum = 0.f;
                unsigned long long vyw = o0 == o_lo ? vy0 : tagged_load(a.vybox + oc);
                for (int g0 = j; g0 < S; g0 += 32 * 4) {
                    unsigned long long wd[4];
                    float wt[4];
                    long long idx[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int g2 = g0 + 32 * u;
                        idx[u] = g2 < S ? (long long)g2 * n + oc : -1;
                        wt[u] = wts[t * S + min(g2, S - 1)];
                    }
                    if (o0 == o_lo && g0 == j) {   // requested before the merge of the statistics
                        bool stale = false;
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            wd[u] = pw4[u];
                            stale = stale || (idx[u] >= 0 && !tagged_ok(wd[u], tag));
                        }
                        if (stale && !wait4(a.pbox, idx, tag, a.spin_limit, wd)) s_abort = 1;
                    } else if (!wait4(a.pbox, idx, tag, a.spin_limit, wd)) {
                        s_abort = 1;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (idx[u] >= 0) sum = fmaf(wt[u], tagged_value(wd[u]), sum);
                }
                sum = sum32(sum);
                if (have && j == 0) {
                    for (int spins = 0; !tagged_ok(vyw, tag); ++spins) {
                        if (spins > a.spin_limit) { s_abort = 1; break; }
                        vyw = tagged_load(a.vybox + oc);
                    }
                    tagged_store(a.gbox + oc, tag, (sum - tagged_value(vyw)) * invN);
                }
            }
        }
        TS(7);
        if (g == S - 1 && wave == 0) {
            float v = lane < T ? lse_s[lane] - zy_s[lane] : 0.f;
            v = sum64(v);
            if (lane == 0 && a.losses) a.losses[w] = v * invN;
        }

        // ---- update of the resident columns: V -= lr Hs^T dZ, c -= lr colsum(dZ) --------------
        {
            f32x4 dz[2];
            float dcs = 0.f;
#pragma unroll
            for (int ps = 0; ps < 2; ++ps) {
                float l[4];
                int yv[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int n = min(16 * ps + 4 * kg + r, T - 1);
                    l[r] = lse_s[n];
                    yv[r] = s_y[n];
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const bool on = 16 * ps + 4 * kg + r < T;
                    const float d = (__expf(zreg[ps][r] - l[r]) - (yv[r] - k0 == cown ? 1.f : 0.f)) * invN;
                    dz[ps][r] = on ? d : 0.f;
                    dcs += dz[ps][r];
                }
            }
            dcs = swap32_sum(swap16_sum(dcs));          // over the four lane groups
            float4 ht[NQ][2];
            float vold[NQ][4];
#pragma unroll
            for (int it = 0; it < NQ; ++it) {
                ht[it][0] = ld4(hsT + (16 * it + m) * HT + 4 * kg);
                ht[it][1] = ld4(hsT + (16 * it + m) * HT + 16 + 4 * kg);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (MODE == 0) {
                        vold[it][r] = Vs[(16 * it + 4 * kg + r) * ES + cown];
                    } else {        // gradient mode: the old gradient when accumulating, else nothing
                        const int i = 16 * it + 4 * kg + r;
                        vold[it][r] = (a.beta && i < H && cown < ncols) ? a.dV[(size_t)i * NV + k0 + cown] : 0.f;
                    }
                }
            }
            const float cold = MODE == 0 ? cs[cown] : ((a.beta && kg == 0 && cown < ncols) ? a.dc[k0 + cown] : 0.f);
#pragma unroll
            for (int it = 0; it < NQ; ++it) {
                f32x4 d = {0.f, 0.f, 0.f, 0.f};
                d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][0].x, dz[0][0], d, 0, 0, 0);
                d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][0].y, dz[0][1], d, 0, 0, 0);
                d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][0].z, dz[0][2], d, 0, 0, 0);
                d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][0].w, dz[0][3], d, 0, 0, 0);
                if (npass > 1) {
                    d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][1].x, dz[1][0], d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][1].y, dz[1][1], d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][1].z, dz[1][2], d, 0, 0, 0);
                    d = __builtin_amdgcn_mfma_f32_16x16x4f32(ht[it][1].w, dz[1][3], d, 0, 0, 0);
                }
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (MODE == 0) {
                        Vs[(16 * it + 4 * kg + r) * ES + cown] = fmaf(-a.lr, d[r], vold[it][r]);
                    } else {
                        const int i = 16 * it + 4 * kg + r;
                        if (i < H && cown < ncols) a.dV[(size_t)i * NV + k0 + cown] = vold[it][r] + d[r];
                    }
                }
            }
            if (MODE == 0) {
                if (kg == 0) cs[cown] = fmaf(-a.lr, dcs, cold);
            } else if (kg == 0 && cown < ncols) {
                a.dc[k0 + cown] = cold + dcs;
            }
        }
        __syncthreads();
        if (s_abort) {   // a wait in the G slice expired
            if (tid == 0) atomicExch(a.status, 1);
            return;
        }
        TS(8);
    }
    TS_FLUSH;

    if (MODE == 1) return;
    // ---- write the columns back --------------------------------------------------------------
    for (int e = tid; e < H * CW; e += NT) {
        const int i = e / CW, cc = e - i * CW;
        if (cc < ncols) a.V[(size_t)i * NV + k0 + cc] = Vs[i * ES + cc];
    }
    if (tid < ncols) a.c[k0 + tid] = cs[tid];
}

// ---------------------------------------------------------------------------------------
// Workgroup 0 in gradient mode: one window, parameters untouched; dWh is accumulated in registers
// (row layout of Wh) one rank-1 term per reverse step, db in a register, the touched rows of dWx
// from the deltas in LDS.
template <int ACT, int NQ>
__device__ __forceinline__ void loop_body_grad(const StreamArgs& a, float* smem) {
    constexpr int HP = 16 * NQ;
    __shared__ int s_ids[MAXT];
    __shared__ int s_first[MAXT];
    __shared__ int4 s_ch[MAXT];
    __shared__ int s_abort;
    const int H = a.H, T = a.T, tid = threadIdx.x;
    const int own = tid >> 2, q = tid & 3;
    const int ownc = min(own, HP - 1);
    const bool live = own < H, lead = live && q == 0;
    const unsigned tag = a.tag0;
    float* Hc = smem;                        // [T+1][HP]  h_{-1} .. h_{T-1}
    float* Dl = Hc + (T + 1) * HP;           // [T][HP] delta_t
    float* Ul = Dl + T * HP;                 // [T][HP] rows of Wx of the window's tokens
    float* Gl = Ul + T * HP;                 // [T][HP] G_t
    const int lds_floats = ((T + 1) + 3 * T) * HP;
    TS_DECL;
    for (int i = tid; i < lds_floats; i += NT) smem[i] = 0.f;

    float4 wf[NQ], wb[NQ], ga[NQ];           // Wh by rows, by columns; dWh by rows
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int k = 4 * (q + 4 * u);
        if ((H & 3) == 0) {
            wf[u] = (live && k < H) ? ld4(a.Wh + (size_t)own * H + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        } else {
            float f[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (live && k + e < H) f[e] = a.Wh[(size_t)own * H + k + e];
            wf[u] = make_float4(f[0], f[1], f[2], f[3]);
        }
        ga[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const float bj = lead ? a.b[own] : 0.f;
    const int myid = tid < T ? a.ids[tid] : 0;
    if (tid == 0) s_abort = 0;
    __syncthreads();
    if (tid < T) s_ids[tid] = myid;
    if (lead) Hc[own] = a.h0 ? a.h0[own] : 0.f;
    __syncthreads();
    if (tid < T) {       // first step with the same token, and the next four
        int f = tid, nc = 0;
        int4 ch = make_int4(-1, -1, -1, -1);
        for (int u0 = 0; u0 < T; u0 += 8) {
            int iv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) iv[k] = s_ids[min(u0 + k, T - 1)];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int idx = u0 + k;
                if (idx < T && iv[k] == myid) {
                    if (idx < f) f = idx;
                    if (idx > tid) {
                        if (nc == 0) ch.x = idx; else if (nc == 1) ch.y = idx;
                        else if (nc == 2) ch.z = idx; else if (nc == 3) ch.w = idx;
                        ++nc;
                    }
                }
            }
        }
        s_first[tid] = f;
        s_ch[tid] = ch;
    }
    if (lead) {
        for (int t0 = 0; t0 < T; t0 += 8) {
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = a.Wx[(size_t)s_ids[min(t0 + u, T - 1)] * H + own];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                consume(v[u]);
                if (t0 + u < T) Ul[(t0 + u) * HP + own] = v[u];
            }
        }
    }
    __syncthreads();
    TS(0);

    for (int s = 0; s < T; ++s) {
        const float4* v4 = reinterpret_cast<const float4*>(Hc + s * HP) + q;
        float4 x[NQ];
#pragma unroll
        for (int u = 0; u < NQ; ++u) x[u] = v4[4 * u];
        const float uin = Ul[s * HP + ownc];
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int u = 0; u < NQ; ++u) {
            if (u & 1) acc1 = dot4(wf[u], x[u], acc1); else acc0 = dot4(wf[u], x[u], acc0);
        }
        const float acc = sum4(acc0 + acc1);
        if (lead) {
            const float hv = activate<ACT>(acc + uin + bj);
            Hc[(s + 1) * HP + own] = hv;
            tagged_store(a.hbox + (size_t)s * H + own, tag, hv);
        }
        lds_barrier();
    }
    TS(1);
    // while the strips work: the column copy of Wh for the reverse loop (strided reads, off the
    // critical path here) and the states the caller asked for
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int k = 4 * (q + 4 * u);
        float g[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (live && k + e < H) g[e] = a.Wh[(size_t)(k + e) * H + own];
        wb[u] = make_float4(g[0], g[1], g[2], g[3]);
    }
    if (lead) {
        if (a.h_all)
            for (int t = 0; t <= T; ++t) a.h_all[(size_t)t * H + own] = Hc[t * HP + own];
        if (a.h_last) a.h_last[own] = Hc[T * HP + own];
    }
    const float dhl = (lead && a.dh_last) ? a.dh_last[own] : 0.f;
    {
        const int n = T * H;
        for (int e0 = tid; e0 < n; e0 += 4 * NT) {
            unsigned long long wd[4];
            long long idx[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) idx[u] = e0 + u * NT < n ? e0 + u * NT : -1;
            if (!wait4(a.gbox, idx, tag, a.spin_limit, wd)) s_abort = 1;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * NT;
                if (e >= n) continue;
                const int t = e / H;
                Gl[t * HP + (e - t * H)] = tagged_value(wd[u]);
            }
        }
    }
    __syncthreads();
    if (s_abort) {
        if (tid == 0) atomicExch(a.status, 1);
        return;
    }
    TS(3);
    float bsum = 0.f;
    if (lead) {
        const float h = Hc[T * HP + own];
        const float d = (Gl[(T - 1) * HP + own] + dhl) * act_grad<ACT>(h);
        Dl[(T - 1) * HP + own] = d;
        bsum = d;
    }
    lds_barrier();
    for (int t = T - 2; t >= 0; --t) {
        const float4* d4 = reinterpret_cast<const float4*>(Dl + (t + 1) * HP) + q;
        const float4* h4 = reinterpret_cast<const float4*>(Hc + (t + 1) * HP) + q;
        float4 x[NQ], hh[NQ];
#pragma unroll
        for (int u = 0; u < NQ; ++u) { x[u] = d4[4 * u]; hh[u] = h4[4 * u]; }
        const float dj = Dl[(t + 1) * HP + ownc];
        const float g = Gl[t * HP + ownc], h = Hc[(t + 1) * HP + ownc];
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int u = 0; u < NQ; ++u) {
            if (u & 1) acc1 = dot4(wb[u], x[u], acc1); else acc0 = dot4(wb[u], x[u], acc0);
        }
        const float acc = sum4(acc0 + acc1);
        if (lead) {
            const float d = (g + acc) * act_grad<ACT>(h);
            Dl[t * HP + own] = d;
            bsum += d;
        }
#pragma unroll
        for (int u = 0; u < NQ; ++u) rank1(ga[u], -dj, hh[u]);   // dWh += delta_{t+1} (x) h_t
        lds_barrier();
    }
    {   // delta_0 (x) h_{-1}, and dh0 = Wh^T delta_0
        const float4* h4 = reinterpret_cast<const float4*>(Hc) + q;
        const float4* d4 = reinterpret_cast<const float4*>(Dl) + q;
        float4 hh[NQ], x[NQ];
#pragma unroll
        for (int u = 0; u < NQ; ++u) { hh[u] = h4[4 * u]; x[u] = d4[4 * u]; }
        const float dj = Dl[ownc];
#pragma unroll
        for (int u = 0; u < NQ; ++u) rank1(ga[u], -dj, hh[u]);
        float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
        for (int u = 0; u < NQ; ++u) {
            if (u & 1) acc1 = dot4(wb[u], x[u], acc1); else acc0 = dot4(wb[u], x[u], acc0);
        }
        const float acc = sum4(acc0 + acc1);
        if (lead && a.dh0) a.dh0[own] = acc;
    }
    TS(4);
    // gradients of the recurrent layer; overwrite and accumulate as separate loops (a load in a
    // storing loop would wait for the previous store's acknowledgement)
    if (live) {
        if ((H & 3) == 0) {
            float4 old[NQ];
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                const int k = 4 * (q + 4 * u);
                old[u] = (a.beta && k < H) ? ld4(a.dWh + (size_t)own * H + k) : make_float4(0.f, 0.f, 0.f, 0.f);
            }
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                const int k = 4 * (q + 4 * u);
                if (k < H)
                    st4(a.dWh + (size_t)own * H + k, make_float4(old[u].x + ga[u].x, old[u].y + ga[u].y,
                                                                 old[u].z + ga[u].z, old[u].w + ga[u].w));
            }
        } else {
            float old[NQ][4];
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                const int k = 4 * (q + 4 * u);
#pragma unroll
                for (int e = 0; e < 4; ++e) old[u][e] = (a.beta && k + e < H) ? a.dWh[(size_t)own * H + k + e] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                const int k = 4 * (q + 4 * u);
                const float f[4] = {ga[u].x, ga[u].y, ga[u].z, ga[u].w};
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (k + e < H) a.dWh[(size_t)own * H + k + e] = old[u][e] + f[e];
            }
        }
    }
    if (lead) a.db[own] = (a.beta ? a.db[own] : 0.f) + bsum;
    if (live) {          // rows of dWx: the four lanes of a hidden unit share the steps
        for (int t = q; t < T; t += 4) {
            if (s_first[t] != t) continue;
            float sum = Dl[t * HP + own];
            int4 c = s_ch[t];
            while (c.x >= 0) {
                const float v0 = Dl[c.x * HP + own], v1 = Dl[max(c.y, 0) * HP + own];
                const float v2 = Dl[max(c.z, 0) * HP + own], v3 = Dl[max(c.w, 0) * HP + own];
                const int4 more = s_ch[max(c.w, 0)];
                sum += v0;
                if (c.y >= 0) sum += v1;
                if (c.z >= 0) sum += v2;
                if (c.w >= 0) sum += v3;
                c = c.w >= 0 ? more : make_int4(-1, -1, -1, -1);
            }
            float* dst = a.dWx + (size_t)s_ids[t] * H + own;
            *dst = (a.beta ? *dst : 0.f) + sum;
        }
    }
    TS(5);
    TS_FLUSH;
}

// The loop workgroup cannot finish a window before every strip has started (each element of G needs
// every strip's share), so it is the one that records the last tag used on these boxes, for the
// next launch on them.
template <int ACT, int NQ>
__global__ __launch_bounds__(NT) void train_stream_kernel(StreamArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    if (blockIdx.x == 0) {
        loop_body<ACT, NQ>(a, smem);
        if (threadIdx.x == 0) tag_word_store(a.tagword, a.tag0 + (unsigned)(a.n_windows - 1));
    } else {
        strip_body<NQ, 0>(a, (int)blockIdx.x - 1, smem);
    }
}

template <int ACT, int NQ>
__global__ __launch_bounds__(NT) void window_kernel(StreamArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    a.tag0 = next_tag(tag_word_load(a.tagword));   // requested first; needed at the first exchange
    if (blockIdx.x == 0) {
        loop_body_grad<ACT, NQ>(a, smem);
        if (threadIdx.x == 0) tag_word_store(a.tagword, a.tag0);
    } else {
        strip_body<NQ, 1>(a, (int)blockIdx.x - 1, smem);
    }
}

template <int ACT>
const void* pick_window_kernel(int nq) {
    switch (nq) {
        case 2: return (const void*)window_kernel<ACT, 2>;
        case 4: return (const void*)window_kernel<ACT, 4>;
        case 7: return (const void*)window_kernel<ACT, 7>;
        default: return (const void*)window_kernel<ACT, 8>;
    }
}

template <int ACT>
const void* pick_kernel(int nq) {
    switch (nq) {
        case 2: return (const void*)train_stream_kernel<ACT, 2>;
        case 4: return (const void*)train_stream_kernel<ACT, 4>;
        case 7: return (const void*)train_stream_kernel<ACT, 7>;
        default: return (const void*)train_stream_kernel<ACT, 8>;
    }
}
int pick_nq(int H) {
    const int need = (H + 15) / 16;
    return need <= 2 ? 2 : need <= 4 ? 4 : need <= 7 ? 7 : 8;
}

struct StreamPlan { size_t status, hbox, gbox, vybox, zybox, statbox, pbox, total; int S; };

StreamPlan stream_plan(const rnn_dims* d) {
    StreamPlan p{};
    const size_t T = (size_t)d->seq_len, H = (size_t)d->hidden;
    p.S = (d->out_dim + CW - 1) / CW;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
    p.status = take(256);
    p.hbox = take(T * H * 8);
    p.gbox = take(T * H * 8);
    p.vybox = take(T * H * 8);
    p.zybox = take(T * 8);
    p.statbox = take(T * p.S * 2 * 8);
    p.pbox = take((size_t)p.S * T * H * 8);
    p.total = off;
    return p;
}

int stream_supported(const rnn_dims* d) {
    if (!d) return RNN_EINVAL;
    if (d->in_dim <= 0 || d->hidden <= 0 || d->out_dim <= 0 || d->seq_len <= 0 || d->batch <= 0)
        return RNN_EINVAL;
    if (d->act != RNN_ACT_SIGMOID && d->act != RNN_ACT_TANH) return RNN_EINVAL;
    if (d->input_kind != RNN_INPUT_TOKENS && d->input_kind != RNN_INPUT_DENSE) return RNN_EINVAL;
    if (d->loss_kind != RNN_LOSS_SOFTMAX_CE && d->loss_kind != RNN_LOSS_LINEAR_MSE) return RNN_EINVAL;
    if (d->flags & ~RNN_FLAG_SYNC) return RNN_EINVAL;
    if (d->input_kind != RNN_INPUT_TOKENS || d->loss_kind != RNN_LOSS_SOFTMAX_CE) return RNN_EUNSUPPORTED;
    if (d->batch != 1 || d->in_dim != d->out_dim) return RNN_EUNSUPPORTED;
    if (d->hidden > MAXH || d->seq_len > MAXT) return RNN_EUNSUPPORTED;
    const int S = (d->out_dim + CW - 1) / CW;
    if (S + 1 > 256 || d->seq_len * S > MAX_TS) return RNN_EUNSUPPORTED;
    if (strip_lds_floats(pick_nq(d->hidden), d->seq_len, S) * 4 > 158 * 1024) return RNN_EUNSUPPORTED;
    if (loop_lds_floats(d->seq_len, pick_nq(d->hidden)) * 4 > 158 * 1024) return RNN_EUNSUPPORTED;
    return RNN_OK;
}

// the fused one-window call accepts what the stream driver accepts, plus different vocabulary
// sizes on the two sides and the accumulate flag
int window_supported(const rnn_dims* d) {
    if (!d) return RNN_EINVAL;
    rnn_dims t = *d;
    if (t.flags & ~(RNN_FLAG_SYNC | RNN_FLAG_ACCUMULATE | RNN_FLAG_COOPERATIVE)) return RNN_EINVAL;
    t.flags &= RNN_FLAG_SYNC;
    if (t.in_dim <= 0) return RNN_EINVAL;
    t.in_dim = t.out_dim;
    return stream_supported(&t);
}

void bind_boxes(StreamArgs& a, void* workspace, const StreamPlan& pl) {
    char* ws = static_cast<char*>(workspace);
    a.S = pl.S;
    a.status = reinterpret_cast<int32_t*>(ws + pl.status);
    a.tagword = reinterpret_cast<unsigned*>(ws + pl.status) + 1;
    a.hbox = reinterpret_cast<unsigned long long*>(ws + pl.hbox);
    a.gbox = reinterpret_cast<unsigned long long*>(ws + pl.gbox);
    a.vybox = reinterpret_cast<unsigned long long*>(ws + pl.vybox);
    a.zybox = reinterpret_cast<unsigned long long*>(ws + pl.zybox);
    a.statbox = reinterpret_cast<unsigned long long*>(ws + pl.statbox);
    a.pbox = reinterpret_cast<unsigned long long*>(ws + pl.pbox);
    a.spin_limit = wait_limit();
}

// dynamic LDS above 64 KB has to be allowed once per kernel
hipError_t allow_lds(const void* fn, size_t bytes) {
    static const void* seen[32];
    static size_t seen_bytes[32];
    static int n_seen = 0;
    if (bytes <= 64 * 1024) return hipSuccess;
    for (int i = 0; i < n_seen; ++i)
        if (seen[i] == fn && seen_bytes[i] >= bytes) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && n_seen < 32) { seen[n_seen] = fn; seen_bytes[n_seen] = bytes; ++n_seen; }
    return e;
}

// Can `blocks` workgroups of this kernel be resident at once on the current device?  The
// one-window kernels wait for each other inside the launch, so a plain launch is only used when
// the whole grid fits the chip by itself; otherwise the launch is cooperative (the runtime then
// refuses what cannot be co-resident instead of letting it spin).  Asked once per kernel and size.
bool fits_the_chip(const void* fn, size_t lds, int blocks) {
    struct Seen { const void* fn; size_t lds; int dev; int capacity; };
    static Seen seen[32];
    static int n_seen = 0;
    static std::mutex mu;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    std::lock_guard<std::mutex> lock(mu);
    for (int i = 0; i < n_seen; ++i)
        if (seen[i].fn == fn && seen[i].lds == lds && seen[i].dev == dev) return blocks <= seen[i].capacity;
    int per_cu = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, NT, lds) != hipSuccess) return false;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
    const int capacity = per_cu * cus;
    if (n_seen < 32) seen[n_seen++] = Seen{fn, lds, dev, capacity};
    return blocks <= capacity;
}

// Argument checks shared by the two forms of the one-window call.
int window_args_ok(const rnn_dims* dims, const rnn_params* params, const int32_t* x, const int32_t* targets,
                   const float* h0, const float* dh_last, const float* h_all, const float* h_last,
                   const float* loss, const rnn_grads* grads, const float* dh0) {
    const int rc = window_supported(dims);
    if (rc != RNN_OK) return rc;
    if (!params || !params->Wx || !params->Wh || !params->b || !params->V || !params->c || !x ||
        !targets || !loss || !grads || !grads->dWx || !grads->dWh || !grads->db || !grads->dV || !grads->dc)
        return RNN_EINVAL;
    auto bad16 = [](const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u); };
    auto bad4 = [](const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 3u); };
    if (bad16(params->Wx) || bad16(params->Wh) || bad16(params->b) || bad16(params->V) || bad16(params->c) ||
        bad16(grads->dWx) || bad16(grads->dWh) || bad16(grads->db) || bad16(grads->dV) || bad16(grads->dc) ||
        bad4(x) || bad4(targets) || bad4(h0) || bad4(dh_last) || bad4(h_all) || bad4(h_last) || bad4(loss) ||
        bad4(dh0))
        return RNN_EINVAL;
    return RNN_OK;
}

// One window on the exchange boxes at `workspace` (checked by the caller).  status_override: where a
// bounded wait that expires leaves its 1 instead of the workspace's own status word.
int launch_window(const rnn_dims* dims, const rnn_params* params, const int32_t* x, const int32_t* targets,
                  const float* h0, const float* dh_last, float* h_all, float* h_last, float* loss,
                  const rnn_grads* grads, float* dh0, void* workspace, const StreamPlan& pl,
                  int32_t* status_override, hipStream_t s) {
    StreamArgs a{};
    a.Wx = const_cast<float*>(params->Wx); a.Wh = const_cast<float*>(params->Wh);
    a.b = const_cast<float*>(params->b); a.V = const_cast<float*>(params->V); a.c = const_cast<float*>(params->c);
    a.ids = x; a.ys = targets; a.n_windows = 1; a.lr = 1.0f; a.tag0 = 0u;   // the kernel reads the tag word
    a.h0 = h0; a.h_last = h_last; a.losses = loss; a.h_all = h_all; a.dh_last = dh_last; a.dh0 = dh0;
    a.dWx = grads->dWx; a.dWh = grads->dWh; a.db = grads->db; a.dV = grads->dV; a.dc = grads->dc;
    a.beta = (dims->flags & RNN_FLAG_ACCUMULATE) ? 1 : 0;
    a.H = dims->hidden; a.NV = dims->out_dim; a.NVin = dims->in_dim; a.T = dims->seq_len;
    bind_boxes(a, workspace, pl);
    if (status_override) a.status = status_override;

    const int nq = pick_nq(a.H);
    const void* fn = dims->act == RNN_ACT_SIGMOID ? pick_window_kernel<0>(nq) : pick_window_kernel<1>(nq);
    size_t lds = loop_lds_floats(a.T, nq);
    if (strip_lds_floats(nq, a.T, a.S) > lds) lds = strip_lds_floats(nq, a.T, a.S);
    lds *= 4;
    if (allow_lds(fn, lds) != hipSuccess) return RNN_EHIP;
    hipError_t e;
    {
        ProfileScope ps(K_WINDOW, s);
        void* args[] = {&a};
        const bool coop = (dims->flags & RNN_FLAG_COOPERATIVE) || !fits_the_chip(fn, lds, 1 + a.S);
        e = coop ? hipLaunchCooperativeKernel(fn, dim3(1 + a.S), dim3(NT), args, (unsigned)lds, s)
                 : hipLaunchKernel(fn, dim3(1 + a.S), dim3(NT), args, lds, s);
    }
    if (e != hipSuccess) return RNN_EHIP;
    if (dims->flags & RNN_FLAG_SYNC)
        if (hipStreamSynchronize(s) != hipSuccess) return RNN_EHIP;
    return RNN_OK;
}


// ---- the general forms: shapes outside the one-launch kernels --------------------------------------
// rnn_window and rnn_train_stream accept every token / softmax-CE shape.  Where the one-launch
// kernels do not reach (hidden > 128, seq_len > 32, batch > 1, very wide vocabularies) the same
// calls enqueue the launches of rnn_forward -> rnn_loss -> rnn_bptt (and, for the stream, one update
// launch per window) on the caller's stream: same results, same arguments, no host work per step.
// Workspace: a 256-byte header (status word first, as in the one-launch form), then what the
// general form keeps itself, then the three calls' own workspace.
constexpr size_t kHeaderBytes = 256;

struct GeneralPlan {
    rnn_dims d3;                       // the dims the three calls see
    size_t hall, state, grads[5], ws3, ws3_bytes, total;
    size_t n_param[5];
};

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// valid for the general form?  (token ids in, softmax cross-entropy out)
int general_supported(const rnn_dims* d, unsigned allowed_flags) {
    if (!d) return RNN_EINVAL;
    if (d->in_dim <= 0 || d->hidden <= 0 || d->out_dim <= 0 || d->seq_len <= 0 || d->batch <= 0) return RNN_EINVAL;
    if (d->act != RNN_ACT_SIGMOID && d->act != RNN_ACT_TANH) return RNN_EINVAL;
    if (d->flags & ~allowed_flags) return RNN_EINVAL;
    if (d->input_kind != RNN_INPUT_TOKENS || d->loss_kind != RNN_LOSS_SOFTMAX_CE) return RNN_EUNSUPPORTED;
    return RNN_OK;
}

int general_plan(const rnn_dims* d, bool stream, GeneralPlan* out) {
    GeneralPlan g{};
    g.d3 = *d;
    g.d3.flags = d->flags & (RNN_FLAG_SYNC | RNN_FLAG_ACCUMULATE);
    if (stream) g.d3.flags = 0;
    if (rnn_workspace_bytes(&g.d3, &g.ws3_bytes) != RNN_OK) return RNN_EUNSUPPORTED;
    const size_t H = d->hidden, B = d->batch, T = d->seq_len;
    size_t off = kHeaderBytes;
    g.hall = off; off += round256((T + 1) * B * H * 4);
    g.state = off; off += round256(2 * B * H * 4);              // stream: the carried state, two slots
    g.n_param[0] = (size_t)d->in_dim * H; g.n_param[1] = H * H; g.n_param[2] = H;
    g.n_param[3] = H * (size_t)d->out_dim; g.n_param[4] = (size_t)d->out_dim;
    for (int i = 0; i < 5; ++i) {
        g.grads[i] = off;
        if (stream) off += round256(g.n_param[i] * 4);
    }
    g.ws3 = off; off += round256(g.ws3_bytes);
    g.total = off;
    *out = g;
    return RNN_OK;
}

// status word of the header |= status word of the three calls' workspace
__global__ void merge_status_kernel(int32_t* __restrict__ header, const int32_t* __restrict__ inner) {
    if (threadIdx.x == 0 && blockIdx.x == 0 && *inner != 0) *header = 1;
}

// params <- params - lr * grads for the five tensors, one launch
struct SgdArgs { float* p[5]; const float* g[5]; size_t n[5]; float lr; };
__global__ __launch_bounds__(256) void sgd_update_kernel(SgdArgs a) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
#pragma unroll
    for (int t = 0; t < 5; ++t)
        for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.n[t]; i += stride)
            a.p[t][i] -= a.lr * a.g[t][i];
}

int general_window(const rnn_dims* dims, const rnn_params* params, const int32_t* x, const int32_t* targets,
                   const float* h0, const float* dh_last, float* h_all, float* h_last, float* loss,
                   const rnn_grads* grads, float* dh0, void* workspace, const GeneralPlan& g, hipStream_t s) {
    char* ws = static_cast<char*>(workspace);
    float* hall = h_all ? h_all : reinterpret_cast<float*>(ws + g.hall);
    void* ws3 = ws + g.ws3;
    int rc = rnn_forward(&g.d3, params, x, h0, hall, h_last, ws3, g.ws3_bytes, s);
    if (rc == RNN_OK) rc = rnn_loss(&g.d3, params, hall, targets, loss, ws3, g.ws3_bytes, s);
    if (rc == RNN_OK) rc = rnn_bptt(&g.d3, params, x, targets, hall, dh_last, grads, dh0, ws3, g.ws3_bytes, s);
    if (rc != RNN_OK) return rc;
    hipLaunchKernelGGL(merge_status_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<int32_t*>(ws),
                       three_call_status_word(&g.d3, ws3));
    return hipGetLastError() == hipSuccess ? RNN_OK : RNN_EHIP;
}

// Address of this device's copy of the fixed scratch array of rnn_window_static.  In host code the
// array's name is only a handle: the address kernels can use comes from hipGetSymbolAddress, once
// per device (every GPU holds its own copy).  The first call on a device also clears the array, on
// the calling stream, ahead of the window kernel.
int static_scratch(hipStream_t s, void** out) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* ptrs[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RNN_EHIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptrs[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RNN_EHIP;
        if (launch_zero_words(static_cast<int32_t*>(p), (int)(kStaticScratchBytes / 4), s) != hipSuccess)
            return RNN_EHIP;
        ptrs[dev] = p;
    }
    *out = ptrs[dev];
    return RNN_OK;
}

}  // namespace
}  // namespace rnn

extern "C" {

int rnn_window_one_launch(const rnn_dims* dims) {
    using namespace rnn;
    const int rc = window_supported(dims);
    if (rc == RNN_OK) return 1;
    if (rc != RNN_EUNSUPPORTED) return rc;
    const int rg = general_supported(dims, RNN_FLAG_SYNC | RNN_FLAG_ACCUMULATE | RNN_FLAG_COOPERATIVE);
    return rg == RNN_OK ? 0 : rg;
}

int rnn_window_workspace_bytes(const rnn_dims* dims, size_t* bytes) {
    using namespace rnn;
    if (!bytes) return RNN_EINVAL;
    const int rc = window_supported(dims);
    if (rc == RNN_EUNSUPPORTED) {
        GeneralPlan g;
        int rg = general_supported(dims, RNN_FLAG_SYNC | RNN_FLAG_ACCUMULATE | RNN_FLAG_COOPERATIVE);
        if (rg == RNN_OK) rg = general_plan(dims, false, &g);
        if (rg != RNN_OK) return rg;
        *bytes = g.total;
        return RNN_OK;
    }
    if (rc != RNN_OK) return rc;
    *bytes = stream_plan(dims).total;
    return RNN_OK;
}

int rnn_window_workspace_init(const rnn_dims* dims, void* workspace, size_t workspace_bytes, void* hip_stream) {
    using namespace rnn;
    const int rc = window_supported(dims);
    if (rc == RNN_EUNSUPPORTED) {
        GeneralPlan g;
        int rg = general_supported(dims, RNN_FLAG_SYNC | RNN_FLAG_ACCUMULATE | RNN_FLAG_COOPERATIVE);
        if (rg == RNN_OK) rg = general_plan(dims, false, &g);
        if (rg != RNN_OK) return rg;
        if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < g.total)
            return RNN_EWORKSPACE;
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        if (launch_zero_words(static_cast<int32_t*>(workspace), (int)(kHeaderBytes / 4), s) != hipSuccess) return RNN_EHIP;
        return rnn_workspace_init(&g.d3, static_cast<char*>(workspace) + g.ws3, g.ws3_bytes, hip_stream);
    }
    if (rc != RNN_OK) return rc;
    const StreamPlan pl = stream_plan(dims);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < pl.total)
        return RNN_EWORKSPACE;
    return launch_zero_words(static_cast<int32_t*>(workspace), (int)(pl.total / 4),
                             static_cast<hipStream_t>(hip_stream)) == hipSuccess ? RNN_OK : RNN_EHIP;
}

int rnn_window(const rnn_dims* dims, const rnn_params* params, const int32_t* x, const int32_t* targets,
               const float* h0, const float* dh_last, float* h_all, float* h_last, float* loss,
               const rnn_grads* grads, float* dh0, void* workspace, size_t workspace_bytes,
               void* hip_stream) {
    using namespace rnn;
    const int rc = window_args_ok(dims, params, x, targets, h0, dh_last, h_all, h_last, loss, grads, dh0);
    if (rc == RNN_EUNSUPPORTED) {      // outside the one-launch kernel: the launches of the three calls
        GeneralPlan g;
        int rg = general_supported(dims, RNN_FLAG_SYNC | RNN_FLAG_ACCUMULATE | RNN_FLAG_COOPERATIVE);
        if (rg == RNN_OK) rg = general_plan(dims, false, &g);
        if (rg != RNN_OK) return rg;
        if (!params || !x || !targets || !loss || !grads) return RNN_EINVAL;
        if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < g.total)
            return RNN_EWORKSPACE;
        return general_window(dims, params, x, targets, h0, dh_last, h_all, h_last, loss, grads, dh0, workspace, g,
                              static_cast<hipStream_t>(hip_stream));
    }
    if (rc != RNN_OK) return rc;
    const StreamPlan pl = stream_plan(dims);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < pl.total)
        return RNN_EWORKSPACE;
    return launch_window(dims, params, x, targets, h0, dh_last, h_all, h_last, loss, grads, dh0, workspace,
                         pl, nullptr, static_cast<hipStream_t>(hip_stream));
}

int rnn_window_static(const rnn_dims* dims, const rnn_params* params, const int32_t* x, const int32_t* targets,
                      const float* h0, const float* dh_last, float* h_all, float* h_last, float* loss,
                      const rnn_grads* grads, float* dh0, int32_t* status, void* hip_stream) {
    using namespace rnn;
    const int rc = window_args_ok(dims, params, x, targets, h0, dh_last, h_all, h_last, loss, grads, dh0);
    if (rc != RNN_OK) return rc;
    if (status && (reinterpret_cast<uintptr_t>(status) & 3u)) return RNN_EINVAL;
    const StreamPlan pl = stream_plan(dims);
    if (pl.total > kStaticScratchBytes) return RNN_ETOOLARGE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    void* ws = nullptr;
    const int rs = static_scratch(s, &ws);
    if (rs != RNN_OK) return rs;
    return launch_window(dims, params, x, targets, h0, dh_last, h_all, h_last, loss, grads, dh0, ws, pl, status, s);
}

int rnn_train_stream_workspace_bytes(const rnn_dims* dims, size_t* bytes) {
    using namespace rnn;
    if (!bytes) return RNN_EINVAL;
    const int rc = stream_supported(dims);
    if (rc == RNN_EUNSUPPORTED) {
        GeneralPlan g;
        int rg = general_supported(dims, RNN_FLAG_SYNC);
        if (rg == RNN_OK && dims->in_dim != dims->out_dim) rg = RNN_EUNSUPPORTED;   // targets are the next ids
        if (rg == RNN_OK) rg = general_plan(dims, true, &g);
        if (rg != RNN_OK) return rg;
        *bytes = g.total;
        return RNN_OK;
    }
    if (rc != RNN_OK) return rc;
    *bytes = stream_plan(dims).total;
    return RNN_OK;
}

int rnn_train_stream(const rnn_dims* dims, const rnn_params_inout* params, const int32_t* ids,
                     int64_t n_windows, float lr, const float* h0, float* h_last, float* losses,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    using namespace rnn;
    const int rc = stream_supported(dims);
    if (rc == RNN_EUNSUPPORTED) {
        // Outside the one-launch kernel: per window the launches of the three calls and one update
        // launch, all enqueued here; the state is carried through two slots of the workspace.
        GeneralPlan g;
        int rg = general_supported(dims, RNN_FLAG_SYNC);
        if (rg == RNN_OK && dims->in_dim != dims->out_dim) rg = RNN_EUNSUPPORTED;   // targets are the next ids
        if (rg == RNN_OK) rg = general_plan(dims, true, &g);
        if (rg != RNN_OK) return rg;
        if (!params || !params->Wx || !params->Wh || !params->b || !params->V || !params->c || !ids) return RNN_EINVAL;
        if (n_windows < 0 || n_windows > (int64_t)0x7fffffff || !(lr == lr)) return RNN_EINVAL;
        if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) || workspace_bytes < g.total)
            return RNN_EWORKSPACE;
        hipStream_t s = static_cast<hipStream_t>(hip_stream);
        char* ws = static_cast<char*>(workspace);
        if (launch_zero_words(reinterpret_cast<int32_t*>(ws), (int)(kHeaderBytes / 4), s) != hipSuccess) return RNN_EHIP;
        int rw = rnn_workspace_init(&g.d3, ws + g.ws3, g.ws3_bytes, hip_stream);
        if (rw != RNN_OK) return rw;
        const size_t bh = (size_t)dims->batch * dims->hidden, tb = (size_t)dims->seq_len * dims->batch;
        float* slot[2] = {reinterpret_cast<float*>(ws + g.state), reinterpret_cast<float*>(ws + g.state) + bh};
        float* hall = reinterpret_cast<float*>(ws + g.hall);
        rnn_params rp{params->Wx, params->Wh, params->b, params->V, params->c};
        rnn_grads gr{reinterpret_cast<float*>(ws + g.grads[0]), reinterpret_cast<float*>(ws + g.grads[1]),
                     reinterpret_cast<float*>(ws + g.grads[2]), reinterpret_cast<float*>(ws + g.grads[3]),
                     reinterpret_cast<float*>(ws + g.grads[4])};
        SgdArgs up{};
        up.p[0] = params->Wx; up.p[1] = params->Wh; up.p[2] = params->b; up.p[3] = params->V; up.p[4] = params->c;
        up.g[0] = gr.dWx; up.g[1] = gr.dWh; up.g[2] = gr.db; up.g[3] = gr.dV; up.g[4] = gr.dc;
        size_t most = 0;
        for (int i = 0; i < 5; ++i) { up.n[i] = g.n_param[i]; if (up.n[i] > most) most = up.n[i]; }
        up.lr = lr;
        const unsigned blocks = (unsigned)((most + 255) / 256 < 2048 ? (most + 255) / 256 : 2048);
        // losses == NULL: the per-window loss still has to land somewhere
        float* loss_sink = reinterpret_cast<float*>(ws) + 8;
        const float* h_prev = h0;
        for (int64_t w = 0; w < n_windows; ++w) {
            const int32_t* xw = ids + (size_t)w * tb;
            float* h_next = (w == n_windows - 1 && h_last) ? h_last : slot[w & 1];
            rw = rnn_forward(&g.d3, &rp, xw, h_prev, hall, h_next, ws + g.ws3, g.ws3_bytes, s);
            if (rw == RNN_OK) rw = rnn_loss(&g.d3, &rp, hall, xw + dims->batch, losses ? losses + w : loss_sink,
                                            ws + g.ws3, g.ws3_bytes, s);
            if (rw == RNN_OK) rw = rnn_bptt(&g.d3, &rp, xw, xw + dims->batch, hall, nullptr, &gr, nullptr,
                                            ws + g.ws3, g.ws3_bytes, s);
            if (rw != RNN_OK) return rw;
            hipLaunchKernelGGL(sgd_update_kernel, dim3(blocks), dim3(256), 0, s, up);
            if (hipGetLastError() != hipSuccess) return RNN_EHIP;
            h_prev = h_next;
        }
        if (n_windows > 0) {
            hipLaunchKernelGGL(merge_status_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<int32_t*>(ws),
                               three_call_status_word(&g.d3, ws + g.ws3));
            if (hipGetLastError() != hipSuccess) return RNN_EHIP;
        } else if (h_last && h0) {
            if (hipMemcpyAsync(h_last, h0, bh * 4, hipMemcpyDeviceToDevice, s) != hipSuccess) return RNN_EHIP;
        }
        if (dims->flags & RNN_FLAG_SYNC)
            if (hipStreamSynchronize(s) != hipSuccess) return RNN_EHIP;
        return RNN_OK;
    }
    if (rc != RNN_OK) return rc;
    if (!params || !params->Wx || !params->Wh || !params->b || !params->V || !params->c || !ids)
        return RNN_EINVAL;
    if (n_windows < 0 || n_windows > (int64_t)0x7fffffff || !(lr == lr)) return RNN_EINVAL;
    auto bad16 = [](const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u); };
    auto bad4 = [](const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 3u); };
    if (bad16(params->Wx) || bad16(params->Wh) || bad16(params->b) || bad16(params->V) ||
        bad16(params->c) || bad4(ids) || bad4(h0) || bad4(h_last) || bad4(losses))
        return RNN_EINVAL;
    const StreamPlan pl = stream_plan(dims);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15u) || workspace_bytes < pl.total)
        return RNN_EWORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (n_windows == 0) return RNN_OK;

    char* ws = static_cast<char*>(workspace);
    StreamArgs a{};
    a.Wx = params->Wx; a.Wh = params->Wh; a.b = params->b; a.V = params->V; a.c = params->c;
    a.ids = ids; a.ys = ids + 1; a.n_windows = n_windows; a.lr = lr; a.tag0 = 1u;
    a.h0 = h0; a.h_last = h_last; a.losses = losses;
    a.H = dims->hidden; a.NV = dims->out_dim; a.NVin = dims->in_dim; a.T = dims->seq_len;
    bind_boxes(a, workspace, pl);

    // tags start at 1 in every call, so the boxes (and the status word) start cleared
    if (launch_zero_words(reinterpret_cast<int32_t*>(ws), (int)(pl.total / 4), s) != hipSuccess) return RNN_EHIP;

    const int nq = pick_nq(a.H);
    const void* fn = dims->act == RNN_ACT_SIGMOID ? pick_kernel<0>(nq) : pick_kernel<1>(nq);
    size_t lds = loop_lds_floats(a.T, nq);
    if (strip_lds_floats(nq, a.T, a.S) > lds) lds = strip_lds_floats(nq, a.T, a.S);
    lds *= 4;
    if (allow_lds(fn, lds) != hipSuccess) return RNN_EHIP;
    hipError_t e;
    {
        ProfileScope ps(K_TRAIN_STREAM, s);
        void* args[] = {&a};
        e = hipLaunchCooperativeKernel(fn, dim3(1 + a.S), dim3(NT), args, (unsigned)lds, s);
    }
    if (e != hipSuccess) return RNN_EHIP;
    if (dims->flags & RNN_FLAG_SYNC)
        if (hipStreamSynchronize(s) != hipSuccess) return RNN_EHIP;
    return RNN_OK;
}

#ifdef RNN_STREAM_TRACE
int rnn_train_stream_trace(long long* host_out, int n) {
    return hipMemcpyFromSymbol(host_out, HIP_SYMBOL(rnn::g_trace), (size_t)n * 8) == hipSuccess ? RNN_OK : RNN_EHIP;
}
#endif

int rnn_train_stream_status(const void* workspace, void* hip_stream, int32_t* status_host) {
    if (!workspace || !status_host) return RNN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(status_host, workspace, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return RNN_EHIP;
    return hipStreamSynchronize(s) == hipSuccess ? RNN_OK : RNN_EHIP;
}

}  // extern "C"
