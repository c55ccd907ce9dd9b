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
// folded into the time loops one rank-1 term per step (row form during the reverse loop, column
// form during the next window's forward loop, same order and same operands, so both copies stay
// bit-identical), where it fills issue slots the latency-bound steps leave idle.
//
// Every wait is bounded; a wait that expires sets the status word and makes its workgroup leave,
// after which the others run into their own limits, so the grid always drains.
#include "../../include/rnn.h"

#include <stdlib.h>

#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

constexpr int NT = 512;          // threads per workgroup (both roles)
constexpr int MAXH = NT / 4;     // four lanes share one hidden unit in the loop workgroup
constexpr int MAXT = 32;         // longest window
constexpr int CW = 128;          // vocabulary columns per strip
constexpr int ES = CW + 16;      // LDS row stride of the strip of V: 16-byte reads by column quads
                                 // (z) and by row groups (P) are both free of bank conflicts
constexpr int HS = 128;          // LDS row stride of the hidden rows kept by a strip
constexpr int MAX_TS = 2048;     // T * strips the strip statistics stage in LDS holds

struct StreamArgs {
    float *Wx, *Wh, *b, *V, *c;          // parameters, updated in place
    const int32_t* ids;                   // [n_windows*T + 1]
    long long n_windows;
    float lr;
    const float* h0;                      // nullable [H]
    float* h_last;                        // nullable [H]
    float* losses;                        // nullable [n_windows]
    int H, NV, T, S;
    unsigned long long *hbox, *gbox, *vybox, *zybox, *statbox, *pbox;
    int32_t* status;
    int spin_limit;
};

__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
// Butterfly stages of a wavefront reduction without LDS traffic.  Stages 1 and 2 permute within
// quads, 4 and 8 mirror within 8 and 16 lanes (equivalent to xor once the smaller stages have
// run), 16 and 32 swap rows / halves of two registers.
__device__ __forceinline__ float sum4(float v) { v += dpp<0xB1>(v); v += dpp<0x4E>(v); return v; }
__device__ __forceinline__ float sum16(float v) { v = sum4(v); v += dpp<0x141>(v); v += dpp<0x140>(v); return v; }
__device__ __forceinline__ float swap16_sum(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float swap32_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float sum32(float v) { return swap16_sum(sum16(v)); }
__device__ __forceinline__ float sum64(float v) { return swap32_sum(sum32(v)); }
__device__ __forceinline__ float max64(float v) {
    v = fmaxf(v, dpp<0xB1>(v)); v = fmaxf(v, dpp<0x4E>(v));
    v = fmaxf(v, dpp<0x141>(v)); v = fmaxf(v, dpp<0x140>(v));
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
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
size_t strip_lds_floats(int H, int T, int S) {
    const int HR = (H + 15) / 16 * 16;
    return (size_t)HR * ES + CW + (size_t)T * HS + (size_t)T * CW + CW + 8 * CW + (size_t)3 * T * S;
}

// ---------------------------------------------------------------------------------------
// Workgroup 0: time loops and the recurrent-layer updates.  NQ = float4 per lane of a row of Wh.
template <int ACT, int NQ>
__device__ __forceinline__ void loop_body(const StreamArgs& a, float* smem) {
    constexpr int HP = 16 * NQ;      // padded vector length
    __shared__ int s_ids[MAXT + 1];
    __shared__ int s_first[MAXT];
    __shared__ int s_abort;
    const int H = a.H, T = a.T, tid = threadIdx.x;
    const int own = tid >> 2, q = tid & 3;
    const int ownc = min(own, HP - 1);
    const bool live = own < H, lead = live && q == 0;
    float* Hl = smem;                        // [2][T+1][HP]  h_{-1} .. h_{T-1}, by window parity
    float* Dl = Hl + 2 * (T + 1) * HP;       // [T][HP] delta_t
    float* Sl = Dl + T * HP;                 // [T][HP] lr * delta_t
    float* Fl = Sl + T * HP;                 // [T][HP] lr * delta summed per distinct token
    float* Ul = Fl + T * HP;                 // [T][HP] rows of Wx of the window's tokens
    float* Gl = Ul + T * HP;                 // [T][HP] G_t
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
    int nid = tid <= T ? a.ids[tid] : 0;     // ids of window 0; later: prefetched a window ahead
    if (tid == 0) s_abort = 0;
    __syncthreads();
    if (lead) Hl[own] = a.h0 ? a.h0[own] : 0.f;

    for (long long w = 0; w < a.n_windows; ++w) {
        const int pw = (int)(w & 1);
        const unsigned tag = (unsigned)(w + 1);
        float* Hc = Hl + pw * (T + 1) * HP;           // this window's states
        const float* Ho = Hl + (pw ^ 1) * (T + 1) * HP;   // the previous window's
        if (tid <= T) {
            s_ids[tid] = nid;
            if (w + 1 < a.n_windows) nid = a.ids[(size_t)(w + 1) * T + tid];
        }
        __syncthreads();
        if (tid < T) {       // first step at which each step's token occurs
            int f = tid;
            for (int u = tid - 1; u >= 0; --u)
                if (s_ids[u] == s_ids[tid]) f = u;
            s_first[tid] = f;
        }
        if (lead) {          // input vectors of the window's tokens, eight requests in flight
            for (int t0 = 0; t0 < T; t0 += 8) {
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    v[u] = dev_load(a.Wx + (size_t)s_ids[min(t0 + u, T - 1)] * H + own);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (t0 + u < T) Ul[(t0 + u) * HP + own] = v[u];
            }
        }
        __syncthreads();

        // ---- forward steps; the column copy of Wh receives the previous window's update ----
        for (int s = 0; s < T; ++s) {
            const float4* v4 = reinterpret_cast<const float4*>(Hc + s * HP) + q;
            float4 x[NQ];
#pragma unroll
            for (int u = 0; u < NQ; ++u) x[u] = v4[4 * u];
            const float uin = lead ? Ul[s * HP + own] : 0.f;
            const int tt = T - 1 - s;                      // term of the previous update
            float4 sd[NQ];
            float ho = 0.f;
            if (w > 0) {
                const float4* s4 = reinterpret_cast<const float4*>(Sl + tt * HP) + q;
#pragma unroll
                for (int u = 0; u < NQ; ++u) sd[u] = s4[4 * u];
                ho = Ho[tt * HP + ownc];
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
            if (w > 0) {
#pragma unroll
                for (int u = 0; u < NQ; ++u) rank1v(wb[u], sd[u], ho);
            }
            lds_barrier();
        }

        // ---- G from the strips -------------------------------------------------------------
        {
            const int n = T * H;
            for (int e0 = tid; e0 < n; e0 += 4 * NT) {
                unsigned long long wd[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) wd[u] = tagged_load(a.gbox + min(e0 + u * NT, n - 1));
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = e0 + u * NT;
                    if (e >= n) continue;
                    for (int spins = 0; !tagged_ok(wd[u], tag); ++spins) {
                        if (spins > a.spin_limit) { s_abort = 1; break; }
                        wd[u] = tagged_load(a.gbox + e);
                    }
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

        // ---- reverse steps; the row copy of Wh receives this window's update ------------------
        float bsum = 0.f;
        if (lead) {
            const float h = Hc[T * HP + own];
            const float d = Gl[(T - 1) * HP + own] * act_grad<ACT>(h);
            Dl[(T - 1) * HP + own] = d;
            Sl[(T - 1) * HP + own] = a.lr * d;
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
            float g = 0.f, h = 0.f;
            if (lead) { g = Gl[t * HP + own]; h = Hc[(t + 1) * HP + own]; }
            float acc0 = 0.f, acc1 = 0.f;
#pragma unroll
            for (int u = 0; u < NQ; ++u) {
                if (u & 1) acc1 = dot4(wb[u], x[u], acc1); else acc0 = dot4(wb[u], x[u], acc0);
            }
            const float acc = sum4(acc0 + acc1);
            if (lead) {
                const float d = (g + acc) * act_grad<ACT>(h);
                Dl[t * HP + own] = d;
                Sl[t * HP + own] = a.lr * d;
                bsum += d;
            }
#pragma unroll
            for (int u = 0; u < NQ; ++u) rank1(wf[u], sj, hh[u]);   // term t+1: delta_{t+1} (x) h_t
            lds_barrier();
        }
        {   // term 0: delta_0 (x) h_{-1}
            const float4* h4 = reinterpret_cast<const float4*>(Hc) + q;
            const float sj = Sl[ownc];
#pragma unroll
            for (int u = 0; u < NQ; ++u) rank1(wf[u], sj, h4[4 * u]);
        }

        // ---- bias, touched rows of Wx, carried state ----------------------------------------
        if (lead) {
            bj = fmaf(-a.lr, bsum, bj);
            for (int t = 0; t < T; ++t) Fl[t * HP + own] = Sl[t * HP + own];
            for (int u = 1; u < T; ++u) {
                const int f = s_first[u];
                if (f != u) Fl[f * HP + own] += Fl[u * HP + own];
            }
            for (int t = 0; t < T; ++t)
                if (s_first[t] == t)
                    dev_store(a.Wx + (size_t)s_ids[t] * H + own, Ul[t * HP + own] - Fl[t * HP + own]);
            Hl[(pw ^ 1) * (T + 1) * HP + own] = Hc[T * HP + own];
        }
        __syncthreads();
    }

    // ---- write the recurrent layer back --------------------------------------------------------
    const int plast = (int)((a.n_windows - 1) & 1);
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
        if (a.h_last) a.h_last[own] = Hl[plast * (T + 1) * HP + T * HP + own];
    }
}

// ---------------------------------------------------------------------------------------
// Workgroups 1..S: one strip of CW vocabulary columns each.
__device__ __forceinline__ void strip_body(const StreamArgs& a, const int g, float* smem) {
    __shared__ int s_y[MAXT];
    __shared__ float lse_s[MAXT];
    __shared__ float zy_s[MAXT];
    __shared__ int s_abort;
    const int H = a.H, T = a.T, S = a.S, NV = a.NV, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int c4 = tid & 31, ig = tid >> 5;          // column quad, group of hidden rows
    const int NU = (H + 15) / 16, HR = 16 * NU;
    const int k0 = g * CW, ncols = min(CW, NV - k0);
    const float invN = 1.0f / (float)T;
    float* Vs = smem;                     // [HR][ES]
    float* cs = Vs + HR * ES;             // [CW]
    float* hs = cs + CW;                  // [T][HS]
    float* Zs = hs + T * HS;              // [T][CW]
    float* es = Zs + T * CW;              // [CW]
    float* red = es + CW;                 // [8][CW]
    float* stage = red + 8 * CW;          // [T][S][2]
    float* wts = stage + 2 * T * S;       // [T][S]

    for (int e = tid; e < HR * CW; e += NT) {
        const int i = e / CW, cc = e - i * CW;
        Vs[i * ES + cc] = (i < H && cc < ncols) ? a.V[(size_t)i * NV + k0 + cc] : 0.f;
    }
    for (int e = tid; e < HR * (ES - CW); e += NT) {
        const int i = e / (ES - CW), cc = e - i * (ES - CW);
        Vs[i * ES + CW + cc] = 0.f;
    }
    if (tid < CW) cs[tid] = tid < ncols ? a.c[k0 + tid] : 0.f;
    for (int e = tid; e < T * HS; e += NT) hs[e] = 0.f;
    int ny = tid < T ? a.ids[tid + 1] : 0;           // targets of window 0
    if (tid == 0) s_abort = 0;
    __syncthreads();

    for (long long w = 0; w < a.n_windows; ++w) {
        const unsigned tag = (unsigned)(w + 1);
        if (tid < T) {
            s_y[tid] = ny;
            if (w + 1 < a.n_windows) ny = a.ids[(size_t)(w + 1) * T + tid + 1];
        }
        // ---- rows, as the hidden states arrive ---------------------------------------------
        for (int t = 0; t < T; ++t) {
            // The last wavefront polls (two words per lane): it publishes nothing in this loop
            // (for H <= 112), so its loads never queue behind stores that await their
            // acknowledgement.
            if (wave == NT / 64 - 1) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int i = lane + 64 * u;
                    if (i < H) {
                        float v = 0.f;
                        if (!tagged_wait(a.hbox + (size_t)t * H + i, tag, a.spin_limit, v)) s_abort = 1;
                        hs[t * HS + i] = v;
                    }
                }
            }
            lds_barrier();
            if (s_abort) {
                if (tid == 0) atomicExch(a.status, 1);
                return;
            }
            // partial logits of a column quad over this thread's hidden rows
            {
                float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (u < NU) {
                        const int i = ig + 16 * u;
                        const float h = hs[t * HS + i];
                        const float4 v = ld4(Vs + i * ES + 4 * c4);
                        acc.x = fmaf(h, v.x, acc.x); acc.y = fmaf(h, v.y, acc.y);
                        acc.z = fmaf(h, v.z, acc.z); acc.w = fmaf(h, v.w, acc.w);
                    }
                }
                acc.x = swap32_sum(acc.x); acc.y = swap32_sum(acc.y);
                acc.z = swap32_sum(acc.z); acc.w = swap32_sum(acc.w);
                if (lane < 32) st4(red + wave * CW + 4 * c4, acc);
            }
            lds_barrier();
            if (wave == 0) {   // logits of the strip, its maximum and sum of exponentials
                float z0 = cs[lane], z1 = cs[64 + lane];
#pragma unroll
                for (int wv = 0; wv < 8; ++wv) { z0 += red[wv * CW + lane]; z1 += red[wv * CW + 64 + lane]; }
                if (lane >= ncols) z0 = -INFINITY;
                if (64 + lane >= ncols) z1 = -INFINITY;
                Zs[t * CW + lane] = z0;
                Zs[t * CW + 64 + lane] = z1;
                const float m = max64(fmaxf(z0, z1));
                const float e0 = __expf(z0 - m), e1 = __expf(z1 - m);
                const float sm = sum64(e0 + e1);
                es[lane] = e0;
                es[64 + lane] = e1;
                if (lane == 0) {
                    unsigned long long* st = a.statbox + ((size_t)t * S + g) * 2;
                    tagged_store(st, tag, m);
                    tagged_store(st + 1, tag, sm);
                }
                const int yl = s_y[t] - k0;
                if (yl >= 0 && yl < CW && lane == (yl & 63))
                    tagged_store(a.zybox + t, tag, yl < 64 ? z0 : z1);
            }
            lds_barrier();
            // share of the softmax part of G, relative to the strip maximum:
            // P[i] = sum_c exp(z_c - m) V[i][c]; four lanes per hidden row
            {
                const int i = tid >> 2, q = tid & 3;
                if (i < HR) {
                    float p0 = 0.f, p1 = 0.f;
#pragma unroll
                    for (int u = 0; u < 8; ++u) {
                        const float4 e4 = ld4(es + 4 * (q + 4 * u));
                        const float4 v4 = ld4(Vs + i * ES + 4 * (q + 4 * u));
                        if (u & 1) p1 = dot4(e4, v4, p1); else p0 = dot4(e4, v4, p0);
                    }
                    const float p = sum4(p0 + p1);
                    if (q == 0 && i < H) {
                        tagged_store(a.pbox + ((size_t)g * T + t) * H + i, tag, p);
                        const int yl = s_y[t] - k0;
                        if (yl >= 0 && yl < CW) tagged_store(a.vybox + (size_t)t * H + i, tag, Vs[i * ES + yl]);
                    }
                }
            }
        }

        // ---- statistics of all strips -> lse per row and the strips' weights -----------------
        {
            const int cnt = T * S * 2;
            for (int w0 = tid; w0 < cnt; w0 += 4 * NT) {
                unsigned long long wd[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) wd[u] = tagged_load(a.statbox + min(w0 + u * NT, cnt - 1));
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int idx = w0 + u * NT;
                    if (idx >= cnt) continue;
                    for (int spins = 0; !tagged_ok(wd[u], tag); ++spins) {
                        if (spins > a.spin_limit) { s_abort = 1; break; }
                        wd[u] = tagged_load(a.statbox + idx);
                    }
                    stage[idx] = tagged_value(wd[u]);
                }
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
        for (int t = wave; t < T; t += NT / 64) {
            float m = -INFINITY, sm = 0.f;
            for (int g2 = lane; g2 < S; g2 += 64)
                lse_merge(m, sm, stage[(t * S + g2) * 2], stage[(t * S + g2) * 2 + 1]);
            lse_merge64(m, sm);
            const float l = m + __logf(sm);
            if (lane == 0) lse_s[t] = l;
            for (int g2 = lane; g2 < S; g2 += 64) wts[t * S + g2] = __expf(stage[(t * S + g2) * 2] - l);
        }
        lds_barrier();

        // ---- this strip's slice of G: 32 lanes per output walk the strips in a fixed order ------
        {
            const int n = T * H, per = (n + S - 1) / S;
            const int o_lo = min(n, g * per), o_hi = min(n, o_lo + per);
            const int j = tid & 31, slot = tid >> 5;
            for (int o0 = o_lo; o0 < o_hi; o0 += NT / 32) {
                const int o = o0 + slot;
                const bool have = o < o_hi;
                const int oc = have ? o : o_hi - 1;
                const int t = oc / H;
                float sum = 0.f;
                for (int g0 = j; g0 < S; g0 += 32 * 4) {
                    unsigned long long wd[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        wd[u] = tagged_load(a.pbox + (size_t)min(g0 + 32 * u, S - 1) * n + oc);
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int g2 = g0 + 32 * u;
                        if (g2 >= S) continue;
                        for (int spins = 0; !tagged_ok(wd[u], tag); ++spins) {
                            if (spins > a.spin_limit) { s_abort = 1; break; }
                            wd[u] = tagged_load(a.pbox + (size_t)g2 * n + oc);
                        }
                        sum = fmaf(wts[t * S + g2], tagged_value(wd[u]), sum);
                    }
                }
                sum = sum32(sum);
                if (have && j == 0) {
                    float vy = 0.f;
                    if (!tagged_wait(a.vybox + oc, tag, a.spin_limit, vy)) s_abort = 1;
                    tagged_store(a.gbox + oc, tag, (sum - vy) * invN);
                }
            }
        }
        if (g == S - 1 && wave == 0) {
            float v = lane < T ? lse_s[lane] - zy_s[lane] : 0.f;
            v = sum64(v);
            if (lane == 0 && a.losses) a.losses[w] = v * invN;
        }

        // ---- update of the resident columns: V -= lr Hs^T dZ, c -= lr colsum(dZ) --------------
        {
            float4 accv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) accv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            float4 dcs = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int n0 = 0; n0 < T; n0 += 8) {
                float4 dz[8];
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    const int n = min(n0 + r, T - 1);
                    const float4 z = ld4(Zs + n * CW + 4 * c4);
                    const float l = lse_s[n];
                    const int yl = s_y[n] - k0 - 4 * c4;
                    float4 d;
                    d.x = (__expf(z.x - l) - (yl == 0 ? 1.f : 0.f)) * invN;
                    d.y = (__expf(z.y - l) - (yl == 1 ? 1.f : 0.f)) * invN;
                    d.z = (__expf(z.z - l) - (yl == 2 ? 1.f : 0.f)) * invN;
                    d.w = (__expf(z.w - l) - (yl == 3 ? 1.f : 0.f)) * invN;
                    if (n0 + r >= T) d = make_float4(0.f, 0.f, 0.f, 0.f);
                    dz[r] = d;
                    dcs.x += d.x; dcs.y += d.y; dcs.z += d.z; dcs.w += d.w;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (u < NU) {
                        const int i = ig + 16 * u;
#pragma unroll
                        for (int r = 0; r < 8; ++r) {
                            const float h = hs[min(n0 + r, T - 1) * HS + i];
                            accv[u].x = fmaf(h, dz[r].x, accv[u].x); accv[u].y = fmaf(h, dz[r].y, accv[u].y);
                            accv[u].z = fmaf(h, dz[r].z, accv[u].z); accv[u].w = fmaf(h, dz[r].w, accv[u].w);
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if (u < NU) {
                    float* p = Vs + (ig + 16 * u) * ES + 4 * c4;
                    float4 v = ld4(p);
                    v.x = fmaf(-a.lr, accv[u].x, v.x); v.y = fmaf(-a.lr, accv[u].y, v.y);
                    v.z = fmaf(-a.lr, accv[u].z, v.z); v.w = fmaf(-a.lr, accv[u].w, v.w);
                    st4(p, v);
                }
            }
            if (ig == 0) {
                float4 v = ld4(cs + 4 * c4);
                v.x = fmaf(-a.lr, dcs.x, v.x); v.y = fmaf(-a.lr, dcs.y, v.y);
                v.z = fmaf(-a.lr, dcs.z, v.z); v.w = fmaf(-a.lr, dcs.w, v.w);
                st4(cs + 4 * c4, v);
            }
        }
        __syncthreads();
        if (s_abort) {   // a wait in the G slice expired
            if (tid == 0) atomicExch(a.status, 1);
            return;
        }
    }

    // ---- write the columns back --------------------------------------------------------------
    for (int e = tid; e < H * CW; e += NT) {
        const int i = e / CW, cc = e - i * CW;
        if (cc < ncols) a.V[(size_t)i * NV + k0 + cc] = Vs[i * ES + cc];
    }
    if (tid < ncols) a.c[k0 + tid] = cs[tid];
}

template <int ACT, int NQ>
__global__ __launch_bounds__(NT) void train_stream_kernel(StreamArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    if (blockIdx.x == 0) loop_body<ACT, NQ>(a, smem);
    else strip_body(a, (int)blockIdx.x - 1, smem);
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
    if (strip_lds_floats(d->hidden, d->seq_len, S) * 4 > 158 * 1024) return RNN_EUNSUPPORTED;
    if (loop_lds_floats(d->seq_len, pick_nq(d->hidden)) * 4 > 158 * 1024) return RNN_EUNSUPPORTED;
    return RNN_OK;
}

}  // namespace
}  // namespace rnn

extern "C" {

int rnn_train_stream_workspace_bytes(const rnn_dims* dims, size_t* bytes) {
    using namespace rnn;
    if (!bytes) return RNN_EINVAL;
    const int rc = stream_supported(dims);
    if (rc != RNN_OK) return rc;
    *bytes = stream_plan(dims).total;
    return RNN_OK;
}

int rnn_train_stream(const rnn_dims* dims, const rnn_params_inout* params, const int32_t* ids,
                     int64_t n_windows, float lr, const float* h0, float* h_last, float* losses,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    using namespace rnn;
    const int rc = stream_supported(dims);
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
    a.ids = ids; a.n_windows = n_windows; a.lr = lr; a.h0 = h0; a.h_last = h_last; a.losses = losses;
    a.H = dims->hidden; a.NV = dims->out_dim; a.T = dims->seq_len; a.S = pl.S;
    a.status = reinterpret_cast<int32_t*>(ws + pl.status);
    a.hbox = reinterpret_cast<unsigned long long*>(ws + pl.hbox);
    a.gbox = reinterpret_cast<unsigned long long*>(ws + pl.gbox);
    a.vybox = reinterpret_cast<unsigned long long*>(ws + pl.vybox);
    a.zybox = reinterpret_cast<unsigned long long*>(ws + pl.zybox);
    a.statbox = reinterpret_cast<unsigned long long*>(ws + pl.statbox);
    a.pbox = reinterpret_cast<unsigned long long*>(ws + pl.pbox);
    a.spin_limit = 1 << 22;
    if (const char* env = getenv("RNN_STREAM_SPIN_LIMIT")) {   // failure-path tests: make waits expire
        const long v = strtol(env, nullptr, 10);
        if (v > 0 && v < (1L << 30)) a.spin_limit = (int)v;
    }

    // tags start at 1 in every call, so the boxes (and the status word) start cleared
    if (launch_zero_words(reinterpret_cast<int32_t*>(ws), (int)(pl.total / 4), s) != hipSuccess) return RNN_EHIP;

    const int nq = pick_nq(a.H);
    const void* fn = dims->act == RNN_ACT_SIGMOID ? pick_kernel<0>(nq) : pick_kernel<1>(nq);
    size_t lds = loop_lds_floats(a.T, nq);
    if (strip_lds_floats(a.H, a.T, a.S) > lds) lds = strip_lds_floats(a.H, a.T, a.S);
    lds *= 4;
    if (lds > 64 * 1024)
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return RNN_EHIP;
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

int rnn_train_stream_status(const void* workspace, void* hip_stream, int32_t* status_host) {
    if (!workspace || !status_host) return RNN_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipMemcpyAsync(status_host, workspace, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return RNN_EHIP;
    return hipStreamSynchronize(s) == hipSuccess ? RNN_OK : RNN_EHIP;
}

}  // extern "C"
