// Device-side pieces of the short-sequence output layer (N = T*B <= 32 rows) that more than one
// kernel uses: the strip geometry, the row loader, the transposed row reduction, and the body
// of the backward strip pass, which runs inside the launch of the reverse time loop.
#pragma once
#include "common.hpp"
#include "internal.hpp"

#include <type_traits>

namespace rnn {
namespace skinny {

constexpr int NR = 16;    // rows held in registers per pass
constexpr int CW = 128;   // vocabulary columns per workgroup
constexpr int NTH = 512;
constexpr int QW = CW / 4;     // column quads per strip (32)
constexpr int IG = NTH / QW;   // groups splitting the H dimension (16)
constexpr int NWV = NTH / 64;  // wavefronts per workgroup (8)
constexpr int NB = 8;          // independent 16-byte loads in flight per thread

// hidden rows of one pass into LDS as hs[i][NR] (zero padded rows)
__device__ __forceinline__ void load_rows(const float* __restrict__ Hs, float* hs, int n0, int N,
                                          int H, int tid) {
    const int n = H * NR;
    for (int base = tid; base < n; base += NB * NTH) {
        float t[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int e = base + u * NTH;
            const int r = e / H, i = e - r * H;            // coalesced along i
            t[u] = (e < n && n0 + r < N) ? Hs[(size_t)(n0 + r) * H + i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int e = base + u * NTH;
            const int r = e / H, i = e - r * H;
            if (e < n) hs[i * NR + r] = t[u];
        }
    }
}

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }

// Sum p[0..15] over the 32 lanes that share lane/32, leaving the total of row
// r = 8*b4 + 4*b3 + 2*b2 + b1 (bits of lane%32) in every lane: each stage halves the number of
// live values, so the whole reduction costs 16 shuffles instead of 80.
__device__ __forceinline__ float quad_rows_reduce(float (&p)[NR], int lane) {
    float q8[8], q4[4], q2[2];
    const bool b4 = lane & 16, b3 = lane & 8, b2 = lane & 4, b1 = lane & 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float send = b4 ? p[j] : p[j + 8], keep = b4 ? p[j + 8] : p[j];
        q8[j] = keep + __shfl_xor(send, 16, kWave);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float send = b3 ? q8[j] : q8[j + 4], keep = b3 ? q8[j + 4] : q8[j];
        q4[j] = keep + __shfl_xor(send, 8, kWave);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const float send = b2 ? q4[j] : q4[j + 2], keep = b2 ? q4[j + 2] : q4[j];
        q2[j] = keep + __shfl_xor(send, 4, kWave);
    }
    const float send = b1 ? q2[0] : q2[1], keep = b1 ? q2[1] : q2[0];
    float v = keep + __shfl_xor(send, 2, kWave);
    v += __shfl_xor(v, 1, kWave);
    return v;
}


// This workgroup's slice of G = (sum over strips of w * share - V[:, y]) / N, w = exp(strip max
// - lse): up to 32 lanes per output walk the strips (fixed order: lane-strided partial sums, then a
// shuffle tree), and the result is published to the reverse loop's workgroup as a tagged word.
__device__ __forceinline__ void reduce_g_slice(const SkinnyArgs& a, int part, int nparts) {
    const int N = a.N, H = a.H, n = N * H, S = (a.O + CW - 1) / CW;
    const int per = (n + nparts - 1) / nparts;
    const int o_lo = part * per, o_hi = min(n, o_lo + per);
    int lpo = 1;                                       // lanes per output: power of two, <= 32
    while (lpo < 32 && lpo < S) lpo *= 2;
    const int tid = threadIdx.x, j = tid % lpo, slot = tid / lpo;
    const float invN = 1.0f / (float)N;
    for (int o0 = o_lo; o0 < o_hi; o0 += NTH / lpo) {
        const int o = o0 + slot;
        const bool live = o < o_hi;
        const int oc = live ? o : o_hi - 1;
        const int t = oc / H;
        const float l = a.lse[t];
        float sum = 0.f;
        for (int g0 = j; g0 < S; g0 += lpo * 4) {     // up to four strips in flight per lane
            float sh[4], m[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int g = min(g0 + lpo * u, S - 1);
                sh[u] = a.gpart[(size_t)g * n + oc];
                m[u] = tagged_value(a.stat_box[((size_t)t * S + g) * 2]);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                consume(sh[u]);
                consume(m[u]);
                if (g0 + lpo * u < S) sum = fmaf(__expf(m[u] - l), sh[u], sum);
            }
        }
        for (int off = lpo / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off, kWave);
        if (live && j == 0) tagged_store(a.g_box + o, a.epoch, (sum - a.vy[o]) * invN);
    }
}

// Backward pass of one strip of 128 vocabulary columns: dZ strip from Z and lse (never written
// back), dc, dV strip = Hs^T dZ, and this workgroup's share of the zero fill of dWx.  It needs
// neither V nor the reverse loop's results, so it runs beside the reverse loop in one launch.
// smem: back_smem(H) bytes.
__device__ __forceinline__ void back_body(const SkinnyArgs& a, int strip, int nstrips, float* smem) {
    const int H = a.H, O = a.O, N = a.N;
    float* hs = smem;                    // [H][NR]
    float* dzs = hs + H * NR;            // [NR][CW]
    const int tid = threadIdx.x, kq = tid % QW, ig = tid / QW;
    const int k0 = strip * CW, k = k0 + 4 * kq;
    const bool kin = k < O;
    const float invN = 1.0f / (float)N;

    reduce_g_slice(a, strip, nstrips);   // first: the reverse loop waits for it

    float4 dc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int n0 = 0; n0 < N; n0 += NR) {
        // requests first: logits, row statistics and targets of row ig
        const int nrow = n0 + ig;                     // IG == NR: group ig produces row ig
        float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        float l = 0.f;
        int y = -1;
        if (nrow < N && kin) {
            z = ld4(a.Z + (size_t)nrow * O + k);
            l = a.lse[nrow];
            y = a.y[nrow] - k;
        }
        __syncthreads();
        load_rows(a.Hs, hs, n0, N, H, tid);
        {
            float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
            if (nrow < N && kin) {
                d.x = (__expf(z.x - l) - (y == 0 ? 1.f : 0.f)) * invN;
                d.y = (__expf(z.y - l) - (y == 1 ? 1.f : 0.f)) * invN;
                d.z = (__expf(z.z - l) - (y == 2 ? 1.f : 0.f)) * invN;
                d.w = (__expf(z.w - l) - (y == 3 ? 1.f : 0.f)) * invN;
            }
            *reinterpret_cast<float4*>(dzs + ig * CW + 4 * kq) = d;
        }
        __syncthreads();
        float4 dz[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) dz[r] = ld4(dzs + r * CW + 4 * kq);
        if (ig == 0) {
#pragma unroll
            for (int r = 0; r < NR; ++r) { dc.x += dz[r].x; dc.y += dz[r].y; dc.z += dz[r].z; dc.w += dz[r].w; }
        }
        // Overwrite and accumulate are separate instantiations: a load of the old dV inside the
        // storing loop would make every iteration wait for the previous store's acknowledgement.
        auto products = [&](auto accumulate) {
            constexpr bool ACC = decltype(accumulate)::value;
            for (int i = ig; i < H; i += IG) {
                // dV[i, quad] (+)= sum_r h[r][i] dz[r]
                const float* hrow = hs + i * NR;
                float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
                for (int r = 0; r < NR; ++r) {
                    const float h = hrow[r];
                    sum.x = fmaf(h, dz[r].x, sum.x);
                    sum.y = fmaf(h, dz[r].y, sum.y);
                    sum.z = fmaf(h, dz[r].z, sum.z);
                    sum.w = fmaf(h, dz[r].w, sum.w);
                }
                if (kin) {
                    float4* dst = reinterpret_cast<float4*>(a.dV + (size_t)i * O + k);
                    if (ACC) {
                        const float4 old = *dst;
                        sum.x += old.x; sum.y += old.y; sum.z += old.z; sum.w += old.w;
                    }
                    *dst = sum;
                }
            }
        };
        if (a.beta || n0 > 0) products(std::true_type{}); else products(std::false_type{});
    }
    if (ig == 0 && kin) {
        float4* dst = reinterpret_cast<float4*>(a.dc + k);
        if (a.beta) { const float4 o = *dst; dc.x += o.x; dc.y += o.y; dc.z += o.z; dc.w += o.w; }
        *dst = dc;
    }

    // Zero fill of the token-gradient matrix (overwrite mode), an even share of its rows per
    // workgroup.  The rows of the tokens that occur in the sequence are left alone: the reverse
    // loop's workgroup writes those rows in full at the end of the same launch, and nothing
    // orders the two workgroups.
    if (a.dWx_zero) {
        __shared__ int s_nskip;
        __shared__ int s_skip[32];
        const int per = (a.NV + nstrips - 1) / nstrips;
        const int r_lo = min(a.NV, strip * per), r_hi = min(a.NV, r_lo + per);
        if (tid == 0) s_nskip = 0;
        __syncthreads();
        if (tid < N) {
            const int id = a.xids[tid];
            if (id >= r_lo && id < r_hi) s_skip[atomicAdd(&s_nskip, 1)] = id;
        }
        __syncthreads();
        const int nskip = s_nskip;
        auto skipped = [&](int row) {
            bool hit = false;
            for (int u = 0; u < nskip; ++u) hit = hit || s_skip[u] == row;
            return hit;
        };
        if ((H & 3) == 0) {                    // rows are 16-byte aligned
            const int H4 = H / 4;
            const int total = (r_hi - r_lo) * H4;
            for (int e = tid; e < total; e += NTH) {
                const int row = r_lo + e / H4, c4 = e - (row - r_lo) * H4;
                if (!skipped(row))
                    reinterpret_cast<float4*>(a.dWx_zero + (size_t)row * H)[c4] = make_float4(0.f, 0.f, 0.f, 0.f);
            }
        } else {
            const int total = (r_hi - r_lo) * H;
            for (int e = tid; e < total; e += NTH) {
                const int row = r_lo + e / H;
                if (!skipped(row)) a.dWx_zero[(size_t)r_lo * H + e] = 0.f;
            }
        }
    }
}

static_assert(IG == NR, "one group per register row");
inline size_t back_smem(int H) { return ((size_t)H * NR + (size_t)NR * CW) * 4; }

}  // namespace skinny
}  // namespace rnn
