// Output layer for a short single sequence (N = T*B <= 32 rows, the paper's batch-1 language
// model benchmark shape): with so few rows the three products with the H x NV output matrix
// are bound by streaming that matrix, not by arithmetic, so they run as column-parallel
// kernels in which every workgroup owns a strip of 128 vocabulary columns, reads its strip of
// V once per kernel with 16-byte loads, and keeps the N hidden rows in LDS.
//
//   skinny_logits : Z strip = Hs V + c, per-row (max, sum exp) of the strip, target logit; the
//                   last strip's workgroup merges the statistics of all strips (passed as
//                   self-validating tagged words) into lse per row and the loss
//   skinny_back   : dZ strip from Z and lse (never written back), dc, dV strip = Hs^T dZ,
//                   partial G = dZ V^T over the strip, and the zero fill of dWx
// The partial G of all strips is summed, in strip order, by the reverse-loop kernel.
//
// Thread layout inside a strip: lane%32 = a quad of 4 adjacent columns, tid/32 = one of 16
// groups that split the hidden dimension.  Requires NV % 4 == 0 (16-byte column quads).
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <type_traits>

namespace rnn {
namespace {

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

__global__ __launch_bounds__(NTH) void skinny_logits_kernel(SkinnyArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int H = a.H, O = a.O, N = a.N;
    float* hs = smem;                 // [H][NR]
    float* red = hs + H * NR;         // [NWV][NR][CW]
    const int tid = threadIdx.x, kq = tid % QW, ig = tid / QW;
    const int lane = tid % kWave, wave = tid / kWave;
    const int k = blockIdx.x * CW + 4 * kq;
    const bool kin = k < O;           // O % 4 == 0: a quad is entirely inside or outside

    // request the strip of V and the bias before waiting for anything
    auto load_v = [&](int i0, float4 (&v)[NB]) {
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int i = i0 + u * IG;
            v[u] = (kin && i < H) ? ld4(a.V + (size_t)i * O + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    float4 v[NB];
    load_v(ig, v);
    const int kc_own = blockIdx.x * CW + tid % CW;          // column of this thread in the combine
    const float cbias = kc_own < O ? a.c[kc_own] : 0.f;
    const bool one_batch = H <= IG * NB;

    for (int n0 = 0; n0 < N; n0 += NR) {
        __syncthreads();
        load_rows(a.Hs, hs, n0, N, H, tid);
        __syncthreads();
        float4 acc[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int i0 = ig; i0 < H; i0 += IG * NB) {
            if (i0 != ig || (n0 > 0 && !one_batch)) load_v(i0, v);
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int i = i0 + u * IG;
                if (i < H) {
                    const float* hrow = hs + i * NR;
#pragma unroll
                    for (int r = 0; r < NR; ++r) {
                        const float h = hrow[r];
                        acc[r].x = fmaf(h, v[u].x, acc[r].x);
                        acc[r].y = fmaf(h, v[u].y, acc[r].y);
                        acc[r].z = fmaf(h, v[u].z, acc[r].z);
                        acc[r].w = fmaf(h, v[u].w, acc[r].w);
                    }
                }
            }
        }
        // the two H-groups of a wavefront combine by shuffle, the four wavefronts through LDS
#pragma unroll
        for (int r = 0; r < NR; ++r) {
            acc[r].x += __shfl_xor(acc[r].x, 32, kWave);
            acc[r].y += __shfl_xor(acc[r].y, 32, kWave);
            acc[r].z += __shfl_xor(acc[r].z, 32, kWave);
            acc[r].w += __shfl_xor(acc[r].w, 32, kWave);
            if (lane < 32) *reinterpret_cast<float4*>(red + (wave * NR + r) * CW + 4 * kq) = acc[r];
        }
        __syncthreads();
        for (int e = tid; e < NR * CW; e += NTH) {   // NTH is a multiple of CW: column = tid % CW
            const int r = e / CW, c = e % CW;
            float z = red[r * CW + c];
#pragma unroll
            for (int w = 1; w < NWV; ++w) z += red[(w * NR + r) * CW + c];
            if (kc_own < O) z += cbias; else z = -INFINITY;
            red[r * CW + c] = z;
            if (kc_own < O && n0 + r < N) a.Z[(size_t)(n0 + r) * O + kc_own] = z;
        }
        __syncthreads();
        // strip statistics: one wavefront per row
        for (int r = wave; r < NR && n0 + r < N; r += NWV) {
            const float z0 = red[r * CW + lane], z1 = red[r * CW + 64 + lane];
            const float m = wave_max(fmaxf(z0, z1));
            const float e = __expf(z0 - m) + __expf(z1 - m);  // exp(-inf) = 0 for padding
            const float s = wave_sum(e);
            if (lane == 0) {
                unsigned long long* st = a.stat_box + ((size_t)(n0 + r) * gridDim.x + blockIdx.x) * 2;
                tagged_store(st, a.epoch, m);
                tagged_store(st + 1, a.epoch, s);
                const int y = a.y[n0 + r] - blockIdx.x * CW;
                if (y >= 0 && y < CW)
                    tagged_store(a.stat_box + (size_t)N * gridDim.x * 2 + n0 + r, a.epoch, red[r * CW + y]);
            }
        }
    }

    // The last strip (usually a short one) merges the statistics of all strips as they arrive:
    // one wavefront per row, lanes over the strips, then the mean row loss.  Only this
    // workgroup waits, and nobody waits for it, so the launch cannot deadlock; the waits are
    // bounded all the same.
    if (blockIdx.x != gridDim.x - 1) return;
    __shared__ float rl[32];
    __shared__ int s_fail;
    if (tid == 0) s_fail = 0;
    __syncthreads();                     // also: `red` is free from here on
    const int strips = gridDim.x;
    const int spin_limit = 1 << 22;
    const unsigned epoch = a.epoch;
    // All words of a group of rows are requested at once (four per thread in flight), parked in
    // LDS, and merged from there: the waiting costs about one memory round trip in total.
    float* stage = red;                  // NWV*NR*CW floats >= 2*strips (checked by the host)
    __shared__ float zys[32];
    const unsigned long long* zybox = a.stat_box + (size_t)N * strips * 2;
    unsigned long long wz = tid < N ? tagged_load(zybox + tid) : 0ull;   // in flight with the rest
    const int rows_per_pass = max(1, (NWV * NR * CW) / (2 * strips));
    for (int n_lo = 0; n_lo < N; n_lo += rows_per_pass) {
        const int n_hi = min(N, n_lo + rows_per_pass);
        const int cnt = (n_hi - n_lo) * strips * 2;
        const unsigned long long* src = a.stat_box + (size_t)n_lo * strips * 2;
        for (int w0 = tid; w0 < cnt; w0 += 4 * NTH) {
            unsigned long long w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) w[u] = tagged_load(src + min(w0 + u * NTH, cnt - 1));
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int idx = w0 + u * NTH;
                if (idx >= cnt) continue;
                for (int spins = 0; !tagged_ok(w[u], epoch); ++spins) {
                    if (spins > spin_limit) { s_fail = 1; break; }
                    w[u] = tagged_load(src + idx);
                }
                stage[idx] = tagged_value(w[u]);
            }
        }
        if (n_lo == 0 && tid < N) {
            for (int spins = 0; !tagged_ok(wz, epoch); ++spins) {
                if (spins > spin_limit) { s_fail = 1; break; }
                wz = tagged_load(zybox + tid);
            }
            zys[tid] = tagged_value(wz);
        }
        __syncthreads();
        for (int n = n_lo + wave; n < n_hi; n += NWV) {
            float m = -INFINITY, sum = 0.f;
            for (int g = lane; g < strips; g += kWave) {
                const float* st = stage + ((size_t)(n - n_lo) * strips + g) * 2;
                lse_merge(m, sum, st[0], st[1]);
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                const float m2 = __shfl_xor(m, off, kWave), s2 = __shfl_xor(sum, off, kWave);
                lse_merge(m, sum, m2, s2);
            }
            if (lane == 0) {
                const float l = m + logf(sum);
                a.lse[n] = l;
                rl[n] = l - zys[n];
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        if (s_fail) atomicExch(a.status, 1);
        float t = 0.f;
        for (int n = 0; n < N; ++n) t += rl[n];
        *a.loss = t / (float)N;
    }
}

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

__global__ __launch_bounds__(NTH) void skinny_back_kernel(SkinnyArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int H = a.H, O = a.O, N = a.N;
    float* hs = smem;                    // [H][NR]
    float* dzs = hs + H * NR;            // [NR][CW]
    float* gs = dzs + NR * CW;           // [NR][H] this strip's partial G
    const int tid = threadIdx.x, kq = tid % QW, ig = tid / QW, lane = tid % kWave;
    const int k0 = blockIdx.x * CW, k = k0 + 4 * kq;
    const bool kin = k < O;
    const float invN = 1.0f / (float)N;
    const int myrow = ((lane & 16) ? 8 : 0) + ((lane & 8) ? 4 : 0) + ((lane & 4) ? 2 : 0) + ((lane & 2) ? 1 : 0);

    auto load_v = [&](int i0, float4 (&v)[NB]) {
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int i = i0 + u * IG;
            v[u] = (kin && i < H) ? ld4(a.V + (size_t)i * O + k) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    const bool one_batch = H <= IG * NB;
    float4 v[NB];

    float4 dc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int n0 = 0; n0 < N; n0 += NR) {
        // requests first: logits, row statistics and targets of row ig, then the strip of V
        const int nrow = n0 + ig;                     // IG == NR: group ig produces row ig
        float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
        float l = 0.f;
        int y = -1;
        if (nrow < N && kin) {
            z = ld4(a.Z + (size_t)nrow * O + k);
            l = a.lse[nrow];
            y = a.y[nrow] - k;
        }
        if (n0 == 0 || !one_batch) load_v(ig, v);
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
            for (int i0 = ig; i0 < H; i0 += IG * NB) {
                if (i0 != ig) load_v(i0, v);
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    const int i = i0 + u * IG;
                    if (i >= H) continue;                       // uniform within a 32-lane group
                    // dV[i, quad] (+)= sum_r h[r][i] dz[r]
                    const float* hrow = hs + i * NR;
                    float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
                    float p[NR];
#pragma unroll
                    for (int r = 0; r < NR; ++r) {
                        const float h = hrow[r];
                        sum.x = fmaf(h, dz[r].x, sum.x);
                        sum.y = fmaf(h, dz[r].y, sum.y);
                        sum.z = fmaf(h, dz[r].z, sum.z);
                        sum.w = fmaf(h, dz[r].w, sum.w);
                        // this quad's share of G[r][i] = sum_c dz[r][c] V[i][c]
                        p[r] = fmaf(dz[r].x, v[u].x, fmaf(dz[r].y, v[u].y, fmaf(dz[r].z, v[u].z, dz[r].w * v[u].w)));
                    }
                    if (kin) {
                        float4* dst = reinterpret_cast<float4*>(a.dV + (size_t)i * O + k);
                        if (ACC) {
                            const float4 old = *dst;
                            sum.x += old.x; sum.y += old.y; sum.z += old.z; sum.w += old.w;
                        }
                        *dst = sum;
                    }
                    const float g = quad_rows_reduce(p, lane);
                    if ((lane & 1) == 0) gs[myrow * H + i] = g;
                }
            }
        };
        if (a.beta || n0 > 0) products(std::true_type{}); else products(std::false_type{});
        __syncthreads();
        for (int e = tid; e < NR * H; e += NTH) {
            const int r = e / H;
            if (n0 + r < N) a.gpart[((size_t)blockIdx.x * N + n0 + r) * H + (e - r * H)] = gs[e];
        }
    }
    if (ig == 0 && kin) {
        float4* dst = reinterpret_cast<float4*>(a.dc + k);
        if (a.beta) { const float4 o = *dst; dc.x += o.x; dc.y += o.y; dc.z += o.z; dc.w += o.w; }
        *dst = dc;
    }

    // zero fill of the token-gradient matrix, an even share per workgroup (overwrite mode)
    if (a.dWx_zero) {
        const size_t total4 = ((size_t)a.NV * H) / 4;  // dWx is 16-byte aligned
        const size_t per = (total4 + gridDim.x - 1) / gridDim.x;
        const size_t b0 = (size_t)blockIdx.x * per;
        const size_t b1 = b0 + per < total4 ? b0 + per : total4;
        float4* z4 = reinterpret_cast<float4*>(a.dWx_zero);
        for (size_t e = b0 + tid; e < b1; e += NTH) z4[e] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (blockIdx.x == 0)
            for (size_t e = total4 * 4 + tid; e < (size_t)a.NV * H; e += NTH) a.dWx_zero[e] = 0.f;
    }
}

static_assert(IG == NR, "one group per register row");
size_t logits_smem(int H) { return ((size_t)H * NR + (size_t)NWV * NR * CW) * 4; }
size_t back_smem(int H) { return ((size_t)H * NR + (size_t)NR * CW + (size_t)NR * H) * 4; }

}  // namespace

int skinny_strips(int O) { return (O + CW - 1) / CW; }

size_t skinny_stat_box_bytes(int N, int O) { return ((size_t)2 * N * skinny_strips(O) + N) * 8; }

bool skinny_supported(int N, int H, int O) {
    if (N > 32 || N < 1 || O % 4 != 0) return false;
    if (2 * skinny_strips(O) > NWV * NR * CW) return false;   // one row of strip statistics fits the LDS stage
    return back_smem(H) <= 64 * 1024 && logits_smem(H) <= 140 * 1024;
}

hipError_t launch_skinny_logits(const SkinnyArgs& a, hipStream_t s) {
    static size_t allowed = 0;
    if (logits_smem(a.H) > 64 * 1024 && logits_smem(a.H) > allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_logits_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)logits_smem(a.H));
        if (e != hipSuccess) return e;
        allowed = logits_smem(a.H);
    }
    ProfileScope ps(K_SKINNY_LOGITS, s);
    hipLaunchKernelGGL(skinny_logits_kernel, dim3(skinny_strips(a.O)), dim3(NTH), logits_smem(a.H), s, a);
    return hipGetLastError();
}

hipError_t launch_skinny_back(const SkinnyArgs& a, hipStream_t s) {
    ProfileScope ps(K_SKINNY_BACK, s);
    hipLaunchKernelGGL(skinny_back_kernel, dim3(skinny_strips(a.O)), dim3(NTH), back_smem(a.H), s, a);
    return hipGetLastError();
}

}  // namespace rnn
