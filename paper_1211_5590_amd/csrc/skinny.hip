// Output layer for a short single sequence (N = T*B <= 32 rows, the paper's batch-1 language
// model benchmark shape): with so few rows the three products with the H x NV output matrix
// are bound by streaming that matrix, not by arithmetic, so they run as column-parallel
// kernels in which every workgroup owns a strip of 128 vocabulary columns, reads its strip of
// V once per kernel with 16-byte loads, and keeps the N hidden rows in LDS.
//
//   skinny_logits : Z strip = Hs V + c, per-row (max, sum exp) of the strip, target logit; the
//                   last strip's workgroup merges the statistics of all strips (passed as
//                   self-validating tagged words) into lse per row and the loss; every strip
//                   also leaves its share of the softmax part of G = dZ V^T, relative to its
//                   own maximum
//   backward strips (skinny_dev.hpp, launched together with the reverse time loop): dZ strip
//                   from Z and lse (never written back), dc, dV strip = Hs^T dZ, zero fill of dWx
// The reverse-loop workgroup combines the strips' shares of G with the weights
// exp(strip max - lse), in strip order.
//
// Thread layout inside a strip: lane%32 = a quad of 4 adjacent columns, tid/32 = one of 16
// groups that split the hidden dimension.  Requires NV % 4 == 0 (16-byte column quads).
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"
#include "skinny_dev.hpp"

#include <type_traits>

namespace rnn {
namespace {

using namespace skinny;

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int ES = CW + 4;   // padded LDS row of 128 columns

__global__ __launch_bounds__(NTH) void skinny_logits_kernel(SkinnyArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    a.epoch = next_tag(tag_word_load(a.epoch_word));   // requested first, needed at the first publish
    const int H = a.H, O = a.O, N = a.N;
    float* hs = smem;                 // [H][NR]
    float* red = hs + H * NR;         // [NWV][NR][CW] partial logits; later a stage for the merge
    float* es = red + NWV * NR * CW;  // [NR][ES] exp(z - strip max), padded rows
    float* Vs = es + NR * ES;         // [IG*NB][ES] one batch of the strip of V, padded rows
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
    __shared__ int s_y[32];
    if (tid < N) s_y[tid] = a.y[tid];

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
        // strip statistics: one wavefront per row; the row's exp(z - strip max) stays in LDS
        for (int r = wave; r < NR; r += NWV) {
            float e0 = 0.f, e1 = 0.f;
            if (n0 + r < N) {
                const float z0 = red[r * CW + lane], z1 = red[r * CW + 64 + lane];
                const float m = wave_max(fmaxf(z0, z1));
                e0 = __expf(z0 - m);          // exp(-inf) = 0 for padding columns
                e1 = __expf(z1 - m);
                const float s = wave_sum(e0 + e1);
                const int y = s_y[n0 + r] - blockIdx.x * CW;
                const float zy = (y >= 0 && y < CW) ? red[r * CW + y] : 0.f;   // read before the overwrite
                if (lane == 0) {
                    unsigned long long* st = a.stat_box + ((size_t)(n0 + r) * gridDim.x + blockIdx.x) * 2;
                    tagged_store(st, a.epoch, m);
                    tagged_store(st + 1, a.epoch, s);
                    if (y >= 0 && y < CW)
                        tagged_store(a.stat_box + (size_t)N * gridDim.x * 2 + n0 + r, a.epoch, zy);
                }
            }
            es[r * ES + lane] = e0;
            es[r * ES + 64 + lane] = e1;
        }
        __syncthreads();
        // Backward needs G = (softmax - onehot) V^T / N.  With w = exp(strip max - lse) the softmax
        // part is sum over strips of w * P, P[r][i] = sum_c exp(z[r][c] - strip max) V[i][c], and P
        // needs only what this workgroup already holds (its strip of V in registers, the
        // exponentials in LDS).  Computing it here takes V and the reverse loop's input out of the
        // backward strip pass, so that pass can run beside the reverse loop instead of before it.
        // It is a [16 x 128] x [128 x H] product, done on the matrix cores: v_mfma_f32_16x16x4 with
        // the rows of exponentials as A and the strip of V, parked in LDS one batch of 128 hidden
        // rows at a time, as B; wavefront w takes the 16 hidden rows 16w.. of the batch.  Lane
        // group g = lane/16 walks the columns 32g..32g+31, so both operands are 16-byte LDS reads
        // (rows are ES = CW+4 words apart: 16 rows spread over all banks).
        {
            bool any_y = false;            // does a target of this pass fall into this strip?
            for (int r = 0; r < NR && n0 + r < N; ++r) {
                const int y = s_y[n0 + r] - blockIdx.x * CW;
                any_y = any_y || (y >= 0 && y < CW);
            }
            const int mrow = lane % 16, g = lane / 16;
            for (int i0 = 0; i0 < H; i0 += IG * NB) {
                if (!one_batch) load_v(i0 + ig, v);
#pragma unroll
                for (int u = 0; u < NB; ++u)     // rows past H are zeros
                    *reinterpret_cast<float4*>(Vs + (IG * u + ig) * ES + 4 * kq) = v[u];
                __syncthreads();
                if (any_y) {               // column y_n of V for the rows whose target is here
                    for (int r = 0; r < NR && n0 + r < N; ++r) {
                        const int y = s_y[n0 + r] - blockIdx.x * CW;
                        if (y < 0 || y >= CW) continue;
                        for (int i = tid; i < IG * NB && i0 + i < H; i += NTH)
                            a.vy[(size_t)(n0 + r) * H + i0 + i] = Vs[i * ES + y];
                    }
                }
                const int itile = i0 + 16 * wave;          // first hidden row of this wavefront's tile
                if (itile < H) {
                    float4 av[8], bv[8];
#pragma unroll
                    for (int m = 0; m < 8; ++m) {
                        av[m] = ld4(es + mrow * ES + 32 * g + 4 * m);
                        bv[m] = ld4(Vs + (16 * wave + mrow) * ES + 32 * g + 4 * m);
                    }
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int m = 0; m < 8; ++m) {
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[m].x, bv[m].x, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[m].y, bv[m].y, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[m].z, bv[m].z, acc, 0, 0, 0);
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[m].w, bv[m].w, acc, 0, 0, 0);
                    }
                    const int i = itile + mrow;            // result: rows 4g..4g+3 of hidden column i
                    if (i < H) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int r = 4 * g + j;
                            if (n0 + r < N) a.gpart[((size_t)blockIdx.x * N + n0 + r) * H + i] = acc[j];
                        }
                    }
                }
                __syncthreads();           // the next batch overwrites Vs
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
    const int spin_limit = a.spin_limit;
    const unsigned epoch = a.epoch;
    // All words of a group of rows are requested at once (four per thread in flight), parked in
    // LDS, and merged from there: the waiting costs about one memory round trip in total.
    float* stage = red;                  // NWV*NR*CW floats >= 2*strips (checked by the host)
    __shared__ float zys[32];
    const unsigned long long* zybox = a.stat_box + (size_t)N * strips * 2;
    unsigned long long wz = tagged_load(zybox + min(tid, N - 1));   // in flight with the rest
    const int rows_per_pass = max(1, (NWV * NR * CW) / (2 * strips));
    for (int n_lo = 0; n_lo < N; n_lo += rows_per_pass) {
        const int n_hi = min(N, n_lo + rows_per_pass);
        const int cnt = (n_hi - n_lo) * strips * 2;
        const unsigned long long* src = a.stat_box + (size_t)n_lo * strips * 2;
        for (int w0 = tid; w0 < cnt; w0 += 4 * NTH) {
            unsigned long long w[4];
            long long idx[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) idx[u] = w0 + u * NTH < cnt ? w0 + u * NTH : -1;
            if (!wait4(src, idx, epoch, spin_limit, w)) s_fail = 1;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (idx[u] >= 0) stage[idx[u]] = tagged_value(w[u]);
        }
        if (n_lo == 0 && tid < N) {
            for (int spins = 0; !tagged_ok(wz, epoch); ++spins) {
                if (spins > spin_limit) { s_fail = 1; break; }
                wz = tagged_load(zybox + tid);
            }
            zys[tid] = tagged_value(wz);
        }
        consume(wz);
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
        // this workgroup has seen every strip's words, so every strip has read the tag: record it
        tag_word_store(a.epoch_word, epoch);
    }
}

size_t logits_smem(int H) { return ((size_t)H * NR + (size_t)NWV * NR * CW + (size_t)(NR + IG * NB) * ES) * 4; }

}  // namespace

int skinny_strips(int O) { return (O + CW - 1) / CW; }

size_t skinny_stat_box_bytes(int N, int O) { return ((size_t)2 * N * skinny_strips(O) + N) * 8; }

bool skinny_supported(int N, int H, int O) {
    if (N > 32 || N < 1 || O % 4 != 0) return false;
    if (2 * skinny_strips(O) > NWV * NR * CW) return false;   // one row of strip statistics fits the LDS stage
    return back_smem(H) <= 64 * 1024 && logits_smem(H) <= 156 * 1024;
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

}  // namespace rnn
