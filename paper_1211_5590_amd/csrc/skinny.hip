// Output layer for a short single sequence (N = T*B <= 32 rows, the paper's batch-1 language
// model benchmark shape): with so few rows the three products with the H x NV output matrix
// are bound by streaming that matrix, not by arithmetic, so they run as column-parallel
// kernels in which every workgroup owns a strip of vocabulary columns, reads its strip of V
// exactly once per kernel, and keeps the N hidden rows in LDS.
//
//   skinny_logits : Z strip = Hs V + c, per-row (max, sum exp) of the strip, target logit
//   skinny_loss   : merges the strip statistics -> lse per row, loss
//   skinny_back   : dZ strip from Z and lse (never written back), dc, dV strip = Hs^T dZ,
//                   partial G = dZ V^T over the strip, and the zero fill of dWx
// The partial G of all strips is summed, in strip order, by the reverse-loop kernel.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

constexpr int NR = 16;    // rows held in registers per pass
constexpr int CW = 128;   // vocabulary columns per workgroup
constexpr int NTH = 256;
constexpr int IG = NTH / CW;  // groups splitting the H dimension

// hidden rows of one pass into LDS as hs[i][NR] (zero padded rows)
__device__ __forceinline__ void load_rows(const float* __restrict__ Hs, float* hs, int n0, int N,
                                          int H, int tid) {
    for (int e = tid; e < H * NR; e += NTH) {
        const int i = e / NR, r = e % NR;
        hs[e] = (n0 + r < N) ? Hs[(size_t)(n0 + r) * H + i] : 0.f;
    }
}

__global__ __launch_bounds__(NTH) void skinny_logits_kernel(SkinnyArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int H = a.H, O = a.O, N = a.N;
    float* hs = smem;                 // [H][NR]
    float* red = hs + H * NR;         // [IG][NR][CW]
    const int tid = threadIdx.x, kk = tid % CW, ig = tid / CW;
    const int k = blockIdx.x * CW + kk;
    const bool kin = k < O;
    const int lane = tid % kWave, wave = tid / kWave;

    for (int n0 = 0; n0 < N; n0 += NR) {
        __syncthreads();
        load_rows(a.Hs, hs, n0, N, H, tid);
        __syncthreads();
        float acc[NR];
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r] = 0.f;
        if (kin) {
#pragma unroll 4
            for (int i = ig; i < H; i += IG) {
                const float v = a.V[(size_t)i * O + k];
                const float4* h4 = reinterpret_cast<const float4*>(hs + i * NR);
#pragma unroll
                for (int r4 = 0; r4 < NR / 4; ++r4) {
                    const float4 h = h4[r4];
                    acc[4 * r4 + 0] = fmaf(h.x, v, acc[4 * r4 + 0]);
                    acc[4 * r4 + 1] = fmaf(h.y, v, acc[4 * r4 + 1]);
                    acc[4 * r4 + 2] = fmaf(h.z, v, acc[4 * r4 + 2]);
                    acc[4 * r4 + 3] = fmaf(h.w, v, acc[4 * r4 + 3]);
                }
            }
        }
#pragma unroll
        for (int r = 0; r < NR; ++r) red[(ig * NR + r) * CW + kk] = acc[r];
        __syncthreads();
        // combine the H-groups, add the bias, store the strip of Z; keep z in red[0]
        for (int e = tid; e < NR * CW; e += NTH) {
            const int r = e / CW, c = e % CW;
            float z = red[r * CW + c];
#pragma unroll
            for (int g = 1; g < IG; ++g) z += red[(g * NR + r) * CW + c];
            const int kc = blockIdx.x * CW + c;
            if (kc < O) z += a.c[kc]; else z = -INFINITY;
            red[r * CW + c] = z;
            if (kc < O && n0 + r < N) a.Z[(size_t)(n0 + r) * O + kc] = z;
        }
        __syncthreads();
        // strip statistics: one wavefront per row
        for (int r = wave; r < NR && n0 + r < N; r += NTH / kWave) {
            const float z0 = red[r * CW + lane], z1 = red[r * CW + 64 + lane];
            const float m = wave_max(fmaxf(z0, z1));
            const float e = __expf(z0 - m) + __expf(z1 - m);  // exp(-inf) = 0 for padding
            const float s = wave_sum(e);
            if (lane == 0) {
                a.pm[(size_t)(n0 + r) * gridDim.x + blockIdx.x] = m;
                a.ps[(size_t)(n0 + r) * gridDim.x + blockIdx.x] = s;
                const int y = a.y[n0 + r] - blockIdx.x * CW;
                if (y >= 0 && y < CW) a.zy[n0 + r] = red[r * CW + y];
            }
        }
    }
}

// one wavefront per row merges the strip statistics; thread 0 then averages the row losses
__global__ __launch_bounds__(NTH) void skinny_loss_kernel(SkinnyArgs a, int strips, float* loss) {
    __shared__ float rl[32];
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    for (int n = wave; n < a.N; n += NTH / kWave) {
        float m = -INFINITY, s = 0.f;
        for (int g = lane; g < strips; g += kWave)
            lse_merge(m, s, a.pm[(size_t)n * strips + g], a.ps[(size_t)n * strips + g]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const float m2 = __shfl_xor(m, off, kWave), s2 = __shfl_xor(s, off, kWave);
            lse_merge(m, s, m2, s2);
        }
        if (lane == 0) {
            const float l = m + logf(s);
            a.lse[n] = l;
            rl[n] = l - a.zy[n];
        }
    }
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int n = 0; n < a.N; ++n) t += rl[n];
        *loss = t / (float)a.N;
    }
}

__global__ __launch_bounds__(NTH) void skinny_back_kernel(SkinnyArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    const int H = a.H, O = a.O, N = a.N;
    float* hs = smem;                    // [H][NR]
    float* dzs = hs + H * NR;            // [CW][NR]
    float* Vs = dzs + CW * NR;           // [H][CW+1]
    float* gred = Vs + H * (CW + 1);     // [IG][NR][H] partial G of the H-groups' column halves
    const int tid = threadIdx.x, kk = tid % CW, ig = tid / CW;
    const int k0 = blockIdx.x * CW, k = k0 + kk;
    const bool kin = k < O;
    const float invN = 1.0f / (float)N;

    // strip of V into LDS (coalesced), reused by every row pass
    for (int e = tid; e < H * CW; e += NTH) {
        const int i = e / CW, c = e % CW;
        Vs[i * (CW + 1) + c] = (k0 + c < O) ? a.V[(size_t)i * O + k0 + c] : 0.f;
    }

    float dc = 0.f;
    for (int n0 = 0; n0 < N; n0 += NR) {
        __syncthreads();
        load_rows(a.Hs, hs, n0, N, H, tid);
        // d loss / d z of the strip for this pass: dzs[c][r]
        for (int e = tid; e < NR * CW; e += NTH) {
            const int r = e / CW, c = e % CW;
            float d = 0.f;
            if (n0 + r < N && k0 + c < O) {
                d = __expf(a.Z[(size_t)(n0 + r) * O + k0 + c] - a.lse[n0 + r]);
                if (a.y[n0 + r] == k0 + c) d -= 1.f;
                d *= invN;
            }
            dzs[c * NR + r] = d;
        }
        __syncthreads();
        float dz[NR];
        {
            const float4* d4 = reinterpret_cast<const float4*>(dzs + kk * NR);
#pragma unroll
            for (int r4 = 0; r4 < NR / 4; ++r4) {
                const float4 d = d4[r4];
                dz[4 * r4] = d.x; dz[4 * r4 + 1] = d.y; dz[4 * r4 + 2] = d.z; dz[4 * r4 + 3] = d.w;
            }
        }
        if (ig == 0) {
#pragma unroll
            for (int r = 0; r < NR; ++r) dc += dz[r];
        }
        // dV[i,k] (+)= sum_r hs[i][r] dz[r]
        if (kin) {
            for (int i = ig; i < H; i += IG) {
                const float4* h4 = reinterpret_cast<const float4*>(hs + i * NR);
                float sum = 0.f;
#pragma unroll
                for (int r4 = 0; r4 < NR / 4; ++r4) {
                    const float4 h = h4[r4];
                    sum = fmaf(h.x, dz[4 * r4], sum);
                    sum = fmaf(h.y, dz[4 * r4 + 1], sum);
                    sum = fmaf(h.z, dz[4 * r4 + 2], sum);
                    sum = fmaf(h.w, dz[4 * r4 + 3], sum);
                }
                float* dst = a.dV + (size_t)i * O + k;
                *dst = (a.beta || n0 > 0) ? *dst + sum : sum;
            }
        }
        // partial G[r][i] = sum over the strip's columns of dz[r][c] V[i][c]; thread = (i, half)
        {
            constexpr int HALF = CW / IG;
            for (int i = tid % CW; i < H; i += CW) {
                float g[NR];
#pragma unroll
                for (int r = 0; r < NR; ++r) g[r] = 0.f;
                const float* vrow = Vs + i * (CW + 1) + ig * HALF;
                for (int c = 0; c < HALF; ++c) {
                    const float v = vrow[c];
                    const float4* d4 = reinterpret_cast<const float4*>(dzs + (ig * HALF + c) * NR);
#pragma unroll
                    for (int r4 = 0; r4 < NR / 4; ++r4) {
                        const float4 d = d4[r4];
                        g[4 * r4 + 0] = fmaf(d.x, v, g[4 * r4 + 0]);
                        g[4 * r4 + 1] = fmaf(d.y, v, g[4 * r4 + 1]);
                        g[4 * r4 + 2] = fmaf(d.z, v, g[4 * r4 + 2]);
                        g[4 * r4 + 3] = fmaf(d.w, v, g[4 * r4 + 3]);
                    }
                }
#pragma unroll
                for (int r = 0; r < NR; ++r) gred[(ig * NR + r) * H + i] = g[r];
            }
        }
        __syncthreads();
        for (int e = tid; e < NR * H; e += NTH) {
            const int r = e / H, i = e % H;
            if (n0 + r >= N) continue;
            float g = gred[r * H + i];
#pragma unroll
            for (int q = 1; q < IG; ++q) g += gred[(q * NR + r) * H + i];
            a.gpart[((size_t)blockIdx.x * N + n0 + r) * H + i] = g;
        }
    }
    if (ig == 0 && kin) a.dc[k] = a.beta ? a.dc[k] + dc : dc;

    // zero fill of the token-gradient matrix, an even share per workgroup (overwrite mode)
    if (a.dWx_zero) {
        const size_t total4 = ((size_t)a.NV * H) / 4;  // NV*H*4 bytes; dWx is 16-byte aligned
        const size_t per = (total4 + gridDim.x - 1) / gridDim.x;
        const size_t b0 = (size_t)blockIdx.x * per;
        const size_t b1 = b0 + per < total4 ? b0 + per : total4;
        float4* z4 = reinterpret_cast<float4*>(a.dWx_zero);
        for (size_t e = b0 + tid; e < b1; e += NTH) z4[e] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (blockIdx.x == 0)
            for (size_t e = total4 * 4 + tid; e < (size_t)a.NV * H; e += NTH) a.dWx_zero[e] = 0.f;
    }
}

}  // namespace

int skinny_strips(int O) { return (O + CW - 1) / CW; }

bool skinny_supported(int N, int H, int O) {
    if (N > 32 || N < 1) return false;
    const size_t back = ((size_t)H * NR + (size_t)CW * NR + (size_t)H * (CW + 1) + (size_t)IG * NR * H) * 4;
    return back <= 150 * 1024 && O >= 1;
}

hipError_t launch_skinny_logits(const SkinnyArgs& a, hipStream_t s) {
    const size_t smem = ((size_t)a.H * NR + (size_t)IG * NR * CW) * 4;
    ProfileScope ps(K_SKINNY_LOGITS, s);
    hipLaunchKernelGGL(skinny_logits_kernel, dim3(skinny_strips(a.O)), dim3(NTH), smem, s, a);
    return hipGetLastError();
}

hipError_t launch_skinny_loss(const SkinnyArgs& a, float* loss, hipStream_t s) {
    ProfileScope ps(K_LOSS_REDUCE, s);
    hipLaunchKernelGGL(skinny_loss_kernel, dim3(1), dim3(NTH), 0, s, a, skinny_strips(a.O), loss);
    return hipGetLastError();
}

hipError_t launch_skinny_back(const SkinnyArgs& a, hipStream_t s) {
    const size_t smem = ((size_t)a.H * NR + (size_t)CW * NR + (size_t)a.H * (CW + 1) + (size_t)IG * NR * a.H) * 4;
    static size_t allowed = 0;
    if (smem > 64 * 1024 && smem > allowed) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(skinny_back_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        allowed = smem;
    }
    ProfileScope ps(K_SKINNY_BACK, s);
    hipLaunchKernelGGL(skinny_back_kernel, dim3(skinny_strips(a.O)), dim3(NTH), smem, s, a);
    return hipGetLastError();
}

}  // namespace rnn
