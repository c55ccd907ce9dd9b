// Batched recurrence for hidden sizes whose matrix does not fit one CU's registers (batch > 4,
// H > 256): one fused matrix-core launch per time step.
//
// With a batch the per-step product is a small GEMM (B x H x H).  The kernel boundary is the
// cheapest device-wide synchronisation measured on this part (a few microseconds -- less than
// an in-kernel release/acquire exchange between XCDs, which has to write back and invalidate
// whole L2s), so every step is one launch; its epilogue applies the input term and activation
// (forward) or the output-layer term and activation derivative (reverse), so the element-wise
// work stays fused into the producing kernel and the host does nothing between steps but
// enqueue.
//
// Tiling of a step: a workgroup of 4 wavefronts owns 16 batch rows x 16 output columns (for
// the 64 x 1024 x 1024 step that is 256 workgroups, one per CU, each streaming its 64 KB slice
// of Wh and 64 KB of state through LDS in K-chunks of 128, double buffered (few, large chunks: every
// chunk costs one L2 round trip that the little arithmetic of a chunk cannot hide); the forward loop uses a
// transposed copy of Wh made once per call so that both directions read the matrix as [k][n]
// and neighbouring workgroups touch neighbouring bytes); a wavefront owns a quarter
// of K as a v_mfma_f32_16x16x4_f32 accumulator pair; the halves meet in LDS.  Inside a chunk K is walked in
// a permuted order (lane group g takes k in [32g, 32g+32)), so a lane's 32 A and 32 B operands
// are 128 contiguous bytes of LDS each.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int SM = 16, SN = 16, SK = 128, SLD = SK + 4, NT = 256;
constexpr int KG = SK / 4;                 // k per lane group inside a chunk
constexpr int RT = SM / 16;                // 16-row tiles per workgroup
constexpr int KSPL = 4 / RT;               // wavefronts sharing a row tile, each a slice of K
constexpr int KW = KG / KSPL;              // k-steps per wavefront per chunk
constexpr int NA4 = SM * SK / 4 / NT;      // float4 of the state chunk per thread (8)
constexpr int NB4 = SN * SK / 4 / NT;      // float4 of the matrix chunk per thread (2)

struct StepArgs {
    const float* A;      // [M,H] previous state (forward) or delta_{t+1} (reverse)
    const float* Wm;     // [H(k),H(n)] matrix of the product: Wh^T (forward) or Wh (reverse)
    float* C;            // [M,H] new state / delta_t
    const float* e0;     // forward: input term rows [M,H], or Wx when ids != NULL; reverse: G_t
    const float* e1;     // forward with ids: bias b; reverse: h_t
    const int32_t* ids;  // forward token input: ids of the M rows, else NULL
    int M, H;
};

template <int ACT, bool BWD, bool VEC>
__global__ __launch_bounds__(NT) void rec_step_kernel(StepArgs p) {
    __shared__ __attribute__((aligned(16))) float As[2][SM][SLD];
    __shared__ __attribute__((aligned(16))) float Bs[2][SN][SLD];
    __shared__ float red[4][kWave][4];          // partial tiles of the kh > 0 wavefronts
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int g = lane / 16, nn = lane % 16;
    const int rt = wave % RT, kh = wave / RT;  // row tile of 16, slice of each lane group's k range
    const int n0 = blockIdx.x * SN, m0 = blockIdx.y * SM;
    const int H = p.H, M = p.M;
    const int nk = (H + SK - 1) / SK;

    float4 ra[NA4], rb[NB4];
    auto load4 = [&](const float* base, int k, int klim) -> float4 {  // 4 floats along k
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if (VEC && k + 3 < klim) return *reinterpret_cast<const float4*>(base + k);
        if (k + 0 < klim) t.x = base[k + 0];
        if (k + 1 < klim) t.y = base[k + 1];
        if (k + 2 < klim) t.z = base[k + 2];
        if (k + 3 < klim) t.w = base[k + 3];
        return t;
    };
    auto fetch = [&](int kc) {
        const int k0 = kc * SK;
#pragma unroll
        for (int i = 0; i < NA4; ++i) {
            const int idx = tid + NT * i, r = idx / (SK / 4), kq = (idx % (SK / 4)) * 4;
            ra[i] = (m0 + r < M) ? load4(p.A + (size_t)(m0 + r) * H, k0 + kq, H)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        // Bs[n][k] = Wm[k0+k][n0+n]: 4 consecutive n of one k; neighbouring workgroups read
        // neighbouring 64-byte pieces of the same matrix rows
#pragma unroll
        for (int i = 0; i < NB4; ++i) {
            const int idx = tid + NT * i, k = idx / 4, nq = (idx % 4) * 4;
            rb[i] = (k0 + k < H) ? load4(p.Wm + (size_t)(k0 + k) * H, n0 + nq, H)
                                 : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto park = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NA4; ++i) {
            const int idx = tid + NT * i, r = idx / (SK / 4), kq = (idx % (SK / 4)) * 4;
            *reinterpret_cast<float4*>(&As[buf][r][kq]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < NB4; ++i) {
            const int idx = tid + NT * i, k = idx / 4, nq = (idx % 4) * 4;
            Bs[buf][nq + 0][k] = rb[i].x;
            Bs[buf][nq + 1][k] = rb[i].y;
            Bs[buf][nq + 2][k] = rb[i].z;
            Bs[buf][nq + 3][k] = rb[i].w;
        }
    };

    // Epilogue operands do not depend on the product: request them before the K loop so their
    // latency (two dependent loads for token input) is hidden behind it.
    const int col = n0 + nn;
    float x0[4], x1[4];
    {
        const int cc = min(col, H - 1);
        int rr[4], id[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) rr[i] = min(m0 + 16 * rt + 4 * g + i, M - 1);
        if (!BWD && p.ids) {
#pragma unroll
            for (int i = 0; i < 4; ++i) id[i] = p.ids[rr[i]];
            const float tb = p.e1[cc];
#pragma unroll
            for (int i = 0; i < 4; ++i) { x0[i] = p.e0[(size_t)id[i] * H + cc] + tb; x1[i] = 0.f; }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                x0[i] = p.e0[(size_t)rr[i] * H + cc];
                x1[i] = BWD ? p.e1[(size_t)rr[i] * H + cc] : 0.f;
            }
        }
    }

    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    fetch(0);
    park(0);
    __syncthreads();
    for (int kc = 0; kc < nk; ++kc) {
        const int cur = kc & 1;
        if (kc + 1 < nk) fetch(kc + 1);
        float a[KW], b[KW];
        const float4* pa = reinterpret_cast<const float4*>(&As[cur][16 * rt + nn][KG * g + KW * kh]);
        const float4* pb = reinterpret_cast<const float4*>(&Bs[cur][nn][KG * g + KW * kh]);
#pragma unroll
        for (int i = 0; i < KW / 4; ++i) {
            const float4 va = pa[i], vb = pb[i];
            a[4 * i] = va.x; a[4 * i + 1] = va.y; a[4 * i + 2] = va.z; a[4 * i + 3] = va.w;
            b[4 * i] = vb.x; b[4 * i + 1] = vb.y; b[4 * i + 2] = vb.z; b[4 * i + 3] = vb.w;
        }
#pragma unroll
        for (int s = 0; s < KW; s += 2) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s], b[s], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s + 1], b[s + 1], acc1, 0, 0, 0);
        }
        if (kc + 1 < nk) park(cur ^ 1);
        __syncthreads();
    }

    // the K slices of a row tile meet in LDS; the kh = 0 wavefront finishes the tile
    if (kh > 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i) red[wave][lane][i] = acc0[i] + acc1[i];
    }
    __syncthreads();
    if (kh > 0) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int row = m0 + 16 * rt + 4 * g + i;
        if (row >= M || col >= H) continue;
        float v = acc0[i] + acc1[i];
#pragma unroll
        for (int w = 1; w < KSPL; ++w) v += red[rt + RT * w][lane][i];
        const float out = BWD ? (v + x0[i]) * act_grad<ACT>(x1[i]) : activate<ACT>(v + x0[i]);
        p.C[(size_t)row * H + col] = out;
    }
}

template <bool BWD>
hipError_t launch_step(const StepArgs& p, int act, hipStream_t s) {
    dim3 grid((p.H + SN - 1) / SN, (p.M + SM - 1) / SM);
    const bool vec = p.H % 4 == 0 && (reinterpret_cast<uintptr_t>(p.A) & 15u) == 0 &&
                     (reinterpret_cast<uintptr_t>(p.Wm) & 15u) == 0;
    ProfileScope ps(BWD ? K_REC_BWD : K_REC_FWD, s);
    if (act == 0) {
        if (vec) hipLaunchKernelGGL((rec_step_kernel<0, BWD, true>), grid, dim3(NT), 0, s, p);
        else hipLaunchKernelGGL((rec_step_kernel<0, BWD, false>), grid, dim3(NT), 0, s, p);
    } else {
        if (vec) hipLaunchKernelGGL((rec_step_kernel<1, BWD, true>), grid, dim3(NT), 0, s, p);
        else hipLaunchKernelGGL((rec_step_kernel<1, BWD, false>), grid, dim3(NT), 0, s, p);
    }
    return hipGetLastError();
}

// dst[0:n) = src ? src : 0
__global__ __launch_bounds__(256) void copy_or_zero_kernel(const float* __restrict__ src,
                                                           float* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x)
        dst[i] = src ? src[i] : 0.f;
}

// delta_{T-1} = (G_{T-1} + dh_last) * act'(h_{T-1})
__global__ __launch_bounds__(256) void bwd_first_kernel(const float* __restrict__ G,
                                                        const float* __restrict__ dh_last,
                                                        const float* __restrict__ h,
                                                        float* __restrict__ delta, size_t n, int act) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x) {
        const float g = G[i] + (dh_last ? dh_last[i] : 0.f);
        delta[i] = g * (act == 0 ? act_grad<0>(h[i]) : act_grad<1>(h[i]));
    }
}

int blocks_for(size_t n) {
    size_t b = (n + 255) / 256;
    return (int)(b > 1024 ? 1024 : (b < 1 ? 1 : b));
}

}  // namespace

hipError_t run_rec_fwd_stepwise(const RecFwdArgs& a, hipStream_t s) {
    const size_t bh = (size_t)a.B * a.H;
    // one transposed copy per call: both directions then stream the matrix in the same
    // channel-friendly [k][n] order
    {
        hipError_t e = launch_transpose(a.Wh, a.WhT, a.H, a.H, s);
        if (e != hipSuccess) return e;
    }
    {
        ProfileScope ps(K_MISC, s);
        hipLaunchKernelGGL(copy_or_zero_kernel, dim3(blocks_for(bh)), dim3(256), 0, s, a.h0, a.hist, bh);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int t = 0; t < a.T; ++t) {
        const size_t in_slot = a.ring ? (size_t)(t & 1) : (size_t)t;
        const size_t out_slot = a.ring ? (size_t)((t + 1) & 1) : (size_t)(t + 1);
        StepArgs p{};
        p.A = a.hist + in_slot * bh; p.Wm = a.WhT; p.C = a.hist + out_slot * bh;
        p.M = a.B; p.H = a.H;
        if (a.U) {
            p.e0 = a.U + (size_t)t * bh;
        } else {
            p.e0 = a.Wx; p.e1 = a.b; p.ids = a.x + (size_t)t * a.B;
        }
        hipError_t e = launch_step<false>(p, a.act, s);
        if (e != hipSuccess) return e;
    }
    if (a.h_last) {
        const size_t last = a.ring ? (size_t)(a.T & 1) : (size_t)a.T;
        ProfileScope ps(K_MISC, s);
        hipLaunchKernelGGL(copy_or_zero_kernel, dim3(blocks_for(bh)), dim3(256), 0, s,
                           (const float*)(a.hist + last * bh), a.h_last, bh);
        return hipGetLastError();
    }
    return hipSuccess;
}

hipError_t run_rec_bwd_stepwise(const RecBwdArgs& a, hipStream_t s) {
    const size_t bh = (size_t)a.B * a.H;
    {
        ProfileScope ps(K_MISC, s);
        hipLaunchKernelGGL(bwd_first_kernel, dim3(blocks_for(bh)), dim3(256), 0, s,
                           a.G + (size_t)(a.T - 1) * bh, a.dh_last, a.h_all + (size_t)a.T * bh,
                           a.Delta + (size_t)(a.T - 1) * bh, bh, a.act);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int t = a.T - 2; t >= 0; --t) {
        StepArgs p{};
        p.A = a.Delta + (size_t)(t + 1) * bh; p.Wm = a.Wh; p.C = a.Delta + (size_t)t * bh;
        p.M = a.B; p.H = a.H;
        p.e0 = a.G + (size_t)t * bh;
        p.e1 = a.h_all + (size_t)(t + 1) * bh;
        hipError_t e = launch_step<true>(p, a.act, s);
        if (e != hipSuccess) return e;
    }
    if (a.dh0) {  // dh0 = delta_0 Wh
        GemmArgs g{};
        g.A = a.Delta; g.B = a.Wh; g.C = a.dh0;
        g.M = a.B; g.N = a.H; g.K = a.H;
        g.lda = a.H; g.ldb = a.H; g.ldc = a.H;
        g.a_t = false; g.b_t = false;
        g.splitk_ws = a.splitk_ws; g.prof_id = K_GEMM_DH0;
        return launch_gemm(g, s);
    }
    return hipSuccess;
}

}  // namespace rnn
