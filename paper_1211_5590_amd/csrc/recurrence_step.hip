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
// A step moves little (for the 64 x 1024 x 1024 step 64 KB of state and 64 KB of matrix per
// workgroup) and computes less, so what it costs is memory round trips: the kernel is built to
// pay ONE.  A workgroup of 16 wavefronts owns 16 batch rows x 16 output columns (256
// workgroups for that step, one per CU); every wavefront takes a 64-wide slice of K and
// requests its whole share of both operands at once, straight into the lane registers the
// matrix instruction (v_mfma_f32_16x16x4_f32) reads them from: lane (r = lane % 16, g = lane / 16)
// holds, as four float4, k = k0 + 16 s + 4 g + e of state row r and of matrix row r, so that the
// four lane groups of one request cover 64 contiguous bytes of a row and both operands walk K in
// the same permuted order.  No LDS staging, no barrier inside the product; the 16 partial tiles
// meet in LDS once.  Both operands are K-contiguous ([n][k]): the forward product reads Wh as it
// is stored, the reverse product a transposed copy made once per call; either way a workgroup's
// slice of the matrix and its state rows are two contiguous 64 KB blocks.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int SM = 16, SN = 16, SKC = 64, SWAVES = 16, NT = SWAVES * kWave;

struct StepArgs {
    const float* A;      // [M,H] previous state (forward) or delta_{t+1} (reverse)
    const float* Wm;     // [H(n),H(k)] matrix of the product, K-contiguous: Wh (forward) or Wh^T (reverse)
    float* C;            // [M,H] new state / delta_t
    const float* e0;     // forward: input term rows [M,H], or Wx when ids != NULL; reverse: G_t
    const float* e1;     // forward with ids: bias b; reverse: h_t
    const int32_t* ids;  // forward token input: ids of the M rows, else NULL
    int M, H;
};

template <bool VEC>
__device__ __forceinline__ float4 load_k4(const float* __restrict__ row, int k, int klim) {
    if (VEC && k + 3 < klim) return *reinterpret_cast<const float4*>(row + k);
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k + 0 < klim) t.x = row[k + 0];
    if (k + 1 < klim) t.y = row[k + 1];
    if (k + 2 < klim) t.z = row[k + 2];
    if (k + 3 < klim) t.w = row[k + 3];
    return t;
}

template <int ACT, bool BWD, bool VEC>
__global__ __launch_bounds__(NT) void rec_step_kernel(StepArgs p) {
    __shared__ float red[SWAVES][4][kWave];     // partial tiles, [wavefront][register][lane]
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int g = lane / 16, nn = lane % 16;
    const int n0 = blockIdx.x * SN, m0 = blockIdx.y * SM;
    const int H = p.H, M = p.M;
    const int nchunks = (H + SKC - 1) / SKC;

    // Epilogue operands do not depend on the product: the four wavefronts that finish the tile
    // request them first (two dependent loads for token input), behind the operand requests.
    // thread (lane, i = wave) of those finishes row 4 g + i, column nn
    const int col = n0 + nn;
    float x0 = 0.f, x1 = 0.f;
    if (wave < 4) {
        const int cc = min(col, H - 1);
        const int rr = min(m0 + 4 * g + wave, M - 1);
        if (!BWD && p.ids) {
            x0 = p.e0[(size_t)p.ids[rr] * H + cc] + p.e1[cc];
        } else {
            x0 = p.e0[(size_t)rr * H + cc];
            if (BWD) x1 = p.e1[(size_t)rr * H + cc];
        }
    }

    const bool a_ok = m0 + nn < M, b_ok = col < H;
    const float* arow = p.A + (size_t)min(m0 + nn, M - 1) * H;
    const float* brow = p.Wm + (size_t)min(col, H - 1) * H;
    f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
    for (int kc = wave; kc < nchunks; kc += SWAVES) {
        const int k0 = kc * SKC + 4 * g;
        float4 a[4], b[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            a[s] = a_ok ? load_k4<VEC>(arow, k0 + 16 * s, H) : make_float4(0.f, 0.f, 0.f, 0.f);
            b[s] = b_ok ? load_k4<VEC>(brow, k0 + 16 * s, H) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].x, b[s].x, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].y, b[s].y, acc1, 0, 0, 0);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].z, b[s].z, acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s].w, b[s].w, acc1, 0, 0, 0);
        }
    }
    // result layout of the 16x16 tile: lane -> column nn; register i -> row 4 g + i
#pragma unroll
    for (int i = 0; i < 4; ++i) red[wave][i][lane] = acc0[i] + acc1[i];
    __syncthreads();
    if (wave >= 4) return;
    const int row = m0 + 4 * g + wave;
    if (row >= M || col >= H) return;
    float v = 0.f;
#pragma unroll
    for (int w = 0; w < SWAVES; ++w) v += red[w][wave][lane];
    p.C[(size_t)row * H + col] = BWD ? (v + x0) * act_grad<ACT>(x1) : activate<ACT>(v + x0);
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
        p.A = a.hist + in_slot * bh; p.Wm = a.Wh; p.C = a.hist + out_slot * bh;
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
        p.A = a.Delta + (size_t)(t + 1) * bh; p.Wm = a.WhT; p.C = a.Delta + (size_t)t * bh;
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
