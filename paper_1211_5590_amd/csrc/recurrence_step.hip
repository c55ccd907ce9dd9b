// Batched recurrence (batch > 4) as one fused MFMA launch per time step.
//
// With a batch the per-step product is a small GEMM (B x H x H); the kernel boundary is the
// cheapest device-wide synchronisation measured on this part (a few microseconds, less than
// an in-kernel release/acquire exchange between XCDs), so every step is one launch of the
// 64x64-tile GEMM whose epilogue applies the input term and activation (forward) or the
// output-layer term and activation derivative (reverse) -- the element-wise work stays fused
// into the producing kernel, and the host still does nothing between steps but enqueue.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

// dst[0:n) = src ? src : 0, and optionally a second copy
__global__ __launch_bounds__(256) void copy_or_zero_kernel(const float* __restrict__ src,
                                                           float* __restrict__ dst,
                                                           float* __restrict__ dst2, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (size_t)gridDim.x * blockDim.x) {
        const float v = src ? src[i] : 0.f;
        dst[i] = v;
        if (dst2) dst2[i] = v;
    }
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
        hipLaunchKernelGGL(copy_or_zero_kernel, dim3(blocks_for(bh)), dim3(256), 0, s, a.h0, a.hist,
                           (float*)nullptr, bh);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int t = 0; t < a.T; ++t) {
        const size_t in_slot = a.ring ? (size_t)(t & 1) : (size_t)t;
        const size_t out_slot = a.ring ? (size_t)((t + 1) & 1) : (size_t)(t + 1);
        GemmArgs g{};
        g.A = a.hist + in_slot * bh; g.B = a.Wh; g.C = a.hist + out_slot * bh;
        g.M = a.B; g.N = a.H; g.K = a.H;
        g.lda = a.H; g.ldb = a.H; g.ldc = a.H;
        g.a_t = false; g.b_t = true;  // h_{t-1} Wh^T
        g.epi = GEMM_EPI_REC_FWD; g.act = a.act;
        if (a.U) {
            g.e0 = a.U + (size_t)t * bh;
        } else {
            g.e0 = a.Wx; g.e1 = a.b; g.ids = a.x + (size_t)t * a.B;
        }
        hipError_t e = launch_gemm(g, s);
        if (e != hipSuccess) return e;
    }
    if (a.h_last) {
        const size_t last = a.ring ? (size_t)(a.T & 1) : (size_t)a.T;
        ProfileScope ps(K_MISC, s);
        hipLaunchKernelGGL(copy_or_zero_kernel, dim3(blocks_for(bh)), dim3(256), 0, s,
                           (const float*)(a.hist + last * bh), a.h_last, (float*)nullptr, bh);
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
        GemmArgs g{};
        g.A = a.Delta + (size_t)(t + 1) * bh; g.B = a.Wh; g.C = a.Delta + (size_t)t * bh;
        g.M = a.B; g.N = a.H; g.K = a.H;
        g.lda = a.H; g.ldb = a.H; g.ldc = a.H;
        g.a_t = false; g.b_t = false;  // delta_{t+1} Wh
        g.epi = GEMM_EPI_REC_BWD; g.act = a.act;
        g.e0 = a.G + (size_t)t * bh;
        g.e1 = a.h_all + (size_t)(t + 1) * bh;
        hipError_t e = launch_gemm(g, s);
        if (e != hipSuccess) return e;
    }
    if (a.dh0) {  // dh0 = delta_0 Wh
        GemmArgs g{};
        g.A = a.Delta; g.B = a.Wh; g.C = a.dh0;
        g.M = a.B; g.N = a.H; g.K = a.H;
        g.lda = a.H; g.ldb = a.H; g.ldc = a.H;
        g.a_t = false; g.b_t = false;
        g.epi = GEMM_EPI_PLAIN; g.splitk_ws = a.splitk_ws;
        return launch_gemm(g, s);
    }
    return hipSuccess;
}

}  // namespace rnn
