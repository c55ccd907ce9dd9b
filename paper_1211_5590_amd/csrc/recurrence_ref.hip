// Shape-agnostic time-loop kernels (any H, any B): one workgroup per batch row runs the whole
// loop on the device, so the host does no work per step (the paper's Scan properties 4 and 5).
// The recurrent matrix is re-read from L2 every step; the resident-weight kernels in
// recurrence.hip replace these for the shapes they cover.  These stay as the fallback and as
// the A/B partner in tests (RNN_FLAG_REFERENCE_KERNELS).
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

__global__ __launch_bounds__(256) void transpose_kernel(const float* __restrict__ src,
                                                        float* __restrict__ dst, int rows, int cols) {
    __shared__ float tile[32][33];
    const int bx = blockIdx.x * 32, by = blockIdx.y * 32;
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int gr = by + r, gc = bx + tx;
        tile[r][tx] = (gr < rows && gc < cols) ? src[(size_t)gr * cols + gc] : 0.f;
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        const int gr = bx + r, gc = by + tx;  // dst is [cols, rows]
        if (gr < cols && gc < rows) dst[(size_t)gr * rows + gc] = tile[tx][r];
    }
}

// out[j] = sum_i Mat[j*H + i] * vec[i] for the rows j this wavefront owns (lanes stride i)
__device__ __forceinline__ float row_dot(const float* __restrict__ row, const float* vec, int H,
                                         int lane) {
    float acc = 0.f;
    for (int i = lane; i < H; i += kWave) acc = fmaf(row[i], vec[i], acc);
    return wave_sum(acc);
}

template <int ACT>
__global__ __launch_bounds__(256) void rec_fwd_ref_kernel(RecFwdArgs a) {
    extern __shared__ float smem[];  // hbuf[2][H]
    const int H = a.H, B = a.B, bb = blockIdx.x;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave, nwaves = blockDim.x / kWave;
    float* hbuf0 = smem;
    float* hbuf1 = smem + H;

    for (int j = tid; j < H; j += blockDim.x) {
        const float v = a.h0 ? a.h0[(size_t)bb * H + j] : 0.f;
        hbuf0[j] = v;
        a.hist[(size_t)bb * H + j] = v;  // slot 0 in both history and ring mode
    }
    __syncthreads();

    for (int t = 0; t < a.T; ++t) {
        const float* hp = (t & 1) ? hbuf1 : hbuf0;
        float* hn = (t & 1) ? hbuf0 : hbuf1;
        const size_t slot = a.ring ? (size_t)((t + 1) & 1) : (size_t)(t + 1);
        float* hout = a.hist + (slot * B + bb) * H;
        const float* in_row = a.U ? a.U + ((size_t)t * B + bb) * H
                                  : a.Wx + (size_t)a.x[(size_t)t * B + bb] * H;
        for (int j = wave; j < H; j += nwaves) {
            const float dot = row_dot(a.Wh + (size_t)j * H, hp, H, lane);
            if (lane == 0) {
                const float pre = dot + in_row[j] + (a.U ? 0.f : a.b[j]);
                const float h = activate<ACT>(pre);
                hn[j] = h;
                hout[j] = h;
            }
        }
        __syncthreads();
    }
    if (a.h_last) {
        const float* hf = (a.T & 1) ? hbuf1 : hbuf0;
        for (int j = tid; j < H; j += blockDim.x) a.h_last[(size_t)bb * H + j] = hf[j];
    }
}

template <int ACT>
__global__ __launch_bounds__(256) void rec_bwd_ref_kernel(RecBwdArgs a) {
    extern __shared__ float smem[];  // carry[H], dlt[H]
    const int H = a.H, B = a.B, bb = blockIdx.x;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave, nwaves = blockDim.x / kWave;
    float* carry = smem;
    float* dlt = smem + H;

    for (int j = tid; j < H; j += blockDim.x)
        carry[j] = a.dh_last ? a.dh_last[(size_t)bb * H + j] : 0.f;
    __syncthreads();

    for (int t = a.T - 1; t >= 0; --t) {
        const size_t row = ((size_t)t * B + bb) * H;
        const float* ht = a.h_all + ((size_t)(t + 1) * B + bb) * H;
        for (int j = tid; j < H; j += blockDim.x) {
            const float d = (a.G[row + j] + carry[j]) * act_grad<ACT>(ht[j]);
            dlt[j] = d;
            a.Delta[row + j] = d;
        }
        __syncthreads();
        if (t > 0 || a.dh0) {
            // carry[i] = sum_j Wh[j,i] dlt[j] = row i of the transposed copy times dlt
            for (int i = wave; i < H; i += nwaves) {
                const float dot = row_dot(a.WhT + (size_t)i * H, dlt, H, lane);
                if (lane == 0) carry[i] = dot;
            }
        }
        __syncthreads();
    }
    if (a.dh0)
        for (int j = tid; j < H; j += blockDim.x) a.dh0[(size_t)bb * H + j] = carry[j];
}

}  // namespace

hipError_t launch_transpose(const float* src, float* dst, int rows, int cols, hipStream_t s) {
    dim3 grid((cols + 31) / 32, (rows + 31) / 32);
    ProfileScope ps(K_TRANSPOSE, s);
    hipLaunchKernelGGL(transpose_kernel, grid, dim3(256), 0, s, src, dst, rows, cols);
    return hipGetLastError();
}

hipError_t launch_rec_fwd_reference(const RecFwdArgs& a, hipStream_t s) {
    const size_t smem = 2 * sizeof(float) * (size_t)a.H;
    if (smem > 64 * 1024) return hipErrorInvalidValue;
    ProfileScope ps(K_REC_FWD, s);
    if (a.act == 0)
        hipLaunchKernelGGL(rec_fwd_ref_kernel<0>, dim3(a.B), dim3(256), smem, s, a);
    else
        hipLaunchKernelGGL(rec_fwd_ref_kernel<1>, dim3(a.B), dim3(256), smem, s, a);
    return hipGetLastError();
}

hipError_t launch_rec_bwd_reference(const RecBwdArgs& a, hipStream_t s) {
    const size_t smem = 2 * sizeof(float) * (size_t)a.H;
    if (smem > 64 * 1024) return hipErrorInvalidValue;
    ProfileScope ps(K_REC_BWD, s);
    if (a.act == 0)
        hipLaunchKernelGGL(rec_bwd_ref_kernel<0>, dim3(a.B), dim3(256), smem, s, a);
    else
        hipLaunchKernelGGL(rec_bwd_ref_kernel<1>, dim3(a.B), dim3(256), smem, s, a);
    return hipGetLastError();
}

}  // namespace rnn
