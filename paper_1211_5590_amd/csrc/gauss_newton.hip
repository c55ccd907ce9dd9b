// Small kernels of the Gauss-Newton-vector product (the paper's section on the R-operator):
// everything heavy in that product is one of the path's existing matrix products or time loops;
// what is left is re-ordering rows in time, adding gathered rows, and applying the Hessian of the
// loss with respect to the outputs to the rows of R z.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

// dst row t = src row T-1-t, rows of `row` floats
__global__ __launch_bounds__(256) void reverse_rows_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                           int T, int row) {
    const int t = blockIdx.y;
    const float* s = src + (size_t)(T - 1 - t) * row;
    float* d = dst + (size_t)t * row;
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < row; i += gridDim.x * blockDim.x) d[i] = s[i];
}

// C[n][:] += M[x[n]][:]
__global__ __launch_bounds__(256) void gather_add_kernel(const int32_t* __restrict__ x, const float* __restrict__ M,
                                                         float* __restrict__ C, int H) {
    const int n = blockIdx.x;
    const float* row = M + (size_t)x[n] * H;
    for (int j = threadIdx.x; j < H; j += blockDim.x) C[(size_t)n * H + j] += row[j];
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float* p, size_t n) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0.f;
}

__global__ __launch_bounds__(256) void scale_kernel(float* p, size_t n, float alpha) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] *= alpha;
}

// One workgroup per row n: RZ_n <- (p * RZ_n - p (p . RZ_n)) * scale with p = softmax(Z_n), the
// product of the cross-entropy's Hessian with respect to the logits and RZ_n.
__global__ __launch_bounds__(256) void gn_softmax_metric_kernel(const float* __restrict__ Z, float* __restrict__ RZ,
                                                                int O, float scale) {
    __shared__ float red[3][4];
    const size_t base = (size_t)blockIdx.x * O;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float m = -INFINITY;
    for (int k = tid; k < O; k += 256) m = fmaxf(m, Z[base + k]);
    m = wave_max(m);
    if (lane == 0) red[0][wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3]));
    float s = 0.f, dot = 0.f;
    for (int k = tid; k < O; k += 256) {
        const float e = __expf(Z[base + k] - m);
        s += e;
        dot = fmaf(e, RZ[base + k], dot);
    }
    s = wave_sum(s);
    dot = wave_sum(dot);
    if (lane == 0) { red[1][wave] = s; red[2][wave] = dot; }
    __syncthreads();
    s = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
    dot = (red[2][0] + red[2][1]) + (red[2][2] + red[2][3]);
    const float inv = 1.0f / s;
    const float pdot = dot * inv;                      // p . RZ
    for (int k = tid; k < O; k += 256) {
        const float p = __expf(Z[base + k] - m) * inv;
        RZ[base + k] = p * (RZ[base + k] - pdot) * scale;
    }
}

int blocks_for(size_t n) {
    const size_t b = (n + 255) / 256;
    return (int)(b < 1 ? 1 : (b > 4096 ? 4096 : b));
}

}  // namespace

hipError_t launch_reverse_rows(const float* src, float* dst, int T, int row, hipStream_t s) {
    ProfileScope ps(K_MISC, s);
    hipLaunchKernelGGL(reverse_rows_kernel, dim3(blocks_for((size_t)row), T), dim3(256), 0, s, src, dst, T, row);
    return hipGetLastError();
}
hipError_t launch_gather_add(const int32_t* x, const float* M, float* C, int N, int H, hipStream_t s) {
    ProfileScope ps(K_MISC, s);
    hipLaunchKernelGGL(gather_add_kernel, dim3(N), dim3(256), 0, s, x, M, C, H);
    return hipGetLastError();
}
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t s) {
    ProfileScope ps(K_MISC, s);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks_for(n)), dim3(256), 0, s, p, n);
    return hipGetLastError();
}
hipError_t launch_scale(float* p, size_t n, float alpha, hipStream_t s) {
    ProfileScope ps(K_GN_METRIC, s);
    hipLaunchKernelGGL(scale_kernel, dim3(blocks_for(n)), dim3(256), 0, s, p, n, alpha);
    return hipGetLastError();
}
hipError_t launch_gn_softmax_metric(const float* Z, float* RZ, int N, int O, float scale, hipStream_t s) {
    ProfileScope ps(K_GN_METRIC, s);
    hipLaunchKernelGGL(gn_softmax_metric_kernel, dim3(N), dim3(256), 0, s, Z, RZ, O, scale);
    return hipGetLastError();
}

}  // namespace rnn
