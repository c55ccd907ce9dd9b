// Persistent batched time loop on the matrix cores with the recurrent matrix resident in
// registers (hidden size <= 256, batch > 4).
//
// Batch rows are independent, so the batch is cut into tiles of 16 rows and every tile gets
// its own workgroup that never talks to another one: no device-wide synchronisation exists
// in this kernel, a step costs one LDS-only workgroup barrier.  The workgroup has 8
// wavefronts; each owns 16*NTW output columns and keeps its share of Wh (forward) or Wh^T
// (reverse) for the whole launch as the B operands of v_mfma_f32_16x16x4_f32 -- HP/4 k-steps
// times NTW column tiles = up to 128 registers per lane.  The state tile (16 x H) lives in
// LDS, double buffered; every wavefront reads all of it once per step as A operands.
//
// K is walked in a permuted order: the MFMA takes k = lane/16 from four lane groups, and
// group g is given the contiguous range [g*HP/4, (g+1)*HP/4), so a lane's A operands for all
// k-steps are HP/4 consecutive floats of one state row (16-byte LDS reads) and its B operands
// HP/4 consecutive weights of one matrix row.  A sum over k does not care about the order.
//
// The per-step epilogue (input term + activation, or output-layer term times the activation
// derivative) is fused, its operands are requested one step ahead, and the new state goes to
// both the history in HBM and the other LDS buffer (the paper's Scan keeps every state for
// the gradient loop: property 1; nothing per step happens on the host: properties 4 and 5).
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int kRows = 16;  // batch rows per workgroup (the MFMA M dimension)

__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int ACT, bool BWD, int HP>
__global__ __launch_bounds__(kThreads) void rec_batch_mfma_kernel(RecMfmaArgs a) {
    constexpr int NTILES = HP / 16;               // column tiles of 16
    constexpr int NTW = (NTILES + 7) / 8;         // column tiles per wavefront
    constexpr int KS = HP / 4;                    // k-steps = floats of one lane's A/B strip
    constexpr int LDH = HP + 4;                   // LDS row stride (rows 4 banks apart)
    __shared__ __attribute__((aligned(16))) float hs[2][kRows][LDH];

    const int H = a.H, B = a.B, T = a.T;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int g = lane / 16, nn = lane % 16;
    const int b0 = blockIdx.x * kRows;
    const size_t bh = (size_t)B * H;

    // ---- resident weights: breg[nt][s] = M[k = KS*g + s][col], M = Wh^T (fwd) or Wh (bwd) ----
    float breg[NTW][KS];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        const int col = (wave * NTW + nt) * 16 + nn;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int k = KS * g + s;
            float w = 0.f;
            if (col < H && k < H) w = BWD ? a.Wh[(size_t)k * H + col] : a.Wh[(size_t)col * H + k];
            breg[nt][s] = w;
        }
    }

    // ---- initial state tile -----------------------------------------------------------------
    for (int i = tid; i < 2 * kRows * LDH; i += kThreads) (&hs[0][0][0])[i] = 0.f;
    __syncthreads();
    for (int i = tid; i < kRows * H; i += kThreads) {
        const int m = i / H, j = i - m * H, row = b0 + m;
        if (row >= B) continue;
        float v;
        if (!BWD) {
            v = a.h0 ? a.h0[(size_t)row * H + j] : 0.f;
            a.hist[(size_t)row * H + j] = v;                       // slot 0
        } else {
            const size_t e = (size_t)(T - 1) * bh + (size_t)row * H + j;
            const float c = a.dh_last ? a.dh_last[(size_t)row * H + j] : 0.f;
            const float h = a.h_all[(size_t)T * bh + (size_t)row * H + j];
            v = (a.G[e] + c) * act_grad<ACT>(h);
            a.Delta[e] = v;
        }
        hs[0][m][j] = v;
    }
    __syncthreads();

    // Epilogue operands of step s for this lane's 4 rows x NTW columns.
    // forward: x0 = input term U[s]; reverse (t = T-2-s): x0 = G[t], x1 = h_t = h_all[t+1].
    const int nsteps = BWD ? T - 1 : T;
    auto load_epi = [&](int s, float (&x0)[NTW][4], float (&x1)[NTW][4]) {
        const int sc = min(s, nsteps - 1);
        const int t = BWD ? T - 2 - sc : sc;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int col = min((wave * NTW + nt) * 16 + nn, H - 1);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = min(b0 + 4 * g + i, B - 1);
                const size_t e = (size_t)t * bh + (size_t)row * H + col;
                if (!BWD) {
                    x0[nt][i] = a.U[e];
                } else {
                    x0[nt][i] = a.G[e];
                    x1[nt][i] = a.h_all[e + bh];
                }
            }
        }
    };
    float n0[NTW][4], n1[NTW][4];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int i = 0; i < 4; ++i) { n0[nt][i] = 0.f; n1[nt][i] = 0.f; }
    if (nsteps > 0) load_epi(0, n0, n1);

    auto product = [&](int cur, f32x4 (&acc)[NTW]) {
        float areg[KS];
        const float4* src = reinterpret_cast<const float4*>(&hs[cur][nn][KS * g]);
#pragma unroll
        for (int i = 0; i < KS / 4; ++i) {
            const float4 v = src[i];
            areg[4 * i] = v.x; areg[4 * i + 1] = v.y; areg[4 * i + 2] = v.z; areg[4 * i + 3] = v.w;
        }
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) acc[nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt)
                acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(areg[s], breg[nt][s], acc[nt], 0, 0, 0);
    };

    int cur = 0;
    for (int s = 0; s < nsteps; ++s) {
        float c0[NTW][4], c1[NTW][4];
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
            for (int i = 0; i < 4; ++i) { c0[nt][i] = n0[nt][i]; c1[nt][i] = n1[nt][i]; }
        if (s + 1 < nsteps) load_epi(s + 1, n0, n1);   // one step ahead

        f32x4 acc[NTW];
        product(cur, acc);

        const int t = BWD ? T - 2 - s : s;
        float* out = BWD ? a.Delta + (size_t)t * bh
                         : a.hist + (size_t)(a.ring ? ((s + 1) & 1) : (s + 1)) * bh;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int col = (wave * NTW + nt) * 16 + nn;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int m = 4 * g + i, row = b0 + m;
                if (col < H && row < B) {
                    const float v = BWD ? (acc[nt][i] + c0[nt][i]) * act_grad<ACT>(c1[nt][i])
                                        : activate<ACT>(acc[nt][i] + c0[nt][i]);
                    out[(size_t)row * H + col] = v;
                    hs[cur ^ 1][m][col] = v;
                }
            }
        }
        lds_barrier();
        cur ^= 1;
    }
    __syncthreads();

    if (!BWD) {
        if (a.h_last)
            for (int i = tid; i < kRows * H; i += kThreads) {
                const int m = i / H, j = i - m * H;
                if (b0 + m < B) a.h_last[(size_t)(b0 + m) * H + j] = hs[cur][m][j];
            }
        return;
    }
    if (a.dh0) {  // dh0 = delta_0 Wh: one more product, no epilogue
        f32x4 acc[NTW];
        product(cur, acc);
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int col = (wave * NTW + nt) * 16 + nn;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = b0 + 4 * g + i;
                if (col < H && row < B) a.dh0[(size_t)row * H + col] = acc[nt][i];
            }
        }
    }
}

// U[n][j] = Wx[x[n]][j] + b[j]: the input term of every step, gathered once outside the loop
__global__ __launch_bounds__(256) void gather_input_kernel(const int32_t* __restrict__ x,
                                                           const float* __restrict__ Wx,
                                                           const float* __restrict__ b,
                                                           float* __restrict__ U, int N, int H) {
    const int n = blockIdx.x;
    const float* row = Wx + (size_t)x[n] * H;
    for (int j = threadIdx.x; j < H; j += blockDim.x) U[(size_t)n * H + j] = row[j] + b[j];
}

template <int ACT, bool BWD>
hipError_t launch_hp(const RecMfmaArgs& a, hipStream_t s) {
    dim3 grid((a.B + kRows - 1) / kRows), block(kThreads);
    if (a.H <= 64) hipLaunchKernelGGL((rec_batch_mfma_kernel<ACT, BWD, 64>), grid, block, 0, s, a);
    else if (a.H <= 128) hipLaunchKernelGGL((rec_batch_mfma_kernel<ACT, BWD, 128>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((rec_batch_mfma_kernel<ACT, BWD, 256>), grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace

bool rec_batch_mfma_supported(int H, int B) { return H <= 256 && B > 4; }

hipError_t launch_gather_input(const int32_t* x, const float* Wx, const float* b, float* U, int N,
                               int H, hipStream_t s) {
    ProfileScope ps(K_MISC, s);
    hipLaunchKernelGGL(gather_input_kernel, dim3(N), dim3(256), 0, s, x, Wx, b, U, N, H);
    return hipGetLastError();
}

hipError_t launch_rec_batch_mfma(const RecMfmaArgs& a, bool bwd, hipStream_t s) {
    if (!rec_batch_mfma_supported(a.H, a.B)) return hipErrorInvalidValue;
    ProfileScope ps(bwd ? K_REC_BWD : K_REC_FWD, s);
    if (!bwd) return a.act == 0 ? launch_hp<0, false>(a, s) : launch_hp<1, false>(a, s);
    return a.act == 0 ? launch_hp<0, true>(a, s) : launch_hp<1, true>(a, s);
}

}  // namespace rnn
