// Persistent batched time loop on the matrix cores with the recurrent matrix resident in
// registers (hidden size <= 256, batch > 4).
//
// Batch rows are independent, so the batch is cut into tiles of 4 rows and every tile gets its
// own workgroup that never talks to another one: no device-wide synchronisation exists in this
// kernel, a step costs one LDS-only workgroup barrier.  The state tile (4 x H) lives in LDS,
// double buffered; the weights (Wh^T forward, Wh reverse) stay in registers for the whole
// launch as B operands of v_mfma_f32_4x4x1_16b_f32.  That instruction computes 16 independent
// 4x4 outer products per issue at the same flop rate as the larger shapes, so a tile of only 4
// batch rows already runs a SIMD at its full fp32 matrix rate, and a batch of 128 spreads over
// 32 compute units instead of the 8 that 16-row tiles would fill.
//
// The per-step epilogue (input term + activation, or output-layer term times the activation
// derivative) is fused, its operands are requested two steps ahead, and the new state goes to
// both the history in HBM and the other LDS buffer (the paper's Scan keeps every state for
// the gradient loop: property 1; nothing per step happens on the host: properties 4 and 5).
//
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

#include <type_traits>

namespace rnn {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Lane layout.  A wavefront owns 32 output columns.  Lane l = 32*hf + 4*blk + i (hf 0..1, blk 0..7, i 0..3):
// blocks blk and 8+blk both produce columns 4*blk .. 4*blk+3 of the 32, for two different k, so
// lane l supplies the B value M[k_hf][col0 + l%32] and receives, in accumulator register r, the
// partial sum over its half's k of row r at that column; the two halves are added with
// v_permlane32_swap, after which the lower lanes hold rows 0,1 and the upper lanes rows 2,3.
// Every block needs the A values h[i][k]; instead of loading each into all blocks, an A register
// holds 16 different k (k = 64q + 32*hf + 4*blk + e in register 4q+e, one 16-byte LDS read per
// q) and the instruction's broadcast field (cbsz = 3: each group of 8 blocks takes A from its
// block abid) selects k = 64q + 32*hf + 4*abid + e.  A lane's weights are HP/2 registers,
// resident for the whole launch; a workgroup is HP/32 wavefronts, two per SIMD at HP = 256.
template <int ACT, bool BWD, int HP>
__global__ __launch_bounds__(2 * HP) void rec_batch_mfma_kernel(RecMfmaArgs a) {
    constexpr int NQ = HP / 64;    // 16-byte A reads per lane and step
    constexpr int LDH = HP + 16;   // LDS row stride: the 4 rows of a read land 16 banks apart
    constexpr int NT = 2 * HP;     // threads
    constexpr int R4 = 4;          // batch rows per workgroup
    __shared__ __attribute__((aligned(16))) float hs[2][R4][LDH];

    const int H = a.H, B = a.B, T = a.T;
    const int tid = threadIdx.x, lane = tid % kWave, wave = tid / kWave;
    const int hf = lane / 32, blk = (lane % 32) / 4, ri = lane % 4;
    const int col = wave * 32 + lane % 32, colc = min(col, H - 1);
    const int b0 = blockIdx.x * R4;
    const size_t bh = (size_t)B * H;

    // ---- resident weights: wreg[(8q+b)*4+e] = M[k][col], k = 64q + 32hf + 4b + e,
    //      M = Wh^T (forward) or Wh (reverse) ------------------------------------------------
    float wreg[HP / 2];
#pragma unroll
    for (int j = 0; j < HP / 2; ++j) {
        const int k = 64 * (j / 32) + 32 * hf + (j % 32);
        const int kc = min(k, H - 1);
        wreg[j] = BWD ? a.Wh[(size_t)kc * H + colc] : a.Wh[(size_t)colc * H + kc];
    }
    // Zero the padding in a second pass, by multiplication: a select would make every load
    // above conditional and serialise them behind a wait each.
    const float colmask = col < H ? 1.f : 0.f;
#pragma unroll
    for (int j = 0; j < HP / 2; ++j) {
        const int k = 64 * (j / 32) + 32 * hf + (j % 32);
        wreg[j] *= k < H ? colmask : 0.f;
    }

    // ---- initial state tile ------------------------------------------------------------------
    for (int i = tid; i < 2 * R4 * LDH; i += NT) (&hs[0][0][0])[i] = 0.f;
    __syncthreads();
    for (int i = tid; i < R4 * HP; i += NT) {
        const int m = i / HP, j = i % HP, row = b0 + m;
        if (row >= B || j >= H) continue;
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

    // Epilogue operands (rows 2hf, 2hf+1 of this lane's column), requested two steps ahead.
    // forward: x0 = input term U[s]; reverse (t = T-2-s): x0 = G[t], x1 = h_t = h_all[t+1].
    const int nsteps = BWD ? T - 1 : T;
    size_t rowoff[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) rowoff[i] = (size_t)min(b0 + 2 * hf + i, B - 1) * H + colc;
    auto load_epi = [&](int s, float (&x0)[2], float (&x1)[2]) {
        const int sc = max(min(s, nsteps - 1), 0);   // clamped: always a valid step to read
        const int t = BWD ? max(T - 2 - sc, 0) : sc;
        const size_t base = (size_t)t * bh;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            if (!BWD) {
                x0[i] = a.U[base + rowoff[i]];
            } else {
                x0[i] = a.G[base + rowoff[i]];
                x1[i] = a.h_all[base + bh + rowoff[i]];
            }
        }
    };
    float n0[2][2], n1[2][2];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int i = 0; i < 2; ++i) { n0[p][i] = 0.f; n1[p][i] = 0.f; }
    load_epi(0, n0[0], n1[0]);
    load_epi(1, n0[1], n1[1]);

    // out[i] = sum_k h[2hf+i][k] * M[k][col] from state buffer CUR
    auto product = [&](auto cur_c, float (&out)[2]) {
        constexpr int CUR = decltype(cur_c)::value;
        float areg[4 * NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const float4 v =
                *reinterpret_cast<const float4*>(&hs[CUR][ri][64 * q + 32 * hf + 4 * blk]);
            areg[4 * q] = v.x; areg[4 * q + 1] = v.y; areg[4 * q + 2] = v.z; areg[4 * q + 3] = v.w;
        }
        f32x4 acc[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
#define RNN_MFMA4_BLOCK(Q, AB)                                                                   \
    _Pragma("unroll") for (int e = 0; e < 4; ++e)                                                \
        acc[e] = __builtin_amdgcn_mfma_f32_4x4x1f32(areg[4 * (Q) + e],                           \
                                                    wreg[(8 * (Q) + (AB)) * 4 + e], acc[e], 3,   \
                                                    (AB), 0);
#define RNN_MFMA4_Q(Q)                                                                           \
    RNN_MFMA4_BLOCK(Q, 0) RNN_MFMA4_BLOCK(Q, 1) RNN_MFMA4_BLOCK(Q, 2) RNN_MFMA4_BLOCK(Q, 3)      \
    RNN_MFMA4_BLOCK(Q, 4) RNN_MFMA4_BLOCK(Q, 5) RNN_MFMA4_BLOCK(Q, 6) RNN_MFMA4_BLOCK(Q, 7)
        RNN_MFMA4_Q(0)
        if constexpr (NQ > 1) { RNN_MFMA4_Q(1) }
        if constexpr (NQ > 2) { RNN_MFMA4_Q(2) RNN_MFMA4_Q(3) }
#undef RNN_MFMA4_Q
#undef RNN_MFMA4_BLOCK
        const f32x4 part = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        // add the two k halves: rows 0,2 in one swap, rows 1,3 in the other
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(part[i]),
                                                            __float_as_uint(part[i + 2]), false,
                                                            false);
            out[i] = __uint_as_float(r[0]) + __uint_as_float(r[1]);
        }
    };

    auto step = [&](int s, auto slot_c) {
        constexpr int SLOT = decltype(slot_c)::value;   // s & 1: state buffer and operand slot
        float acc[2];
        product(slot_c, acc);

        const int t = BWD ? T - 2 - s : s;
        float* out = BWD ? a.Delta + (size_t)t * bh
                         : a.hist + (size_t)(a.ring ? ((s + 1) & 1) : (s + 1)) * bh;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = 2 * hf + i;
            const float v = BWD ? (acc[i] + n0[SLOT][i]) * act_grad<ACT>(n1[SLOT][i])
                                : activate<ACT>(acc[i] + n0[SLOT][i]);
            if (col < H) {
                hs[SLOT ^ 1][m][col] = v;
                if (b0 + m < B) out[(size_t)(b0 + m) * H + col] = v;
            }
        }
        // The slot is free again: request the operands of step s + 2 into the same registers.
        // Unconditional (the step index is clamped) so that the wait counts stay exact.
        load_epi(s + 2, n0[SLOT], n1[SLOT]);
        lds_barrier();
    };

    // pairs of steps with no branch between them (exact wait counts), then the odd one out
    int s2 = 0;
    for (; s2 + 1 < nsteps; s2 += 2) {
        step(s2, std::integral_constant<int, 0>{});
        step(s2 + 1, std::integral_constant<int, 1>{});
    }
    if (s2 < nsteps) step(s2, std::integral_constant<int, 0>{});
    __syncthreads();
    const int cur = nsteps > 0 ? (nsteps & 1) : 0;

    if (!BWD) {
        if (a.h_last)
            for (int i = tid; i < R4 * HP; i += NT) {
                const int m = i / HP, j = i % HP;
                if (b0 + m < B && j < H) a.h_last[(size_t)(b0 + m) * H + j] = hs[cur][m][j];
            }
        return;
    }
    if (a.dh0) {  // dh0 = delta_0 Wh: one more product, no epilogue
        float acc[2];
        if (cur == 0) product(std::integral_constant<int, 0>{}, acc);
        else product(std::integral_constant<int, 1>{}, acc);
        if (col < H)
#pragma unroll
            for (int i = 0; i < 2; ++i)
                if (b0 + 2 * hf + i < B) a.dh0[(size_t)(b0 + 2 * hf + i) * H + col] = acc[i];
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
    dim3 grid((a.B + 3) / 4);
    if (a.H <= 64) hipLaunchKernelGGL((rec_batch_mfma_kernel<ACT, BWD, 64>), grid, dim3(128), 0, s, a);
    else if (a.H <= 128) hipLaunchKernelGGL((rec_batch_mfma_kernel<ACT, BWD, 128>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((rec_batch_mfma_kernel<ACT, BWD, 256>), grid, dim3(512), 0, s, a);
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
