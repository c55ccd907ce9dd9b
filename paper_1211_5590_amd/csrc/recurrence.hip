// Persistent time-loop kernels with the recurrent matrix resident on chip (batch 1 .. 4).
//
// The paper's Scan runs its loop as one graph node whose per-step bookkeeping is done in
// compiled code, keeps every state for the gradient loop, and hoists everything that does not
// depend on the previous state out of the loop (Scan properties 1, 5, 8).  Here one launch
// runs all T steps; what stays inside the loop is only the product of Wh (forward) or Wh^T
// (reverse) with the previous state, a fused bias/activation (or activation-derivative)
// epilogue, and the store of the new state.
//
// Work split: P workgroups per batch row, each holding R = ceil(H/P) rows of the matrix in LDS
// for the whole launch (loaded once).  A row's dot product is shared by L lanes that read the
// row and the state vector as float4 and combine with wavefront shuffles.  P = 1: the state
// lives in LDS and a step costs one workgroup barrier.  P > 1: every workgroup stores its
// slice of the new state to global memory, publishes a per-workgroup step counter with
// release semantics, waits (bounded) for the other P-1 counters, and re-reads the full vector.
// The launch is cooperative, so all P*B workgroups are co-resident; a wait that exceeds its
// spin limit sets the status word and makes the whole workgroup leave, so every wavefront
// terminates whatever happens.
#include "common.hpp"
#include "internal.hpp"
#include "prof.hpp"

namespace rnn {
namespace {

constexpr int kThreads = 512;

template <int ACT, bool BWD>
__global__ __launch_bounds__(kThreads) void rec_resident_kernel(RecResArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ int s_abort;
    const int H = a.H, P = a.P, R = a.R, ldw = a.ldw, L = a.L, B = a.B, T = a.T;
    const int p = blockIdx.x, bb = blockIdx.y;
    const int tid = threadIdx.x;
    const int r0 = p * R;
    const int rows = max(0, min(R, H - r0));
    const int H4 = (H + 3) / 4, Hp = H4 * 4;
    float* W = smem;                       // [R][ldw], zero padded
    float* vbuf = smem + a.w_floats;       // [2][Hp], zero padded
    const int q = tid % L, grp = tid / L, ngrp = kThreads / L;

    if (tid == 0) s_abort = 0;
    for (int i = tid; i < R * ldw; i += kThreads) W[i] = 0.f;
    for (int i = tid; i < 2 * Hp; i += kThreads) vbuf[i] = 0.f;
    __syncthreads();
    if (!BWD) {
        for (int i = tid; i < rows * H; i += kThreads) {
            const int r = i / H, k = i - r * H;
            W[r * ldw + k] = a.Wh[(size_t)(r0 + r) * H + k];
        }
    } else {  // rows of Wh^T: W[r][k] = Wh[k][r0 + r]
        for (int i = tid; i < rows * H; i += kThreads) {
            const int k = i / rows, r = i - k * rows;
            W[r * ldw + k] = a.Wh[(size_t)k * H + r0 + r];
        }
    }

    // sum of the per-strip partial G (fixed strip order) when the output layer ran column-split
    if (BWD && a.gpart) {
        const int n = T * B * H;
        for (int e = tid; e < n; e += kThreads) {
            float g = 0.f;
#pragma unroll 8
            for (int sidx = 0; sidx < a.gstrips; ++sidx) g += a.gpart[(size_t)sidx * n + e];
            a.Gw[e] = g;
        }
        __syncthreads();
    }

    // ---- initial vector ------------------------------------------------------------------
    // forward: h_{-1} = h0 (or zeros), also stored as slot 0 of the history.
    // reverse: delta_{T-1} = (G_{T-1} + dh_last) * act'(h_{T-1}), stored as Delta[T-1].
    if (!BWD) {
        for (int j = tid; j < H; j += kThreads) {
            const float v = a.h0 ? a.h0[(size_t)bb * H + j] : 0.f;
            vbuf[j] = v;
            if (j >= r0 && j < r0 + rows) a.hist[(size_t)bb * H + j] = v;
        }
    } else {
        const size_t row = ((size_t)(T - 1) * B + bb) * H;
        const float* ht = a.h_all + ((size_t)T * B + bb) * H;
        for (int j = tid; j < H; j += kThreads) {
            const float c = a.dh_last ? a.dh_last[(size_t)bb * H + j] : 0.f;
            const float d = (a.G[row + j] + c) * act_grad<ACT>(ht[j]);
            vbuf[j] = d;
            if (j >= r0 && j < r0 + rows) a.Delta[row + j] = d;
        }
    }
    __syncthreads();

    // Steps.  forward: s = 0..T-1 computes h_s from h_{s-1}.  reverse: s = 0..T-2 computes
    // delta_t for t = T-2-s from delta_{t+1}.
    const int nsteps = BWD ? T - 1 : T;
    int cur = 0;
    // first-row operands of the epilogue are fetched one step ahead (latency off the chain)
    const bool lead = (q == 0) && grp < rows;
    float pre0 = 0.f, pre1 = 0.f;  // fwd: input term; bwd: G_t and h_t
    auto fetch = [&](int s, int j, float& x0, float& x1) {
        if (!BWD) {
            const size_t n = (size_t)s * B + bb;
            x0 = a.U ? a.U[n * H + j] : a.Wx[(size_t)a.x[n] * H + j] + a.b[j];
            x1 = 0.f;
        } else {
            const int t = T - 2 - s;
            x0 = a.G[((size_t)t * B + bb) * H + j];
            x1 = a.h_all[((size_t)(t + 1) * B + bb) * H + j];
        }
    };
    if (lead && nsteps > 0) fetch(0, r0 + grp, pre0, pre1);

    for (int s = 0; s < nsteps; ++s) {
        const float c0 = pre0, c1 = pre1;
        if (lead && s + 1 < nsteps) fetch(s + 1, r0 + grp, pre0, pre1);
        const float4* v4 = reinterpret_cast<const float4*>(vbuf + cur * Hp);
        float* vnext = vbuf + (cur ^ 1) * Hp;
        const int t = BWD ? T - 2 - s : s;
        float* out_row = BWD ? a.Delta + ((size_t)t * B + bb) * H
                             : a.hist + ((size_t)(a.ring ? ((s + 1) & 1) : (s + 1)) * B + bb) * H;
        for (int row = grp; row < rows; row += ngrp) {
            const float4* w4 = reinterpret_cast<const float4*>(W + row * ldw);
            float acc = 0.f;
            for (int c = q; c < H4; c += L) {
                const float4 w = w4[c], x = v4[c];
                acc = fmaf(w.x, x.x, acc);
                acc = fmaf(w.y, x.y, acc);
                acc = fmaf(w.z, x.z, acc);
                acc = fmaf(w.w, x.w, acc);
            }
            for (int off = L >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
            if (q == 0) {
                const int j = r0 + row;
                float x0 = c0, x1 = c1;
                if (row != grp) fetch(s, j, x0, x1);
                const float v = BWD ? (x0 + acc) * act_grad<ACT>(x1) : activate<ACT>(acc + x0);
                out_row[j] = v;
                vnext[j] = v;
            }
        }
        if (P > 1) {
            const int step = s + 1;
            __threadfence();
            __syncthreads();
            int32_t* fl = a.flags + (size_t)bb * P;
            if (tid == 0) __hip_atomic_store(fl + p, step, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
            if (tid < P) {
                int spins = 0;
                while (__hip_atomic_load(fl + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < step) {
                    if (++spins > a.spin_limit) { s_abort = 1; break; }
                    __builtin_amdgcn_s_sleep(1);
                }
            }
            __syncthreads();
            if (s_abort) {
                if (tid == 0) atomicExch(a.status, 1);
                return;  // uniform: the whole workgroup leaves
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            for (int j = tid; j < H; j += kThreads) vnext[j] = out_row[j];
        }
        __syncthreads();
        cur ^= 1;
    }

    const float* vfin = vbuf + cur * Hp;
    if (!BWD) {
        if (a.h_last)
            for (int j = r0 + tid; j < r0 + rows; j += kThreads) a.h_last[(size_t)bb * H + j] = vfin[j];
        return;
    }
    if (a.dh0) {  // dh0 = Wh^T delta_0
        const float4* v4 = reinterpret_cast<const float4*>(vfin);
        for (int row = grp; row < rows; row += ngrp) {
            const float4* w4 = reinterpret_cast<const float4*>(W + row * ldw);
            float acc = 0.f;
            for (int c = q; c < H4; c += L) {
                const float4 w = w4[c], x = v4[c];
                acc = fmaf(w.x, x.x, acc);
                acc = fmaf(w.y, x.y, acc);
                acc = fmaf(w.z, x.z, acc);
                acc = fmaf(w.w, x.w, acc);
            }
            for (int off = L >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, kWave);
            if (q == 0) a.dh0[(size_t)bb * H + r0 + row] = acc;
        }
    }
    if (!a.fuse_post) return;

    // ---- fused weight gradients for a short single sequence (P == 1, B == 1) -----------------
    // dWh = sum_t delta_t (x) h_{t-1},  db = sum_t delta_t,  dWx rows by token id.
    __syncthreads();               // everyone is done with W and vbuf
    float* D = smem;               // [T][H] delta rows
    float* Hprev = smem + T * H;   // [T][H] h_{t-1} rows
    for (int i = tid; i < T * H; i += kThreads) {
        D[i] = a.Delta[i];
        Hprev[i] = a.h_all[i];
    }
    __syncthreads();
    for (int j = tid; j < H; j += kThreads) {
        float sum = 0.f;
        for (int t = 0; t < T; ++t) sum += D[t * H + j];
        a.db[j] = a.beta ? a.db[j] + sum : sum;
    }
    for (int e = tid; e < H * H; e += kThreads) {
        const int j = e / H, i = e - j * H;
        float sum = 0.f;
        for (int t = 0; t < T; ++t) sum = fmaf(D[t * H + j], Hprev[t * H + i], sum);
        a.dWh[e] = a.beta ? a.dWh[e] + sum : sum;
    }
    // token rows: the first occurrence of an id sums all its steps in ascending order
    for (int t = 0; t < T; ++t) {
        const int id = a.x[t];
        bool first = true;
        for (int u = 0; u < t; ++u) first = first && (a.x[u] != id);
        if (!first) continue;      // uniform across the workgroup
        for (int j = tid; j < H; j += kThreads) {
            float sum = 0.f;
            for (int u = t; u < T; ++u)
                if (a.x[u] == id) sum += D[u * H + j];
            float* dst = a.dWx + (size_t)id * H + j;
            *dst = a.beta ? *dst + sum : sum;
        }
    }
}

__global__ void zero_words_kernel(int32_t* p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0;
}

template <typename K>
hipError_t allow_lds(K kernel, size_t bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

int pow2_floor(int v) {
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}

}  // namespace

hipError_t launch_zero_words(int32_t* p, int n, hipStream_t s) {
    ProfileScope ps(K_MISC, s);
    hipLaunchKernelGGL(zero_words_kernel, dim3(1), dim3(256), 0, s, p, n);
    return hipGetLastError();
}

bool rec_resident_plan(int H, int B, int T, bool fuse_post, RecResPlan* out) {
    if (B > 4 || H > 4096) return false;
    constexpr size_t kLdsBudget = 150 * 1024;  // of 160 KB per CU
    const int Hp = (H + 3) / 4 * 4;
    for (int P = 1; P <= 128; P *= 2) {
        if (P * B > 128) break;
        const int R = (H + P - 1) / P;
        int L = pow2_floor(kThreads / R);
        if (L < 1) L = 1;
        if (L > 64) L = 64;
        int ldw = Hp;
        if (L < 8) while (ldw % 32 != (4 * L) % 32) ldw += 4;
        size_t w_floats = (size_t)R * ldw;
        if (fuse_post && P == 1 && (size_t)2 * T * H > w_floats) w_floats = (size_t)2 * T * H;
        w_floats = (w_floats + 3) / 4 * 4;  // keeps the state vectors 16-byte aligned
        const size_t bytes = (w_floats + 2 * (size_t)Hp) * 4;
        if (bytes <= kLdsBudget) {
            out->P = P; out->R = R; out->L = L; out->ldw = ldw;
            out->w_floats = (int)w_floats; out->smem = bytes;
            return true;
        }
        if (fuse_post) return false;  // the fused tail needs the single-workgroup form
    }
    return false;
}

hipError_t launch_rec_resident(RecResArgs a, const RecResPlan& pl, bool bwd, hipStream_t s) {
    a.P = pl.P; a.R = pl.R; a.L = pl.L; a.ldw = pl.ldw; a.w_floats = pl.w_floats;
    if (a.spin_limit <= 0) a.spin_limit = 1 << 22;
    if (pl.P > 1) {
        hipError_t e = launch_zero_words(a.flags, pl.P * a.B, s);
        if (e != hipSuccess) return e;
    }
    const void* fn;
    if (!bwd) fn = a.act == 0 ? (const void*)rec_resident_kernel<0, false> : (const void*)rec_resident_kernel<1, false>;
    else fn = a.act == 0 ? (const void*)rec_resident_kernel<0, true> : (const void*)rec_resident_kernel<1, true>;
    static size_t allowed[4] = {0, 0, 0, 0};
    const int slot = (bwd ? 2 : 0) + (a.act == 0 ? 0 : 1);
    if (pl.smem > 64 * 1024 && pl.smem > allowed[slot]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.smem);
        if (e != hipSuccess) return e;
        allowed[slot] = pl.smem;
    }
    ProfileScope ps(bwd ? K_REC_BWD : K_REC_FWD, s);
    dim3 grid(pl.P, a.B), block(kThreads);
    if (pl.P > 1) {
        void* args[] = {&a};
        return hipLaunchCooperativeKernel(fn, grid, block, args, (unsigned)pl.smem, s);
    }
    if (!bwd) {
        if (a.act == 0) hipLaunchKernelGGL((rec_resident_kernel<0, false>), grid, block, pl.smem, s, a);
        else hipLaunchKernelGGL((rec_resident_kernel<1, false>), grid, block, pl.smem, s, a);
    } else {
        if (a.act == 0) hipLaunchKernelGGL((rec_resident_kernel<0, true>), grid, block, pl.smem, s, a);
        else hipLaunchKernelGGL((rec_resident_kernel<1, true>), grid, block, pl.smem, s, a);
    }
    return hipGetLastError();
}

}  // namespace rnn
