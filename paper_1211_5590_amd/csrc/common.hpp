// Device-side helpers shared by the gfx950 kernels of the Elman-RNN training path.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rnn {

constexpr int kWave = 64;  // CDNA wavefront width

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

__device__ __forceinline__ float sigmoidf_fast(float a) {
    // 1/(1+e^-a); e^-a overflows to +inf for a < -88 and the reciprocal then gives 0.
    return fast_rcp(1.0f + __expf(-a));
}

__device__ __forceinline__ float tanhf_fast(float a) {
    // sign(a) (1-t)/(1+t) with t = e^{-2|a|} in (0,1]: no overflow for any a.
    const float t = __expf(-2.0f * fabsf(a));
    const float r = (1.0f - t) * fast_rcp(1.0f + t);
    return copysignf(r, a);
}

template <int ACT>
__device__ __forceinline__ float activate(float a) {
    return ACT == 0 ? sigmoidf_fast(a) : tanhf_fast(a);
}

// derivative of the activation expressed through its output h
template <int ACT>
__device__ __forceinline__ float act_grad(float h) {
    return ACT == 0 ? h * (1.0f - h) : 1.0f - h * h;
}

// merge two (max, sum of exp relative to max) pairs of a log-sum-exp
__device__ __forceinline__ void lse_merge(float& m, float& s, float m2, float s2) {
    const float mn = fmaxf(m, m2);
    // a pair with s == 0 carries m = -inf; guard the -inf - -inf case
    const float a = (m == mn) ? s : s * __expf(m - mn);
    const float b = (m2 == mn) ? s2 : s2 * __expf(m2 - mn);
    m = mn;
    s = a + b;
}

// ---------------------------------------------------------------------------------------
// Self-validating words for exchanges between workgroups of one launch.  A 32-bit value
// travels with a 32-bit tag in one naturally aligned 64-bit word that is written and read with
// relaxed device-scope atomics, so a reader that sees the expected tag has the value that was
// written with it: no separate flag, no fence, one memory round trip.  A tag is never 0
// (cleared memory) and is unique to the launch or step that writes it.
__device__ __forceinline__ void tagged_store(unsigned long long* p, unsigned tag, float v) {
    __hip_atomic_store(p, ((unsigned long long)tag << 32) | (unsigned long long)__float_as_uint(v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long tagged_load(const unsigned long long* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool tagged_ok(unsigned long long w, unsigned tag) {
    return (unsigned)(w >> 32) == tag;
}
__device__ __forceinline__ float tagged_value(unsigned long long w) {
    return __uint_as_float((unsigned)w);
}
// polls until the tag shows up; false when the bounded wait expires
__device__ __forceinline__ bool tagged_wait(const unsigned long long* p, unsigned tag, int spin_limit,
                                            float& v) {
    unsigned long long w = tagged_load(p);
    for (int spins = 0; !tagged_ok(w, tag); ++spins) {
        if (spins > spin_limit) return false;
        w = tagged_load(p);
    }
    v = tagged_value(w);
    return true;
}

}  // namespace rnn
