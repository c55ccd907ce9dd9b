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

// Workgroup barrier that waits for this wavefront's LDS traffic only.  __syncthreads() also waits
// for every outstanding global access (vmcnt(0)), which would expose the full memory latency of
// requests that were issued on purpose several iterations ahead of their use.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Four consecutive 16-byte aligned LDS words, read with an LDS instruction and waited for through the
// LDS counter alone.  A volatile read through an ordinary pointer becomes a flat load, whose wait is
// vmcnt(0): a spin on an LDS flag would then also wait for every global store and prefetch in flight.
__device__ __forceinline__ int4 lds_peek4(const int* p) {
    int4 v;
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"((unsigned)(size_t)p) : "memory");
    return v;
}

template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
// Butterfly stages of a wavefront reduction without LDS traffic.  Stages 1 and 2 permute within
// quads, 4 and 8 mirror within 8 and 16 lanes (equivalent to xor once the smaller stages have
// run), 16 and 32 swap rows / halves of two registers.
__device__ __forceinline__ float sum4(float v) { v += dpp<0xB1>(v); v += dpp<0x4E>(v); return v; }
__device__ __forceinline__ float sum16(float v) { v = sum4(v); v += dpp<0x141>(v); v += dpp<0x140>(v); return v; }
__device__ __forceinline__ float swap16_sum(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float swap32_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float sum32(float v) { return swap16_sum(sum16(v)); }
__device__ __forceinline__ float sum64(float v) { return swap32_sum(sum32(v)); }
__device__ __forceinline__ float max64(float v) {
    v = fmaxf(v, dpp<0xB1>(v)); v = fmaxf(v, dpp<0x4E>(v));
    v = fmaxf(v, dpp<0x141>(v)); v = fmaxf(v, dpp<0x140>(v));
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float max16(float v) {
    v = fmaxf(v, dpp<0xB1>(v)); v = fmaxf(v, dpp<0x4E>(v));
    v = fmaxf(v, dpp<0x141>(v)); v = fmaxf(v, dpp<0x140>(v));
    return v;
}
__device__ __forceinline__ float max32(float v) {
    v = max16(v);
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
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
// Tags of consecutive launches on one set of boxes are device state: a word next to the boxes holds
// the tag the previous launch used; every workgroup of a launch reads it on entry, uses the next
// tag, and one workgroup that can only finish after all the others have started stores the new
// value at its end.  (A tag drawn on the host would be baked into the launch's arguments, and a
// replayed HIP graph would then meet its own tag in the words its previous replay left behind.)
__device__ __forceinline__ unsigned next_tag(unsigned previous) {
    const unsigned t = previous + 1u;
    return t ? t : 1u;           // 0 is what cleared memory holds: never a tag
}
__device__ __forceinline__ unsigned tag_word_load(const unsigned* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void tag_word_store(unsigned* p, unsigned tag) {
    __hip_atomic_store(p, tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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


// Every requested word is "used" here, also the clamped duplicates a batch requests past the end
// of its range: a load whose result is never read stays pending in the compiler's bookkeeping,
// and the wait it later inserts before reusing the register (in some unrelated loop) would also
// wait for every store issued since.
__device__ __forceinline__ void consume(unsigned long long v) { asm volatile("" ::"v"(v)); }
__device__ __forceinline__ void consume(float v) { asm volatile("" ::"v"(v)); }

// Waits for N tagged words at once (act[u] false marks an unused slot).  All stale words are
// requested again together, so words that arrive while the batch is being polled cost one more
// round trip in total, not one each.  Returns false when the bounded wait expires.
template <int N>
__device__ __forceinline__ bool wait_n(const unsigned long long* const (&ptr)[N], const bool (&act)[N],
                                       unsigned tag, int spin_limit, unsigned long long (&w)[N]) {
#pragma unroll
    for (int u = 0; u < N; ++u) w[u] = tagged_load(ptr[u]);
    bool ok = true;
    for (int spins = 0;; ++spins) {
        bool stale = false;
#pragma unroll
        for (int u = 0; u < N; ++u) stale = stale || (act[u] && !tagged_ok(w[u], tag));
        if (!stale) break;
        if (spins > spin_limit) { ok = false; break; }
        __builtin_amdgcn_s_sleep(1);   // a short pause keeps the pollers from crowding the memory pipeline
#pragma unroll
        for (int u = 0; u < N; ++u)
            if (act[u] && !tagged_ok(w[u], tag)) w[u] = tagged_load(ptr[u]);
    }
#pragma unroll
    for (int u = 0; u < N; ++u) consume(w[u]);
    return ok;
}
// four words base[idx[u]]; idx[u] < 0 marks an unused slot
__device__ __forceinline__ bool wait4(const unsigned long long* base, const long long (&idx)[4], unsigned tag,
                                      int spin_limit, unsigned long long (&w)[4]) {
    const unsigned long long* ptr[4];
    bool act[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) { act[u] = idx[u] >= 0; ptr[u] = base + (act[u] ? idx[u] : 0); }
    return wait_n<4>(ptr, act, tag, spin_limit, w);
}


}  // namespace rnn
