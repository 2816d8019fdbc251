// Cross-workgroup hand-over of scan aggregates through global memory (gfx950), shared by the scan
// kernels and by the projection GEMM that scans its own output tile.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssm {

__device__ __forceinline__ float2 cmul(float2 a, float2 b)
{
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
// a * b + c
__device__ __forceinline__ float2 cfma(float2 a, float2 b, float2 c)
{
    return make_float2(fmaf(a.x, b.x, fmaf(-a.y, b.y, c.x)), fmaf(a.x, b.y, fmaf(a.y, b.x, c.y)));
}

// Cross-workgroup hand-over without fences: every descriptor word is one 64-bit value that
// carries a float in its upper half and a tag in its lower half, written and read with relaxed
// device-scope atomics (write-through / cache-bypassing accesses).  A word whose tag is non-zero
// is complete by construction, so no ordering between different words is ever needed and no
// cache write-back or invalidate is paid.
//   tag 1: aggregate (state for zero incoming state), no reset among the workgroup's steps
//   tag 2: aggregate, a reset among the steps (the product of the transition is zero)
//   tag 3: inclusive state
__device__ __forceinline__ void publish_word(unsigned long long *w, float v, unsigned tag)
{
    __hip_atomic_store(w, ((unsigned long long)__float_as_uint(v) << 32) | tag, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long poll_word(const unsigned long long *w)
{
    return __hip_atomic_load(w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float word_value(unsigned long long w) { return __uint_as_float((unsigned)(w >> 32)); }
__device__ __forceinline__ unsigned word_tag(unsigned long long w) { return (unsigned)(w & 0xffffffffu); }

// Waits (bounded) until both words of a pair carry a tag >= min_tag.  Returns false on give-up.
__device__ __forceinline__ bool wait_pair(const unsigned long long *w, unsigned min_tag, unsigned spin_limit,
                                          float2 &value, unsigned &tag)
{
    unsigned spins = 0;
    while (true) {
        const unsigned long long w0 = poll_word(w), w1 = poll_word(w + 1);
        if (word_tag(w0) >= min_tag && word_tag(w1) >= min_tag) {
            value = make_float2(word_value(w0), word_value(w1));
            tag = word_tag(w0);
            return true;
        }
        if (spins >= spin_limit) return false;
        ++spins;
        __builtin_amdgcn_s_sleep(2);
    }
}

}  // namespace ssm
