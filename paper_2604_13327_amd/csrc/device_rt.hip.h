// Device-side event-tensor runtime (paper Sec. 3.3): an event tensor is an int32 array in HBM;
// notify = device-scope atomic decrement, wait = wavefront-level spin until zero with bounded
// backoff.  Plus small numeric helpers shared by the task bodies.
#pragma once
#include <hip/hip_runtime.h>

#include "etc_types.h"

namespace etc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);      // round to nearest even (inputs are finite)
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    return (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ int ev_peek(const int32_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Records the first error; later waits see it and give up at once, so the kernel always drains.
__device__ __forceinline__ void raise_error(const Params &P, int code, int fn, int ev)
{
    int expected = 0;
    if (__hip_atomic_compare_exchange_strong(P.error_word, &expected, code, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT)) {
        __hip_atomic_store(P.error_word + 1, fn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(P.error_word + 2, ev, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(P.error_word + 3, (int)blockIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// E[ev].wait() for one wavefront: lane 0 polls, backing off with s_sleep; every lane then passes an
// acquire fence so that loads issued after the wait observe what the notifying tasks wrote.
// Returns false when the spin budget ran out or another wave already raised an error.
__device__ __forceinline__ bool wave_wait(const Params &P, int ev, int fn)
{
    int ok = 1;
    if (ev >= 0) {
        if (lane_id() == 0) {
            const int32_t *p = P.ev_cur + ev;
            long long spins = 0;
            while (ev_peek(p) > 0) {
                if (spins < 64) __builtin_amdgcn_s_sleep(1); else __builtin_amdgcn_s_sleep(8);
                ++spins;
                if ((spins & 255) == 0 && ev_peek(P.error_word) != 0) { ok = 0; break; }
                if (spins > P.spin_budget) { raise_error(P, ERR_WAIT_TIMEOUT, fn, ev); ok = 0; break; }
            }
        }
        ok = __builtin_amdgcn_readfirstlane(ok);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    return ok != 0;
}

// Makes the calling workgroup's global stores visible device-wide; call before notifying.
// Every thread drains its own stores, the barrier collects the workgroup, thread 0 publishes.
__device__ __forceinline__ void wg_release()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
}

// E[ev].notify(): returns the value before the decrement (1 means this call fired the event).
__device__ __forceinline__ int ev_notify(const Params &P, int ev)
{
    return __hip_atomic_fetch_sub(P.ev_cur + ev, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

}  // namespace etc
