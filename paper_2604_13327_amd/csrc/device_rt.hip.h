// Device-side event-tensor runtime (paper Sec. 3.3): an event tensor is an int32 array in HBM;
// notify = device-scope atomic decrement, wait = spin until zero with bounded backoff.
//
// Coherence design for MI355X.  The 8 XCDs have private L2 caches, and a device-scope release or
// acquire FENCE writes back / invalidates a whole L2: measured at 15-30 us per hop, far more than the
// work between two events.  So no such fence is ever executed here.  Instead every datum that
// crosses tasks inside a launch (activations, partial results, event counters, queue slots) is
// written with device-scope write-through stores and read with device-scope loads (relaxed atomics
// of 2, 4 or 8 bytes: the "sc1" forms), which bypass the non-coherent level.  Ordering is then just:
//   producer: all threads drain their stores (s_waitcnt), workgroup barrier, one atomic decrement;
//   consumer: poll the counter with device-scope loads, then issue its (device-scope) data loads.
// Weights and cached KV pages are read-only during a launch and use ordinary (cached, streaming) loads.
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

// v ~= hi + lo with hi, lo bf16: 16 mantissa bits survive, so bf16 MFMA operands lose ~2^-17 instead of 2^-9
__device__ __forceinline__ void split_bf16(float v, uint16_t &hi, uint16_t &lo)
{
    hi = f32_to_bf16_bits(v);
    lo = f32_to_bf16_bits(v - bf16_bits_to_f32(hi));
}

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// An argument of an out-of-line function arrives in vector registers, one copy per lane, even when every lane
// holds the same value (task records, tile descriptors, event ids): the function then computes addresses and
// branches per lane and runs out of vector registers.  This moves such a value back into scalar registers.
template <class T>
__device__ __forceinline__ T wave_uniform(const T &v)
{
    static_assert(sizeof(T) % 4 == 0, "whole 32-bit words");
    struct Words { uint32_t w[sizeof(T) / 4]; };
    Words a = __builtin_bit_cast(Words, v);
#pragma unroll
    for (unsigned i = 0; i < sizeof(T) / 4; ++i) a.w[i] = __builtin_amdgcn_readfirstlane(a.w[i]);
    return __builtin_bit_cast(T, a);
}

// A plain-data struct to and from LDS, word by word (a struct in LDS is not assignable as a whole).
template <class T>
__device__ __forceinline__ void lds_put(T *dst, const T &v)
{
    static_assert(sizeof(T) % 4 == 0, "whole 32-bit words");
    struct Words { uint32_t w[sizeof(T) / 4]; };
    const Words a = __builtin_bit_cast(Words, v);
    __attribute__((address_space(3))) uint32_t *d = (__attribute__((address_space(3))) uint32_t *)dst;
#pragma unroll
    for (unsigned i = 0; i < sizeof(T) / 4; ++i) d[i] = a.w[i];
}
template <class T>
__device__ __forceinline__ T lds_get_uniform(const T *src)
{
    static_assert(sizeof(T) % 4 == 0, "whole 32-bit words");
    struct Words { uint32_t w[sizeof(T) / 4]; };
    Words a;
    const __attribute__((address_space(3))) uint32_t *s = (const __attribute__((address_space(3))) uint32_t *)src;
#pragma unroll
    for (unsigned i = 0; i < sizeof(T) / 4; ++i) a.w[i] = __builtin_amdgcn_readfirstlane(s[i]);
    return __builtin_bit_cast(T, a);
}

// ---- explicit address spaces ---------------------------------------------------------------------
// Pointers that were themselves loaded from memory (weight tables, scratch pointers of an LDS copy of
// the parameters) are generic to the compiler, which would then emit FLAT loads; those count against
// the LDS wait counter as well, so every LDS wait would also wait for the newest weight load.  Every
// accessor therefore states its address space.
#define ETC_AS_GLOBAL __attribute__((address_space(1)))
#define ETC_AS_LDS __attribute__((address_space(3)))
template <class T> __device__ __forceinline__ const ETC_AS_GLOBAL T *as_global(const T *p) { return (const ETC_AS_GLOBAL T *)p; }
template <class T> __device__ __forceinline__ ETC_AS_GLOBAL T *as_global(T *p) { return (ETC_AS_GLOBAL T *)p; }
template <class T> __device__ __forceinline__ ETC_AS_LDS T *as_lds(T *p) { return (ETC_AS_LDS T *)p; }

__device__ __forceinline__ u32x4 gld_16B(const void *p) { return *as_global(reinterpret_cast<const u32x4 *>(p)); }
__device__ __forceinline__ u32x4 gld_16B_nt(const void *p)
{
    return __builtin_nontemporal_load(as_global(reinterpret_cast<const u32x4 *>(p)));
}
__device__ __forceinline__ int gld_i32(const int32_t *p) { return *as_global(p); }
__device__ __forceinline__ uint16_t gld_u16(const uint16_t *p) { return *as_global(p); }
__device__ __forceinline__ void gst_u16(uint16_t *p, uint16_t v) { *as_global(p) = v; }
__device__ __forceinline__ void gst_f32(float *p, float v) { *as_global(p) = v; }

// ---- device-scope (cross-XCD coherent) accessors ----------------------------------------------
#define ETC_SCOPE __HIP_MEMORY_SCOPE_AGENT
__device__ __forceinline__ float ld_f32(const float *p) { return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, ETC_SCOPE); }
__device__ __forceinline__ int ld_i32(const int32_t *p) { return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, ETC_SCOPE); }
__device__ __forceinline__ uint64_t ld_u64(const void *p)
{
    return __hip_atomic_load(as_global(reinterpret_cast<const uint64_t *>(p)), __ATOMIC_RELAXED, ETC_SCOPE);
}
__device__ __forceinline__ void ld_f32x2(const float *p, float &a, float &b)
{
    const uint64_t v = ld_u64(p);
    a = __uint_as_float((uint32_t)v);
    b = __uint_as_float((uint32_t)(v >> 32));
}
__device__ __forceinline__ u32x4 ld_16B(const void *p)      // 16 bytes as two 8-byte device-scope loads
{
    const uint64_t a = ld_u64(p), b = ld_u64(reinterpret_cast<const uint64_t *>(p) + 1);
    return u32x4{(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)};
}
__device__ __forceinline__ void st_f32(float *p, float v) { __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, ETC_SCOPE); }
__device__ __forceinline__ void st_i32(int32_t *p, int v) { __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, ETC_SCOPE); }
__device__ __forceinline__ void st_u64(void *p, uint64_t v)
{
    __hip_atomic_store(as_global(reinterpret_cast<uint64_t *>(p)), v, __ATOMIC_RELAXED, ETC_SCOPE);
}
__device__ __forceinline__ void st_u16(uint16_t *p, uint16_t v) { __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, ETC_SCOPE); }

__device__ __forceinline__ int ev_peek(const int32_t *p) { return ld_i32(p); }

// Records the first error; later waits see it and give up at once, so the kernel always drains.
__device__ __forceinline__ void raise_error(const Params &P, int code, int fn, int ev)
{
    int expected = 0;
    if (__hip_atomic_compare_exchange_strong(as_global(P.error_word), &expected, code, __ATOMIC_RELAXED, __ATOMIC_RELAXED, ETC_SCOPE)) {
        st_i32(P.error_word + 1, fn);
        st_i32(P.error_word + 2, ev);
        st_i32(P.error_word + 3, (int)blockIdx.x);
        // mirrored to pinned host memory: the host sees it without a device call (one store over the bus, error case only)
        if (P.error_host != nullptr) __hip_atomic_store(as_global(P.error_host), code, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Spin of one lane until E[ev] reaches zero: bounded backoff, bounded budget.
__device__ __forceinline__ void spin_until_zero(const Params &P, int ev, int fn)
{
    const int32_t *p = P.ev_cur + ev;
    long long spins = 0;
    while (ev_peek(p) > 0) {
        if (spins < 16) __builtin_amdgcn_s_sleep(1); else __builtin_amdgcn_s_sleep(4);
        ++spins;
        if ((spins & 255) == 0 && ev_peek(P.error_word) != 0) break;
        if (spins > P.spin_budget) { raise_error(P, ERR_WAIT_TIMEOUT, fn, ev); break; }
    }
}

// E[ev].wait() for one wavefront (lane 0 polls).  A wait that gives up records the error and the task
// still runs (on stale data), so every wave keeps the same barrier sequence and the kernel drains.
__device__ __forceinline__ void wave_wait(const Params &P, int ev, int fn)
{
    if (ev < 0) return;
    if (lane_id() == 0) spin_until_zero(P, ev, fn);
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");    // orders later loads after the poll (no cache op)
}

// E[ev0].wait(), E[ev1].wait() for the whole workgroup: one polling lane, then a barrier.
__device__ __forceinline__ void wg_wait(const Params &P, int ev0, int ev1, int fn)
{
    if (ev0 < 0 && ev1 < 0) return;
    if (threadIdx.x == 0) {
        if (ev0 >= 0) spin_until_zero(P, ev0, fn);
        if (ev1 >= 0) spin_until_zero(P, ev1, fn);
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

// Before a notify: every thread drains its (write-through) stores, then the workgroup meets.
// s_waitcnt vmcnt(0) as a builtin (not inline asm), so that the compiler's own wait-count bookkeeping
// knows nothing is outstanding afterwards: only then can it keep fine-grained vmcnt(N) waits inside the
// weight-streaming loops instead of draining at every loop header.
__device__ __forceinline__ void drain_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

__device__ __forceinline__ void wg_release()
{
    drain_vmem();
    __syncthreads();
}

// E[ev].notify(): returns the value before the decrement (1 means this call fired the event).
__device__ __forceinline__ int ev_notify(const Params &P, int ev)
{
    return __hip_atomic_fetch_sub(as_global(P.ev_cur + ev), 1, __ATOMIC_RELAXED, ETC_SCOPE);
}

// Per-task trace mark (debug): thread 0 stamps the device wall clock.
__device__ __forceinline__ void trace_mark(const Params &P, int task_id, int slot)
{
    if (P.trace != nullptr && threadIdx.x == 0 && task_id >= 0)
        as_global(P.trace)[(size_t)task_id * 8 + slot] = slot == 7 ? (uint64_t)blockIdx.x : (uint64_t)wall_clock64();
}

// ---- ready queue of the dynamic scheduler: what the kernel's loop and a triggering task share ----
__device__ __forceinline__ uint64_t q_slot_word(const Params &P, int task_id)
{
    return ((uint64_t)P.epoch << 32) | (uint64_t)(uint32_t)(task_id + 1);
}

// Reserves `cnt` tickets (lane 0) and returns the first one to every lane, or -1 when the queue is full.
__device__ __forceinline__ int q_reserve_wave(const Params &P, int cnt)
{
    int base = 0;
    if (lane_id() == 0) base = __hip_atomic_fetch_add(as_global(P.q_ctrl_cur + 1), cnt, __ATOMIC_RELAXED, ETC_SCOPE);
    base = __builtin_amdgcn_readfirstlane(base);
    if (base + cnt > P.q_capacity) {
        if (lane_id() == 0) raise_error(P, ERR_QUEUE_OVERFLOW, 0, base);
        return -1;
    }
    return base;
}

// ---- sums across lanes ---------------------------------------------------------------------------------
// Cross-lane data-parallel-primitive (DPP) moves inside a row of 16 lanes: the two quad exchanges, then the
// mirror of each half row, then the mirror of the row.  Each is one VALU instruction; a wavefront shuffle goes
// through the LDS crossbar instead, and a chain of dependent ones costs a memory-like round trip each.
template <int CTRL> __device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}
template <int CTRL> __device__ __forceinline__ int dpp_i32(int v) { return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, false); }

// Sum over N (8 or 16) consecutive lanes, aligned to N, result in every one of them.
template <int N>
__device__ __forceinline__ float lanes_sum(float s)
{
    static_assert(N == 8 || N == 16, "8 or 16 lanes");
    s += dpp_f32<0xB1>(s);                    // quad_perm [1,0,3,2]
    s += dpp_f32<0x4E>(s);                    // quad_perm [2,3,0,1]
    s += dpp_f32<0x141>(s);                   // row_half_mirror
    if (N == 16) s += dpp_f32<0x140>(s);      // row_mirror
    return s;
}

// Sum over the wavefront, the same value in every lane: the four row sums are read as scalars.
__device__ __forceinline__ float wave_sum(float v)
{
    v = lanes_sum<16>(v);
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ int wave_sum_i(int v)
{
    v += dpp_i32<0xB1>(v);
    v += dpp_i32<0x4E>(v);
    v += dpp_i32<0x141>(v);
    v += dpp_i32<0x140>(v);
    return (__builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16)) +
           (__builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48));
}

}  // namespace etc
