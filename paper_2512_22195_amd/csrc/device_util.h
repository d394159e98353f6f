// Small device helpers shared by every kernel file: bf16 rounding, loads through the global
// address space, agent-scope accesses and the arrival counter built on them.
#pragma once

#include "matkv_internal.h"

namespace matkv {
namespace dev {

typedef unsigned int u32x2v __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));

// fp32 -> bf16, round to nearest even on the bit pattern; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// 16-byte load through the global address space (a pointer rebuilt from an integer would
// otherwise be treated as generic and loaded with the slower flat instructions).
__device__ __forceinline__ uint4 ldg16(const void* p) {
    typedef const __attribute__((address_space(1))) u32x4v* gptr;
    const u32x4v r = *(gptr)(uintptr_t)p;
    return make_uint4(r.x, r.y, r.z, r.w);
}

// 8-byte load through the global address space.
__device__ __forceinline__ uint2 ldg8(const void* p) {
    typedef const __attribute__((address_space(1))) u32x2v* gptr;
    const u32x2v r = *(gptr)(uintptr_t)p;
    return make_uint2(r.x, r.y);
}

// Agent-scope relaxed accesses: coherent across the chip's L2 slices without cache flushes.
__device__ __forceinline__ void st_agent2(float* p, float x, float y) {
    const uint64_t v = (uint64_t)__float_as_uint(x) | ((uint64_t)__float_as_uint(y) << 32);
    __hip_atomic_store(reinterpret_cast<uint64_t*>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_agent2(const float* p) {
    const uint64_t r = __hip_atomic_load(reinterpret_cast<const uint64_t*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((uint32_t)r), __uint_as_float((uint32_t)(r >> 32)));
}

// One workgroup's arrival at a counter: every thread has waited for its own agent-scope stores,
// the barrier orders them before thread 0's ticket.  Returns true in every thread of the
// workgroup that arrived last of `expected`.
__device__ __forceinline__ bool arrive_at(int32_t* counter, int expected, int* sm_last) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const int prev = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *sm_last = (prev == expected - 1);
    }
    __syncthreads();
    return *sm_last != 0;
}
// (by the workgroup that arrived last: ready for the next launch)
__device__ __forceinline__ void reset_counter_at(int32_t* counter) {
    if (threadIdx.x == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace dev
}  // namespace matkv
