// How workgroups of one launch hand data to each other on a GPU whose XCDs have separate,
// mutually non-coherent L2 caches: the writer uses device-scope write-through stores and waits
// for their completion before it takes a ticket on a device-scope counter; the workgroup that
// draws the last ticket reads with device-scope loads, which do not trust its own XCD's caches.
// The loads are buffer loads: they take the scope as a cache-policy operand (bit 4 = sc1 on
// gfx942 / gfx950) while staying ordinary tracked loads, so many of them can be in flight at once
// (atomic loads are issued one at a time), and 8- and 16-byte forms exist.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tidal {
namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
constexpr int kCachePolicySc1 = 16;

__device__ __forceinline__ void publish(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish(uint32_t *p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish(uint64_t *p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// A buffer resource over [base, base + bytes); base is wave-uniform.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t coherent_window(const void *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ u32x4_t coherent_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, kCachePolicySc1);
}
__device__ __forceinline__ u32x2_t coherent_load8(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset) {
    return __builtin_amdgcn_raw_buffer_load_b64(r, byte_offset, 0, kCachePolicySc1);
}
__device__ __forceinline__ uint32_t coherent_load4(__amdgpu_buffer_rsrc_t r, uint32_t byte_offset) {
    return __builtin_amdgcn_raw_buffer_load_b32(r, byte_offset, 0, kCachePolicySc1);
}

// Every store of this wave has completed (write-through stores have reached memory).
__device__ __forceinline__ void wait_for_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

}  // namespace
}  // namespace tidal
