// Device-side helpers shared by the kernels: vector types, wave-level sums, buffer addressing, streaming stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lf {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __bf16 v4bf __attribute__((ext_vector_type(4)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// A 128-bit load that is known to hit global memory.  Pointers that travel through LDS or a table
// lose their address space; a generic ("flat") load would then be counted against the LDS counter
// as well, and the next LDS wait would also wait for every such load in flight.
typedef const __attribute__((address_space(1))) v4f* global_v4f_ptr;
__device__ __forceinline__ v4f load_global_v4f(const float* p) { return *(global_v4f_ptr)(p); }
// A relaxed atomic load of workgroup scope: an ordinary load instruction, but one the compiler leaves
// where the source puts it.  A plain load would be sunk next to its first use, with the whole memory
// latency then in front of that use.
__device__ __forceinline__ float load_global_f32_here(const float* p) {
    return __hip_atomic_load((const __attribute__((address_space(1))) float*)(p), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_WORKGROUP);
}
// Buffer addressing: the base lives in four scalar registers, each load supplies one 32-bit byte
// offset, and an offset at or past `bytes` makes the load return zeros instead of touching memory.
// The pointer is made wave-uniform first (a resource in vector registers would be loaded lane by lane).
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buffer(const void* p, unsigned bytes) {
    const unsigned long long a = reinterpret_cast<unsigned long long>(p);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)a);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32));
    void* q = reinterpret_cast<void*>(((unsigned long long)hi << 32) | lo);
    return __builtin_amdgcn_make_buffer_rsrc(q, 0, __builtin_amdgcn_readfirstlane(bytes), 0x00020000);
}
__device__ __forceinline__ v4f buffer_load_v4f(__amdgpu_buffer_rsrc_t r, unsigned byte_offset) {
    return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, 0));
}

// The same load marked non-temporal (NT) or not: for data that is read once and is too large to stay in the caches.
template <bool NT>
__device__ __forceinline__ v4f buffer_load_v4f_as(__amdgpu_buffer_rsrc_t r, unsigned byte_offset) {
    return __builtin_bit_cast(v4f, __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, NT ? 2 : 0));
}

// Streaming (non-temporal) 128-bit store through a buffer resource: an offset at or past the buffer's size
// makes the store a no-op, so rows past the end need no branch.  (aux bit 1 = non-temporal.)
__device__ __forceinline__ void buffer_store_nt_v4f(__amdgpu_buffer_rsrc_t r, unsigned byte_offset, v4f v) {
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(v4u, v), r, byte_offset, 0, 2);
}

// Streaming (non-temporal) 128-bit store to global memory.
__device__ __forceinline__ void store_global_nt_v4f(float* p, v4f v) {
    __builtin_nontemporal_store(v, (__attribute__((address_space(1))) v4f*)(p));
}
__device__ __forceinline__ void store_global_f32(float* p, float v) {
    *(__attribute__((address_space(1))) float*)(p) = v;
}

// sigma(z) = 1/(1+e^-z), section 2.  Accurate expf and an IEEE division: the
// O(N) epilogues are never the bottleneck.
__device__ __forceinline__ float sigmoidf(float z) { return 1.0f / (1.0f + expf(-z)); }

// v of the lane N places to the right within the lane's row of 16 lanes, cyclically (a data-parallel
// move, a few cycles; a general cross-lane shuffle goes through the LDS crossbar and takes a hundred).
template <int N>
__device__ __forceinline__ float row_rotate(float v) {
    static_assert(N >= 1 && N <= 15, "rotation within a row of 16 lanes");
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x120 + N,
                                                                 0xF, 0xF, false));
}
// Sum over those lanes of the row whose lane number is congruent to this lane's modulo STEP (a power of
// two up to 16); every lane gets its class's sum.  Fixed order.
template <int STEP>
__device__ __forceinline__ float row_class_sum(float v) {
    if constexpr (STEP <= 1) v += row_rotate<1>(v);
    if constexpr (STEP <= 2) v += row_rotate<2>(v);
    if constexpr (STEP <= 4) v += row_rotate<4>(v);
    if constexpr (STEP <= 8) v += row_rotate<8>(v);
    return v;
}
// Sum over the 64 lanes in a fixed order; every lane gets the result.
__device__ __forceinline__ float wave_sum(float v) {
    v = row_class_sum<1>(v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return ((r0 + r1) + r2) + r3;
}

}  // namespace lf
