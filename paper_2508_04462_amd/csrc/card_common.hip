// Shared device helpers of libcard (gfx950 / CDNA4, 64-wide wavefronts).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "card_layout.h"

namespace card {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) unsigned int uint4v;

// Data handed from one workgroup to another inside a kernel goes through device-scope accesses:
// the store writes through the compute die's own L2, the load bypasses it.  (A full device fence
// would write back and invalidate the whole L2 on every call - tens of microseconds.)
__device__ __forceinline__ void st_agent(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// order-preserving map float -> uint32 (larger float, larger key)
__device__ __forceinline__ uint32_t float_key(float v) {
    const uint32_t b = __float_as_uint(v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
// fp32 -> bf16 high part + bf16 remainder: two matrix instructions then see ~16 mantissa bits
__device__ __forceinline__ void split_bf16(float v, __bf16& hi, __bf16& lo) {
    hi = static_cast<__bf16>(v);
    lo = static_cast<__bf16>(v - static_cast<float>(hi));
}
// element (head element j, token t) inside the V block of one page and head: pairs of 16-row
// tiles are interleaved so that one 16-byte load per lane feeds two P*V matrix instructions
__device__ __forceinline__ int v_page_index(int j, int t) {
    return ((((j >> 5) * 64) + (t >> 2) * 16 + (j & 15)) << 3) + ((j >> 4) & 1) * 4 + (t & 3);
}

}  // namespace card
