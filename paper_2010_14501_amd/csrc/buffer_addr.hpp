// Buffer addressing: address = base (a resource descriptor in scalar registers) + a 32-bit per-lane byte offset + a 32-bit
// scalar byte offset.  The part of an address that is the same for every lane so costs no vector instruction -- on this chip
// every vector instruction takes its cycles from the fp32 matrix pipe of the same SIMD, whichever wave issues it.
// The descriptors span the whole 32-bit offset range: every access made through them is in bounds by construction, the
// hardware's range check is not relied upon.  Word 3 is the plain 32-bit data format of this GPU family.
#pragma once
#include <hip/hip_runtime.h>

namespace monet {

typedef float bf4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t buffer_of(const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, -1, 0x00020000);
}
__device__ __forceinline__ float buffer_load(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
}
__device__ __forceinline__ bf4 buffer_load4(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {
    return __builtin_bit_cast(bf4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0));
}
__device__ __forceinline__ void buffer_store4(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff, bf4 v) {
    typedef unsigned int word4 __attribute__((__vector_size__(16)));
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(word4, v), r, (int)voff, (int)soff, 0);
}
__device__ __forceinline__ void buffer_store(__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff, float v) {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, v), r, (int)voff, (int)soff, 0);
}

}  // namespace monet
