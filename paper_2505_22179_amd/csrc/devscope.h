// Coherent-at-device-scope accesses for partial results that one workgroup writes and another reads
// inside the same kernel (last-arriver reductions).  They bypass the per-XCD L2's non-coherent lines
// one access at a time, so no whole-cache write-back or invalidate is needed.  A region is addressed
// through a buffer descriptor (wavefront-uniform base) and a byte offset or the index of a 16-byte quad.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace w4 {

typedef __amdgpu_buffer_rsrc_t PartialBuffer;
constexpr int kDeviceScope = 16;   // cache-policy bit sc1

__device__ __forceinline__ PartialBuffer partial_buffer(const float *base)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(base), 0, 0x7FFFFFFF, 0x00020000);
}
__device__ __forceinline__ void store_partial(PartialBuffer b, int quad, float __attribute__((ext_vector_type(4))) v)
{
    typedef uint32_t u32x4_ __attribute__((ext_vector_type(4)));
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_, v), b, quad * 16, 0, kDeviceScope);
}
__device__ __forceinline__ float __attribute__((ext_vector_type(4))) load_partial(PartialBuffer b, int quad)
{
    typedef float float4v_ __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(float4v_, __builtin_amdgcn_raw_buffer_load_b128(b, quad * 16, 0, kDeviceScope));
}
__device__ __forceinline__ void store_partial_f32(PartialBuffer b, int index, float v)
{
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), b, index * 4, 0, kDeviceScope);
}
__device__ __forceinline__ float load_partial_f32(PartialBuffer b, int index)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(b, index * 4, 0, kDeviceScope));
}

}  // namespace w4
