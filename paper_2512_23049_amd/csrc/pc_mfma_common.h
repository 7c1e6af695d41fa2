// Small device helpers shared by the bf16 MFMA kernels (gfx950).
#ifndef PC_MFMA_COMMON_H_
#define PC_MFMA_COMMON_H_

#include "pc_kernels.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define PC_D 128

// fp32 -> fp16 bits, round to nearest even (split partials are stored normalised in fp16:
// 11 significant bits, four times finer than the bf16 the final output is rounded to)
__device__ __forceinline__ uint16_t to_f16(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }
__device__ __forceinline__ uint32_t pack_f16(float a, float b) { return (uint32_t)to_f16(a) | ((uint32_t)to_f16(b) << 16); }

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    bf16x2 r = {(__bf16)a, (__bf16)b};
    return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ uint16_t to_bf16(float a)
{
    __bf16 r = (__bf16)a;
    return __builtin_bit_cast(uint16_t, r);
}
__device__ __forceinline__ uint4 ldg16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }


#endif
