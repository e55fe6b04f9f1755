// Device helpers shared by every MXFP4 GEMM kernel: vector types, the FP4 operand of the block-scaled matrix
// instruction, and the bf16 rounding of the epilogue.
#ifndef DUQPP_MXFP4_DEVICE_H
#define DUQPP_MXFP4_DEVICE_H

#include "duqpp_internal.h"

namespace duqpp {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The instruction takes eight registers per operand; FP4 fills the first four (32 values of 4 bits).
__device__ __forceinline__ i32x8 fp4_operand(const u32x4& v) {
    i32x8 r = {(int)v[0], (int)v[1], (int)v[2], (int)v[3], 0, 0, 0, 0};
    return r;
}
__device__ __forceinline__ i32x8 fp4_operand(const uint4& v) {
    i32x8 r = {(int)v.x, (int)v.y, (int)v.z, (int)v.w, 0, 0, 0, 0};
    return r;
}

// fp32 -> bf16 bits, round to nearest even (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace duqpp
#endif
