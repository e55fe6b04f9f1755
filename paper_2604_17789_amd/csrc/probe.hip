// Measurement aid: the rate the chip sustains on the block-scaled FP4 MFMA alone, with operands held in
// registers -- no memory traffic, no LDS, one wave per SIMD on every CU.  It is the ceiling of any MXFP4 GEMM
// at the clock the chip settles to under that load, to set beside the nominal peak.
#include "duqpp_internal.h"

namespace duqpp {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_fp4_mfma_kernel(ProbeParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    // operand bit patterns from the caller's code bytes (16 bytes per lane and operand), scale bytes 127 +- 3
    const u32x4 va = *(const u32x4*)(p.codes + ((blockIdx.x * 4 + wave) % p.pieces) * 2048 + lane * 16);
    const u32x4 vb = *(const u32x4*)(p.codes + ((blockIdx.x * 4 + wave) % p.pieces) * 2048 + 1024 + lane * 16);
    const i32x8 a = {(int)va[0], (int)va[1], (int)va[2], (int)va[3], 0, 0, 0, 0};
    const i32x8 b = {(int)vb[0], (int)vb[1], (int)vb[2], (int)vb[3], 0, 0, 0, 0};
    const int sa = 0x7C7E7F80 + (lane & 1), sb = 0x807F7E7D - (lane & 1);
    f32x16 acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
    for (int64_t it = 0; it < p.iters; ++it) {
        // the scale byte selector is an immediate: the four choices written out
        acc[0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[0], 4, 4, 0, sa, 0, sb);
        acc[1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[1], 4, 4, 1, sa, 1, sb);
        acc[2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[2], 4, 4, 2, sa, 2, sb);
        acc[3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[3], 4, 4, 3, sa, 3, sb);
        acc[4] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[4], 4, 4, 0, sa, 0, sb);
        acc[5] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[5], 4, 4, 1, sa, 1, sb);
        acc[6] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[6], 4, 4, 2, sa, 2, sb);
        acc[7] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[7], 4, 4, 3, sa, 3, sb);
    }
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    p.out[blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_probe_fp4_mfma(const ProbeParams& p, hipStream_t stream) {
    hipLaunchKernelGGL(probe_fp4_mfma_kernel, dim3(kNumCU), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace duqpp
