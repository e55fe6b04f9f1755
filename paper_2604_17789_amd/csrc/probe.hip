// Measurement aid: the rate the chip sustains on the block-scaled FP4 MFMA alone, with operands held in
// registers -- no memory traffic, no LDS, one wave per SIMD on every CU.  It is the ceiling of any MXFP4 GEMM
// under that load, to set beside the nominal peak.  Two patterns: one operand pair held for every instruction,
// and four activation-side times four weight-side fragments with every instruction taking a different pair in
// the order of the GEMM kernels' inner loop (one operand changes per instruction).  The second is the honest
// ceiling: how fast the matrix cores issue depends on how much their operands switch, not only on their values.
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

// 16 instructions per iteration: acc[i][j] += a[i] . b[j], rows alternately forwards and backwards
__global__ __launch_bounds__(256) void probe_fp4_mfma_switching_kernel(ProbeParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    i32x8 a[4], b[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int piece = ((blockIdx.x * 4 + wave) * 4 + k) % p.pieces;
        const u32x4 va = *(const u32x4*)(p.codes + piece * 2048 + lane * 16);
        const u32x4 vb = *(const u32x4*)(p.codes + piece * 2048 + 1024 + lane * 16);
        a[k] = i32x8{(int)va[0], (int)va[1], (int)va[2], (int)va[3], 0, 0, 0, 0};
        b[k] = i32x8{(int)vb[0], (int)vb[1], (int)vb[2], (int)vb[3], 0, 0, 0, 0};
    }
    const int sa = 0x7C7E7F80 + (lane & 1), sb = 0x807F7E7D - (lane & 1);
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
#define DUQPP_PROBE_ROW(I, J0, J1, J2, J3, SEL)                                                                    \
    acc[I][J0] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[I], b[J0], acc[I][J0], 4, 4, SEL, sa, SEL, sb); \
    acc[I][J1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[I], b[J1], acc[I][J1], 4, 4, SEL, sa, SEL, sb); \
    acc[I][J2] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[I], b[J2], acc[I][J2], 4, 4, SEL, sa, SEL, sb); \
    acc[I][J3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[I], b[J3], acc[I][J3], 4, 4, SEL, sa, SEL, sb)
    for (int64_t it = 0; it < p.iters; ++it) {
        DUQPP_PROBE_ROW(0, 0, 1, 2, 3, 0);
        DUQPP_PROBE_ROW(1, 3, 2, 1, 0, 1);
        DUQPP_PROBE_ROW(2, 0, 1, 2, 3, 2);
        DUQPP_PROBE_ROW(3, 3, 2, 1, 0, 3);
    }
#undef DUQPP_PROBE_ROW
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) s += acc[i][j][e];
    p.out[blockIdx.x * 256 + threadIdx.x] = s;
}

hipError_t launch_probe_fp4_mfma(const ProbeParams& p, hipStream_t stream) {
    if (p.switching) hipLaunchKernelGGL(probe_fp4_mfma_switching_kernel, dim3(kNumCU), dim3(256), 0, stream, p);
    else hipLaunchKernelGGL(probe_fp4_mfma_kernel, dim3(kNumCU), dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace duqpp
