// Device helpers shared by the tiled MXFP4 GEMM kernels: LDS-DMA transfers issued from asm, hand-placed
// waits, the block-scaled FP4 MFMA.
#ifndef DUQPP_GEMM_TILED_COMMON_H
#define DUQPP_GEMM_TILED_COMMON_H

#include "duqpp_internal.h"
#include "mxfp4_device.h"

namespace duqpp {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));   // fp32 pairs convert to it in one instruction, round to nearest even

constexpr int kTileStepBytes = 8 * 512;                 // codes of one row tile for one K step (8 groups)

// M0 carries the LDS destination of an LDS-DMA transfer; the compiler reserves the register but
// has no use for it in this kernel, and the clobber tells it the value does not survive.
#pragma clang diagnostic ignored "-Winline-asm"

// Four KiB-sized LDS-DMA transfers: global [src, src + 4096) (64 lanes x 16 B per transfer) to LDS
// [lds_dst, lds_dst + 4096).  The immediate offset advances both addresses.
__device__ __forceinline__ void dma_4k(const uint8_t* src_lane, uint32_t lds_dst) {
    asm volatile(
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, off\n\t"
        "global_load_lds_dwordx4 %0, off offset:1024\n\t"
        "global_load_lds_dwordx4 %0, off offset:2048\n\t"
        "global_load_lds_dwordx4 %0, off offset:3072"
        :
        : "v"(src_lane), "s"(lds_dst)
        : "memory", "m0");
}

// One KiB-sized transfer with a compile-time offset applied to both addresses.
template <int OFF>
__device__ __forceinline__ void dma_1k_at(const uint8_t* src_lane, uint32_t lds_dst) {
    asm volatile(
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, off offset:%2"
        :
        : "v"(src_lane), "s"(lds_dst), "n"(OFF)
        : "memory", "m0");
}

__device__ __forceinline__ void dma_1k(const uint8_t* src_lane, uint32_t lds_dst) {
    asm volatile(
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %0, off"
        :
        : "v"(src_lane), "s"(lds_dst)
        : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Every LDS access this wave has issued has completed, then workgroup barrier: what a wave writes to LDS
// after the barrier cannot overtake a read another wave issued before it.
__device__ __forceinline__ void workgroup_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

#define DUQPP_MFMA(ACC, A, B, SA, SB, SEL) \
    ACC = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(A), fp4_operand(B), ACC, 4, 4, SEL, (int)(SA), SEL, (int)(SB))

// One 256-byte transfer (64 lanes x 4 B): the scale words of one row tile for one K step.
__device__ __forceinline__ void dma_256(const uint8_t* src_lane, uint32_t lds_dst) {
    asm volatile(
        "s_mov_b32 m0, %1\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dword %0, off"
        :
        : "v"(src_lane), "s"(lds_dst)
        : "memory", "m0");
}

}  // namespace duqpp
#endif
