// Device code shared by the kernels that rotate and quantise (rotq.hip, rotq_gemm_fused.hip): the rotation of a
// 32-token x 32-channel tile on the bf16 matrix cores at fp32 accuracy (Eq. 4 / Eq. 5) and the MXFP4 quantiser of one
// group (Eq. 2).  One definition, so that every kernel produces the same codes from the same inputs.
#ifndef DUQPP_ROTQ_DEVICE_H
#define DUQPP_ROTQ_DEVICE_H

#include "duqpp_internal.h"

namespace duqpp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// R^T pieces of one block in MFMA A-operand form: [k-step] x {hi, mid, lo}
struct RotOperand {
    bf16x8 hi[2], mid[2], lo[2];
};

// Exact split v = hi + mid + lo with each piece a bf16 (truncation keeps the three pieces
// non-overlapping: 8 significant bits each out of fp32's 24).
__device__ __forceinline__ void split3(float v, uint32_t& hi, uint32_t& mid, uint32_t& lo) {
    uint32_t bh = __float_as_uint(v) & 0xFFFF0000u;
    float r1 = v - __uint_as_float(bh);
    uint32_t bm = __float_as_uint(r1) & 0xFFFF0000u;
    float r2 = r1 - __uint_as_float(bm);
    uint32_t bl = __float_as_uint(r2) & 0xFFFF0000u;
    hi = bh >> 16; mid = bm >> 16; lo = bl >> 16;
}

// Lane (c = lane & 31, h = lane >> 5) holds, for k-step s, R[r = 16 s + 8 h + i][c], i = 0..7.
__device__ __forceinline__ void load_rot_operand(const float* __restrict__ Rb, int c, int h, RotOperand& op) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        u32x4 vh, vm, vl;
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            uint32_t h0, m0, l0, h1, m1, l1;
            split3(Rb[(16 * s + 8 * h + i) * 32 + c], h0, m0, l0);
            split3(Rb[(16 * s + 8 * h + i + 1) * 32 + c], h1, m1, l1);
            vh[i / 2] = h0 | (h1 << 16);
            vm[i / 2] = m0 | (m1 << 16);
            vl[i / 2] = l0 | (l1 << 16);
        }
        op.hi[s] = __builtin_bit_cast(bf16x8, vh);
        op.mid[s] = __builtin_bit_cast(bf16x8, vm);
        op.lo[s] = __builtin_bit_cast(bf16x8, vl);
    }
}

// The same operand from the packed form duqpp_pack_rotation writes offline (the blocks are calibrated offline,
// Sec. 4.2, like the weights): per block 6 KiB as [piece: lo, mid, hi][k-step][lane][8 bf16], i.e. each of the six
// registers quads of a lane is one 16-byte load and a wave-level load is one contiguous KiB.  No split, no strided
// 4-byte loads at the head of every launch.
constexpr int kPackedBlockBytes = 3 * 2 * 64 * 16;
static_assert(kPackedBlockBytes == kPackedRotationBlockBytes, "size the ABI reports for a packed block");
__device__ __forceinline__ void load_rot_operand_packed(const uint8_t* __restrict__ Pb, int lane, RotOperand& op) {
    const u32x4* q = (const u32x4*)Pb + lane;
    op.lo[0] = __builtin_bit_cast(bf16x8, q[0 * 64]);
    op.lo[1] = __builtin_bit_cast(bf16x8, q[1 * 64]);
    op.mid[0] = __builtin_bit_cast(bf16x8, q[2 * 64]);
    op.mid[1] = __builtin_bit_cast(bf16x8, q[3 * 64]);
    op.hi[0] = __builtin_bit_cast(bf16x8, q[4 * 64]);
    op.hi[1] = __builtin_bit_cast(bf16x8, q[5 * 64]);
}

// acc[i] of lane (t = lane & 31, h) is y[token t][channel 8 (i / 4) + 4 h + i % 4] of one block.
__device__ __forceinline__ f32x16 rotate_tile(const RotOperand& op, const u32x4 xv[2]) {
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    bf16x8 b0 = __builtin_bit_cast(bf16x8, xv[0]);
    bf16x8 b1 = __builtin_bit_cast(bf16x8, xv[1]);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op.lo[0], b0, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op.lo[1], b1, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op.mid[0], b0, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op.mid[1], b1, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op.hi[0], b0, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op.hi[1], b1, acc, 0, 0, 0);
    return acc;
}

// Eq. 2 on one token's 32 values spread over lanes l and l^32 (16 each, layout of rotate_tile): the E8M0 byte of the
// group, and this lane's own 16 codes -- acc[2 k], acc[2 k + 1] in the low and high nibble of byte k of p0 (k < 4),
// acc[8 + 2 k], acc[9 + 2 k] likewise in p1.
__device__ __forceinline__ uint32_t quantize_lane(const f32x16& acc, uint32_t& p0, uint32_t& p1) {
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(acc[i]));
    m = fmaxf(m, __shfl_xor(m, 32));
    // floor(log2 amax) - 2 from the exponent field; fields 0..2 (amax < 2^-124) clamp to 2^-127
    uint32_t ef = __float_as_uint(m) >> 23;
    uint32_t byte = (ef > 2u ? ef : 2u) - 2u;
    float sc = __uint_as_float(byte << 23);
    p0 = 0;
    p1 = 0;
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[0], acc[1], sc, 0);
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[2], acc[3], sc, 1);
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[4], acc[5], sc, 2);
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[6], acc[7], sc, 3);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[8], acc[9], sc, 0);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[10], acc[11], sc, 1);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[12], acc[13], sc, 2);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[14], acc[15], sc, 3);
    return byte;
}

// The same with the codes in the order of the operand layouts.  Returns the E8M0 byte; `out` receives this lane's 8
// bytes of the group's 16 code bytes (h = 0: bytes 0..7, h = 1: bytes 8..15).
__device__ __forceinline__ uint32_t quantize_group(const f32x16& acc, uint2& out) {
    uint32_t p0, p1;
    const uint32_t byte = quantize_lane(acc, p0, p1);
    // p0 = code bytes {2h, 2h+1, 4+2h, 5+2h}, p1 = {8+2h, 9+2h, 12+2h, 13+2h}.
    // Swap p0 of the upper half-wave with p1 of the lower: h = 0 then holds both p0s, h = 1 both p1s.
    auto sw = __builtin_amdgcn_permlane32_swap(p0, p1, false, false);
    uint32_t a = sw[0], b = sw[1];        // a: from h = 0, b: from h = 1
    out.x = (a & 0xFFFFu) | (b << 16);
    out.y = (a >> 16) | (b & 0xFFFF0000u);
    return byte;
}

}  // namespace duqpp
#endif
