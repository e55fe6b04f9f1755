// One-kernel form of the online path, shaped for up to 32 tokens: rotate (Eq. 4 / Eq. 5), quantise (Eq. 2) and
// multiply (Eq. 5) in a single launch, with no activation operand in memory between the stages.  More tokens run as
// independent tiles of 32 along blockIdx.y, each streaming the weights again.
//
// Shape.  As the weight-streaming kernel (gemm_decode.hip): one workgroup of 8 waves per 32 output channels, the
// waves split K into contiguous runs of 256-wide steps, each accumulates one 32 x 32 tile, and the eight partial
// tiles are summed through LDS in a fixed order.  What differs is where a wave's activation fragments come from:
// instead of loading codes and scales that an earlier launch wrote, it makes them -- for each K step it loads the
// eight 32-channel blocks of x (bf16) and their rotation blocks (packed form), rotates each on the bf16 matrix
// cores, quantises each group, and moves the 16 code bytes of (token t, group) into the lane the block-scaled
// instruction wants them in.  The device functions are the ones of the two-launch path (rotq_device.h), so the
// codes are the same bit for bit; they can be written out for inspection by the first workgroup.
//
// Cost.  Every workgroup needs the whole quantised activation tile, so each of the N / 32 workgroups repeats the
// rotation of all K / 32 blocks: N / 32 times the matrix-core and quantiser work of the separate launch, and, with
// one rotation block per group, N / 32 reads of all of R through the L2.  That is why the library's default path
// stays two launches; this kernel exists so that the comparison can be measured, and it is never chosen by shape.
#include "duqpp_internal.h"
#include "mxfp4_device.h"
#include "rotq_device.h"

namespace duqpp {

constexpr int kFusedWaves = 8;

// The two FP4 operands of lanes (t, 0) and (t, 1) from the quantiser's output for two blocks: oA / oB hold, in lane
// (t, h), code bytes 8 h .. 8 h + 7 of token t for block A / block B.  Afterwards lane (t, 0) holds all 16 bytes of
// block A and lane (t, 1) all 16 bytes of block B.
__device__ __forceinline__ u32x4 gather_operand(uint2 oA, uint2 oB) {
    // permlane32_swap(a, b): lanes 32..63 of a trade places with lanes 0..31 of b
    auto x = __builtin_amdgcn_permlane32_swap(oA.x, oB.x, false, false);
    auto y = __builtin_amdgcn_permlane32_swap(oA.y, oB.y, false, false);
    // x[0]: lane (t, 0) = A bytes 0..3, lane (t, 1) = B bytes 0..3;  x[1]: A bytes 8..11 | B bytes 8..11; y likewise + 4
    u32x4 r = {x[0], y[0], x[1], y[1]};
    return r;
}

template <bool OUT_BF16>
__global__ __launch_bounds__(kFusedWaves * 64) void rotq_gemm_fused_decode_kernel(FusedDecodeParams p) {
    __shared__ float part[kFusedWaves][16][64];            // [wave][accumulator register][lane]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int t = lane & 31, g = lane >> 5;                // token (activation side) or channel (weight side), half
    const int rt = blockIdx.x;                             // weight row tile
    const int mt = blockIdx.y;                             // token tile
    const int NI = p.GP / 8;
    const int per = (NI + kFusedWaves - 1) / kFusedWaves;
    const int s0 = wave * per;
    int s1 = s0 + per;
    if (s1 > NI) s1 = NI;

    const uint8_t* b_codes = p.b_codes + (int64_t)rt * p.GP * 512 + g * 2048 + t * 16;
    const uint8_t* b_scales = p.b_scales + (int64_t)rt * NI * 256 + lane * 4;
    // lanes without a token of their own rotate token 0 again (same cache lines); their operand is then replaced by
    // the padding of the tiled layout (code 0, scale 127), exactly what the separate launch writes for such rows
    const bool own = 32 * mt + t < p.T;
    const uint16_t* xrow = p.x + (int64_t)(own ? 32 * mt + t : 0) * p.ldx + 8 * g;
    const uint8_t* rp = p.r_packed;
    const bool shared_r = p.r_stride == 0;
    RotOperand opS;
    if (shared_r) load_rot_operand_packed(rp, lane, opS);

    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;

    for (int s = s0; s < s1; ++s) {
        // weight fragments of this step first: their latency hides behind the rotation below
        u32x4 b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) b[i] = __builtin_nontemporal_load((const u32x4*)(b_codes + (int64_t)s * 4096 + i * 512));
        const uint32_t sb = *(const uint32_t*)(b_scales + (int64_t)s * 256);
        u32x4 a[4];
        uint32_t sa = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // MFMA i of the step takes group 8 s + 4 g + i from lane (t, g): blocks jA (g = 0) and jB (g = 1)
            const int jA = 8 * s + i, jB = jA + 4;
            const int cA = jA < p.G ? jA : p.G - 1, cB = jB < p.G ? jB : p.G - 1;       // padding groups: any valid block
            u32x4 xA[2], xB[2];
            xA[0] = *(const u32x4*)(xrow + 32 * cA);
            xA[1] = *(const u32x4*)(xrow + 32 * cA + 16);
            xB[0] = *(const u32x4*)(xrow + 32 * cB);
            xB[1] = *(const u32x4*)(xrow + 32 * cB + 16);
            f32x16 yA, yB;
            if (shared_r) {
                yA = rotate_tile(opS, xA);
                yB = rotate_tile(opS, xB);
            } else {
                RotOperand opA, opB;
                load_rot_operand_packed(rp + (int64_t)cA * p.r_stride, lane, opA);
                load_rot_operand_packed(rp + (int64_t)cB * p.r_stride, lane, opB);
                yA = rotate_tile(opA, xA);
                yB = rotate_tile(opB, xB);
            }
            uint2 oA, oB;
            uint32_t byteA = quantize_group(yA, oA);
            uint32_t byteB = quantize_group(yB, oB);
            if (!own || jA >= p.G) { oA = make_uint2(0, 0); byteA = 127; }
            if (!own || jB >= p.G) { oB = make_uint2(0, 0); byteB = 127; }
            a[i] = gather_operand(oA, oB);
            sa |= (g ? byteB : byteA) << (8 * i);
        }
        if (p.dbg_codes && blockIdx.x == 0) {
            // the activation operand as the separate launch would have written it
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *(u32x4*)(p.dbg_codes + (((int64_t)mt * p.GP + 8 * s + 4 * g + i) * 32 + t) * 16) = a[i];
            *(uint32_t*)(p.dbg_scales + ((((int64_t)mt * NI + s) * 2 + g) * 32 + t) * 4) = sa;
        }
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(a[0]), fp4_operand(b[0]), acc, 4, 4, 0, (int)sa, 0, (int)sb);
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(a[1]), fp4_operand(b[1]), acc, 4, 4, 1, (int)sa, 1, (int)sb);
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(a[2]), fp4_operand(b[2]), acc, 4, 4, 2, (int)sa, 2, (int)sb);
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(a[3]), fp4_operand(b[3]), acc, 4, 4, 3, (int)sa, 3, (int)sb);
    }

    // the eight partial tiles through LDS, summed in a fixed order (as in the weight-streaming kernel)
#pragma unroll
    for (int e = 0; e < 16; ++e) part[wave][e][lane] = acc[e];
    __syncthreads();
    // acc[e] of lane (r, g): token 8 (e / 4) + 4 g + e % 4, output channel 32 rt + r
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int e = (threadIdx.x >> 6) + 8 * h;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kFusedWaves; ++w) sum += part[w][e][lane];
        const int tok = 32 * mt + 8 * (e / 4) + 4 * g + (e % 4);
        const int col = rt * 32 + t;
        if (tok < p.T && col < p.N) {
            if (OUT_BF16) ((uint16_t*)p.y)[(int64_t)tok * p.ldy + col] = f32_to_bf16_rne(sum);
            else ((float*)p.y)[(int64_t)tok * p.ldy + col] = sum;
        }
    }
}

hipError_t launch_rotq_gemm_fused_decode(const FusedDecodeParams& p, hipStream_t stream) {
    if (p.T < 1 || p.T > kFusedMaxT) return hipErrorInvalidValue;
    dim3 grid((unsigned)((p.N + 31) / 32), (unsigned)((p.T + 31) / 32)), block(kFusedWaves * 64);
    return p.out_bf16 ? launch(rotq_gemm_fused_decode_kernel<true>, grid, block, 0, stream, p)
                      : launch(rotq_gemm_fused_decode_kernel<false>, grid, block, 0, stream, p);
}

}  // namespace duqpp
