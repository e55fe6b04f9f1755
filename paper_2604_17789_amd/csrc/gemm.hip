// W4A4 MXFP4 GEMM (the Q(X^) . Q(W^) product of the paper's Eq. 5) on gfx950's block-scaled
// matrix cores: v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in FP4 (E2M1) and one
// E8M0 scale per lane.
//
// Operand form of the instruction for FP4: lane l supplies, for row (l & 31) of its matrix,
// the 32 consecutive K values of k-block (l >> 5) as 16 bytes (element 2i in the low nibble
// of byte i) plus one scale byte that applies to exactly those 32 values -- i.e. one MXFP4
// group of the row-major [rows, K/2] / [rows, K/32] layout is one lane's operand.
// K is a summation index, so the order in which groups meet the instruction is free: a lane
// reads FOUR consecutive groups of its row (64 bytes of codes, one 32-bit word of scales) and
// feeds them to four MFMAs that pick scale byte 0..3 of the word; half-wave g handles groups
// 4g .. 4g+3 of every run of 8.
#include "duqpp_internal.h"
#include "mxfp4_device.h"

namespace duqpp {

#define DUQPP_MFMA_FP4(acc, a, b, sa, sb, sel) \
    acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(a), fp4_operand(b), acc, 4, 4, sel, (int)(sa), sel, (int)(sb))

// Four consecutive groups (kb .. kb+3) of one row: 64 code bytes + 4 scale bytes.
struct RowFrag {
    uint4 q[4];
    uint32_t s;
};

__device__ __forceinline__ void load_frag(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                          int64_t row, int G, int kb, bool fast, RowFrag& f) {
    const uint8_t* cr = codes + (row * G + kb) * 16;
    const uint8_t* sr = scales + row * G + kb;
    if (fast) {
        f.q[0] = *(const uint4*)(cr);
        f.q[1] = *(const uint4*)(cr + 16);
        f.q[2] = *(const uint4*)(cr + 32);
        f.q[3] = *(const uint4*)(cr + 48);
        f.s = *(const uint32_t*)sr;
    } else {
        // ragged tail (or a scale row that is not word aligned): groups past G contribute zero
        f.s = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (kb + i < G) {
                f.q[i] = *(const uint4*)(cr + 16 * i);
                f.s |= (uint32_t)sr[i] << (8 * i);
            } else {
                f.q[i] = make_uint4(0, 0, 0, 0);
                f.s |= 127u << (8 * i);
            }
        }
    }
}

// Direct-from-global kernel: 4 waves as 2 x 2, each wave a 64 x 64 output tile (2 x 2 MFMA
// tiles), operands read straight from global memory in the canonical layout.
constexpr int kDirTileM = 128, kDirTileN = 128;

template <bool OUT_BF16>
__global__ __launch_bounds__(256) void gemm_direct_kernel(GemmParams p) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int r = lane & 31, g = lane >> 5;
    const int m0 = blockIdx.y * kDirTileM + (wave >> 1) * 64;
    const int n0 = blockIdx.x * kDirTileN + (wave & 1) * 64;
    if (m0 >= p.T || n0 >= p.N) return;

    int64_t arow[2], brow[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        int a = m0 + 32 * t + r, b = n0 + 32 * t + r;
        arow[t] = a < p.T ? a : p.T - 1;
        brow[t] = b < p.N ? b : p.N - 1;
    }
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int G = p.G;
    // whole-word scale loads need word-aligned scale rows on both operands
    const bool aligned = (G % 4) == 0 && (((uintptr_t)p.a_scales | (uintptr_t)p.b_scales) & 3) == 0;
    for (int kb0 = 0; kb0 < G; kb0 += 8) {
        const int kb = kb0 + 4 * g;
        const bool fast = aligned && (kb0 + 8 <= G);
        RowFrag fa[2], fb[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            load_frag(p.a_codes, p.a_scales, arow[t], G, kb, fast, fa[t]);
            load_frag(p.b_codes, p.b_scales, brow[t], G, kb, fast, fb[t]);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                DUQPP_MFMA_FP4(acc[i][j], fa[i].q[0], fb[j].q[0], fa[i].s, fb[j].s, 0);
                DUQPP_MFMA_FP4(acc[i][j], fa[i].q[1], fb[j].q[1], fa[i].s, fb[j].s, 1);
                DUQPP_MFMA_FP4(acc[i][j], fa[i].q[2], fb[j].q[2], fa[i].s, fb[j].s, 2);
                DUQPP_MFMA_FP4(acc[i][j], fa[i].q[3], fb[j].q[3], fa[i].s, fb[j].s, 3);
            }
    }
    // acc[i][j][e] of lane (r, g): row m0 + 32 i + 8 (e / 4) + 4 g + e % 4, column n0 + 32 j + r
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + 32 * j + r;
            if (col >= p.N) continue;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int row = m0 + 32 * i + 8 * (e / 4) + 4 * g + (e % 4);
                if (row < p.T) {
                    if (OUT_BF16) ((uint16_t*)p.y)[(int64_t)row * p.ldy + col] = f32_to_bf16_rne(acc[i][j][e]);
                    else ((float*)p.y)[(int64_t)row * p.ldy + col] = acc[i][j][e];
                }
            }
        }
}


hipError_t launch_gemm(const GemmParams& p, hipStream_t stream) {
    dim3 grid((unsigned)((p.N + kDirTileN - 1) / kDirTileN), (unsigned)((p.T + kDirTileM - 1) / kDirTileM)), block(256);
    return p.out_bf16 ? launch(gemm_direct_kernel<true>, grid, block, 0, stream, p)
                      : launch(gemm_direct_kernel<false>, grid, block, 0, stream, p);
}

}  // namespace duqpp
