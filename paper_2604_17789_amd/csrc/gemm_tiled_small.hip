// W4A4 MXFP4 GEMM (Eq. 5) on tiled operands for shapes that give the 128 x 256 tiling too few tiles to
// occupy the chip (a few hundred tokens against a few thousand output channels): the same block-scaled
// FP4 instruction, K permutation and LDS-DMA feeding as gemm_tiled.hip, on 64 x 128 tiles.
//
//   workgroup  4 waves as 2 x 2, output tile 64 (tokens) x 128 (output channels); each wave owns 32 x 64 =
//              1 x 2 MFMA tiles.  A stage holds (2 + 4) row tiles x 4 KiB of codes and 8 x 256 B of scale
//              words (six used); three stages are 78 KiB, so two workgroups share a CU when there are
//              more tiles than CUs, and their eight waves cover each other's waits.
//   transfers  per K step a wave moves six KiB of codes and two 256-byte rows of scale words (waves 2 and
//              3: one real row and one repeated into the padding, which keeps the count per wave uniform).
// Per flop this tile moves twice the bytes of the large one from L2 to LDS, so it runs at about half its
// per-CU rate -- on four times as many CUs when the large tiling would leave most of them idle.
#include <atomic>

#include "duqpp_internal.h"
#include "gemm_tiled_common.h"

namespace duqpp {

constexpr int kSBM = 64, kSBN = 128;
constexpr int kSMT = kSBM / 32, kSNT = kSBN / 32;           // row tiles of A / B per workgroup
constexpr int kSRowTiles = kSMT + kSNT;                     // 6
constexpr int kSScalesOff = kSRowTiles * kTileStepBytes;    // scale words follow the codes in a stage
constexpr int kSStageBytes = kSScalesOff + 8 * 256;
constexpr int kSStages = 3;                                 // 79872 B: two workgroups per CU (six stages for
                                                            // a lone workgroup per CU measured 5 % slower)
constexpr int kSGroupM = 8;
constexpr int kSDmaOps = 8;                                 // transfers per wave per step

// at most 8 * k transfers outstanding, k <= MAXK (uniform over the wave)
template <int MAXK>
__device__ __forceinline__ void wait_steps_outstanding(int k) {
    if constexpr (MAXK == 0) {
        wait_vmcnt<0>();
    } else {
        if (k >= MAXK) wait_vmcnt<kSDmaOps * MAXK>();
        else wait_steps_outstanding<MAXK - 1>(k);
    }
}

template <bool OUT_BF16, int STAGES>
__global__ __launch_bounds__(256, STAGES == 3 ? 2 : 1) void gemm_tiled_small_kernel(TiledGemmParams p) {
    static_assert(kSDmaOps * (STAGES - 2) <= 63, "the wait counter holds 63");
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    const int tiles_m = (p.T + kSBM - 1) / kSBM, tiles_n = (p.N + kSBN - 1) / kSBN;
    // XCD-contiguous renumbering, then groups of kSGroupM M-tiles swept along N
    int pid;
    {
        const int id = blockIdx.x, n = gridDim.x;
        const int per = n / kNumXCD, rem = n % kNumXCD;
        const int xcd = id % kNumXCD, slot = id / kNumXCD;
        pid = xcd * per + (xcd < rem ? xcd : rem) + slot;
    }
    const int group_sz = kSGroupM * tiles_n;
    const int first_m = (pid / group_sz) * kSGroupM;
    const int gm = (tiles_m - first_m) < kSGroupM ? (tiles_m - first_m) : kSGroupM;
    const int tile_m = first_m + (pid % group_sz) % gm;
    const int tile_n = (pid % group_sz) / gm;

    const int RTa = (p.T + 31) / 32, RTb = (p.N + 31) / 32;
    const int NI = p.GP / 8;                               // K steps
    const int64_t tile_bytes = (int64_t)p.GP * 512;        // codes of one row tile
    const int64_t tile_sbytes = (int64_t)NI * 256;         // scale words of one row tile

    // row tile q of the stage (0, 1: A; 2..5: B) -> its codes / scale words in global memory; tiles past the
    // ragged edge are replaced by the last valid one (their outputs are never stored)
    auto codes_of = [&](int q) -> const uint8_t* {
        if (q < kSMT) {
            int rt = tile_m * kSMT + q;
            if (rt >= RTa) rt = RTa - 1;
            return p.a_codes + rt * tile_bytes;
        }
        int rt = tile_n * kSNT + (q - kSMT);
        if (rt >= RTb) rt = RTb - 1;
        return p.b_codes + rt * tile_bytes;
    };
    auto scales_of = [&](int q) -> const uint8_t* {
        if (q < kSMT) {
            int rt = tile_m * kSMT + q;
            if (rt >= RTa) rt = RTa - 1;
            return p.a_scales + rt * tile_sbytes;
        }
        int rt = tile_n * kSNT + (q - kSMT);
        if (rt >= RTb) rt = RTb - 1;
        return p.b_scales + rt * tile_sbytes;
    };

    // ---- LDS-DMA duty of this wave per step: the KiB pieces 6 w .. 6 w + 5 of the 24 (piece i = KiB i % 4
    // of row tile i / 4) and the scale rows 2 w, 2 w + 1 (rows 6, 7 do not exist: row 5 again, into the padding)
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const void*)lds);
    const uint8_t* dma_src[6];
    uint32_t dma_dst[6];
#pragma unroll
    for (int k = 0; k < 6; ++k) {
        const int piece = wave * 6 + k;
        dma_src[k] = codes_of(piece / 4) + (piece % 4) * 1024 + lane * 16;
        dma_dst[k] = lds0 + piece * 1024;
    }
    const uint8_t* sdma_src[2];
    uint32_t sdma_dst[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int row = wave * 2 + k;
        sdma_src[k] = scales_of(row < kSRowTiles ? row : kSRowTiles - 1) + lane * 4;
        sdma_dst[k] = lds0 + kSScalesOff + row * 256;
    }
    auto issue_dma = [&](int step, int stage) {
        const uint32_t so = stage * kSStageBytes;
#pragma unroll
        for (int k = 0; k < 6; ++k) dma_1k(dma_src[k] + (int64_t)step * kTileStepBytes, dma_dst[k] + so);
#pragma unroll
        for (int k = 0; k < 2; ++k) dma_256(sdma_src[k] + (int64_t)step * 256, sdma_dst[k] + so);
    };

    // ---- LDS read addresses: lane (r, g) reads group 4 g + i of row r at (4 g + i) * 512 + r * 16;
    // its scale word of row tile q at kSScalesOff + q * 256 + lane * 4
    const uint8_t* pa0 = lds + g * 2048 + r * 16 + wm * kTileStepBytes;
    const uint8_t* pb0 = lds + g * 2048 + r * 16 + (kSMT + wn * 2) * kTileStepBytes;
    const uint8_t* psa0 = lds + kSScalesOff + wm * 256 + lane * 4;
    const uint8_t* psb0 = lds + kSScalesOff + (kSMT + wn * 2) * 256 + lane * 4;

    f32x16 acc[2];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

    // ---- prologue: STAGES - 1 steps in flight.  Transfers complete in issue order, so "at most 8 k
    // outstanding" means everything but the newest k steps' transfers has landed.
    constexpr int P = STAGES - 1;
#pragma unroll
    for (int d = 0; d < P; ++d)
        if (d < NI) issue_dma(d, d);
    wait_steps_outstanding<P - 1>((NI < P ? NI : P) - 1);
    workgroup_barrier();

    int stage = 0;
    for (int it = 0; it < NI; ++it) {
        // refill the stage consumed in the previous step (free since the barrier that ended it)
        if (it + P < NI) issue_dma(it + P, stage >= 1 ? stage - 1 : STAGES - 1);
        const uint8_t* pa = pa0 + stage * kSStageBytes;
        const uint8_t* pb = pb0 + stage * kSStageBytes;
        const uint32_t sa = *(const uint32_t*)(psa0 + stage * kSStageBytes);
        const uint32_t sb0 = *(const uint32_t*)(psb0 + stage * kSStageBytes);
        const uint32_t sb1 = *(const uint32_t*)(psb0 + stage * kSStageBytes + 256);
        u32x4 fa[4], fb0[4], fb1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            fa[q] = *(const u32x4*)(pa + q * 512);
            fb0[q] = *(const u32x4*)(pb + q * 512);
            fb1[q] = *(const u32x4*)(pb + 4096 + q * 512);
        }
        DUQPP_MFMA(acc[0], fa[0], fb0[0], sa, sb0, 0);
        DUQPP_MFMA(acc[1], fa[0], fb1[0], sa, sb1, 0);
        DUQPP_MFMA(acc[0], fa[1], fb0[1], sa, sb0, 1);
        DUQPP_MFMA(acc[1], fa[1], fb1[1], sa, sb1, 1);
        DUQPP_MFMA(acc[0], fa[2], fb0[2], sa, sb0, 2);
        DUQPP_MFMA(acc[1], fa[2], fb1[2], sa, sb1, 2);
        DUQPP_MFMA(acc[0], fa[3], fb0[3], sa, sb0, 3);
        DUQPP_MFMA(acc[1], fa[3], fb1[3], sa, sb1, 3);
        if (it + 1 < NI) {
            // the next step's stage has landed for this wave (the steps issued after it may be outstanding),
            // then for all; and every wave is done reading this step's stage before the next step refills it.
            // (Reading the next step's operands under the second half of these MFMAs, from a second register
            // set, measured 20 % slower.)
            const int last_issued = it + P < NI ? it + P : NI - 1;
            wait_steps_outstanding<P - 1>(last_issued - (it + 1));
            workgroup_barrier();
        }
        stage = stage + 1 == STAGES ? 0 : stage + 1;
    }

    // ---- epilogue: acc[j][e] of lane (r, g) is row 8 (e / 4) + 4 g + e % 4, column 32 j + r of the wave's tile
    const int m0 = tile_m * kSBM + wm * 32, n0 = tile_n * kSBN + wn * 64;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = n0 + 32 * j + r;
        if (col >= p.N) continue;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int row = m0 + 8 * (e / 4) + 4 * g + (e % 4);
            if (row < p.T) {
                if (OUT_BF16) ((uint16_t*)p.y)[(int64_t)row * p.ldy + col] = f32_to_bf16_rne(acc[j][e]);
                else ((float*)p.y)[(int64_t)row * p.ldy + col] = acc[j][e];
            }
        }
    }
}

constexpr int kSLdsBytes = kSStages * kSStageBytes;

hipError_t setup_gemm_tiled_small() {
    static PerDeviceOnce once;
    return once.run([] {
        hipError_t e = allow_dynamic_lds((const void*)gemm_tiled_small_kernel<true, kSStages>, kSLdsBytes);
        if (e != hipSuccess) return e;
        return allow_dynamic_lds((const void*)gemm_tiled_small_kernel<false, kSStages>, kSLdsBytes);
    });
}

hipError_t launch_gemm_tiled_small(const TiledGemmParams& p, hipStream_t stream) {
    hipError_t e = setup_gemm_tiled_small();
    if (e != hipSuccess) return e;
    const int tiles_m = (p.T + kSBM - 1) / kSBM, tiles_n = (p.N + kSBN - 1) / kSBN;
    dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    return p.out_bf16 ? launch(gemm_tiled_small_kernel<true, kSStages>, grid, block, kSLdsBytes, stream, p)
                      : launch(gemm_tiled_small_kernel<false, kSStages>, grid, block, kSLdsBytes, stream, p);
}

}  // namespace duqpp
