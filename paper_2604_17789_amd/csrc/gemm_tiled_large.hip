// W4A4 MXFP4 GEMM (Eq. 5) on 256 x 256 output tiles, for shapes with enough of them to occupy the chip.
//
// Why a second tiling.  With 128 x 256 tiles (gemm_tiled.hip) a CU moves 52 KiB from L2 into LDS and reads
// 96 KiB back out of LDS for every 1024 matrix-core cycles; both rates are close to what the path from L2
// (about 32 B per clock and CU on this access pattern) and the LDS (128 B per clock) deliver, and on real
// operands every byte moved beside the MFMAs lowers the rate the chip sustains (measured: the transfers cost
// 17 % of the 128 x 256 kernel's time, the fragment reads 4-5 %).  A wave tile of 128 x 128 instead of 64 x 128
// reuses every fragment twice as often: per 1024 matrix-core cycles the CU moves 34 KiB in and reads 64 KiB out.
//
// Shape of the kernel
//   workgroup  4 waves (one per SIMD) as 2 x 2, output tile 256 x 256; each wave owns 128 x 128 = 4 x 4 MFMA
//              tiles = 256 fp32 accumulators per lane (the whole accumulation half of the register file).
//   K loop     steps of 128 (4 MXFP4 groups): 16 row tiles x 2 KiB of codes and 16 x 128 B of scale words per
//              step, moved by LDS-DMA into one of four stages; three steps are in flight while one is
//              consumed.
//   operands   lane (r, g) feeds group 2 g + i of row r to MFMA i (i = 0, 1) of a step: one ds_read_b128 at
//              (2 g + i) * 512 + r * 16 of the row tile's 2 KiB.  Its scale bytes are bytes 2 g + i of the row's
//              scale word of that step: each half-wave reads its own 16 bits of the word, and the byte select
//              of the instruction is i for every lane.
// K is a summation index: the order in which groups meet the instruction only changes the order of the fp32
// additions.
#include <type_traits>

#include "duqpp_internal.h"
#include "gemm_tiled_common.h"

namespace duqpp {
namespace large {

constexpr int kBM = 256, kBN = 256;
constexpr int kMT = kBM / 32, kNT = kBN / 32;            // row tiles of A / B per workgroup
constexpr int kStepBytes = 4 * 512;                      // codes of one row tile for one K step (4 groups)
constexpr int kCodesBytes = (kMT + kNT) * kStepBytes;    // 32 KiB
constexpr int kScalesBytes = (kMT + kNT) * 128;          // one word per row and step
constexpr int kStageBytes = kCodesBytes + kScalesBytes;  // 34 KiB
constexpr int kStages = 4;
constexpr int kEpPitch = 144;                            // 64 bf16 of a row + 16 bytes, so that rows 4 apart differ in bank
constexpr int kEpBytes = 32 * kEpPitch;                  // per-wave scratch of the bf16 transpose
constexpr int kEpOff = kStages * kStageBytes;
constexpr int kLdsBytes = kEpOff + 4 * kEpBytes;         // 157696 of the CU's 163840
constexpr int kDmaOps = 10;                              // transfers per wave per step: 8 x 1 KiB of codes, 2 x 256 B of scales
constexpr int kGroupM = 8;                               // M tiles per group in the workgroup ordering

struct Frags {
    u32x4 a[4], b[4];
};
struct Scales {
    uint32_t a[4], b[4];
};

template <bool OUT_BF16>
__global__ __launch_bounds__(256) void gemm_tiled_large_kernel(TiledGemmParams p) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    const int tiles_m = (p.T + kBM - 1) / kBM, tiles_n = (p.N + kBN - 1) / kBN;
    const int total = tiles_m * tiles_n;
    const int RTa = (p.T + 31) / 32, RTb = (p.N + 31) / 32;
    const int NI = p.GP / 4;                               // K steps per tile
    const int64_t tile_bytes = (int64_t)p.GP * 512;        // codes of one row tile
    const int64_t tile_sbytes = (int64_t)p.GP * 32;        // scale words of one row tile

    // ---- which output tiles: as in the 128 x 256 kernel, one persistent workgroup per CU, XCD-contiguous
    // renumbering, tiles grouped kGroupM M-tiles x N so that the workgroups of an L2 share operand rows
    const int nwg = gridDim.x;                             // <= total
    int slot;
    {
        const int id = blockIdx.x;
        const int per = nwg / kNumXCD, rem = nwg % kNumXCD;
        const int xcd = id % kNumXCD, sl = id / kNumXCD;
        slot = xcd * per + (xcd < rem ? xcd : rem) + sl;
    }
    const int nt = (total - 1 - slot) / nwg + 1;           // tiles of this workgroup
    const int S = nt * NI;                                 // its K steps, all tiles in a row
    auto tile_of = [&](int j, int& tile_m, int& tile_n) {
        const int pid = j * nwg + slot;
        const int group_sz = kGroupM * tiles_n;
        const int first_m = (pid / group_sz) * kGroupM;
        const int gm = (tiles_m - first_m) < kGroupM ? (tiles_m - first_m) : kGroupM;
        tile_m = first_m + (pid % group_sz) % gm;
        tile_n = (pid % group_sz) / gm;
    };

    // ---- LDS-DMA duty of wave w per step: row tiles 4 w .. 4 w + 3 of the stage's 16 (0..7: A, 8..15: B),
    // 2 KiB of codes each, and their scale words (two transfers of 64 words: lanes 0..31 one row tile, lanes
    // 32..63 the next).
    const uint8_t* csrc[4];
    const uint8_t* ssrc[2];
    uint32_t cdst[4], sdst[2];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const void*)lds);
#pragma unroll
    for (int k = 0; k < 4; ++k) cdst[k] = lds0 + (wave * 4 + k) * kStepBytes;
#pragma unroll
    for (int x = 0; x < 2; ++x) sdst[x] = lds0 + kCodesBytes + (wave * 4 + 2 * x) * 128;
    auto operand_tile = [&](int tq, int tile_m, int tile_n, const uint8_t*& codes, const uint8_t*& scales) {
        if (tq < kMT) {
            int rt = tile_m * kMT + tq;
            if (rt >= RTa) rt = RTa - 1;                   // ragged M: any valid tile, its rows are never stored
            codes = p.a_codes + rt * tile_bytes;
            scales = p.a_scales + rt * tile_sbytes;
        } else {
            int rt = tile_n * kNT + (tq - kMT);
            if (rt >= RTb) rt = RTb - 1;
            codes = p.b_codes + rt * tile_bytes;
            scales = p.b_scales + rt * tile_sbytes;
        }
    };
    auto set_dma_tile = [&](int j) {
        int tile_m, tile_n;
        tile_of(j, tile_m, tile_n);
        const uint8_t *c, *s;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            operand_tile(wave * 4 + k, tile_m, tile_n, c, s);
            csrc[k] = c + lane * 16;
        }
#pragma unroll
        for (int x = 0; x < 2; ++x) {
            operand_tile(wave * 4 + 2 * x + (lane >> 5), tile_m, tile_n, c, s);
            ssrc[x] = s + (lane & 31) * 4;
        }
    };
    // The transfers run three steps ahead of the MFMAs and carry on into the workgroup's next tile while the
    // current one finishes.  Past the last step of the run the sources stay where they are: the last step is
    // transferred again, into stages that nobody reads any more, so every step issues and awaits the same
    // number of transfers and one loop body serves all of them.
    int dma_j = 0, dma_it = 0;                             // tile and step within it that the sources point at
    int dma_left = S - 1;                                  // steps after that one
    set_dma_tile(0);
    auto advance_dma = [&]() {
        if (dma_left == 0) return;
        --dma_left;
#pragma unroll
        for (int k = 0; k < 4; ++k) csrc[k] += kStepBytes;
#pragma unroll
        for (int x = 0; x < 2; ++x) ssrc[x] += 128;
        if (++dma_it == NI) {
            dma_it = 0;
            set_dma_tile(++dma_j);
        }
    };
    auto issue_dma = [&](int stage) {
        const uint32_t so = stage * kStageBytes;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            dma_1k_at<0>(csrc[k], cdst[k] + so);
            dma_1k_at<1024>(csrc[k], cdst[k] + so);
        }
        dma_256(ssrc[0], sdst[0] + so);
        dma_256(ssrc[1], sdst[1] + so);
        advance_dma();
    };

    // ---- LDS read addresses of lane (r, g): codes of group 2 g + i of row r at (2 g + i) * 512 + r * 16 of a
    // row tile; scale bytes of groups 2 g, 2 g + 1 of row r at r * 4 + 2 g of the row tile's 128 bytes (read as 16 bits:
    // the byte select of MFMA i is then i for every lane)
    const uint8_t* pa0 = lds + (wm * 4) * kStepBytes + g * 1024 + r * 16;
    const uint8_t* pb0 = lds + (kMT + wn * 4) * kStepBytes + g * 1024 + r * 16;
    const uint8_t* psa0 = lds + kCodesBytes + (wm * 4) * 128 + r * 4 + g * 2;
    const uint8_t* psb0 = lds + kCodesBytes + (kMT + wn * 4) * 128 + r * 4 + g * 2;

    // ---- prologue: three steps in flight; transfers complete in issue order, so "at most 2 kDmaOps
    // outstanding" means all but the two newest steps' transfers have landed
    issue_dma(0);
    issue_dma(1);
    issue_dma(2);
    wait_vmcnt<2 * kDmaOps>();
    workgroup_barrier();
    Frags f0, f1;
    Scales scs[2];                                         // scale bytes of the current / next step, swapped by parity
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        f0.a[t] = *(const u32x4*)(pa0 + t * kStepBytes);
        f0.b[t] = *(const u32x4*)(pb0 + t * kStepBytes);
        scs[0].a[t] = *(const uint16_t*)(psa0 + t * 128);
        scs[0].b[t] = *(const uint16_t*)(psb0 + t * 128);
    }

    int stage = 0;                                         // stage of the step to compute next
    for (int j = 0; j < nt; ++j) {                         // ---- one output tile per iteration
    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

    // One K step.  PAR: parity of the step within the tile (every tile has an even number of steps); the step's
    // scale bytes are in scs[PAR] and it reads the next step's into scs[PAR ^ 1], so nothing is copied between steps.
    auto step = [&](int stage, auto par_c) {
        constexpr int PAR = decltype(par_c)::value;
        Scales& sc = scs[PAR];
        Scales& sn = scs[PAR ^ 1];
        const int stage1 = (stage + 1) & (kStages - 1);
        const int stage3 = (stage + 3) & (kStages - 1);
        const uint8_t* pa = pa0 + stage * kStageBytes;
        const uint8_t* pb = pb0 + stage * kStageBytes;
        const uint32_t so3 = stage3 * kStageBytes;
        // transfer k of the ten that refill the stage consumed in the previous step (every wave has passed the
        // barrier that followed its last read of it)
        auto dma_slot = [&](auto kc) {
            constexpr int k = decltype(kc)::value;
            if constexpr (k < 8) dma_1k_at<(k % 2) * 1024>(csrc[k / 2], cdst[k / 2] + so3);
            else dma_256(ssrc[k - 8], sdst[k - 8] + so3);
        };
#define DUQPP_PIN __builtin_amdgcn_sched_barrier(0)
#define DUQPP_DMA(K) dma_slot(std::integral_constant<int, K>{}); DUQPP_PIN
        // four MFMAs of one row of tile pairs, left to the scheduler (the group barriers below place them)
#define DUQPP_ROW_FREE(F, I, SEL, J0, J1, J2, J3)                            \
        DUQPP_MFMA(acc[I][J0], F.a[I], F.b[J0], sc.a[I], sc.b[J0], SEL);   \
        DUQPP_MFMA(acc[I][J1], F.a[I], F.b[J1], sc.a[I], sc.b[J1], SEL);   \
        DUQPP_MFMA(acc[I][J2], F.a[I], F.b[J2], sc.a[I], sc.b[J2], SEL);   \
        DUQPP_MFMA(acc[I][J3], F.a[I], F.b[J3], sc.a[I], sc.b[J3], SEL)
        // ---- first half: groups 2 g of every row tile; the fragments of the second half are read meanwhile
        f1.a[0] = *(const u32x4*)(pa + 512);
        f1.b[0] = *(const u32x4*)(pb + 512);
        DUQPP_PIN;
        DUQPP_MFMA(acc[0][0], f0.a[0], f0.b[0], sc.a[0], sc.b[0], 0); DUQPP_PIN;
        f1.b[1] = *(const u32x4*)(pb + kStepBytes + 512); DUQPP_PIN;
        DUQPP_MFMA(acc[0][1], f0.a[0], f0.b[1], sc.a[0], sc.b[1], 0); DUQPP_PIN;
        f1.b[2] = *(const u32x4*)(pb + 2 * kStepBytes + 512); DUQPP_PIN;
        DUQPP_MFMA(acc[0][2], f0.a[0], f0.b[2], sc.a[0], sc.b[2], 0); DUQPP_PIN;
        f1.b[3] = *(const u32x4*)(pb + 3 * kStepBytes + 512); DUQPP_PIN;
        DUQPP_MFMA(acc[0][3], f0.a[0], f0.b[3], sc.a[0], sc.b[3], 0); DUQPP_PIN;
        f1.a[1] = *(const u32x4*)(pa + kStepBytes + 512); DUQPP_PIN;
        DUQPP_MFMA(acc[1][3], f0.a[1], f0.b[3], sc.a[1], sc.b[3], 0); DUQPP_PIN;
        f1.a[2] = *(const u32x4*)(pa + 2 * kStepBytes + 512); DUQPP_PIN;
        DUQPP_MFMA(acc[1][2], f0.a[1], f0.b[2], sc.a[1], sc.b[2], 0); DUQPP_PIN;
        f1.a[3] = *(const u32x4*)(pa + 3 * kStepBytes + 512); DUQPP_PIN;
        DUQPP_MFMA(acc[1][1], f0.a[1], f0.b[1], sc.a[1], sc.b[1], 0); DUQPP_PIN;
        DUQPP_DMA(0);
        DUQPP_MFMA(acc[1][0], f0.a[1], f0.b[0], sc.a[1], sc.b[0], 0); DUQPP_PIN;
        DUQPP_MFMA(acc[2][0], f0.a[2], f0.b[0], sc.a[2], sc.b[0], 0); DUQPP_PIN;
        DUQPP_DMA(1);
        DUQPP_MFMA(acc[2][1], f0.a[2], f0.b[1], sc.a[2], sc.b[1], 0); DUQPP_PIN;
        DUQPP_MFMA(acc[2][2], f0.a[2], f0.b[2], sc.a[2], sc.b[2], 0); DUQPP_PIN;
        DUQPP_DMA(2);
        DUQPP_MFMA(acc[2][3], f0.a[2], f0.b[3], sc.a[2], sc.b[3], 0); DUQPP_PIN;
        DUQPP_MFMA(acc[3][3], f0.a[3], f0.b[3], sc.a[3], sc.b[3], 0); DUQPP_PIN;
        DUQPP_DMA(3);
        DUQPP_MFMA(acc[3][2], f0.a[3], f0.b[2], sc.a[3], sc.b[2], 0); DUQPP_PIN;
        DUQPP_MFMA(acc[3][1], f0.a[3], f0.b[1], sc.a[3], sc.b[1], 0); DUQPP_PIN;
        DUQPP_DMA(4);
        DUQPP_MFMA(acc[3][0], f0.a[3], f0.b[0], sc.a[3], sc.b[0], 0); DUQPP_PIN;
        // ---- second half: groups 2 g + 1; the remaining transfers, then the next step's first fragments
        DUQPP_MFMA(acc[0][0], f1.a[0], f1.b[0], sc.a[0], sc.b[0], 1); DUQPP_PIN;
        DUQPP_DMA(5);
        DUQPP_MFMA(acc[0][1], f1.a[0], f1.b[1], sc.a[0], sc.b[1], 1); DUQPP_PIN;
        DUQPP_MFMA(acc[0][2], f1.a[0], f1.b[2], sc.a[0], sc.b[2], 1); DUQPP_PIN;
        DUQPP_DMA(6);
        DUQPP_MFMA(acc[0][3], f1.a[0], f1.b[3], sc.a[0], sc.b[3], 1); DUQPP_PIN;
        DUQPP_MFMA(acc[1][3], f1.a[1], f1.b[3], sc.a[1], sc.b[3], 1); DUQPP_PIN;
        DUQPP_DMA(7);
        DUQPP_MFMA(acc[1][2], f1.a[1], f1.b[2], sc.a[1], sc.b[2], 1); DUQPP_PIN;
        DUQPP_DMA(8);
        DUQPP_MFMA(acc[1][1], f1.a[1], f1.b[1], sc.a[1], sc.b[1], 1); DUQPP_PIN;
        DUQPP_DMA(9);
        DUQPP_MFMA(acc[1][0], f1.a[1], f1.b[0], sc.a[1], sc.b[0], 1); DUQPP_PIN;
        advance_dma();
        {
            // the next step has landed for this wave, then for all; every LDS read of the current stage has
            // been issued and has returned before any later transfer can touch it
            wait_vmcnt<2 * kDmaOps>();
            workgroup_barrier();
            const uint8_t* na = pa0 + stage1 * kStageBytes;
            const uint8_t* nb = pb0 + stage1 * kStageBytes;
            const uint8_t* nsa = psa0 + stage1 * kStageBytes;
            const uint8_t* nsb = psb0 + stage1 * kStageBytes;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                f0.a[t] = *(const u32x4*)(na + t * kStepBytes);
                f0.b[t] = *(const u32x4*)(nb + t * kStepBytes);
                sn.a[t] = *(const uint16_t*)(nsa + t * 128);
                sn.b[t] = *(const uint16_t*)(nsb + t * 128);
            }
        }
        DUQPP_ROW_FREE(f1, 2, 1, 0, 1, 2, 3);
        DUQPP_ROW_FREE(f1, 3, 1, 3, 2, 1, 0);
        // the 16 reads above, two at a time ahead of each of the eight MFMAs
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        DUQPP_PIN;
#undef DUQPP_ROW_FREE
#undef DUQPP_DMA
#undef DUQPP_PIN
    };

    // ---- a finished tile: acc[i][jj][e] of lane (r, g) is row 32 i + 8 (e / 4) + 4 g + e % 4, column 32 jj + r
    // of the wave's 128 x 128.  The scratch of the bf16 transpose is a region of its own, private to the wave.
    auto store_tile = [&](int j) {
        int tile_m, tile_n;
        tile_of(j, tile_m, tile_n);
        const int m0 = tile_m * kBM + wm * 128, n0 = tile_n * kBN + wn * 128;
        if constexpr (OUT_BF16) {
            // Each 32 x 64 piece of the wave's tile is transposed through LDS and leaves as 16-byte pieces,
            // 128 contiguous bytes per row (a direct store would write 2 bytes per lane).  The launch code
            // sends only 16-byte aligned outputs with N % 8 == 0 here, so a piece is inside or outside as a whole.
            uint8_t* ep = lds + kEpOff + wave * kEpBytes;
            uint8_t* wp = ep + (4 * g) * kEpPitch + r * 2;                 // this lane's column in the scratch
            const uint8_t* rp = ep + (lane >> 3) * kEpPitch + (lane & 7) * 16;   // its 16-byte piece of rows lane / 8 + 8 k
            const int gcol = n0 + (lane & 7) * 8;
            uint16_t* dst0 = (uint16_t*)p.y + (int64_t)(m0 + (lane >> 3)) * p.ldy + gcol;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int hh = 0; hh < 2; ++hh) {
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                        for (int e = 0; e < 16; e += 2) {
                            // rows 8 (e / 4) + 4 g + e % 4 and the next one: the two halves of one packed convert
                            const f32x2 v = {acc[i][2 * hh + jj][e], acc[i][2 * hh + jj][e + 1]};
                            const bf16x2 b = __builtin_convertvector(v, bf16x2);
                            const uint32_t u = __builtin_bit_cast(uint32_t, b);
                            uint8_t* q = wp + (8 * (e / 4) + (e % 4)) * kEpPitch + 64 * jj;
                            *(uint16_t*)q = (uint16_t)u;
                            *(uint16_t*)(q + kEpPitch) = (uint16_t)(u >> 16);
                        }
                    // same wave wrote and reads: program order suffices within a wave
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const u32x4 v = *(const u32x4*)(rp + 8 * k * kEpPitch);
                        const int grow = m0 + 32 * i + 8 * k + (lane >> 3);
                        if (grow < p.T && gcol + 64 * hh < p.N)
                            // streamed: the result is not read again here, the operands' lines are (2-3 % at T = 8192)
                            __builtin_nontemporal_store(v, (u32x4*)(dst0 + (int64_t)(32 * i + 8 * k) * p.ldy + 64 * hh));
                    }
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    const int col = n0 + 32 * jj + r;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int row = m0 + 32 * i + 8 * (e / 4) + 4 * g + (e % 4);
                        if (row < p.T && col < p.N) ((float*)p.y)[(int64_t)row * p.ldy + col] = acc[i][jj][e];
                    }
                }
        }
    };

    // Steps of this tile, in pairs of opposite parity.
    for (int it = 0; it < NI; it += 2) {
        step(stage, std::integral_constant<int, 0>{});
        stage = (stage + 1) & (kStages - 1);
        step(stage, std::integral_constant<int, 1>{});
        stage = (stage + 1) & (kStages - 1);
    }
    store_tile(j);
    }                                                      // ---- tile loop
    wait_vmcnt<0>();                                       // the surplus transfers of the last steps
}

}  // namespace large

// bf16 outputs leave as 16-byte pieces: the output must be 16-byte aligned with N and ldy multiples of 8
bool gemm_tiled_large_accepts(const TiledGemmParams& p) {
    if (!p.out_bf16) return true;
    return (reinterpret_cast<uintptr_t>(p.y) & 15) == 0 && (p.ldy % 8) == 0 && (p.N % 8) == 0;
}

hipError_t setup_gemm_tiled_large() {
    using namespace large;
    static PerDeviceOnce once;
    return once.run([] {
        hipError_t e = allow_dynamic_lds((const void*)gemm_tiled_large_kernel<true>, kLdsBytes);
        if (e != hipSuccess) return e;
        return allow_dynamic_lds((const void*)gemm_tiled_large_kernel<false>, kLdsBytes);
    });
}

hipError_t launch_gemm_tiled_large(const TiledGemmParams& p, hipStream_t stream) {
    using namespace large;
    if (!gemm_tiled_large_accepts(p)) return hipErrorInvalidValue;
    hipError_t e = setup_gemm_tiled_large();
    if (e != hipSuccess) return e;
    const int tiles_m = (p.T + kBM - 1) / kBM, tiles_n = (p.N + kBN - 1) / kBN;
    const int total = tiles_m * tiles_n;
    dim3 grid((unsigned)(total < kNumCU ? total : kNumCU)), block(256);
    return p.out_bf16 ? launch(gemm_tiled_large_kernel<true>, grid, block, kLdsBytes, stream, p)
                      : launch(gemm_tiled_large_kernel<false>, grid, block, kLdsBytes, stream, p);
}

}  // namespace duqpp
