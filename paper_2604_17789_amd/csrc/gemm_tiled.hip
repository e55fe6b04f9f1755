// W4A4 MXFP4 GEMM (the Q(X^) . Q(W^) product of the paper's Eq. 5) for operands in the tiled
// layout, on gfx950's block-scaled matrix cores (v_mfma_scale_f32_32x32x64_f8f6f4, FP4 x FP4).
//
// Shape of the kernel
//   workgroup  4 waves (one per SIMD) as 2 x 2, output tile 128 (tokens) x 256 (output channels);
//              each wave owns 64 x 128 = 2 x 4 MFMA tiles = 128 fp32 accumulators per lane.
//   tiles      one workgroup per CU walks its output tiles one after the other; the operand transfers of the
//              next tile start while the current one finishes, so only the store of a tile interrupts the
//              matrix cores, not the refill of the pipeline.
//   K loop     steps of 256 (8 MXFP4 groups).  The codes of a step, (4 + 8) row tiles x 4 KiB, and
//              their scale words, 12 x 256 B, go from global memory straight into LDS by LDS-DMA
//              (each code transfer moves one contiguous KiB); three such stages rotate, two in
//              flight while one is consumed.
//   operands   in the tiled layout the 16 code bytes of (row r, group j) of a row tile sit at
//              (j * 32 + r) * 16, so the FP4 operand of lane (r, g) for MFMA i of a step -- group
//              4 g + i of row r -- is one ds_read_b128 and 32 lanes read 512 contiguous bytes.
//   scales     lane (r, g) needs the four E8M0 bytes of groups 4 g .. 4 g + 3: one 32-bit word,
//              stored lane-linear per (row tile, step); the four MFMAs of a step select bytes
//              0..3 of it.
// K is a summation index, so feeding groups to the instruction in this permuted order changes
// nothing but the order of the fp32 additions.
//
// The LDS-DMA transfers are issued from asm statements and their completion is awaited by hand
// (s_waitcnt vmcnt before the workgroup barrier): were they visible to the compiler as LDS writes, it
// would drain the whole DMA queue before every LDS read it cannot disambiguate, i.e. serialise the
// pipeline.  No other vector-memory load is issued inside the K loop, so the compiler places no
// vmcnt wait of its own there; LDS reads and MFMAs are ordinary code with compiler-managed waits.
#include <type_traits>

#include "duqpp_internal.h"
#include "gemm_tiled_common.h"

namespace duqpp {

constexpr int kBM = 128, kBN = 256;
constexpr int kMT = kBM / 32, kNT = kBN / 32;           // row tiles of A / B per workgroup
constexpr int kStageBytes = (kMT + kNT) * kTileStepBytes + 4 * 1024;   // codes + scale words
constexpr int kStages = 3;
constexpr int kGemmLdsBytes = kStages * kStageBytes;    // 159744 of the CU's 163840
constexpr int kGroupM = 8;                              // M tiles per group in the workgroup ordering: an XCD's 32 workgroups form an 8 x 4 block (1024 x 1024 outputs), the shape with the fewest operand rows

constexpr int kScaleRegionBytes = 4 * 1024;               // 12 x 256 B of scale words + 1 KiB of padding
constexpr int kScalesOff = (kMT + kNT) * kTileStepBytes;  // scale words follow the codes in a stage

struct Frags {
    u32x4 a[2], b[4];
};

struct Scales {
    uint32_t a[2], b[4];
};

// the eight MFMAs of one quarter step: groups 4 g + SEL of every row tile pair, in an order that changes one
// operand at a time (the second row runs backwards): operands that switch cost matrix-core time
#define DUQPP_MFMA8(F, S, SEL)                                    \
    DUQPP_MFMA(acc[0][0], F.a[0], F.b[0], S.a[0], S.b[0], SEL);   \
    DUQPP_MFMA(acc[0][1], F.a[0], F.b[1], S.a[0], S.b[1], SEL);   \
    DUQPP_MFMA(acc[0][2], F.a[0], F.b[2], S.a[0], S.b[2], SEL);   \
    DUQPP_MFMA(acc[0][3], F.a[0], F.b[3], S.a[0], S.b[3], SEL);   \
    DUQPP_MFMA(acc[1][3], F.a[1], F.b[3], S.a[1], S.b[3], SEL);   \
    DUQPP_MFMA(acc[1][2], F.a[1], F.b[2], S.a[1], S.b[2], SEL);   \
    DUQPP_MFMA(acc[1][1], F.a[1], F.b[1], S.a[1], S.b[1], SEL);   \
    DUQPP_MFMA(acc[1][0], F.a[1], F.b[0], S.a[1], S.b[0], SEL)

// fragments of quarter Q of the stage whose per-lane base addresses are pa (A tiles) and pb (B tiles)
template <int Q>
__device__ __forceinline__ void read_frags(Frags& f, const uint8_t* pa, const uint8_t* pb) {
    f.a[0] = *(const u32x4*)(pa + Q * 512);
    f.a[1] = *(const u32x4*)(pa + 4096 + Q * 512);
    f.b[0] = *(const u32x4*)(pb + Q * 512);
    f.b[1] = *(const u32x4*)(pb + 4096 + Q * 512);
    f.b[2] = *(const u32x4*)(pb + 8192 + Q * 512);
    f.b[3] = *(const u32x4*)(pb + 12288 + Q * 512);
}

template <bool OUT_BF16>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(TiledGemmParams p) {
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 31, g = lane >> 5;
    const int wm = wave >> 1, wn = wave & 1;

    const int tiles_m = (p.T + kBM - 1) / kBM, tiles_n = (p.N + kBN - 1) / kBN;
    const int total = tiles_m * tiles_n;
    const int RTa = (p.T + 31) / 32, RTb = (p.N + 31) / 32;
    const int NI = p.GP / 8;                               // K steps per tile
    const int64_t tile_bytes = (int64_t)p.GP * 512;        // codes of one row tile
    const int64_t tile_sbytes = (int64_t)NI * 256;         // scale words of one row tile

    // ---- which output tiles.  The launch has at most one workgroup per CU; workgroup `slot` takes tiles
    // slot, slot + nwg, ...  Within each such round the workgroups are renumbered so that an XCD holds a
    // contiguous range, and tile numbers run through groups of kGroupM M-tiles swept along N, so that the
    // 32 workgroups sharing an L2 cover a compact block of the output.
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

    // ---- LDS-DMA duty of this wave per step: three whole row tiles of codes (12 transfers of 1 KiB)
    // and one KiB of scale words (the words of four row tiles; wave 3 has only padding to move, which
    // keeps the number of transfers per wave uniform for the waits below).  The transfers run two steps
    // ahead of the MFMAs and carry on into the workgroup's next tile while the current one finishes.
    const uint8_t* dma_src[3];                             // this lane's source of the step to transfer next
    const uint8_t* sdma_src;
    uint32_t dma_dst[3];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) const void*)lds);
#pragma unroll
    for (int k = 0; k < 3; ++k) dma_dst[k] = lds0 + (wave * 3 + k) * kTileStepBytes;
    const uint32_t sdma_dst = lds0 + kScalesOff + wave * 1024;
    auto set_dma_tile = [&](int j) {
        int tile_m, tile_n;
        tile_of(j, tile_m, tile_n);
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const int tq = wave * 3 + k;                   // 0..3: A row tiles, 4..11: B row tiles
            const uint8_t* base;
            if (tq < kMT) {
                int rt = tile_m * kMT + tq;
                if (rt >= RTa) rt = RTa - 1;               // ragged M: any valid tile, its rows are never stored
                base = p.a_codes + rt * tile_bytes;
            } else {
                int rt = tile_n * kNT + (tq - kMT);
                if (rt >= RTb) rt = RTb - 1;
                base = p.b_codes + rt * tile_bytes;
            }
            dma_src[k] = base + lane * 16;
        }
        // scale words: lane l of wave w moves 16 bytes = the words of lanes 4 (l % 16) .. + 3 of row tile
        // 4 w + l / 16 (tiles 0..3: A, 4..11: B, 12..15: none -- wave 3 re-reads tile 11 into the padding)
        int tq = wave * 4 + (lane >> 4);
        if (tq > kMT + kNT - 1) tq = kMT + kNT - 1;
        const uint8_t* base;
        if (tq < kMT) {
            int rt = tile_m * kMT + tq;
            if (rt >= RTa) rt = RTa - 1;
            base = p.a_scales + rt * tile_sbytes;
        } else {
            int rt = tile_n * kNT + (tq - kMT);
            if (rt >= RTb) rt = RTb - 1;
            base = p.b_scales + rt * tile_sbytes;
        }
        sdma_src = base + (lane & 15) * 16;
    };
    int dma_j = 0, dma_it = 0;                             // tile and step within it that the sources point at
    set_dma_tile(0);
    auto advance_dma = [&]() {
#pragma unroll
        for (int k = 0; k < 3; ++k) dma_src[k] += kTileStepBytes;
        sdma_src += 256;
        if (++dma_it == NI) {
            dma_it = 0;
            if (++dma_j < nt) set_dma_tile(dma_j);
        }
    };
    constexpr int kDmaOps = 13;                            // transfers per wave per step
    auto issue_dma = [&](int stage) {
        const uint32_t so = stage * kStageBytes;
#pragma unroll
        for (int k = 0; k < 3; ++k) dma_4k(dma_src[k], dma_dst[k] + so);
        dma_1k(sdma_src, sdma_dst + so);
        advance_dma();
    };

    // ---- LDS read addresses: lane (r, g) reads group 4 g + i of row r at (4 g + i) * 512 + r * 16;
    // its scale word of row tile t at kScalesOff + t * 256 + lane * 4
    const uint8_t* pa0 = lds + g * 2048 + r * 16 + (wm * 2) * kTileStepBytes;
    const uint8_t* pb0 = lds + g * 2048 + r * 16 + (kMT + wn * 4) * kTileStepBytes;
    const uint8_t* psa0 = lds + kScalesOff + (wm * 2) * 256 + lane * 4;
    const uint8_t* psb0 = lds + kScalesOff + (kMT + wn * 4) * 256 + lane * 4;
    auto read_scales = [&](Scales& s, int stage) {
        const uint8_t* qa = psa0 + stage * kStageBytes;
        const uint8_t* qb = psb0 + stage * kStageBytes;
        s.a[0] = *(const uint32_t*)(qa);
        s.a[1] = *(const uint32_t*)(qa + 256);
        s.b[0] = *(const uint32_t*)(qb);
        s.b[1] = *(const uint32_t*)(qb + 256);
        s.b[2] = *(const uint32_t*)(qb + 512);
        s.b[3] = *(const uint32_t*)(qb + 768);
    };

    // ---- prologue: the first two stages.  Transfers complete in issue order, so "at most 13
    // outstanding" means everything but the newest step's transfers has landed.
    issue_dma(0);
    if (S > 1) {
        issue_dma(1);
        wait_vmcnt<kDmaOps>();
    } else {
        wait_vmcnt<0>();
    }
    workgroup_barrier();
    Frags f0, f1;
    Scales sc, sn;
    read_frags<0>(f0, pa0, pb0);
    read_scales(sc, 0);
    sn = sc;

    int stage = 0;                                         // stage of the step to compute next
    for (int j = 0; j < nt; ++j) {                         // ---- one output tile per iteration
    // The accumulators live and die inside one iteration: nothing but the transfer pipeline, the stage
    // counter and the prefetched fragments of the next step is carried from tile to tile.
    f32x16 acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

    // One K step.  MORE1 / MORE2: a next step / a step after that exists (in this tile or the next).
    auto step = [&](int stage, auto more1_c, auto more2_c) {
        constexpr bool MORE1 = decltype(more1_c)::value, MORE2 = decltype(more2_c)::value;
        const int stage1 = stage + 1 == kStages ? 0 : stage + 1;
        const int stage2 = stage1 + 1 == kStages ? 0 : stage1 + 1;
        // The 13 transfers that refill the stage consumed in the previous step (every wave has passed
        // the barrier that followed its last read of it) are spread over the first three quarters, one
        // every other MFMA: the CU's one texture path moves 64 B/clk, i.e. a step's 52 KiB take 832 of
        // the step's 1024 MFMA cycles, and a wave that issues its transfers in a burst sits behind the
        // other waves' bursts with its MFMAs waiting.
        const uint8_t* d0 = dma_src[0];
        const uint8_t* d1 = dma_src[1];
        const uint8_t* d2 = dma_src[2];
        const uint8_t* d3 = sdma_src;
        const uint32_t so2 = stage2 * kStageBytes;
        auto dma_slot = [&](auto kc) {
            constexpr int k = decltype(kc)::value;
            if constexpr (MORE2) {
                if constexpr (k < 4) dma_1k_at<(k % 4) * 1024>(d0, dma_dst[0] + so2);
                else if constexpr (k < 8) dma_1k_at<(k % 4) * 1024>(d1, dma_dst[1] + so2);
                else if constexpr (k < 12) dma_1k_at<(k % 4) * 1024>(d2, dma_dst[2] + so2);
                else dma_1k_at<0>(d3, sdma_dst + so2);
            }
        };
        const uint8_t* pa = pa0 + stage * kStageBytes;
        const uint8_t* pb = pb0 + stage * kStageBytes;
#define DUQPP_PIN __builtin_amdgcn_sched_barrier(0)
#define DUQPP_DMA(K) dma_slot(std::integral_constant<int, K>{}); DUQPP_PIN
        // quarter Q (fragments CUR) while the fragments of quarter Q + 1 (NXT) are read; D0..D3: transfers
#define DUQPP_QUARTER(Q, CUR, NXT, D0, D1, D2, D3)                                            \
        DUQPP_DMA(D0);                                                                         \
        NXT.a[0] = *(const u32x4*)(pa + (Q + 1) * 512);                                         \
        DUQPP_MFMA(acc[0][0], CUR.a[0], CUR.b[0], sc.a[0], sc.b[0], Q); DUQPP_PIN;              \
        NXT.b[0] = *(const u32x4*)(pb + (Q + 1) * 512);                                         \
        DUQPP_MFMA(acc[0][1], CUR.a[0], CUR.b[1], sc.a[0], sc.b[1], Q); DUQPP_PIN;              \
        DUQPP_DMA(D1);                                                                         \
        NXT.b[1] = *(const u32x4*)(pb + 4096 + (Q + 1) * 512);                                  \
        DUQPP_MFMA(acc[0][2], CUR.a[0], CUR.b[2], sc.a[0], sc.b[2], Q); DUQPP_PIN;              \
        NXT.b[2] = *(const u32x4*)(pb + 8192 + (Q + 1) * 512);                                  \
        DUQPP_MFMA(acc[0][3], CUR.a[0], CUR.b[3], sc.a[0], sc.b[3], Q); DUQPP_PIN;              \
        DUQPP_DMA(D2);                                                                         \
        NXT.b[3] = *(const u32x4*)(pb + 12288 + (Q + 1) * 512);                                 \
        DUQPP_MFMA(acc[1][3], CUR.a[1], CUR.b[3], sc.a[1], sc.b[3], Q); DUQPP_PIN;              \
        NXT.a[1] = *(const u32x4*)(pa + 4096 + (Q + 1) * 512);                                  \
        DUQPP_MFMA(acc[1][2], CUR.a[1], CUR.b[2], sc.a[1], sc.b[2], Q); DUQPP_PIN;              \
        DUQPP_DMA(D3);                                                                         \
        DUQPP_MFMA(acc[1][1], CUR.a[1], CUR.b[1], sc.a[1], sc.b[1], Q);                         \
        DUQPP_MFMA(acc[1][0], CUR.a[1], CUR.b[0], sc.a[1], sc.b[0], Q); DUQPP_PIN
        DUQPP_DMA(12);
        DUQPP_QUARTER(0, f0, f1, 0, 1, 2, 3);
        DUQPP_QUARTER(1, f1, f0, 4, 5, 6, 7);
        DUQPP_QUARTER(2, f0, f1, 8, 9, 10, 11);
#undef DUQPP_QUARTER
#undef DUQPP_DMA
        if constexpr (MORE2) advance_dma();
        if constexpr (MORE1) {
            // next stage landed for this wave, then for all; every LDS read of the current stage has
            // been issued and returns before any later transfer can touch it
            if constexpr (MORE2) wait_vmcnt<kDmaOps>();
            else wait_vmcnt<0>();
            workgroup_barrier();
            read_frags<0>(f0, pa0 + stage1 * kStageBytes, pb0 + stage1 * kStageBytes);
            read_scales(sn, stage1);
        }
        DUQPP_MFMA8(f1, sc, 3);
        if constexpr (MORE1) {
            // the reads above (6 fragments, 3 paired scale reads) two at a time ahead of the MFMAs
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            }
        }
        DUQPP_PIN;
#undef DUQPP_PIN
        sc = sn;
    };

    // ---- a finished tile: acc[i][j][e] of lane (r, g) is row 32 i + 8 (e / 4) + 4 g + e % 4, column 32 j + r.
    // `stage` is the stage the tile's last step consumed: no wave reads it any more (`synced`: they have all
    // passed a barrier since), and the only transfers that will write bytes [12288 w, 12288 (w + 1)) of it are
    // wave w's own, issued later in program order -- so that range is wave w's scratch for the bf16 transpose.
    auto store_tile = [&](int j, int stage, bool synced) {
        int tile_m, tile_n;
        tile_of(j, tile_m, tile_n);
        const int m0 = tile_m * kBM + wm * 64, n0 = tile_n * kBN + wn * 128;
        if constexpr (OUT_BF16) {
            // A direct store would write 2 bytes per lane, 64 contiguous bytes per instruction and row.
            // Instead each 32 x 128 half of the wave's tile is transposed through LDS and leaves as 16-byte
            // pieces, 256 contiguous bytes per row.  Rows are padded to 272 bytes so that the two
            // half-waves (four rows apart) fall on different banks.
            const bool vec_ok = ((reinterpret_cast<uintptr_t>(p.y) & 15) == 0) && (p.ldy % 8) == 0;
            if (vec_ok) {
                constexpr int kRowPitch = 272;
                static_assert(32 * kRowPitch <= 3 * kTileStepBytes, "scratch within the wave's own transfer range");
                if (!synced) workgroup_barrier();
                uint8_t* ep = lds + stage * kStageBytes + wave * (3 * kTileStepBytes);
#pragma unroll
                for (int i = 0; i < 2; ++i) {
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                        for (int e = 0; e < 16; e += 2) {
                            // rows 8 (e / 4) + 4 g + e % 4 and the next one: the two halves of one packed convert
                            const bf16x2 b = __builtin_convertvector((f32x2){acc[i][jj][e], acc[i][jj][e + 1]}, bf16x2);
                            const uint32_t u = __builtin_bit_cast(uint32_t, b);
                            uint8_t* q = ep + (8 * (e / 4) + 4 * g + (e % 4)) * kRowPitch + (32 * jj + r) * 2;
                            *(uint16_t*)q = (uint16_t)u;
                            *(uint16_t*)(q + kRowPitch) = (uint16_t)(u >> 16);
                        }
                    // same wave wrote and reads: program order suffices within a wave
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const int row = k * 4 + (lane >> 4), ch = lane & 15;
                        const int grow = m0 + 32 * i + row, gcol = n0 + ch * 8;
                        const u32x4 v = *(const u32x4*)(ep + row * kRowPitch + ch * 16);
                        if (grow < p.T && gcol < p.N) {
                            uint16_t* dst = (uint16_t*)p.y + (int64_t)grow * p.ldy + gcol;
                            if (gcol + 8 <= p.N) {
                                __builtin_nontemporal_store(v, (u32x4*)dst);   // streamed: keeps the operands' lines in L2 (1-5 % at the LLaMA-3-8B shapes)
                            } else {                       // ragged right edge
                                for (int c = 0; c < 8 && gcol + c < p.N; ++c) dst[c] = (uint16_t)(v[c / 2] >> (16 * (c & 1)));
                            }
                        }
                    }
                }
                return;
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                const int col = n0 + 32 * jj + r;
                if (col >= p.N) continue;
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row = m0 + 32 * i + 8 * (e / 4) + 4 * g + (e % 4);
                    if (row < p.T) {
                        if (OUT_BF16) ((uint16_t*)p.y)[(int64_t)row * p.ldy + col] = f32_to_bf16_rne(acc[i][jj][e]);
                        else ((float*)p.y)[(int64_t)row * p.ldy + col] = acc[i][jj][e];
                    }
                }
            }
    };

    // Steps of this tile.  All but the last two steps of the whole run have two successors.
    const int s0 = j * NI;
    int hot = S - 2 - s0;
    hot = hot < 0 ? 0 : (hot > NI ? NI : hot);
    int it = 0;
    for (; it < hot; ++it) {
        step(stage, std::true_type{}, std::true_type{});
        stage = stage + 1 == kStages ? 0 : stage + 1;
    }
    for (; it < NI; ++it) {
        if (s0 + it + 1 < S) step(stage, std::true_type{}, std::false_type{});
        else step(stage, std::false_type{}, std::false_type{});
        stage = stage + 1 == kStages ? 0 : stage + 1;
    }
    // a step with a successor ends behind a barrier
    store_tile(j, stage == 0 ? kStages - 1 : stage - 1, s0 + NI < S);
    }                                                      // ---- tile loop
}

// 128 x 256 tiles, persistent workgroups, any shape.
hipError_t setup_gemm_tiled_mid() {
    static PerDeviceOnce once;
    return once.run([] {
        hipError_t e = allow_dynamic_lds((const void*)gemm_tiled_kernel<true>, kGemmLdsBytes);
        if (e != hipSuccess) return e;
        return allow_dynamic_lds((const void*)gemm_tiled_kernel<false>, kGemmLdsBytes);
    });
}

hipError_t launch_gemm_tiled_mid(const TiledGemmParams& p, hipStream_t stream) {
    hipError_t e = setup_gemm_tiled_mid();
    if (e != hipSuccess) return e;
    const int tiles_m = (p.T + kBM - 1) / kBM, tiles_n = (p.N + kBN - 1) / kBN;
    // persistent workgroups: the 156 KiB of LDS allow one per CU, and each walks its tiles with the
    // transfer pipeline running across tile boundaries
    const int total = tiles_m * tiles_n;
    dim3 grid((unsigned)(total < kNumCU ? total : kNumCU)), block(256);
    return p.out_bf16 ? launch(gemm_tiled_kernel<true>, grid, block, kGemmLdsBytes, stream, p)
                      : launch(gemm_tiled_kernel<false>, grid, block, kGemmLdsBytes, stream, p);
}

// Which kernel runs a shape.
int choose_gemm_kernel(const TiledGemmParams& p) {
    // Weight-streaming shapes go to the decode kernel: always up to 32 tokens, up to 64 unless the 64 x 128 tiles fill
    // the chip (N beyond about 24 k); from 65 to 128 (two passes
    // over the weights) when that beats the 128 x 256 kernel, which then has at most N / 256 of the 256 CUs busy
    // for GP / 8 steps of about a microsecond.  Times in microseconds, fitted to measurements at the LLaMA-3-8B shapes.
    if (p.T <= 32) return DUQPP_GEMM_KERNEL_DECODE;
    if (p.T <= 64) {
        // Two activation row tiles per wave stream the weights at about 4 TB/s; the 64 x 128 tiles take about 0.8 us
        // per K step of 256 once there are enough of them for every CU, whatever the byte count (N = 28672, K = 8192,
        // T = 48: 27.9 us against 33.9 us; N = 14336, K = 4096: 12.1 us against 11.1 us).
        const double t_decode = 2.5 + (double)p.N * p.GP * 17.0 / 4.0e6;
        const int64_t small_tiles = (int64_t)((p.T + 63) / 64) * ((p.N + 127) / 128);
        const double t_small = 2.5 + 0.8 * (p.GP / 8) * (double)((small_tiles + 2 * kNumCU - 1) / (2 * kNumCU));
        return t_decode <= t_small ? DUQPP_GEMM_KERNEL_DECODE : DUQPP_GEMM_KERNEL_SMALL;
    }
    const int64_t mid_tiles = (int64_t)((p.T + kBM - 1) / kBM) * ((p.N + kBN - 1) / kBN);
    if (p.T <= kDecodeMaxT) {
        const double weight_bytes = (double)p.N * p.GP * 17.0;
        const double t_decode = 2.0 * (2.5 + weight_bytes / 2.8e6);
        const int tiles = (p.N + kBN - 1) / kBN;
        const double t_prefill = 3.0 + 1.05 * (p.GP / 8) * ((tiles + kNumCU - 1) / kNumCU);
        if (t_decode < t_prefill) return DUQPP_GEMM_KERNEL_DECODE;
    }
    // Too few 128 x 256 tiles to occupy the chip: 64 x 128 tiles, four times as many, two workgroups per CU.
    if (mid_tiles < kNumCU / 2) return DUQPP_GEMM_KERNEL_SMALL;
    // 256 x 256 tiles do a flop in about 0.8 of the time of 128 x 256 tiles (less L2 and LDS traffic per flop),
    // i.e. a tile with twice the work costs 1.6 of a 128 x 256 tile: they win when the rounds over the 256 CUs come out
    // cheaper, which needs at least 256 of them or so.
    // (N a multiple of 8 for either output type, so that the fp32 and the bf16 result of a shape come from the same
    // kernel and the second is the rounding of the first.)
    if ((p.N % 8) == 0 && gemm_tiled_large_accepts(p)) {
        const int64_t large_tiles = (int64_t)((p.T + 255) / 256) * ((p.N + 255) / 256);
        const double t_mid = (double)((mid_tiles + kNumCU - 1) / kNumCU);
        const double t_large = 1.6 * (double)((large_tiles + kNumCU - 1) / kNumCU);
        if (t_large < t_mid) return DUQPP_GEMM_KERNEL_LARGE;
    }
    return DUQPP_GEMM_KERNEL_MID;
}

hipError_t launch_gemm_tiled_as(const TiledGemmParams& p, int kernel, hipStream_t stream) {
    switch (kernel) {
        case DUQPP_GEMM_KERNEL_AUTO: return launch_gemm_tiled_as(p, choose_gemm_kernel(p), stream);
        case DUQPP_GEMM_KERNEL_DECODE: return p.T <= kDecodeMaxT ? launch_gemm_decode(p, stream) : hipErrorInvalidValue;
        case DUQPP_GEMM_KERNEL_SMALL: return launch_gemm_tiled_small(p, stream);
        case DUQPP_GEMM_KERNEL_MID: return launch_gemm_tiled_mid(p, stream);
        case DUQPP_GEMM_KERNEL_LARGE: return launch_gemm_tiled_large(p, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm_tiled(const TiledGemmParams& p, hipStream_t stream) {
    return launch_gemm_tiled_as(p, DUQPP_GEMM_KERNEL_AUTO, stream);
}

}  // namespace duqpp
