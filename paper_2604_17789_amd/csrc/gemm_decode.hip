// Decode-shape W4A4 MXFP4 GEMM (Eq. 5 with a handful of tokens): T <= 128, so the activations are one to
// four row tiles (MT = 1 or 2 per workgroup, one or two passes over the weights along blockIdx.y) and the
// product is bound by streaming the weights from HBM (N * K * 17/32 bytes).  Tiled operand layout, same instruction and K permutation as the prefill kernel.
//
// One workgroup of 8 waves per ROWS = 32 or 16 output channels of a weight row tile: the streaming rate
// a single CU sustains is a small fraction of the chip's, so the launch wants at least one workgroup per
// CU, and with fewer row tiles than CUs each tile is cut into 2 workgroups.  With more than 16 tokens such a
// workgroup still issues the 32-row instruction; its lanes r >= ROWS re-read rows 0..15 and their results are dropped
// (up to 16 tokens: gemm_decode16_kernel below, on the 16-row instruction).  The waves split K: each owns a
// contiguous range of K steps, loads its weight fragments straight from global memory into registers
// (512 contiguous bytes per half-wave and load, every byte read once chip-wide), its activation
// fragments from the L2-resident activation tile, and accumulates one 32 x 32 tile.  The eight
// partial tiles are then summed through LDS in a fixed order (deterministic) and the first T rows
// are stored.
#include "duqpp_internal.h"
#include "mxfp4_device.h"

namespace duqpp {

constexpr int kDecWaves = 8;

#define DUQPP_DEC_MFMA(ACC, A, B, SA, SB, SEL) \
    ACC = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fp4_operand(A), fp4_operand(B), ACC, 4, 4, SEL, (int)(SA), SEL, (int)(SB))

template <int MT>
struct DecStep {
    u32x4 a[MT][4], b[4];
    uint32_t sa[MT], sb;
};

// One K step's fragments.  No lane is switched off: a branch around a load makes the compiler wait for every
// outstanding load at the join (s_waitcnt vmcnt(0)), i.e. for the step just requested as well as for the one about
// to be multiplied, and the two steps in flight collapse into one.  Lanes without a token of their own re-read
// row 0 of the first activation tile (a_off / a_soff of such a lane point there): the same cache lines as lane 0, so
// no extra traffic -- fetching all 32 rows of a tile that holds a handful of tokens would be more traffic into the CU
// than the weights -- and their results fall on tokens >= T and are never stored.  Likewise the lanes beyond a
// half-tile workgroup's 16 rows re-read rows 0..15 (lane_code_b is built from r % ROWS).
template <int ROWS, int MT>
__device__ __forceinline__ void dec_load(DecStep<MT>& d, const uint8_t* a_codes, const uint8_t* a_scales,
                                         const int64_t (&a_off)[MT], const int64_t (&a_soff)[MT],
                                         const uint8_t* b_codes, const uint8_t* b_scales, int step, int lane_code_b,
                                         int lane4_b) {
    const uint8_t* pb = b_codes + (int64_t)step * 4096 + lane_code_b;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const uint8_t* pa = a_codes + a_off[m] + (int64_t)step * 4096;
#pragma unroll
        for (int i = 0; i < 4; ++i) d.a[m][i] = *(const u32x4*)(pa + i * 512);
        d.sa[m] = *(const uint32_t*)(a_scales + a_soff[m] + (int64_t)step * 256);
    }
    // weights are read once
#pragma unroll
    for (int i = 0; i < 4; ++i) d.b[i] = __builtin_nontemporal_load((const u32x4*)(pb + i * 512));
    d.sb = *(const uint32_t*)(b_scales + (int64_t)step * 256 + lane4_b);
}

template <bool OUT_BF16, int ROWS, int MT>
__global__ __launch_bounds__(kDecWaves * 64) void gemm_decode_kernel(TiledGemmParams p) {
    static_assert(ROWS == 32 || ROWS == 16, "a row tile is cut into 1 or 2 workgroups");
    __shared__ float part[kDecWaves][16][64];              // [wave][accumulator register][lane]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = lane & 31, g = lane >> 5;
    constexpr int kCuts = 32 / ROWS;
    const int rt = blockIdx.x / kCuts;                     // weight row tile
    const int rb = (blockIdx.x % kCuts) * ROWS + (r & (ROWS - 1));   // row of the tile lane r < ROWS supplies
    const int NI = p.GP / 8;
    const int per = (NI + kDecWaves - 1) / kDecWaves;
    const int s0 = wave * per;
    int s1 = s0 + per;
    if (s1 > NI) s1 = NI;

    const uint8_t* b_codes = p.b_codes + (int64_t)rt * p.GP * 512;
    const uint8_t* b_scales = p.b_scales + (int64_t)rt * NI * 256;
    const int64_t a_tile_bytes = (int64_t)p.GP * 512, a_tile_sbytes = (int64_t)NI * 256;
    // this workgroup's activation row tiles: MT of them from m0; one past the last tile is all zeros
    // (its results fall on tokens >= T and are dropped)
    const int RTa = (p.T + 31) / 32;
    const int m0 = blockIdx.y * MT;
    // A operand (activations): group 4 g + i of row r sits at (4 g + i) * 512 + r * 16, its scale word at
    // (32 g + r) * 4; B operand (weights): the same with row rb
    const int lane_code = g * 2048 + r * 16, lane_code_b = g * 2048 + rb * 16;
    const int lane4 = lane * 4, lane4_b = (g * 32 + rb) * 4;
    // per activation row tile: this lane's token row, or row 0 of the first tile when it has none
    int64_t a_off[MT], a_soff[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int mt = m0 + m;
        const bool own = mt < RTa && r < p.T - 32 * mt;
        a_off[m] = own ? mt * a_tile_bytes + lane_code : (int64_t)g * 2048;
        a_soff[m] = own ? mt * a_tile_sbytes + lane4 : (int64_t)g * 128;
    }

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[m][e] = 0.f;

    // The loads of step s + 1 are issued before the MFMAs of step s.
    auto mfmas = [&](const DecStep<MT>& d) {
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            DUQPP_DEC_MFMA(acc[m], d.a[m][0], d.b[0], d.sa[m], d.sb, 0);
            DUQPP_DEC_MFMA(acc[m], d.a[m][1], d.b[1], d.sa[m], d.sb, 1);
            DUQPP_DEC_MFMA(acc[m], d.a[m][2], d.b[2], d.sa[m], d.sb, 2);
            DUQPP_DEC_MFMA(acc[m], d.a[m][3], d.b[3], d.sa[m], d.sb, 3);
        }
    };
    if constexpr (ROWS == 32 && MT == 1) {
        // Whole row tiles, one activation tile: a wave has few steps (two at K = 4096), and the plain loop measured
        // 1-4 % faster than the two-set form below (8192 x 8192, T = 32: 8.7 against 9.0 us).
        if (s0 < s1) {
            DecStep<MT> cur, nxt;
            dec_load<ROWS, MT>(cur, p.a_codes, p.a_scales, a_off, a_soff, b_codes, b_scales, s0, lane_code_b, lane4_b);
            for (int s = s0; s < s1; ++s) {
                if (s + 1 < s1)
                    dec_load<ROWS, MT>(nxt, p.a_codes, p.a_scales, a_off, a_soff, b_codes, b_scales, s + 1, lane_code_b, lane4_b);
                mfmas(cur);
                cur = nxt;
            }
        }
    } else if (s0 < s1) {
        // Two register sets taking turns, two steps per round and no branch in the round: with a branch around a
        // load, or a copy from one set to the other, the compiler's wait covers the loads just issued as well and
        // only one step is ever in flight (N = 4096, K = 14336, T = 64: 13.7 -> 12.8 us).
        DecStep<MT> even, odd;
        dec_load<ROWS, MT>(even, p.a_codes, p.a_scales, a_off, a_soff, b_codes, b_scales, s0, lane_code_b, lane4_b);
        int s = s0;
        for (; s + 2 < s1; s += 2) {
            // (the barriers keep the scheduler from gathering all loads of the round at its top, which again ends
            // every round with nothing in flight)
            dec_load<ROWS, MT>(odd, p.a_codes, p.a_scales, a_off, a_soff, b_codes, b_scales, s + 1, lane_code_b, lane4_b);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(even);
            __builtin_amdgcn_sched_barrier(0);
            dec_load<ROWS, MT>(even, p.a_codes, p.a_scales, a_off, a_soff, b_codes, b_scales, s + 2, lane_code_b, lane4_b);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(odd);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (s + 1 < s1) {
            dec_load<ROWS, MT>(odd, p.a_codes, p.a_scales, a_off, a_soff, b_codes, b_scales, s + 1, lane_code_b, lane4_b);
            mfmas(even);
            mfmas(odd);
        } else {
            mfmas(even);
        }
    }
    // per activation row tile: the eight partial tiles through LDS, summed in a fixed order
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        if (m > 0) __syncthreads();                        // the previous tile's partials have been read
#pragma unroll
        for (int e = 0; e < 16; ++e) part[wave][e][lane] = acc[m][e];
        __syncthreads();
        // acc[e] of lane (r, g): token 32 (m0 + m) + 8 (e / 4) + 4 g + e % 4, output channel 32 rt + rb (lanes r < ROWS).
        // 1024 outputs, 512 threads: thread t sums register e = t / 64 and e + 8 of lane t % 64 over the waves.
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int e = (threadIdx.x >> 6) + 8 * h;
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < kDecWaves; ++w) sum += part[w][e][lane];
            const int tok = 32 * (m0 + m) + 8 * (e / 4) + 4 * g + (e % 4);
            const int col = rt * 32 + rb;
            if (r < ROWS && tok < p.T && col < p.N) {
                if (OUT_BF16) ((uint16_t*)p.y)[(int64_t)tok * p.ldy + col] = f32_to_bf16_rne(sum);
                else ((float*)p.y)[(int64_t)tok * p.ldy + col] = sum;
            }
        }
    }
}

// ---- Up to 16 tokens against fewer weight row tiles than CUs: half row tiles on the 16 x 16 x 128 instruction.
// A row tile is cut into two workgroups of 16 output channels, as above, but here every lane loads: lane
// (c, g) = (lane % 16, lane / 16) supplies group 4 q + g of channel c for MFMA q = 0, 1 of a K step (a wave-level load is
// four runs of 256 contiguous bytes), and token lane % 16 in the same way on the activation side, so a half-tile
// workgroup moves as many bytes per load instruction as a whole-tile one.  The lane's scale byte is the one of its own
// group, fetched as a byte, and the instruction's byte select is 0.  acc[i] of lane (c, g) is token 4 g + i, channel c.
typedef float f32x4 __attribute__((ext_vector_type(4)));

struct Dec16Step {
    u32x4 a[2], b[2];
    uint32_t sa[2], sb[2];
};

__device__ __forceinline__ void dec16_load(Dec16Step& d, const uint8_t* a_codes, const uint8_t* a_scales,
                                           const uint8_t* b_codes, const uint8_t* b_scales, int step, int off_a,
                                           int soff_a, int off_b, int soff_b) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        d.a[q] = *(const u32x4*)(a_codes + (int64_t)step * 4096 + q * 2048 + off_a);
        d.sa[q] = a_scales[(int64_t)step * 256 + q * 128 + soff_a];
        d.b[q] = __builtin_nontemporal_load((const u32x4*)(b_codes + (int64_t)step * 4096 + q * 2048 + off_b));
        d.sb[q] = b_scales[(int64_t)step * 256 + q * 128 + soff_b];
    }
}

template <bool OUT_BF16>
__global__ __launch_bounds__(kDecWaves * 64) void gemm_decode16_kernel(TiledGemmParams p) {
    __shared__ float part[kDecWaves][4][64];               // [wave][accumulator register][lane]
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int rt = blockIdx.x >> 1;                        // weight row tile
    const int rb = (blockIdx.x & 1) * 16 + c;              // row of the tile this lane supplies
    const int NI = p.GP / 8;
    const int per = (NI + kDecWaves - 1) / kDecWaves;
    const int s0 = wave * per;
    int s1 = s0 + per;
    if (s1 > NI) s1 = NI;
    const uint8_t* b_codes = p.b_codes + (int64_t)rt * p.GP * 512;
    const uint8_t* b_scales = p.b_scales + (int64_t)rt * NI * 256;
    // group 4 q + g of row r of a step: codes at (4 q + g) * 512 + r * 16, scale byte at q * 128 + r * 4 + g
    // (lanes without a token re-read token 0: no branch around a load, no extra cache line; their results are tokens >= T)
    const int ca = c < p.T ? c : 0;
    const int off_a = g * 512 + ca * 16, soff_a = ca * 4 + g;
    const int off_b = g * 512 + rb * 16, soff_b = rb * 4 + g;

    f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    auto mfmas = [&](const Dec16Step& d) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
            acc[q] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fp4_operand(d.a[q]), fp4_operand(d.b[q]), acc[q],
                                                                      4, 4, 0, (int)d.sa[q], 0, (int)d.sb[q]);
    };
    if (s0 < s1) {                                         // two register sets taking turns, as above
        Dec16Step even, odd;
        dec16_load(even, p.a_codes, p.a_scales, b_codes, b_scales, s0, off_a, soff_a, off_b, soff_b);
        int s = s0;
        for (; s + 2 < s1; s += 2) {
            dec16_load(odd, p.a_codes, p.a_scales, b_codes, b_scales, s + 1, off_a, soff_a, off_b, soff_b);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(even);
            __builtin_amdgcn_sched_barrier(0);
            dec16_load(even, p.a_codes, p.a_scales, b_codes, b_scales, s + 2, off_a, soff_a, off_b, soff_b);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(odd);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (s + 1 < s1) {
            dec16_load(odd, p.a_codes, p.a_scales, b_codes, b_scales, s + 1, off_a, soff_a, off_b, soff_b);
            mfmas(even);
            mfmas(odd);
        } else {
            mfmas(even);
        }
    }
    // the eight waves' partial tiles (two each) through LDS, summed in a fixed order
#pragma unroll
    for (int i = 0; i < 4; ++i) part[wave][i][lane] = acc[0][i] + acc[1][i];
    __syncthreads();
    if (threadIdx.x < 256) {
        const int i = threadIdx.x >> 6;                    // `lane` is threadIdx.x % 64 here as well
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kDecWaves; ++w) sum += part[w][i][lane];
        const int tok = 4 * g + i, col = rt * 32 + rb;
        if (tok < p.T && col < p.N) {
            if (OUT_BF16) ((uint16_t*)p.y)[(int64_t)tok * p.ldy + col] = f32_to_bf16_rne(sum);
            else ((float*)p.y)[(int64_t)tok * p.ldy + col] = sum;
        }
    }
}

template <int ROWS, int MT>
static hipError_t launch_decode_rows(const TiledGemmParams& p, unsigned tiles, unsigned passes, hipStream_t stream) {
    dim3 grid(tiles * (32 / ROWS), passes), block(kDecWaves * 64);
    return p.out_bf16 ? launch(gemm_decode_kernel<true, ROWS, MT>, grid, block, 0, stream, p)
                      : launch(gemm_decode_kernel<false, ROWS, MT>, grid, block, 0, stream, p);
}

hipError_t launch_gemm_decode(const TiledGemmParams& p, hipStream_t stream) {
    if (p.T > kDecodeMaxT) return hipErrorInvalidValue;
    const unsigned tiles = (unsigned)((p.N + 31) / 32);
    // Fewer row tiles than CUs: half tiles, twice the workgroups (N = 4096, K = 14336, T = 32: 9.6 us; whole tiles on
    // half the CUs are slower from 9 tokens on).  Quartering the tiles, 16 waves per workgroup or register rings three
    // and four steps deep all lost when they were measured.
    // Up to 16 tokens and fewer row tiles than CUs: half tiles on the 16 x 16 x 128 instruction, whose loads are whole
    // (N = 4096, K = 14336: T = 1 9.0 -> 7.1 us, T = 16 9.1 -> 7.9 us; N = K = 4096: 4.3 -> 3.7 us).
    if (p.T <= 16 && tiles < (unsigned)kNumCU) {
        dim3 grid(tiles * 2), block(kDecWaves * 64);
        return p.out_bf16 ? launch(gemm_decode16_kernel<true>, grid, block, 0, stream, p)
                          : launch(gemm_decode16_kernel<false>, grid, block, 0, stream, p);
    }
    const bool cut = tiles < (unsigned)kNumCU;              // (more than 16 tokens here)
    // 65..128 tokens: two passes of two row tiles each (blockIdx.y), the weights of the second mostly from cache
    const unsigned passes = p.T <= 64 ? 1u : 2u;
    if (p.T <= 32) return cut ? launch_decode_rows<16, 1>(p, tiles, passes, stream) : launch_decode_rows<32, 1>(p, tiles, passes, stream);
    return cut ? launch_decode_rows<16, 2>(p, tiles, passes, stream) : launch_decode_rows<32, 2>(p, tiles, passes, stream);
}

}  // namespace duqpp
