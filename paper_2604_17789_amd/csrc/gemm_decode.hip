// Decode-shape W4A4 MXFP4 GEMM (Eq. 5 with a handful of tokens): T <= 128, so the activations are one to
// four row tiles (MT = 1 or 2 per workgroup, one or two passes over the weights along blockIdx.y) and the
// product is bound by streaming the weights from HBM (N * K * 17/32 bytes).  Tiled operand layout, same instruction and K permutation as the prefill kernel.
//
// One workgroup of 8 waves per ROWS = 32 or 16 output channels of a weight row tile: the streaming rate
// a single CU sustains is a small fraction of the chip's, so the launch wants at least one workgroup per
// CU, and with fewer row tiles than CUs each tile is cut into 2 workgroups.  Such a workgroup still issues the
// 32-row instruction; its lanes r >= ROWS load nothing, feed zeros, and their results are dropped.  The waves split K: each owns a
// contiguous range of K steps, loads its weight fragments straight from global memory into registers
// (512 contiguous bytes per half-wave and load, every byte read once chip-wide), its activation
// fragments from the L2-resident activation tile, and accumulates one 32 x 32 tile.  The eight
// partial tiles are then summed through LDS in a fixed order (deterministic) and the first T rows
// are stored.
#include "duqpp_internal.h"

namespace duqpp {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kDecWaves = 8;

__device__ __forceinline__ i32x8 dec_fp4_operand(const u32x4& v) {
    i32x8 r = {(int)v[0], (int)v[1], (int)v[2], (int)v[3], 0, 0, 0, 0};
    return r;
}

#define DUQPP_DEC_MFMA(ACC, A, B, SA, SB, SEL) \
    ACC = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(dec_fp4_operand(A), dec_fp4_operand(B), ACC, 4, 4, SEL, (int)(SA), SEL, (int)(SB))

template <int MT>
struct DecStep {
    u32x4 a[MT][4], b[4];
    uint32_t sa[MT], sb;
};

// a_tile_bytes / a_tile_sbytes: distance between the activations' row tiles (codes / scale words)
template <int ROWS, int MT>
__device__ __forceinline__ void dec_load(DecStep<MT>& d, const uint8_t* a_codes, const uint8_t* a_scales,
                                         int64_t a_tile_bytes, int64_t a_tile_sbytes, int m0, int rta, int T,
                                         const uint8_t* b_codes, const uint8_t* b_scales, int step, int lane_code,
                                         int lane4, int lane_code_b, int lane4_b, int r) {
    const uint8_t* pb = b_codes + (int64_t)step * 4096 + lane_code_b;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        // Only the lanes of real tokens fetch activations: every workgroup reads the whole activation tile from
        // L2, which with a handful of tokens would otherwise be more traffic per CU than the weights themselves
        // (32 rows of mostly padding against ROWS rows of weights).  The other lanes feed zeros; their results
        // fall on tokens >= T and are dropped.
        const int mt = m0 + m;
        if (mt < rta && r < T - 32 * mt) {
            const uint8_t* pa = a_codes + mt * a_tile_bytes + (int64_t)step * 4096 + lane_code;
#pragma unroll
            for (int i = 0; i < 4; ++i) d.a[m][i] = *(const u32x4*)(pa + i * 512);
            d.sa[m] = *(const uint32_t*)(a_scales + mt * a_tile_sbytes + (int64_t)step * 256 + lane4);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) d.a[m][i] = u32x4{0u, 0u, 0u, 0u};
            d.sa[m] = 0x7F7F7F7Fu;
        }
    }
    // weights are read once; lanes beyond the workgroup's rows load nothing and feed zeros
    if (ROWS == 32 || r < ROWS) {
#pragma unroll
        for (int i = 0; i < 4; ++i) d.b[i] = __builtin_nontemporal_load((const u32x4*)(pb + i * 512));
        d.sb = *(const uint32_t*)(b_scales + (int64_t)step * 256 + lane4_b);
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) d.b[i] = u32x4{0u, 0u, 0u, 0u};
        d.sb = 0x7F7F7F7Fu;
    }
}

__device__ __forceinline__ uint16_t dec_f32_to_bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
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

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[m][e] = 0.f;

    // two steps in flight per wave: the loads of step s + 1 are issued before the MFMAs of step s.
    // (Deeper register rings measured slower: they cost the occupancy that hides the latency better.)
    DecStep<MT> cur, nxt;
    if (s0 < s1)
        dec_load<ROWS, MT>(cur, p.a_codes, p.a_scales, a_tile_bytes, a_tile_sbytes, m0, RTa, p.T, b_codes, b_scales, s0, lane_code,
                           lane4, lane_code_b, lane4_b, r);
    for (int s = s0; s < s1; ++s) {
        if (s + 1 < s1)
            dec_load<ROWS, MT>(nxt, p.a_codes, p.a_scales, a_tile_bytes, a_tile_sbytes, m0, RTa, p.T, b_codes, b_scales, s + 1,
                               lane_code, lane4, lane_code_b, lane4_b, r);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            DUQPP_DEC_MFMA(acc[m], cur.a[m][0], cur.b[0], cur.sa[m], cur.sb, 0);
            DUQPP_DEC_MFMA(acc[m], cur.a[m][1], cur.b[1], cur.sa[m], cur.sb, 1);
            DUQPP_DEC_MFMA(acc[m], cur.a[m][2], cur.b[2], cur.sa[m], cur.sb, 2);
            DUQPP_DEC_MFMA(acc[m], cur.a[m][3], cur.b[3], cur.sa[m], cur.sb, 3);
        }
        cur = nxt;
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
                if (OUT_BF16) ((uint16_t*)p.y)[(int64_t)tok * p.ldy + col] = dec_f32_to_bf16_rne(sum);
                else ((float*)p.y)[(int64_t)tok * p.ldy + col] = sum;
            }
        }
    }
}

template <int ROWS, int MT>
static void launch_decode_rows(const TiledGemmParams& p, unsigned tiles, unsigned passes, hipStream_t stream) {
    dim3 grid(tiles * (32 / ROWS), passes), block(kDecWaves * 64);
    if (p.out_bf16) hipLaunchKernelGGL((gemm_decode_kernel<true, ROWS, MT>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((gemm_decode_kernel<false, ROWS, MT>), grid, block, 0, stream, p);
}

hipError_t launch_gemm_decode(const TiledGemmParams& p, hipStream_t stream) {
    if (p.T > kDecodeMaxT) return hipErrorInvalidValue;
    const unsigned tiles = (unsigned)((p.N + 31) / 32);
    // Measured at N = 4096, K = 14336: with more than a few tokens halving the row tiles (256 workgroups instead
    // of 128) gains 4 % (T = 16: 9.4 -> 9.0 us); with up to 8 tokens whole tiles win (T = 1: 8.8 -> 8.6 us), as a
    // half-tile workgroup issues the same loads for half the bytes (K = 4096, N = 14336 forced to half tiles:
    // 7.1 -> 9.6 us).  Quartering the tiles, 16 waves per workgroup or register rings three and four steps deep
    // all lose.
    const bool cut = tiles < (unsigned)kNumCU && p.T > 8;
    // 65..128 tokens: two passes of two row tiles each (blockIdx.y), the weights of the second mostly from cache
    const unsigned passes = p.T <= 64 ? 1u : 2u;
    if (p.T <= 32) {
        if (cut) launch_decode_rows<16, 1>(p, tiles, passes, stream);
        else launch_decode_rows<32, 1>(p, tiles, passes, stream);
    } else {
        if (cut) launch_decode_rows<16, 2>(p, tiles, passes, stream);
        else launch_decode_rows<32, 2>(p, tiles, passes, stream);
    }
    return hipGetLastError();
}

}  // namespace duqpp
