// Rotate + MXFP4-quantise kernel (the online X -> Q(X . R^) of the paper's Eq. 5 / Remark 2,
// with Q from Eq. 2), hand-written for gfx950.
//
// Mapping.  One wavefront owns two adjacent 32-channel blocks and walks down 32-token tiles.
// The 32x32 rotation of a tile runs on the matrix cores as  Y^T = R^T . X^T  with
// v_mfma_f32_32x32x16_bf16: the A operand is R^T (M = output channel), the B operand is the
// token tile (N = token), so the 32 rotated channels of one token land in just two lanes
// (l and l^32), which makes the group amax one cross-lane step.
// fp32 accuracy on bf16 matrix cores: X is bf16 already; each fp32 entry of R is split
// exactly into three bf16 pieces (8 + 8 + 8 significant bits), so every product is exact in
// fp32 and only the fp32 accumulation order differs from a plain fp32 dot product.
// The quantiser uses the hardware E2M1 convert (v_cvt_scalef32_pk_fp4_f32), which rounds to
// nearest even, saturates at 6, keeps the sign of zero and divides by the power of two held
// in the exponent field of its scale operand (field 0 meaning 2^-127).
#include "duqpp_internal.h"

namespace duqpp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kRotqWaves = 8;              // wavefronts per workgroup
constexpr int kBlocksPerWave = 2;
constexpr int kBlocksPerWG = kRotqWaves * kBlocksPerWave;

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

// acc[i] of lane (t = lane & 31, h) is y[token t][channel 8 (i / 4) + 4 h + i % 4] of one block.
__device__ __forceinline__ f32x16 rotate_tile(const RotOperand& op, const uint4 xv[2]) {
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

// Eq. 2 on one token's 32 values spread over lanes l and l^32 (16 each, layout of rotate_tile).
// Returns the E8M0 byte; `out` receives this lane's 8 bytes of the group's 16 code bytes
// (h = 0: bytes 0..7, h = 1: bytes 8..15).
__device__ __forceinline__ uint32_t quantize_group(const f32x16& acc, uint2& out) {
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) m = fmaxf(m, fabsf(acc[i]));
    m = fmaxf(m, __shfl_xor(m, 32));
    // floor(log2 amax) - 2 from the exponent field; fields 0..2 (amax < 2^-124) clamp to 2^-127
    uint32_t ef = __float_as_uint(m) >> 23;
    uint32_t byte = (ef > 2u ? ef : 2u) - 2u;
    float sc = __uint_as_float(byte << 23);
    uint32_t p0 = 0, p1 = 0;
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[0], acc[1], sc, 0);
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[2], acc[3], sc, 1);
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[4], acc[5], sc, 2);
    p0 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p0, acc[6], acc[7], sc, 3);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[8], acc[9], sc, 0);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[10], acc[11], sc, 1);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[12], acc[13], sc, 2);
    p1 = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p1, acc[14], acc[15], sc, 3);
    // p0 = code bytes {2h, 2h+1, 4+2h, 5+2h}, p1 = {8+2h, 9+2h, 12+2h, 13+2h}.
    // Swap p0 of the upper half-wave with p1 of the lower: h = 0 then holds both p0s, h = 1 both p1s.
    auto sw = __builtin_amdgcn_permlane32_swap(p0, p1, false, false);
    uint32_t a = sw[0], b = sw[1];        // a: from h = 0, b: from h = 1
    out.x = (a & 0xFFFFu) | (b << 16);
    out.y = (a >> 16) | (b & 0xFFFF0000u);
    return byte;
}

__device__ __forceinline__ void logical_workgroup(int& logical) {
    // Workgroups are dealt round-robin to the 8 XCDs; renumber so that each XCD gets a
    // contiguous range (same column chunk -> same R blocks and output lines in one L2).
    int id = blockIdx.x, n = gridDim.x;
    int per = n / kNumXCD, rem = n % kNumXCD;
    int xcd = id % kNumXCD, slot = id / kNumXCD;
    logical = xcd * per + (xcd < rem ? xcd : rem) + slot;
}

__global__ __launch_bounds__(kRotqWaves * 64) void rotq_kernel(RotqParams p) {
    int logical;
    logical_workgroup(logical);
    const int chunk = logical / p.ngroups;
    const int tg = logical % p.ngroups;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int c = lane & 31, h = lane >> 5;

    const int j0 = (chunk * kRotqWaves + wave) * kBlocksPerWave;
    if (j0 >= p.G) return;
    const bool two = (j0 + 1) < p.G;
    const int j1 = two ? j0 + 1 : j0;

    const int tile0 = tg * p.tiles_per_wg;
    int tile1 = tile0 + p.tiles_per_wg;
    if (tile1 > p.ntiles) tile1 = p.ntiles;
    if (tile0 >= tile1) return;

    const int last_row = p.rows - 1;
    const int64_t Kh = (int64_t)p.G * 16;   // code bytes per row

    // first tile's activations go out before the R blocks are fetched and split
    uint4 xn[2][2];
    {
        int row = tile0 * 32 + c;
        if (row > last_row) row = last_row;
        const uint16_t* xr = p.x + (int64_t)row * p.ldx + 8 * h;
        xn[0][0] = *(const uint4*)(xr + 32 * j0);
        xn[0][1] = *(const uint4*)(xr + 32 * j0 + 16);
        xn[1][0] = *(const uint4*)(xr + 32 * j1);
        xn[1][1] = *(const uint4*)(xr + 32 * j1 + 16);
    }
    RotOperand op0, op1;
    load_rot_operand(p.R + (int64_t)j0 * p.r_stride, c, h, op0);
    load_rot_operand(p.R + (int64_t)j1 * p.r_stride, c, h, op1);

    for (int tile = tile0; tile < tile1; ++tile) {
        uint4 xc[2][2] = {{xn[0][0], xn[0][1]}, {xn[1][0], xn[1][1]}};
        if (tile + 1 < tile1) {
            int row = (tile + 1) * 32 + c;
            if (row > last_row) row = last_row;
            const uint16_t* xr = p.x + (int64_t)row * p.ldx + 8 * h;
            xn[0][0] = *(const uint4*)(xr + 32 * j0);
            xn[0][1] = *(const uint4*)(xr + 32 * j0 + 16);
            xn[1][0] = *(const uint4*)(xr + 32 * j1);
            xn[1][1] = *(const uint4*)(xr + 32 * j1 + 16);
        }
        f32x16 acc0 = rotate_tile(op0, xc[0]);
        f32x16 acc1 = rotate_tile(op1, xc[1]);
        uint2 o0, o1;
        uint32_t byte0 = quantize_group(acc0, o0);
        uint32_t byte1 = quantize_group(acc1, o1);

        const int row = tile * 32 + c;
        if (row <= last_row) {
            uint8_t* cr = p.codes + (int64_t)row * Kh + 8 * h;
            *(uint2*)(cr + 16 * j0) = o0;
            if (two) *(uint2*)(cr + 16 * j1) = o1;
            // lower half-wave writes block j0's scale, upper half-wave block j1's
            if (h == 0) p.scales[(int64_t)row * p.G + j0] = (uint8_t)byte0;
            else if (two) p.scales[(int64_t)row * p.G + j1] = (uint8_t)byte1;
            if (p.ydbg) {
                float* yr = p.ydbg + (int64_t)row * p.G * 32 + 4 * h;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    *(float4*)(yr + 32 * j0 + 8 * q) = make_float4(acc0[4 * q], acc0[4 * q + 1], acc0[4 * q + 2], acc0[4 * q + 3]);
                    if (two) *(float4*)(yr + 32 * j1 + 8 * q) = make_float4(acc1[4 * q], acc1[4 * q + 1], acc1[4 * q + 2], acc1[4 * q + 3]);
                }
            }
        }
    }
}

void plan_rotq(RotqParams& p) {
    p.ntiles = (p.rows + 31) / 32;
    p.nchunks = (p.G + kBlocksPerWG - 1) / kBlocksPerWG;
    // Aim for one resident round: about 4 workgroups of 8 waves per CU.
    const int64_t slots = (int64_t)kNumCU * 4;
    int64_t units = (int64_t)p.ntiles * p.nchunks;
    int tpw = (int)((units + slots - 1) / slots);
    if (tpw < 1) tpw = 1;
    p.tiles_per_wg = tpw;
    p.ngroups = (p.ntiles + tpw - 1) / tpw;
}

hipError_t launch_rotq(const RotqParams& p, hipStream_t stream) {
    dim3 grid((unsigned)((int64_t)p.nchunks * p.ngroups)), block(kRotqWaves * 64);
    hipLaunchKernelGGL(rotq_kernel, grid, block, 0, stream, p);
    return hipGetLastError();
}

// Test-only: the same quantize_group on fp32 values read from memory in the accumulator layout.
__global__ __launch_bounds__(64) void quant_dbg_kernel(QuantDbgParams p) {
    const int lane = threadIdx.x, c = lane & 31, h = lane >> 5;
    const int j = blockIdx.x;
    const int row = blockIdx.y * 32 + c;
    const int rl = row < p.rows ? row : p.rows - 1;
    const float* yr = p.y + (int64_t)rl * p.ldy + 32 * j + 4 * h;
    f32x16 acc;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        float4 v = *(const float4*)(yr + 8 * q);
        acc[4 * q] = v.x; acc[4 * q + 1] = v.y; acc[4 * q + 2] = v.z; acc[4 * q + 3] = v.w;
    }
    uint2 o;
    uint32_t byte = quantize_group(acc, o);
    if (row < p.rows) {
        *(uint2*)(p.codes + (int64_t)row * p.G * 16 + 16 * j + 8 * h) = o;
        if (h == 0) p.scales[(int64_t)row * p.G + j] = (uint8_t)byte;
    }
}

hipError_t launch_quant_dbg(const QuantDbgParams& p, hipStream_t stream) {
    dim3 grid((unsigned)p.G, (unsigned)((p.rows + 31) / 32)), block(64);
    hipLaunchKernelGGL(quant_dbg_kernel, grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace duqpp
