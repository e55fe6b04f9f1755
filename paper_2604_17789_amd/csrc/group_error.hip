// Per-group normalised quantisation error -- the statistic of Fig. 1 (Sec. 4.1): for every token and every group of
// 32 channels ||Q(y) - y||_2 / ||y||_2, where y is the group after the block rotation of Eq. 4 (or the group itself:
// the figure's "Original" setting) and Q the MXFP4 quantiser of Eq. 2.  An analysis tool beside the hot path: it
// rotates and quantises with the hot path's own device functions (rotq_device.h), so the error it reports is the
// error of the codes the hot path produces.
#include "duqpp_internal.h"
#include "rotq_device.h"

namespace duqpp {

// value of an E2M1 code (sign, two exponent bits, one mantissa bit): 0, 0.5, 1, 1.5, 2, 3, 4, 6
__device__ __forceinline__ double e2m1_value(uint32_t nib) {
    const uint32_t e = (nib >> 1) & 3u, m = nib & 1u;
    const double mag = e == 0u ? 0.5 * m : (1.0 + 0.5 * m) * (double)(1u << (e - 1u));
    return (nib & 8u) ? -mag : mag;
}

// One wave per (tile of 32 tokens, group): lane (c, h) holds 16 of token c's 32 values, as in rotate_tile.
__global__ __launch_bounds__(64) void group_error_kernel(GroupErrorParams p) {
    const int lane = threadIdx.x, c = lane & 31, h = lane >> 5;
    const int j = blockIdx.x;
    const int token = blockIdx.y * 32 + c;
    const int tl = token < p.rows ? token : p.rows - 1;      // rows past the end: a valid row, never stored
    const uint16_t* xr = p.x + (int64_t)tl * p.ldx + 32 * j;
    f32x16 acc;
    if (p.R) {
        RotOperand op;
        load_rot_operand(p.R + (int64_t)j * p.r_stride, c, h, op);
        u32x4 xv[2];
        xv[0] = *(const u32x4*)(xr + 8 * h);
        xv[1] = *(const u32x4*)(xr + 8 * h + 16);
        acc = rotate_tile(op, xv);
    } else {
        // no rotation: acc[i] is channel 8 (i / 4) + 4 h + i % 4 of the group, the layout rotate_tile would give
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint2 v = *(const uint2*)(xr + 8 * q + 4 * h);
            acc[4 * q + 0] = __uint_as_float(v.x << 16);
            acc[4 * q + 1] = __uint_as_float(v.x & 0xFFFF0000u);
            acc[4 * q + 2] = __uint_as_float(v.y << 16);
            acc[4 * q + 3] = __uint_as_float(v.y & 0xFFFF0000u);
        }
    }
    uint32_t p0, p1;
    const uint32_t byte = quantize_lane(acc, p0, p1);
    // 2^(byte - 127) as a double (the fp32 form of 2^-127 would be subnormal)
    const double scale = __longlong_as_double((long long)(byte + 896u) << 52);
    double num = 0.0, den = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const uint32_t nib = ((i < 8 ? p0 : p1) >> (4 * (i & 7))) & 15u;
        const double y = (double)acc[i];
        const double d = e2m1_value(nib) * scale - y;
        num += d * d;
        den += y * y;
    }
    num += __shfl_xor(num, 32);
    den += __shfl_xor(den, 32);
    if (h == 0 && token < p.rows) p.err[(int64_t)token * p.G + j] = den > 0.0 ? (float)sqrt(num / den) : -1.0f;
}

// Mean of the ratios over the groups that have one (err >= 0), summed in a fixed order: thread t takes elements
// t, t + 1024, ..., then a tree over the 1024 partial sums.
__global__ __launch_bounds__(1024) void group_error_mean_kernel(GroupErrorMeanParams p) {
    const float* err = p.err;
    const int64_t n = p.n;
    __shared__ double ssum[1024];
    __shared__ double scnt[1024];
    double s = 0.0, cnt = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 1024) {
        const float e = err[i];
        if (e >= 0.f) { s += (double)e; cnt += 1.0; }
    }
    ssum[threadIdx.x] = s;
    scnt[threadIdx.x] = cnt;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            ssum[threadIdx.x] += ssum[threadIdx.x + w];
            scnt[threadIdx.x] += scnt[threadIdx.x + w];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) *p.mean = scnt[0] > 0.0 ? ssum[0] / scnt[0] : 0.0;
}

hipError_t launch_group_error(const GroupErrorParams& p, hipStream_t stream) {
    const int64_t tiles = ((int64_t)p.rows + 31) / 32;
    if (p.G < 1 || p.rows < 1 || tiles > kGroupErrorMaxTiles) return hipErrorInvalidValue;
    hipError_t e = launch(group_error_kernel, dim3((unsigned)p.G, (unsigned)tiles), dim3(64), 0, stream, p);
    if (e != hipSuccess || !p.mean) return e;
    const GroupErrorMeanParams m{p.err, (int64_t)p.rows * p.G, p.mean};
    return launch(group_error_mean_kernel, dim3(1), dim3(1024), 0, stream, m);
}

}  // namespace duqpp
