// Conversions between the row-major MXFP4 operand layout of the ABI and the tiled layout the
// fast GEMM reads (see duqpp_internal.h).  Pure byte permutations.
#include "duqpp_internal.h"

namespace duqpp {

// one thread per (row tile, group, row): moves 16 code bytes and 1 scale byte
__global__ __launch_bounds__(256) void tile_kernel(LayoutParams p) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int RT = (p.rows + 31) / 32;
    const int64_t total = (int64_t)RT * p.GP * 32;
    if (idx >= total) return;
    const int r = (int)(idx & 31);
    const int j = (int)((idx >> 5) % p.GP);
    const int rt = (int)((idx >> 5) / p.GP);
    const int row = rt * 32 + r;
    uint4 c = make_uint4(0, 0, 0, 0);
    uint8_t s = 127;
    if (row < p.rows && j < p.G) {
        c = *(const uint4*)(p.src_codes + ((int64_t)row * p.G + j) * 16);
        s = p.src_scales[(int64_t)row * p.G + j];
    }
    *(uint4*)(p.dst_codes + idx * 16) = c;
    p.dst_scales[((((int64_t)rt * (p.GP / 8) + j / 8) * 2 + (j % 8) / 4) * 32 + r) * 4 + (j % 4)] = s;
}

__global__ __launch_bounds__(256) void untile_kernel(LayoutParams p) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over (row, group)
    const int64_t total = (int64_t)p.rows * p.G;
    if (idx >= total) return;
    const int j = (int)(idx % p.G);
    const int row = (int)(idx / p.G);
    const int rt = row / 32, r = row % 32;
    *(uint4*)(p.dst_codes + idx * 16) = *(const uint4*)(p.src_codes + (((int64_t)rt * p.GP + j) * 32 + r) * 16);
    p.dst_scales[idx] = p.src_scales[((((int64_t)rt * (p.GP / 8) + j / 8) * 2 + (j % 8) / 4) * 32 + r) * 4 + (j % 4)];
}

hipError_t launch_tile(const LayoutParams& p, hipStream_t stream) {
    const int64_t total = (int64_t)((p.rows + 31) / 32) * p.GP * 32;
    return launch(tile_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p);
}

hipError_t launch_untile(const LayoutParams& p, hipStream_t stream) {
    const int64_t total = (int64_t)p.rows * p.G;
    return launch(untile_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p);
}

}  // namespace duqpp
