// Internal declarations shared by the translation units of libduqpp (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include <atomic>

#include "duqpp.h"

namespace duqpp {

constexpr int kBlock = 32;        // rotation block == MXFP4 group (Eq. 4, B = 32)
constexpr int kNumCU = 256;       // MI355X
constexpr int kNumXCD = 8;
constexpr int kMaxDevices = 64;   // devices of one process the per-device set-up keeps track of

// A launch that reports its own status.  The runtime's per-thread error state, which may still hold an error left by
// the caller's earlier work, is neither consulted nor cleared.
template <typename P>
inline hipError_t launch(void (*kernel)(P), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, const P& p) {
    P arg = p;
    void* args[] = {&arg};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, args, lds_bytes, stream);
}
template <typename P, typename Q>
inline hipError_t launch(void (*kernel)(P, Q), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, const P& p,
                         const Q& q) {
    P a0 = p;
    Q a1 = q;
    void* args[] = {&a0, &a1};
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, args, lds_bytes, stream);
}

// Set-up that has to happen once on every device a kernel runs on (a function attribute belongs to the device's
// copy of the code): f runs with the calling thread's current device, once per device and process.
struct PerDeviceOnce {
    std::atomic<int> done[kMaxDevices];
    template <typename F>
    hipError_t run(F&& f) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
        if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
        e = f();
        if (e == hipSuccess) done[dev].store(1, std::memory_order_release);
        return e;
    }
};
inline hipError_t allow_dynamic_lds(const void* kernel, int bytes) {
    return hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// Per-device set-up of each translation unit's kernels (what duqpp_init runs; the launchers run it themselves on
// first use).
hipError_t setup_rotq();
hipError_t setup_gemm_tiled_mid();
hipError_t setup_gemm_tiled_small();
hipError_t setup_gemm_tiled_large();

// ---- rotate + quantise (rotq.hip) ------------------------------------------------------
struct RotqParams {
    const uint16_t* x;   // bf16 [rows, K], stride ldx
    int64_t ldx;
    int rows;
    int G;               // K / 32
    const float* R;      // [n_rblocks, 32, 32]; with r_packed the packed blocks of duqpp_pack_rotation
    int r_stride;        // floats (bytes when r_packed) between consecutive blocks of R (0 when one block is shared)
    int r_packed;        // R holds packed blocks (tiled output only)
    uint8_t* codes;      // [rows, K/2], or the tiled codes when tiled != 0
    uint8_t* scales;     // [rows, G], or the tiled scales
    int tiled;           // output placement
    int GP;              // groups padded to a multiple of 8 (tiled layout)
    float* ydbg;         // nullable [rows, K]
    int ntiles;          // ceil(rows / 32)
    int tiles_per_wg;
    int ngroups;         // ceil(ntiles / tiles_per_wg)
    int nchunks;         // column chunks (each covers waves*2 blocks)
    int waves;           // wavefronts per workgroup
    int by_columns;      // tiled-output kernel: an XCD owns column chunks (1) or token runs (0)
    int stages;          // tiled-output kernel: depth of a wave's ring of token tiles (2 or 3)
};
hipError_t launch_rotq(const RotqParams& p, hipStream_t stream);
void plan_rotq(RotqParams& p);    // fills ntiles / tiles_per_wg / ngroups / nchunks / waves / by_columns / stages

constexpr int kPackedRotationBlockBytes = 6144;   // three bf16 pieces of a 32 x 32 block
struct PackRotationParams {
    const float* R; uint8_t* packed; int n_blocks;
};
hipError_t launch_pack_rotation(const PackRotationParams& p, hipStream_t stream);

// ---- per-group normalised quantisation error (group_error.hip) --------------------------
struct GroupErrorParams {
    const uint16_t* x;   // bf16 [rows, K], stride ldx
    int64_t ldx;
    int rows;
    int G;               // K / 32
    const float* R;      // fp32 blocks, or null: no rotation
    int r_stride;        // floats between consecutive blocks (0 when one block is shared)
    float* err;          // [rows, G]
    double* mean;        // nullable
};
struct GroupErrorMeanParams {
    const float* err; int64_t n; double* mean;
};
constexpr int64_t kGroupErrorMaxTiles = 65535;   // token tiles along blockIdx.y
hipError_t launch_group_error(const GroupErrorParams& p, hipStream_t stream);

struct QuantDbgParams {
    const float* y; int64_t ldy; int rows; int G; uint8_t* codes; uint8_t* scales;
};
hipError_t launch_quant_dbg(const QuantDbgParams& p, hipStream_t stream);

// ---- MXFP4 GEMM (gemm.hip) ------------------------------------------------------------
struct GemmParams {
    const uint8_t* a_codes; const uint8_t* a_scales;   // [T, K/2], [T, G]
    const uint8_t* b_codes; const uint8_t* b_scales;   // [N, K/2], [N, G]
    int T, N, G;
    void* y; int64_t ldy; int out_bf16;
};
hipError_t launch_gemm(const GemmParams& p, hipStream_t stream);

}  // namespace duqpp

// ---- tiled operand layout (layout.hip, gemm_tiled.hip) ----------------------------------
// An MXFP4 operand with `rows` rows and G groups, padded to RT = ceil(rows/32) row tiles and
// GP = ceil(G/8)*8 groups:
//   codes   [RT][GP][32 rows][16 bytes]            one group of one row = 16 contiguous bytes,
//                                                  the 32 rows of a tile adjacent (512 B), then the next group
//   scales  [RT][GP/8][2][32 rows][4 bytes]        byte b of the word at [rt][q][g][r] is the scale of
//                                                  row 32 rt + r, group 8 q + 4 g + b
// Padding rows and groups hold code 0 and scale 127 (= 1.0), so they contribute exact zeros.
namespace duqpp {

inline int64_t tiled_row_tiles(int64_t rows) { return (rows + 31) / 32; }
inline int64_t tiled_groups(int64_t G) { return (G + 7) / 8 * 8; }
inline size_t tiled_codes_bytes(int64_t rows, int64_t G) { return (size_t)tiled_row_tiles(rows) * tiled_groups(G) * 512; }
inline size_t tiled_scales_bytes(int64_t rows, int64_t G) { return (size_t)tiled_row_tiles(rows) * tiled_groups(G) * 32; }

struct LayoutParams {
    const uint8_t* src_codes; const uint8_t* src_scales;
    uint8_t* dst_codes; uint8_t* dst_scales;
    int rows, G, GP;
};
hipError_t launch_tile(const LayoutParams& p, hipStream_t stream);     // row-major -> tiled (writes the padding too)
hipError_t launch_untile(const LayoutParams& p, hipStream_t stream);   // tiled -> row-major

// ---- smoothing merged into the rotation blocks (smooth.hip) ---------------------------------
struct FoldParams {
    const float* R; int r_stride;      // [G or 1][32][32]; floats between blocks (0 when shared)
    const float* lambda;               // [32 G]
    float* R_act; float* R_wgt;        // [G][32][32] each
    int G;
};
hipError_t launch_fold_smoothing(const FoldParams& p, hipStream_t stream);

// ---- offline construction of the shared rotation block (construct.hip) ------------------------------
struct ConstructParams {
    const uint16_t* x; int64_t ldx; int64_t T; int64_t K;   // calibration activations, bf16 [T, K]
    const double* q_steps; int steps;                       // [steps][31][31] orthogonal draws
    float* R_out; int32_t* info; double* peaks;             // [32][32]; {block, steps kept}; nullable [steps + 1]
    void* workspace;
};
size_t construct_workspace_bytes(int64_t T, int steps);
hipError_t launch_construct_rotation(const ConstructParams& p, hipStream_t stream);

struct TiledGemmParams {
    const uint8_t* a_codes; const uint8_t* a_scales;   // tiled, T rows
    const uint8_t* b_codes; const uint8_t* b_scales;   // tiled, N rows
    int T, N, GP;
    void* y; int64_t ldy; int out_bf16;
};
hipError_t launch_gemm_tiled(const TiledGemmParams& p, hipStream_t stream);     // picks the kernel by shape
int choose_gemm_kernel(const TiledGemmParams& p);                              // the DUQPP_GEMM_KERNEL_* it picks
hipError_t launch_gemm_tiled_as(const TiledGemmParams& p, int kernel, hipStream_t stream);   // a named kernel
hipError_t launch_gemm_tiled_small(const TiledGemmParams& p, hipStream_t stream);   // 64 x 128 tiles
hipError_t launch_gemm_tiled_large(const TiledGemmParams& p, hipStream_t stream);   // 256 x 256 tiles
bool gemm_tiled_large_accepts(const TiledGemmParams& p);                           // output alignment the large kernel needs
// ---- one-kernel rotate + quantise + multiply for up to 32 tokens (rotq_gemm_fused.hip) ----------------------
struct FusedDecodeParams {
    const uint16_t* x; int64_t ldx; int T;               // bf16 [T, K]
    const uint8_t* r_packed; int r_stride;                // packed rotation blocks; bytes between them (0 = one shared block)
    const uint8_t* b_codes; const uint8_t* b_scales;      // tiled weights
    int N, G, GP;
    void* y; int64_t ldy; int out_bf16;
    uint8_t* dbg_codes; uint8_t* dbg_scales;              // nullable: the activation operand (tiled, T rows)
};
constexpr int kFusedMaxT = 32 * 65535;                    // token tiles run along blockIdx.y
hipError_t launch_rotq_gemm_fused_decode(const FusedDecodeParams& p, hipStream_t stream);

constexpr int kDecodeMaxT = 128;   // up to four activation row tiles go to the weight-streaming kernel
hipError_t launch_gemm_decode(const TiledGemmParams& p, hipStream_t stream);    // T <= kDecodeMaxT

}  // namespace duqpp
