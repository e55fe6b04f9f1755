// Internal declarations shared by the translation units of libduqpp (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "duqpp.h"

namespace duqpp {

constexpr int kBlock = 32;        // rotation block == MXFP4 group (Eq. 4, B = 32)
constexpr int kNumCU = 256;       // MI355X
constexpr int kNumXCD = 8;

// ---- rotate + quantise (rotq.hip) ------------------------------------------------------
struct RotqParams {
    const uint16_t* x;   // bf16 [rows, K], stride ldx
    int64_t ldx;
    int rows;
    int G;               // K / 32
    const float* R;      // [n_rblocks, 32, 32]
    int r_stride;        // floats between consecutive blocks of R (0 when one block is shared)
    uint8_t* codes;      // [rows, K/2]
    uint8_t* scales;     // [rows, G]
    float* ydbg;         // nullable [rows, K]
    int ntiles;          // ceil(rows / 32)
    int tiles_per_wg;
    int ngroups;         // ceil(ntiles / tiles_per_wg)
    int nchunks;         // column chunks (each covers waves*2 blocks)
};
hipError_t launch_rotq(const RotqParams& p, hipStream_t stream);
void plan_rotq(RotqParams& p);    // fills ntiles / tiles_per_wg / ngroups / nchunks

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
    void* workspace; size_t workspace_bytes;
};
hipError_t launch_gemm(const GemmParams& p, hipStream_t stream);
size_t gemm_workspace_bytes(int64_t T, int64_t N, int64_t K);

}  // namespace duqpp
