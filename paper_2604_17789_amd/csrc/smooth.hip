// Merge of the smoothing diagonal of the paper's Eq. 3 into the rotation blocks of Eq. 4, so that the
// operands of Eq. 5, X Lambda^-1 R^ and R^T Lambda W, come out of the unchanged rotate+quantise kernels:
//     (x / lambda) . R_j = x . (diag(1 / lambda_j) R_j),     (w * lambda) . R_j = w . (diag(lambda_j) R_j)
// Offline work, one thread per block entry.
#include "duqpp_internal.h"

namespace duqpp {

__global__ __launch_bounds__(256) void fold_smoothing_kernel(FoldParams p) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over [G][32 (r: input channel)][32 (c)]
    if (idx >= (int64_t)p.G * 1024) return;
    const int j = (int)(idx >> 10), r = (int)((idx >> 5) & 31);
    const float v = p.R[(int64_t)j * p.r_stride + (idx & 1023)];
    const float l = p.lambda[32 * j + r];
    p.R_act[idx] = v / l;                                      // IEEE division (hipcc's default for fp32)
    p.R_wgt[idx] = v * l;
}

hipError_t launch_fold_smoothing(const FoldParams& p, hipStream_t stream) {
    const int64_t total = (int64_t)p.G * 1024;
    return launch(fold_smoothing_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, p);
}

}  // namespace duqpp
