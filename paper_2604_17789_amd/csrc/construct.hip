// Offline: greedy outlier-aware construction of the shared 32x32 rotation block (paper Sec. 4.2, paragraph
// "Fine-grained Block-diagonal Rotation", steps (1)-(3); all blocks share the matrix built from the block that
// holds the largest outlier).  The paper gives the construction as a sketch; the reading implemented here:
//   b*  = block of 32 channels with the largest |x| (smallest index among equals);  Z_0 = X[:, b*],  R^(0) = I
//   for t = 1 .. steps:  d = channel of Z_{t-1} with the largest magnitude (smallest index among equals)
//                        R_t = E_d . H . diag(1, Q'_t) . E_d      E_d exchanges coordinates 0 and d, H is the
//                              normalised Sylvester-Hadamard matrix (uniform first row: what sits in coordinate 0
//                              is spread evenly), Q'_t a caller-drawn orthogonal 31 x 31 matrix
//                        Z_t = Z_{t-1} . R_t,   R^(t) = R^(t-1) . R_t,   peak_t = max |Z_t|
//   result R^(t*), t* = the step count with the smallest peak (smallest t among equals; t = 0 keeps the identity)
// Arithmetic: fp64, every dot product accumulated in index order from zero with one rounding per multiply and per
// add (contraction into fused multiply-adds is switched off for this file), so that the argmax / argmin decisions
// and the result do not depend on how the work is spread over the chip.  Maxima are taken with integer atomics on
// the bit patterns of |z| (order-independent).
//
// One kernel launch per step: the step needs the column maxima of the whole previous state.  That is 130 short
// launches for the paper's 128 steps; the call is offline.
#include "duqpp_internal.h"

#pragma clang fp contract(off)

namespace duqpp {

namespace {

constexpr double kHadamardEntry = 0.17677669529663687;   // 1 / sqrt(32)
constexpr int kStepRowsPerWG = 64;

__device__ __forceinline__ double hadamard_entry(int i, int k) { return (__popc(i & k) & 1) ? -kHadamardEntry : kHadamardEntry; }

// workspace: [header 64 B: u64 block key][colmax (S + 1) x 32 u64][Rhist (S + 1) x 1024 f64][Z T x 32 f64]
struct Workspace {
    unsigned long long* key;
    unsigned long long* colmax;
    double* rhist;
    double* z;
};
__host__ __device__ inline Workspace carve(void* ws, int steps) {
    Workspace w;
    uint8_t* p = static_cast<uint8_t*>(ws);
    w.key = reinterpret_cast<unsigned long long*>(p);
    w.colmax = reinterpret_cast<unsigned long long*>(p + 64);
    w.rhist = reinterpret_cast<double*>(p + 64 + (size_t)(steps + 1) * 256);
    w.z = reinterpret_cast<double*>(p + 64 + (size_t)(steps + 1) * 256 + (size_t)(steps + 1) * 8192);
    return w;
}

__global__ __launch_bounds__(256) void construct_init_kernel(ConstructParams p) {
    Workspace w = carve(p.workspace, p.steps);
    const int n = 8 + (p.steps + 1) * 32;                    // header and column maxima, as 64-bit words
    unsigned long long* base = w.key;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) base[i] = 0ull;
}

// largest |x| per block of 32 channels -> one 64-bit key: magnitude bits above, inverted block index below, so
// that the integer maximum is the largest magnitude in the smallest block
__global__ __launch_bounds__(256) void construct_blockmax_kernel(ConstructParams p) {
    Workspace w = carve(p.workspace, p.steps);
    const int64_t chunks_per_row = p.K / 8;                  // 16-byte pieces of 8 bf16; 4 per block
    const int64_t total = (int64_t)p.T * chunks_per_row;
    unsigned long long best = 0ull;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t row = i / chunks_per_row, ch = i - row * chunks_per_row;
        const uint4 v = *reinterpret_cast<const uint4*>(p.x + row * p.ldx + ch * 8);
        const uint32_t words[4] = {v.x, v.y, v.z, v.w};
        uint32_t m = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint32_t lo = words[k] & 0x7FFFu, hi = (words[k] >> 16) & 0x7FFFu;
            m = m > lo ? m : lo;
            m = m > hi ? m : hi;
        }
        const unsigned long long key = ((unsigned long long)m << 32) | (0xFFFFFFFFu - (uint32_t)(ch / 4));
        best = best > key ? best : key;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const unsigned long long o = __shfl_xor(best, off);
        best = best > o ? best : o;
    }
    if ((threadIdx.x & 63) == 0 && best) atomicMax(w.key, best);
}

__device__ __forceinline__ int chosen_block(const Workspace& w) { return (int)(0xFFFFFFFFu - (uint32_t)(*w.key & 0xFFFFFFFFull)); }

// column maxima of 8 rows x 32 columns held by a workgroup of 256 (thread = (row slot, column)) into colmax[32]
__device__ __forceinline__ void column_max_to_global(unsigned long long mine, unsigned long long* red /* LDS [256] */,
                                                     unsigned long long* colmax) {
    red[threadIdx.x] = mine;
    __syncthreads();
    if (threadIdx.x < 32) {
        unsigned long long m = 0ull;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const unsigned long long o = red[s * 32 + threadIdx.x];
            m = m > o ? m : o;
        }
        if (m) atomicMax(colmax + threadIdx.x, m);
    }
    __syncthreads();
}

__device__ __forceinline__ unsigned long long abs_bits(double v) { return (unsigned long long)__double_as_longlong(v) & 0x7FFFFFFFFFFFFFFFull; }

// Z_0 = the chosen block's columns as doubles, their column maxima, R^(0) = I
__global__ __launch_bounds__(256) void construct_extract_kernel(ConstructParams p) {
    __shared__ unsigned long long red[256];
    Workspace w = carve(p.workspace, p.steps);
    const int b = chosen_block(w);
    const int c = threadIdx.x & 31, slot = threadIdx.x >> 5;
    unsigned long long mine = 0ull;
    for (int64_t row = (int64_t)blockIdx.x * 8 + slot; row < p.T; row += (int64_t)gridDim.x * 8) {
        const uint32_t bits = p.x[row * p.ldx + 32 * b + c];
        const double v = (double)__uint_as_float(bits << 16);
        w.z[row * 32 + c] = v;
        const unsigned long long a = abs_bits(v);
        mine = mine > a ? mine : a;
    }
    column_max_to_global(mine, red, w.colmax);
    if (blockIdx.x == 0)
        for (int e = threadIdx.x; e < 1024; e += 256) w.rhist[e] = (e / 32 == e % 32) ? 1.0 : 0.0;
}

// one greedy step t >= 1
__global__ __launch_bounds__(256) void construct_step_kernel(ConstructParams p, int t) {
    __shared__ double M[32 * 32];                            // H . diag(1, Q'_t)
    __shared__ double rows[8 * 32];
    __shared__ unsigned long long red[256];
    __shared__ int sigma[32];
    Workspace w = carve(p.workspace, p.steps);
    // (1) the channel with the largest magnitude in the previous state, smallest index among equals
    if (threadIdx.x == 0) {
        const unsigned long long* cm = w.colmax + (size_t)(t - 1) * 32;
        int d = 0;
        unsigned long long best = cm[0];
        for (int c = 1; c < 32; ++c)
            if (cm[c] > best) { best = cm[c]; d = c; }
        for (int c = 0; c < 32; ++c) sigma[c] = c;
        sigma[0] = d;
        sigma[d] = 0;
    }
    // (2) M = H . diag(1, Q'): column 0 passes through, the others sum terms k = 1 .. 31 in order
    const double* q = p.q_steps + (size_t)(t - 1) * 31 * 31;
    for (int e = threadIdx.x; e < 1024; e += 256) {
        const int i = e >> 5, j = e & 31;
        double acc;
        if (j == 0) {
            acc = hadamard_entry(i, 0);
        } else {
            acc = 0.0;
            for (int k = 1; k < 32; ++k) acc = acc + hadamard_entry(i, k) * q[(k - 1) * 31 + (j - 1)];
        }
        M[e] = acc;
    }
    __syncthreads();
    // R_t[r][c] = M[sigma(r)][sigma(c)]  (E_d . M . E_d)
    const int c = threadIdx.x & 31, slot = threadIdx.x >> 5;
    const int sc = sigma[c];
    // (3) Z <- Z . R_t for this workgroup's rows, 8 at a time, and the new column maxima
    unsigned long long mine = 0ull;
    const int64_t row0 = (int64_t)blockIdx.x * kStepRowsPerWG;
    for (int pass = 0; pass < kStepRowsPerWG / 8; ++pass) {
        const int64_t row = row0 + pass * 8 + slot;
        const bool ok = row < p.T;
        rows[threadIdx.x] = ok ? w.z[row * 32 + c] : 0.0;
        __syncthreads();
        double acc = 0.0;
        for (int r = 0; r < 32; ++r) acc = acc + rows[slot * 32 + r] * M[sigma[r] * 32 + sc];
        if (ok) {
            w.z[row * 32 + c] = acc;
            const unsigned long long a = abs_bits(acc);
            mine = mine > a ? mine : a;
        }
        __syncthreads();
    }
    column_max_to_global(mine, red, w.colmax + (size_t)t * 32);
    // R^(t) = R^(t-1) . R_t, by the first workgroup
    if (blockIdx.x == 0) {
        const double* prev = w.rhist + (size_t)(t - 1) * 1024;
        double* next = w.rhist + (size_t)t * 1024;
        for (int e = threadIdx.x; e < 1024; e += 256) {
            const int i = e >> 5, j = e & 31;
            const int sj = sigma[j];
            double acc = 0.0;
            for (int r = 0; r < 32; ++r) acc = acc + prev[i * 32 + r] * M[sigma[r] * 32 + sj];
            next[e] = acc;
        }
    }
}

// peaks, the first minimum, the kept product rounded to fp32
__global__ __launch_bounds__(256) void construct_final_kernel(ConstructParams p) {
    __shared__ int best_t;
    Workspace w = carve(p.workspace, p.steps);
    if (threadIdx.x == 0) {
        unsigned long long best = ~0ull;
        int bt = 0;
        for (int t = 0; t <= p.steps; ++t) {
            unsigned long long peak = 0ull;
            for (int c = 0; c < 32; ++c) {
                const unsigned long long v = w.colmax[(size_t)t * 32 + c];
                peak = peak > v ? peak : v;
            }
            if (p.peaks) p.peaks[t] = __longlong_as_double((long long)peak);
            if (peak < best) { best = peak; bt = t; }
        }
        best_t = bt;
        p.info[0] = chosen_block(w);
        p.info[1] = bt;
    }
    __syncthreads();
    const double* r = w.rhist + (size_t)best_t * 1024;
    for (int e = threadIdx.x; e < 1024; e += 256) p.R_out[e] = (float)r[e];
}

}  // namespace

size_t construct_workspace_bytes(int64_t T, int steps) {
    return 64 + (size_t)(steps + 1) * 256 + (size_t)(steps + 1) * 8192 + (size_t)T * 256;
}

hipError_t launch_construct_rotation(const ConstructParams& p, hipStream_t stream) {
    hipError_t e = launch(construct_init_kernel, dim3(8), dim3(256), 0, stream, p);
    if (e != hipSuccess) return e;
    const int64_t chunks = (int64_t)p.T * (p.K / 8);
    int grid = (int)((chunks + 255) / 256 < 2048 ? (chunks + 255) / 256 : 2048);
    e = launch(construct_blockmax_kernel, dim3(grid), dim3(256), 0, stream, p);
    if (e != hipSuccess) return e;
    grid = (int)((p.T + 7) / 8 < 1024 ? (p.T + 7) / 8 : 1024);
    e = launch(construct_extract_kernel, dim3(grid), dim3(256), 0, stream, p);
    if (e != hipSuccess) return e;
    const int step_grid = (int)((p.T + kStepRowsPerWG - 1) / kStepRowsPerWG);
    for (int t = 1; t <= p.steps; ++t) {
        e = launch(construct_step_kernel, dim3(step_grid), dim3(256), 0, stream, p, t);
        if (e != hipSuccess) return e;
    }
    return launch(construct_final_kernel, dim3(1), dim3(256), 0, stream, p);
}

}  // namespace duqpp
