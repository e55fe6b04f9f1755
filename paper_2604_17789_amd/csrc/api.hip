// C ABI of libduqpp: argument validation on the host, then kernel launches on the caller's stream.
#include <cstring>

#include "duqpp_internal.h"

using namespace duqpp;

// Scratch of duqpp_rotq_gemm_tiled_noalloc: the activation operand between its two kernels.  One copy per GPU,
// held from the moment the library's code is loaded there until the process ends.  In host code the name is only a
// handle for hipGetSymbolAddress; the device address it yields (g_scratch_ptr) is what kernels and copies are given.
// (No `used` attribute: the compiler gives a static device variable that host code refers to external linkage in the
// code object, which the runtime's look-up by name needs; `used` would keep it a local symbol.)
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

namespace {

inline bool aligned_to(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// One gfx950 check per device, cached.  0 = unknown, 1 = ok, 2 = wrong architecture.
std::atomic<int> g_arch_state[64];

int check_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return DUQPP_ERR_HIP; }
    if (dev < 0 || dev >= 64) return DUQPP_ERR_HIP;
    int st = g_arch_state[dev].load(std::memory_order_relaxed);
    if (st == 0) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess) { (void)hipGetLastError(); return DUQPP_ERR_HIP; }
        st = (std::strncmp(prop.gcnArchName, "gfx950", 6) == 0) ? 1 : 2;
        g_arch_state[dev].store(st, std::memory_order_relaxed);
    }
    return st == 1 ? DUQPP_OK : DUQPP_ERR_ARCH;
}

// Device address of `scratch` on each device, looked up once per device with that device current.
uint8_t* g_scratch_ptr[kMaxDevices];
PerDeviceOnce g_scratch_once;

hipError_t setup_scratch() {
    return g_scratch_once.run([] {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = static_cast<uint8_t*>(ptr);
        return hipSuccess;
    });
}

int validate_rows_K(int64_t rows, int64_t K, int64_t ld, int64_t n_rblocks) {
    if (rows < 1 || rows > (int64_t)1 << 30) return DUQPP_ERR_SHAPE;
    if (K < 32 || (K % 32) != 0 || K > (int64_t)1 << 30) return DUQPP_ERR_SHAPE;
    if (ld < K) return DUQPP_ERR_SHAPE;
    if (n_rblocks != 1 && n_rblocks != K / 32) return DUQPP_ERR_SHAPE;
    return DUQPP_OK;
}

// R: fp32 blocks, or with `packed` the blocks in the form duqpp_pack_rotation writes (tiled output only).
int rotate_quantize_impl(const void* x, int64_t rows, int64_t K, int64_t ldx, const void* R, int64_t n_rblocks,
                         uint8_t* codes, uint8_t* scales, float* ydbg, void* stream, bool tiled = false,
                         bool packed = false) {
    int st = duqpp_validate_rotate_quantize(x, rows, K, ldx, static_cast<const float*>(R), n_rblocks, codes, scales);
    if (st != DUQPP_OK) return st;
    if (ydbg && !aligned_to(ydbg, 16)) return DUQPP_ERR_ALIGN;
    if (tiled && (!aligned_to(codes, 256) || !aligned_to(scales, 256))) return DUQPP_ERR_ALIGN;
    if (packed && (!tiled || !aligned_to(R, 16))) return tiled ? DUQPP_ERR_ALIGN : DUQPP_ERR_SHAPE;
    st = check_device();
    if (st != DUQPP_OK) return st;
    RotqParams p{};
    p.x = static_cast<const uint16_t*>(x);
    p.ldx = ldx;
    p.rows = (int)rows;
    p.G = (int)(K / 32);
    p.R = static_cast<const float*>(R);
    p.r_packed = packed ? 1 : 0;
    p.r_stride = (n_rblocks == 1) ? 0 : (packed ? kPackedRotationBlockBytes : 32 * 32);
    p.codes = codes;
    p.scales = scales;
    p.ydbg = ydbg;
    p.tiled = tiled ? 1 : 0;
    p.GP = (int)tiled_groups(K / 32);
    plan_rotq(p);
    return launch_rotq(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

// Scratch of the row-major GEMM calls: both operands in the tiled layout, each part rounded up to 256 bytes:
// A codes, A scales, B codes, B scales.
size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }
struct TiledScratch {
    size_t a_codes, a_scales, b_codes, b_scales;           // byte offsets
    size_t total;
};
TiledScratch tiled_scratch(int64_t T, int64_t N, int64_t K) {
    TiledScratch w{};
    const int64_t G = K / 32;
    w.a_codes = 0;
    w.a_scales = w.a_codes + round256(tiled_codes_bytes(T, G));
    w.b_codes = w.a_scales + round256(tiled_scales_bytes(T, G));
    w.b_scales = w.b_codes + round256(tiled_codes_bytes(N, G));
    w.total = w.b_scales + round256(tiled_scales_bytes(N, G));
    return w;
}

// The fused call on tiled weights with the activation operand in a_codes / a_scales (256-byte aligned scratch of
// the sizes duqpp_tiled_bytes reports): every argument of both stages is checked before the first launch.
int rotq_gemm_tiled_impl(const void* x_bf16, int64_t ldx, const void* R, int64_t n_rblocks, uint8_t* a_codes,
                         uint8_t* a_scales, const uint8_t* b_codes_t, const uint8_t* b_scales_t, int64_t T, int64_t N,
                         int64_t K, void* y, int out_dtype, int64_t ldy, void* stream, bool packed = false) {
    int st = duqpp_validate_rotate_quantize(x_bf16, T, K, ldx, static_cast<const float*>(R), n_rblocks, a_codes, a_scales);
    if (st != DUQPP_OK) return st;
    if (packed && !aligned_to(R, 16)) return DUQPP_ERR_ALIGN;
    st = duqpp_validate_mxfp4_gemm(a_codes, a_scales, b_codes_t, b_scales_t, T, N, K, y, out_dtype, ldy, nullptr, 0, 2);
    if (st != DUQPP_OK) return st;
    if (!aligned_to(b_codes_t, 256) || !aligned_to(b_scales_t, 256)) return DUQPP_ERR_ALIGN;
    st = rotate_quantize_impl(x_bf16, T, K, ldx, R, n_rblocks, a_codes, a_scales, nullptr, stream, true, packed);
    if (st != DUQPP_OK) return st;
    return duqpp_mxfp4_gemm_tiled(a_codes, a_scales, b_codes_t, b_scales_t, T, N, K, y, out_dtype, ldy, stream);
}

}  // namespace

extern "C" {

int duqpp_init(void) {
    int st = check_device();
    if (st != DUQPP_OK) return st;
    if (setup_rotq() != hipSuccess || setup_gemm_tiled_mid() != hipSuccess || setup_gemm_tiled_small() != hipSuccess ||
        setup_gemm_tiled_large() != hipSuccess || setup_scratch() != hipSuccess)
        return DUQPP_ERR_HIP;
    return DUQPP_OK;
}

size_t duqpp_noalloc_scratch_bytes(void) { return kStaticScratchBytes; }

int duqpp_rotq_gemm_tiled_noalloc(const void* x_bf16, int64_t ldx, const float* R, int64_t n_rblocks,
                                  const uint8_t* b_codes_t, const uint8_t* b_scales_t, int64_t T, int64_t N, int64_t K,
                                  void* y, int out_dtype, int64_t ldy, void* stream) {
    if (!x_bf16 || !R || !b_codes_t || !b_scales_t || !y) return DUQPP_ERR_NULL;
    int st = validate_rows_K(T, K, ldx, n_rblocks);
    if (st != DUQPP_OK) return st;
    const size_t cb = round256(tiled_codes_bytes(T, K / 32));
    const size_t sb = round256(tiled_scales_bytes(T, K / 32));
    if (cb + sb > kStaticScratchBytes) return DUQPP_ERR_TOO_LARGE;
    st = check_device();
    if (st != DUQPP_OK) return st;
    if (setup_scratch() != hipSuccess) return DUQPP_ERR_HIP;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return DUQPP_ERR_HIP;
    uint8_t* a_codes = g_scratch_ptr[dev];                   // the device address, never the array's name
    uint8_t* a_scales = a_codes + cb;
    // The rotate+quantise kernel writes every byte of the operand the GEMM reads, padding included, so nothing of an
    // earlier call's contents is read and nothing has to be cleared.
    return rotq_gemm_tiled_impl(x_bf16, ldx, R, n_rblocks, a_codes, a_scales, b_codes_t, b_scales_t, T, N, K, y, out_dtype,
                                ldy, stream);
}

int duqpp_validate_rotate_quantize(const void* x, int64_t T, int64_t K, int64_t ldx, const float* R,
                                   int64_t n_rblocks, const uint8_t* codes, const uint8_t* scales) {
    if (!x || !R || !codes || !scales) return DUQPP_ERR_NULL;
    int st = validate_rows_K(T, K, ldx, n_rblocks);
    if (st != DUQPP_OK) return st;
    if (!aligned_to(x, 16) || (ldx % 8) != 0) return DUQPP_ERR_ALIGN;
    if (!aligned_to(R, 4) || !aligned_to(codes, 16)) return DUQPP_ERR_ALIGN;
    return DUQPP_OK;
}

int duqpp_validate_mxfp4_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                              const uint8_t* b_scales, int64_t T, int64_t N, int64_t K, const void* y,
                              int out_dtype, int64_t ldy, const void* workspace, size_t workspace_bytes,
                              int fused) {
    if (!a_codes || !b_codes || !b_scales || !y) return DUQPP_ERR_NULL;
    if (!fused && !a_scales) return DUQPP_ERR_NULL;
    if (T < 1 || N < 1 || T > (int64_t)1 << 30 || N > (int64_t)1 << 30) return DUQPP_ERR_SHAPE;
    if (K < 32 || (K % 32) != 0 || K > (int64_t)1 << 30) return DUQPP_ERR_SHAPE;
    if (ldy < N) return DUQPP_ERR_SHAPE;
    if (out_dtype != DUQPP_F32 && out_dtype != DUQPP_BF16) return DUQPP_ERR_DTYPE;
    if (!aligned_to(b_codes, 16)) return DUQPP_ERR_ALIGN;
    if (!fused && !aligned_to(a_codes, 16)) return DUQPP_ERR_ALIGN;
    if (!aligned_to(y, out_dtype == DUQPP_F32 ? 4 : 2)) return DUQPP_ERR_ALIGN;
    if (fused == 2) return DUQPP_OK;   // tiled operands: no workspace
    // the fused call needs its scratch; the separate call runs a slower direct kernel without one
    if (!workspace && !fused) return DUQPP_OK;
    if (!workspace || workspace_bytes < duqpp_gemm_workspace_bytes(T, N, K, fused)) return DUQPP_ERR_WORKSPACE;
    if (!aligned_to(workspace, 256)) return DUQPP_ERR_ALIGN;
    return DUQPP_OK;
}

size_t duqpp_gemm_workspace_bytes(int64_t T, int64_t N, int64_t K, int /*fused*/) {
    if (T < 1 || N < 1 || K < 32 || (K % 32) != 0) return 0;
    return tiled_scratch(T, N, K).total;
}

int duqpp_rotate_quantize(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const float* R,
                          int64_t n_rblocks, uint8_t* x_codes, uint8_t* x_scales, float* y_rot_dbg,
                          void* stream) {
    return rotate_quantize_impl(x_bf16, T, K, ldx, R, n_rblocks, x_codes, x_scales, y_rot_dbg, stream);
}

int duqpp_quantize_weights(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, const float* R,
                           int64_t n_rblocks, uint8_t* w_codes, uint8_t* w_scales, void* stream) {
    return rotate_quantize_impl(w_bf16, N, K, ldw, R, n_rblocks, w_codes, w_scales, nullptr, stream);
}

int duqpp_mxfp4_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* b_codes,
                     const uint8_t* b_scales, int64_t T, int64_t N, int64_t K, void* y, int out_dtype,
                     int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    int st = duqpp_validate_mxfp4_gemm(a_codes, a_scales, b_codes, b_scales, T, N, K, y, out_dtype, ldy,
                                       workspace, workspace_bytes, 0);
    if (st != DUQPP_OK) return st;
    st = check_device();
    if (st != DUQPP_OK) return st;
    hipStream_t hs = static_cast<hipStream_t>(stream);
    if (!workspace) {
        GemmParams p{};
        p.a_codes = a_codes; p.a_scales = a_scales; p.b_codes = b_codes; p.b_scales = b_scales;
        p.T = (int)T; p.N = (int)N; p.G = (int)(K / 32);
        p.y = y; p.ldy = ldy; p.out_bf16 = (out_dtype == DUQPP_BF16);
        return launch_gemm(p, hs) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
    }
    // re-tile both operands into the scratch, then the tiled kernel
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const TiledScratch w = tiled_scratch(T, N, K);
    const int G = (int)(K / 32), GP = (int)tiled_groups(G);
    LayoutParams la{a_codes, a_scales, ws + w.a_codes, ws + w.a_scales, (int)T, G, GP};
    LayoutParams lb{b_codes, b_scales, ws + w.b_codes, ws + w.b_scales, (int)N, G, GP};
    if (launch_tile(la, hs) != hipSuccess || launch_tile(lb, hs) != hipSuccess) return DUQPP_ERR_HIP;
    TiledGemmParams p{ws + w.a_codes, ws + w.a_scales, ws + w.b_codes, ws + w.b_scales, (int)T, (int)N, GP,
                      y, ldy, out_dtype == DUQPP_BF16};
    return launch_gemm_tiled(p, hs) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_rotq_gemm(const void* x_bf16, int64_t ldx, const float* R, int64_t n_rblocks,
                    const uint8_t* b_codes, const uint8_t* b_scales, int64_t T, int64_t N, int64_t K,
                    void* y, int out_dtype, int64_t ldy, void* workspace, size_t workspace_bytes,
                    void* stream) {
    if (!x_bf16 || !R) return DUQPP_ERR_NULL;
    // the A-side codes live in the workspace: validate the GEMM part with it standing in for them
    int st = duqpp_validate_mxfp4_gemm(static_cast<const uint8_t*>(workspace), nullptr, b_codes, b_scales, T, N, K,
                                       y, out_dtype, ldy, workspace, workspace_bytes, 1);
    if (st == DUQPP_ERR_NULL && !workspace && b_codes && b_scales && y) st = DUQPP_ERR_WORKSPACE;
    if (st != DUQPP_OK) return st;
    st = check_device();
    if (st != DUQPP_OK) return st;
    // activations are rotated and quantised straight into the tiled layout; the row-major weights are re-tiled
    hipStream_t hs = static_cast<hipStream_t>(stream);
    uint8_t* ws = static_cast<uint8_t*>(workspace);
    const TiledScratch w = tiled_scratch(T, N, K);
    const int G = (int)(K / 32), GP = (int)tiled_groups(G);
    st = rotate_quantize_impl(x_bf16, T, K, ldx, R, n_rblocks, ws + w.a_codes, ws + w.a_scales, nullptr, stream, true);
    if (st != DUQPP_OK) return st;
    LayoutParams lb{b_codes, b_scales, ws + w.b_codes, ws + w.b_scales, (int)N, G, GP};
    if (launch_tile(lb, hs) != hipSuccess) return DUQPP_ERR_HIP;
    TiledGemmParams p{ws + w.a_codes, ws + w.a_scales, ws + w.b_codes, ws + w.b_scales, (int)T, (int)N, GP,
                      y, ldy, out_dtype == DUQPP_BF16};
    return launch_gemm_tiled(p, hs) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_group_error(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const float* R, int64_t n_rblocks,
                      float* err, double* mean, void* stream) {
    if (!x_bf16 || !err) return DUQPP_ERR_NULL;
    int st = validate_rows_K(T, K, ldx, R ? n_rblocks : 1);
    if (st != DUQPP_OK) return st;
    if ((T + 31) / 32 > kGroupErrorMaxTiles) return DUQPP_ERR_TOO_LARGE;
    if (!aligned_to(x_bf16, 16) || (ldx % 8) != 0) return DUQPP_ERR_ALIGN;
    if ((R && !aligned_to(R, 4)) || !aligned_to(err, 4) || (mean && !aligned_to(mean, 8))) return DUQPP_ERR_ALIGN;
    st = check_device();
    if (st != DUQPP_OK) return st;
    GroupErrorParams p{};
    p.x = static_cast<const uint16_t*>(x_bf16);
    p.ldx = ldx;
    p.rows = (int)T;
    p.G = (int)(K / 32);
    p.R = R;
    p.r_stride = (n_rblocks == 1) ? 0 : 32 * 32;
    p.err = err;
    p.mean = mean;
    return launch_group_error(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_quantize_f32_dbg(const float* y, int64_t rows, int64_t K, int64_t ldy, uint8_t* codes,
                           uint8_t* scales, void* stream) {
    if (!y || !codes || !scales) return DUQPP_ERR_NULL;
    int st = validate_rows_K(rows, K, ldy, 1);
    if (st != DUQPP_OK) return st;
    if (!aligned_to(y, 16) || (ldy % 4) != 0 || !aligned_to(codes, 16)) return DUQPP_ERR_ALIGN;
    st = check_device();
    if (st != DUQPP_OK) return st;
    QuantDbgParams p{y, ldy, (int)rows, (int)(K / 32), codes, scales};
    return launch_quant_dbg(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_tiled_bytes(int64_t rows, int64_t K, size_t* codes_bytes, size_t* scales_bytes) {
    if (rows < 1 || K < 32 || (K % 32) != 0 || rows > (int64_t)1 << 30 || K > (int64_t)1 << 30) return DUQPP_ERR_SHAPE;
    if (codes_bytes) *codes_bytes = tiled_codes_bytes(rows, K / 32);
    if (scales_bytes) *scales_bytes = tiled_scales_bytes(rows, K / 32);
    return DUQPP_OK;
}

static int layout_call(const uint8_t* src_c, const uint8_t* src_s, int64_t rows, int64_t K, uint8_t* dst_c,
                       uint8_t* dst_s, void* stream, bool to_tiled) {
    if (!src_c || !src_s || !dst_c || !dst_s) return DUQPP_ERR_NULL;
    int st = validate_rows_K(rows, K, K, 1);
    if (st != DUQPP_OK) return st;
    const uint8_t* tc = to_tiled ? dst_c : src_c;
    const uint8_t* ts = to_tiled ? dst_s : src_s;
    const uint8_t* rc = to_tiled ? src_c : dst_c;
    if (!aligned_to(tc, 256) || !aligned_to(ts, 256) || !aligned_to(rc, 16)) return DUQPP_ERR_ALIGN;
    st = check_device();
    if (st != DUQPP_OK) return st;
    LayoutParams p{src_c, src_s, dst_c, dst_s, (int)rows, (int)(K / 32), (int)tiled_groups(K / 32)};
    hipError_t e = to_tiled ? launch_tile(p, static_cast<hipStream_t>(stream)) : launch_untile(p, static_cast<hipStream_t>(stream));
    return e == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_tile_operand(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K, uint8_t* codes_t,
                       uint8_t* scales_t, void* stream) {
    return layout_call(codes, scales, rows, K, codes_t, scales_t, stream, true);
}

int duqpp_untile_operand(const uint8_t* codes_t, const uint8_t* scales_t, int64_t rows, int64_t K, uint8_t* codes,
                         uint8_t* scales, void* stream) {
    return layout_call(codes_t, scales_t, rows, K, codes, scales, stream, false);
}

int duqpp_quantize_weights_tiled(const void* w_bf16, int64_t N, int64_t K, int64_t ldw, const float* R,
                                 int64_t n_rblocks, uint8_t* w_codes_t, uint8_t* w_scales_t, void* stream) {
    return rotate_quantize_impl(w_bf16, N, K, ldw, R, n_rblocks, w_codes_t, w_scales_t, nullptr, stream, true);
}

int duqpp_rotate_quantize_tiled(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const float* R,
                                int64_t n_rblocks, uint8_t* x_codes_t, uint8_t* x_scales_t, void* stream) {
    return rotate_quantize_impl(x_bf16, T, K, ldx, R, n_rblocks, x_codes_t, x_scales_t, nullptr, stream, true);
}

int duqpp_mxfp4_gemm_tiled(const uint8_t* a_codes_t, const uint8_t* a_scales_t, const uint8_t* b_codes_t,
                           const uint8_t* b_scales_t, int64_t T, int64_t N, int64_t K, void* y, int out_dtype,
                           int64_t ldy, void* stream) {
    int st = duqpp_validate_mxfp4_gemm(a_codes_t, a_scales_t, b_codes_t, b_scales_t, T, N, K, y, out_dtype, ldy,
                                       nullptr, 0, 2);
    if (st != DUQPP_OK) return st;
    if (!aligned_to(a_codes_t, 256) || !aligned_to(a_scales_t, 256) || !aligned_to(b_codes_t, 256) ||
        !aligned_to(b_scales_t, 256))
        return DUQPP_ERR_ALIGN;
    st = check_device();
    if (st != DUQPP_OK) return st;
    TiledGemmParams p{a_codes_t, a_scales_t, b_codes_t, b_scales_t, (int)T, (int)N, (int)tiled_groups(K / 32),
                      y, ldy, out_dtype == DUQPP_BF16};
    return launch_gemm_tiled(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_mxfp4_gemm_tiled_on(int kernel, const uint8_t* a_codes_t, const uint8_t* a_scales_t,
                              const uint8_t* b_codes_t, const uint8_t* b_scales_t, int64_t T, int64_t N, int64_t K,
                              void* y, int out_dtype, int64_t ldy, void* stream) {
    if (kernel < DUQPP_GEMM_KERNEL_AUTO || kernel > DUQPP_GEMM_KERNEL_LARGE) return DUQPP_ERR_SHAPE;
    int st = duqpp_validate_mxfp4_gemm(a_codes_t, a_scales_t, b_codes_t, b_scales_t, T, N, K, y, out_dtype, ldy,
                                       nullptr, 0, 2);
    if (st != DUQPP_OK) return st;
    if (!aligned_to(a_codes_t, 256) || !aligned_to(a_scales_t, 256) || !aligned_to(b_codes_t, 256) ||
        !aligned_to(b_scales_t, 256))
        return DUQPP_ERR_ALIGN;
    TiledGemmParams p{a_codes_t, a_scales_t, b_codes_t, b_scales_t, (int)T, (int)N, (int)tiled_groups(K / 32),
                      y, ldy, out_dtype == DUQPP_BF16};
    if (kernel == DUQPP_GEMM_KERNEL_DECODE && T > kDecodeMaxT) return DUQPP_ERR_SHAPE;
    if (kernel == DUQPP_GEMM_KERNEL_LARGE && !gemm_tiled_large_accepts(p)) return DUQPP_ERR_SHAPE;
    st = check_device();
    if (st != DUQPP_OK) return st;
    return launch_gemm_tiled_as(p, kernel, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_gemm_kernel_for(int64_t T, int64_t N, int64_t K, int out_dtype) {
    if (T < 1 || N < 1 || K < 32 || (K % 32) != 0 || T > (int64_t)1 << 30 || N > (int64_t)1 << 30 || K > (int64_t)1 << 30)
        return DUQPP_ERR_SHAPE;
    if (out_dtype != DUQPP_F32 && out_dtype != DUQPP_BF16) return DUQPP_ERR_DTYPE;
    TiledGemmParams p{nullptr, nullptr, nullptr, nullptr, (int)T, (int)N, (int)tiled_groups(K / 32),
                      nullptr, N, out_dtype == DUQPP_BF16};
    return choose_gemm_kernel(p);
}

int duqpp_rotq_gemm_tiled(const void* x_bf16, int64_t ldx, const float* R, int64_t n_rblocks,
                          const uint8_t* b_codes_t, const uint8_t* b_scales_t, int64_t T, int64_t N, int64_t K,
                          void* y, int out_dtype, int64_t ldy, void* workspace, size_t workspace_bytes,
                          void* stream) {
    if (!x_bf16 || !R || !b_codes_t || !b_scales_t || !y) return DUQPP_ERR_NULL;
    int st = validate_rows_K(T, K, ldx, n_rblocks);
    if (st != DUQPP_OK) return st;
    const size_t cb = round256(tiled_codes_bytes(T, K / 32));
    const size_t sb = round256(tiled_scales_bytes(T, K / 32));
    if (!workspace || workspace_bytes < cb + sb) return DUQPP_ERR_WORKSPACE;
    if (!aligned_to(workspace, 256)) return DUQPP_ERR_ALIGN;
    uint8_t* a_codes = static_cast<uint8_t*>(workspace);
    uint8_t* a_scales = a_codes + cb;
    return rotq_gemm_tiled_impl(x_bf16, ldx, R, n_rblocks, a_codes, a_scales, b_codes_t, b_scales_t, T, N, K, y, out_dtype,
                                ldy, stream);
}

size_t duqpp_packed_rotation_bytes(int64_t n_rblocks) {
    if (n_rblocks < 1 || n_rblocks > (int64_t)1 << 25) return 0;
    return (size_t)n_rblocks * kPackedRotationBlockBytes;
}

int duqpp_pack_rotation(const float* R, int64_t n_rblocks, void* R_packed, void* stream) {
    if (!R || !R_packed) return DUQPP_ERR_NULL;
    if (n_rblocks < 1 || n_rblocks > (int64_t)1 << 25) return DUQPP_ERR_SHAPE;
    if (!aligned_to(R, 4) || !aligned_to(R_packed, 16)) return DUQPP_ERR_ALIGN;
    int st = check_device();
    if (st != DUQPP_OK) return st;
    PackRotationParams p{R, static_cast<uint8_t*>(R_packed), (int)n_rblocks};
    return launch_pack_rotation(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_rotate_quantize_tiled_packed(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const void* R_packed,
                                       int64_t n_rblocks, uint8_t* x_codes_t, uint8_t* x_scales_t, void* stream) {
    return rotate_quantize_impl(x_bf16, T, K, ldx, R_packed, n_rblocks, x_codes_t, x_scales_t, nullptr, stream, true, true);
}

int duqpp_rotq_gemm_tiled_packed(const void* x_bf16, int64_t ldx, const void* R_packed, int64_t n_rblocks,
                                 const uint8_t* b_codes_t, const uint8_t* b_scales_t, int64_t T, int64_t N, int64_t K,
                                 void* y, int out_dtype, int64_t ldy, void* workspace, size_t workspace_bytes,
                                 void* stream) {
    if (!x_bf16 || !R_packed || !b_codes_t || !b_scales_t || !y) return DUQPP_ERR_NULL;
    int st = validate_rows_K(T, K, ldx, n_rblocks);
    if (st != DUQPP_OK) return st;
    const size_t cb = round256(tiled_codes_bytes(T, K / 32));
    const size_t sb = round256(tiled_scales_bytes(T, K / 32));
    if (!workspace || workspace_bytes < cb + sb) return DUQPP_ERR_WORKSPACE;
    if (!aligned_to(workspace, 256)) return DUQPP_ERR_ALIGN;
    uint8_t* a_codes = static_cast<uint8_t*>(workspace);
    return rotq_gemm_tiled_impl(x_bf16, ldx, R_packed, n_rblocks, a_codes, a_codes + cb, b_codes_t, b_scales_t, T, N, K, y,
                                out_dtype, ldy, stream, true);
}

int duqpp_rotq_gemm_fused_decode(const void* x_bf16, int64_t ldx, const void* R_packed, int64_t n_rblocks,
                                 const uint8_t* b_codes_t, const uint8_t* b_scales_t, int64_t T, int64_t N, int64_t K,
                                 void* y, int out_dtype, int64_t ldy, uint8_t* a_codes_t_dbg, uint8_t* a_scales_t_dbg,
                                 void* stream) {
    if (!x_bf16 || !R_packed || !b_codes_t || !b_scales_t || !y) return DUQPP_ERR_NULL;
    if ((a_codes_t_dbg == nullptr) != (a_scales_t_dbg == nullptr)) return DUQPP_ERR_NULL;
    int st = validate_rows_K(T, K, ldx, n_rblocks);
    if (st != DUQPP_OK) return st;
    if (T > kFusedMaxT || N < 1 || N > (int64_t)1 << 30 || ldy < N) return DUQPP_ERR_SHAPE;
    if (out_dtype != DUQPP_F32 && out_dtype != DUQPP_BF16) return DUQPP_ERR_DTYPE;
    if (!aligned_to(x_bf16, 16) || (ldx % 8) != 0 || !aligned_to(R_packed, 16) || !aligned_to(b_codes_t, 256) ||
        !aligned_to(b_scales_t, 256) || !aligned_to(y, out_dtype == DUQPP_F32 ? 4 : 2) ||
        (a_codes_t_dbg && (!aligned_to(a_codes_t_dbg, 256) || !aligned_to(a_scales_t_dbg, 256))))
        return DUQPP_ERR_ALIGN;
    st = check_device();
    if (st != DUQPP_OK) return st;
    FusedDecodeParams p{static_cast<const uint16_t*>(x_bf16), ldx, (int)T, static_cast<const uint8_t*>(R_packed),
                        n_rblocks == 1 ? 0 : kPackedRotationBlockBytes, b_codes_t, b_scales_t, (int)N, (int)(K / 32),
                        (int)tiled_groups(K / 32), y, ldy, out_dtype == DUQPP_BF16, a_codes_t_dbg, a_scales_t_dbg};
    return launch_rotq_gemm_fused_decode(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

int duqpp_fold_smoothing(const float* R, int64_t n_rblocks, const float* lambda, int64_t K, float* R_act,
                         float* R_wgt, void* stream) {
    if (!R || !lambda || !R_act || !R_wgt) return DUQPP_ERR_NULL;
    if (K < 32 || (K % 32) != 0 || K > (int64_t)1 << 30) return DUQPP_ERR_SHAPE;
    if (n_rblocks != 1 && n_rblocks != K / 32) return DUQPP_ERR_SHAPE;
    if (!aligned_to(R, 4) || !aligned_to(lambda, 4) || !aligned_to(R_act, 4) || !aligned_to(R_wgt, 4))
        return DUQPP_ERR_ALIGN;
    int st = check_device();
    if (st != DUQPP_OK) return st;
    FoldParams p{R, n_rblocks == 1 ? 0 : 1024, lambda, R_act, R_wgt, (int)(K / 32)};
    return launch_fold_smoothing(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

size_t duqpp_construct_rotation_workspace_bytes(int64_t T, int max_steps) {
    if (T < 1 || T > (int64_t)1 << 30 || max_steps < 0 || max_steps > 4096) return 0;
    return construct_workspace_bytes(T, max_steps);
}

int duqpp_construct_rotation(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const double* q_steps,
                             int max_steps, float* R_out, int32_t* info, double* peaks, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (!x_bf16 || !R_out || !info || (max_steps > 0 && !q_steps)) return DUQPP_ERR_NULL;
    int st = validate_rows_K(T, K, ldx, 1);
    if (st != DUQPP_OK) return st;
    if (max_steps < 0 || max_steps > 4096) return DUQPP_ERR_SHAPE;
    if (!aligned_to(x_bf16, 16) || (ldx % 8) != 0 || !aligned_to(q_steps, 8) || !aligned_to(R_out, 4) ||
        !aligned_to(info, 4) || !aligned_to(peaks, 8))
        return DUQPP_ERR_ALIGN;
    if (!workspace || workspace_bytes < construct_workspace_bytes(T, max_steps)) return DUQPP_ERR_WORKSPACE;
    if (!aligned_to(workspace, 256)) return DUQPP_ERR_ALIGN;
    st = check_device();
    if (st != DUQPP_OK) return st;
    ConstructParams p{static_cast<const uint16_t*>(x_bf16), ldx, T, K, q_steps, max_steps, R_out, info, peaks, workspace};
    return launch_construct_rotation(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DUQPP_OK : DUQPP_ERR_HIP;
}

const char* duqpp_status_string(int status) {
    switch (status) {
        case DUQPP_OK: return "ok";
        case DUQPP_ERR_NULL: return "null pointer";
        case DUQPP_ERR_SHAPE: return "bad shape";
        case DUQPP_ERR_ALIGN: return "misaligned pointer or stride";
        case DUQPP_ERR_DTYPE: return "bad output dtype";
        case DUQPP_ERR_WORKSPACE: return "workspace missing or too small";
        case DUQPP_ERR_ARCH: return "device is not gfx950";
        case DUQPP_ERR_HIP: return "HIP runtime error";
        case DUQPP_ERR_TOO_LARGE: return "problem exceeds the fixed scratch of the entry point that allocates nothing";
        default: return "unknown status";
    }
}

const char* duqpp_version(void) { return "duqpp 0.1 (gfx950)"; }

}  // extern "C"
