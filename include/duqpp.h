/*
 * duqpp.h -- C ABI of the DuQuant++ online inference hot path for AMD MI355X (gfx950).
 *
 * The path is the reformulated linear layer of the paper's Eq. 5 (Sec. 4.2):
 *
 *     Y = Q(X . R^) . Q(R^T . W)
 *
 * where R^ = BlockDiag(R_1 .. R_G) is orthogonal with 32x32 blocks aligned to the MXFP4
 * groups (Eq. 4, B = 32) and Q is MXFP4 quantisation (Sec. 3.2, Eq. 2): every 32
 * consecutive values along the reduction axis K share one E8M0 power-of-two scale
 * 2^(floor(log2 amax) - 2) and are stored as 4-bit E2M1 codes (round to nearest, ties to
 * even, saturating at +-6).  The smoothing diagonal of Eq. 3 enters through the rotation blocks
 * (duqpp_fold_smoothing); the kernels take any 32x32 fp32 blocks, orthogonal or not.
 *
 * Conventions (all entry points)
 *   - Every pointer is a DEVICE pointer unless its comment says "host".  The caller owns
 *     every buffer; the library allocates nothing.  What it keeps per device is set-up only: the
 *     architecture check and the kernels' shared-memory attributes (made at duqpp_init or at the first
 *     call on that device); no call leaves data behind that a later call reads.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work and return; they never synchronise.
 *   - Layouts are row-major with K contiguous.  G = K / 32.
 *       X       bf16  [T, K]      row stride ldx (elements)
 *       W       bf16  [N, K]      row n = output channel n (a Linear's weight), stride ldw
 *       R       fp32  [n_rblocks, 32, 32], R[j][r][c]: r = input channel of block j,
 *               c = output channel, so y[32j + c] = sum_r x[32j + r] * R[j][r][c]
 *               (row-vector form X . R^ of Eq. 5).  n_rblocks == G, or 1 when every
 *               group shares one block (the shared-matrix variant of Sec. 4.2).
 *       codes   uint8 [rows, K/2] element 2i in the LOW nibble of byte i, 2i+1 in the high
 *               nibble; code = sign<<3 | magnitude index into {0, .5, 1, 1.5, 2, 3, 4, 6}
 *       scales  uint8 [rows, G]   E8M0: value 2^(byte - 127); 0xFF is never produced
 *       Y       fp32 or bf16 [T, N], row stride ldy (elements)
 *   - Requirements checked on the host before any launch (of every stage, for the fused calls): pointers non-null, T/N >= 1,
 *     K >= 32 and K % 32 == 0, n_rblocks in {1, K/32}, ld >= the row length, X/W bases and
 *     row strides 16-byte aligned, codes bases 16-byte aligned, Y base aligned to its element.
 *   - Inputs must be finite; NaN/Inf are outside the contract.
 *   - Return value: DUQPP_OK or a negative duqpp_status; nothing throws or aborts.  DUQPP_ERR_HIP reports a
 *     failure of the call's own launches or runtime calls; an error that the caller's earlier work left in the
 *     runtime's error state is neither reported nor cleared.
 *   - Results are deterministic: the same inputs give bit-identical outputs on every call.
 */
#ifndef DUQPP_H
#define DUQPP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DUQPP_OK = 0,
    DUQPP_ERR_NULL = -1,      /* a required pointer is null */
    DUQPP_ERR_SHAPE = -2,     /* bad T/N/K/ld/n_rblocks */
    DUQPP_ERR_ALIGN = -3,     /* base pointer or stride not aligned as required */
    DUQPP_ERR_DTYPE = -4,     /* out_dtype is not a duqpp_dtype */
    DUQPP_ERR_WORKSPACE = -5, /* workspace missing or smaller than duqpp_gemm_workspace_bytes */
    DUQPP_ERR_ARCH = -6,      /* the current device is not gfx950 */
    DUQPP_ERR_HIP = -7,       /* a HIP runtime call or launch failed */
    DUQPP_ERR_TOO_LARGE = -8  /* duqpp_rotq_gemm_tiled_noalloc: the activations do not fit its fixed scratch */
} duqpp_status;

typedef enum { DUQPP_F32 = 0, DUQPP_BF16 = 1 } duqpp_dtype;

/*
 * Optional: the per-device set-up (architecture check, shared-memory attributes of the kernels) for the calling
 * thread's current device, so that no entry point has to do it at its first call -- e.g. before a stream capture.
 * Once per device is enough; further calls return at once.  Every entry point runs the part it needs by itself.
 */
int duqpp_init(void);

/*
 * Offline weight transform of Eq. 5: W^ = R^T . W, then Eq. 2 along K.  With W stored
 * [N, K], each row is rotated exactly like a token (W^T . R^).
 *   w_bf16   in   [N, K] bf16, stride ldw
 *   R        in   [n_rblocks, 32, 32] fp32
 *   w_codes  out  [N, K/2];  w_scales out [N, K/32]
 */
int duqpp_quantize_weights(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                           const float* R, int64_t n_rblocks,
                           uint8_t* w_codes, uint8_t* w_scales, void* stream);

/*
 * Online activation transform of Eq. 5 (Remark 2: the only online extra is X -> X . R^):
 * rotate every 32-channel block of every token by its block of R^ (Eq. 4), then quantise
 * to MXFP4 (Eq. 2).
 *   x_bf16     in   [T, K] bf16, stride ldx
 *   x_codes    out  [T, K/2];  x_scales out [T, K/32]
 *   y_rot_dbg  out  nullable; when given, [T, K] fp32 (stride K) receives the rotated values
 *                   the quantiser saw (used by parity tests; costs extra HBM traffic)
 */
int duqpp_rotate_quantize(const void* x_bf16, int64_t T, int64_t K, int64_t ldx,
                          const float* R, int64_t n_rblocks,
                          uint8_t* x_codes, uint8_t* x_scales,
                          float* y_rot_dbg, void* stream);

/*
 * W4A4 MXFP4 product of Eq. 5: Y[t, n] = sum_k val_a[t, k] * val_b[n, k], where val is the
 * value a code and its group scale stand for.  Products of E2M1 values are exact; sums are
 * accumulated in fp32 on the block-scaled matrix cores.
 *   a_codes/a_scales  in   [T, K/2], [T, K/32]   (from duqpp_rotate_quantize)
 *   b_codes/b_scales  in   [N, K/2], [N, K/32]   (from duqpp_quantize_weights)
 *   y                 out  [T, N] of out_dtype (duqpp_dtype), stride ldy; bf16 output is the
 *                          round-to-nearest-even of the fp32 result
 *   workspace         optional scratch of at least duqpp_gemm_workspace_bytes(T, N, K, 0) bytes, 256-byte
 *                     aligned.  With it the operands are first re-tiled into the scratch (see the tiled
 *                     layout below) and the fast kernel runs; with NULL a slower kernel reads the row-major
 *                     operands directly.  Same result either way up to the order of the fp32 additions.
 *                     A non-null workspace that is too small is an error (DUQPP_ERR_WORKSPACE).
 */
int duqpp_mxfp4_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                     const uint8_t* b_codes, const uint8_t* b_scales,
                     int64_t T, int64_t N, int64_t K,
                     void* y, int out_dtype, int64_t ldy,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Fused form of the online path: Y = Q(X . R^) . Q(W^) in one call, producing exactly the
 * codes duqpp_rotate_quantize would and the product duqpp_mxfp4_gemm would (two kernels on the stream
 * plus the re-tiling of the row-major weights; callers that keep the weights tiled use
 * duqpp_rotq_gemm_tiled and skip that).
 *   workspace  required: at least duqpp_gemm_workspace_bytes(T, N, K, 1) bytes, 256-byte aligned
 */
int duqpp_rotq_gemm(const void* x_bf16, int64_t ldx, const float* R, int64_t n_rblocks,
                    const uint8_t* b_codes, const uint8_t* b_scales,
                    int64_t T, int64_t N, int64_t K,
                    void* y, int out_dtype, int64_t ldy,
                    void* workspace, size_t workspace_bytes, void* stream);

/*
 * Offline: the rotation blocks in the form the tiled-output kernel consumes directly.  The blocks are calibrated
 * offline like the weights (Sec. 4.2), so what every online launch would otherwise redo at its start -- fetching each
 * 32 x 32 fp32 block and splitting every entry exactly into three bf16 pieces for the matrix cores (Eq. 4 / Eq. 5 at
 * fp32 accuracy) -- is done once here.  Same pieces, so the *_packed calls below return bit for bit what their
 * counterparts return for the fp32 blocks.
 *   R         in   [n_rblocks, 32, 32] fp32 (any n_rblocks >= 1)
 *   R_packed  out  duqpp_packed_rotation_bytes(n_rblocks) = 6144 * n_rblocks bytes, 16-byte aligned; per block
 *                  [piece: low, middle, high][half of the 32 input channels][lane 0..63][8 bf16], lane (c + 32 h)
 *                  holding R[16 s + 8 h + i][c] for i = 0..7 -- an opaque operand form, not an interchange format
 */
size_t duqpp_packed_rotation_bytes(int64_t n_rblocks);   /* host, pure; 0 for invalid arguments */
int duqpp_pack_rotation(const float* R, int64_t n_rblocks, void* R_packed, void* stream);

/*
 * Per-group normalised quantisation error, the statistic of Fig. 1 (Sec. 4.1): for every token t and every group j
 * of 32 channels, ||Q(y) - y||_2 / ||y||_2 with y the group after the block rotation of Eq. 4 and Q the quantiser of
 * Eq. 2 -- rotated and quantised by the same device code as duqpp_rotate_quantize, so it is the error of the codes
 * that call produces.  An analysis tool, not a step of the online path.
 *   x_bf16  in   [T, K] bf16, row stride ldx elements (multiple of 8), 16-byte aligned; T <= 32 * 65535
 *   R       in   [n_rblocks, 32, 32] fp32 with n_rblocks == K/32 or 1, or NULL: no rotation (y = x, the figure's
 *                unrotated setting; n_rblocks is then ignored)
 *   err     out  [T, K/32] fp32; -1 for a group whose 32 values are all zero (it has no ratio)
 *   mean    out  nullable; one double in device memory, 8-byte aligned: the mean of err over the groups that have a
 *                ratio (what the figure plots), summed in a fixed order; 0 when no group has one
 */
int duqpp_group_error(const void* x_bf16, int64_t T, int64_t K, int64_t ldx, const float* R, int64_t n_rblocks,
                      float* err, double* mean, void* stream);

/*
 * TEST ONLY: runs the quantiser stage of duqpp_rotate_quantize (group amax, E8M0 scale,
 * E2M1 rounding, packing -- Eq. 2) on caller-supplied fp32 values, so that every fp32 bit
 * pattern can be swept through the device code.
 *   y  in  [rows, K] fp32, stride ldy (elements, multiple of 4)
 */
int duqpp_quantize_f32_dbg(const float* y, int64_t rows, int64_t K, int64_t ldy,
                           uint8_t* codes, uint8_t* scales, void* stream);

/*
 * ---- Tiled operand layout: the fast path ---------------------------------------------------
 * The row-major [rows, K/2] + [rows, K/32] form above is the interchange contract.  The GEMM's
 * matrix-core operand for one lane is one MXFP4 group of one row (16 code bytes + 1 scale byte),
 * so the kernels run fastest on a layout that keeps the 32 rows of a row tile adjacent per group.
 * With RT = ceil(rows / 32) and GP = ceil((K/32) / 8) * 8:
 *     codes_t   uint8 [RT][GP][32][16]        16 code bytes of (row 32 rt + r, group j) at
 *                                             ((rt * GP + j) * 32 + r) * 16
 *     scales_t  uint8 [RT][GP/8][2][32][4]    scale of (row 32 rt + r, group j) at
 *                                             (((rt * GP/8 + j/8) * 2 + (j%8)/4) * 32 + r) * 4 + j%4
 * Padding rows and groups hold code 0 and scale 127.  Sizes come from duqpp_tiled_bytes; bases
 * must be 256-byte aligned.  The *_tiled entry points compute exactly what their row-major
 * counterparts compute (Eq. 5 / Eq. 2); only the placement of the bytes differs.
 */

/* Host, pure: bytes of the tiled codes and scales of a [rows, K] operand (either pointer may be null). */
int duqpp_tiled_bytes(int64_t rows, int64_t K, size_t* codes_bytes, size_t* scales_bytes);

/* Row-major -> tiled (writes the padding too) and back.  Pure byte permutations. */
int duqpp_tile_operand(const uint8_t* codes, const uint8_t* scales, int64_t rows, int64_t K,
                       uint8_t* codes_t, uint8_t* scales_t, void* stream);
int duqpp_untile_operand(const uint8_t* codes_t, const uint8_t* scales_t, int64_t rows, int64_t K,
                         uint8_t* codes, uint8_t* scales, void* stream);

/* duqpp_quantize_weights / duqpp_rotate_quantize with tiled outputs. */
int duqpp_quantize_weights_tiled(const void* w_bf16, int64_t N, int64_t K, int64_t ldw,
                                 const float* R, int64_t n_rblocks,
                                 uint8_t* w_codes_t, uint8_t* w_scales_t, void* stream);
int duqpp_rotate_quantize_tiled(const void* x_bf16, int64_t T, int64_t K, int64_t ldx,
                                const float* R, int64_t n_rblocks,
                                uint8_t* x_codes_t, uint8_t* x_scales_t, void* stream);

/* duqpp_rotate_quantize_tiled on packed rotation blocks (duqpp_pack_rotation; n_rblocks == K/32, or 1 for a shared block). */
int duqpp_rotate_quantize_tiled_packed(const void* x_bf16, int64_t T, int64_t K, int64_t ldx,
                                       const void* R_packed, int64_t n_rblocks,
                                       uint8_t* x_codes_t, uint8_t* x_scales_t, void* stream);

/* duqpp_mxfp4_gemm on tiled operands (no workspace). */
int duqpp_mxfp4_gemm_tiled(const uint8_t* a_codes_t, const uint8_t* a_scales_t,
                           const uint8_t* b_codes_t, const uint8_t* b_scales_t,
                           int64_t T, int64_t N, int64_t K,
                           void* y, int out_dtype, int64_t ldy, void* stream);

/*
 * NOT PART OF THE CONTRACT -- a hook for tests and measurements that may change with the kernels:
 * duqpp_mxfp4_gemm_tiled on one named kernel instead of the one the library would
 * pick for the shape, so that every kernel can be checked at every shape.  Same arguments, checks and result.
 * A kernel that cannot run the call returns DUQPP_ERR_SHAPE: the decode kernel takes T <= 128; the 256 x 256
 * kernel with bf16 output needs y 16-byte aligned and N, ldy multiples of 8.
 * duqpp_gemm_kernel_for reports (host, pure) which kernel DUQPP_GEMM_KERNEL_AUTO resolves to; it assumes an
 * aligned output.
 */
enum {
    DUQPP_GEMM_KERNEL_AUTO = 0,
    DUQPP_GEMM_KERNEL_DECODE = 1,   /* weight streaming, T <= 128 */
    DUQPP_GEMM_KERNEL_SMALL = 2,    /* 64 x 128 tiles */
    DUQPP_GEMM_KERNEL_MID = 3,      /* 128 x 256 tiles */
    DUQPP_GEMM_KERNEL_LARGE = 4     /* 256 x 256 tiles */
};
int duqpp_mxfp4_gemm_tiled_on(int kernel,
                              const uint8_t* a_codes_t, const uint8_t* a_scales_t,
                              const uint8_t* b_codes_t, const uint8_t* b_scales_t,
                              int64_t T, int64_t N, int64_t K,
                              void* y, int out_dtype, int64_t ldy, void* stream);
int duqpp_gemm_kernel_for(int64_t T, int64_t N, int64_t K, int out_dtype);

/*
 * duqpp_rotq_gemm with tiled weights.  workspace: at least the two sizes duqpp_tiled_bytes(T, K)
 * reports, each rounded up to 256, 256-byte aligned.
 */
int duqpp_rotq_gemm_tiled(const void* x_bf16, int64_t ldx, const float* R, int64_t n_rblocks,
                          const uint8_t* b_codes_t, const uint8_t* b_scales_t,
                          int64_t T, int64_t N, int64_t K,
                          void* y, int out_dtype, int64_t ldy,
                          void* workspace, size_t workspace_bytes, void* stream);

/* duqpp_rotq_gemm_tiled on packed rotation blocks. */
int duqpp_rotq_gemm_tiled_packed(const void* x_bf16, int64_t ldx, const void* R_packed, int64_t n_rblocks,
                                 const uint8_t* b_codes_t, const uint8_t* b_scales_t,
                                 int64_t T, int64_t N, int64_t K,
                                 void* y, int out_dtype, int64_t ldy,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * The online path of Eq. 5 as ONE kernel, shaped for up to 32 tokens: every workgroup rotates (Eq. 4) and quantises
 * (Eq. 2) the activations it needs in the prologue of its K steps and multiplies them with its 32 output channels of
 * the tiled weights; no activation operand exists in memory and no workspace is needed.  More than 32 tokens run as
 * independent tiles of 32 tokens, each streaming the weights again.  Same device code for rotation
 * and quantiser as duqpp_rotate_quantize_tiled, hence the same codes bit for bit; the product is that of
 * duqpp_mxfp4_gemm_tiled on those codes up to the order of the fp32 additions.
 * Each of the N / 32 workgroups repeats the rotation of the whole token tile, so this form is slower than the two
 * launches of duqpp_rotq_gemm_tiled at every benchmark shape (LLaMA-3-8B decode, 1 to 16 tokens: 27-52 us against
 * 10-11 us on one MI355X; prefill shapes: tens of milliseconds against tenths) and the library never picks it by itself: it is here so that the one-kernel form can be
 * checked and measured.
 *   T                    1 .. 32 * 65535
 *   R_packed             from duqpp_pack_rotation; n_rblocks == K/32, or 1 for a shared block
 *   a_codes_t_dbg, a_scales_t_dbg   nullable (both or neither): receive the activation operand the product was formed
 *                        from, in the tiled layout for T rows (duqpp_tiled_bytes(T, K)), 256-byte aligned
 */
int duqpp_rotq_gemm_fused_decode(const void* x_bf16, int64_t ldx, const void* R_packed, int64_t n_rblocks,
                                 const uint8_t* b_codes_t, const uint8_t* b_scales_t,
                                 int64_t T, int64_t N, int64_t K,
                                 void* y, int out_dtype, int64_t ldy,
                                 uint8_t* a_codes_t_dbg, uint8_t* a_scales_t_dbg, void* stream);

/*
 * duqpp_rotq_gemm_tiled for callers that cannot allocate or cannot hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without the workspace), same
 * checks, same kernels and bit-identical results; the activation operand between the two kernels lives in a
 * fixed array of duqpp_noalloc_scratch_bytes() = 8 MiB that is part of the library's device code (one copy per GPU,
 * held until the process ends).  The call allocates and frees nothing.
 *   - Limit: the two sizes duqpp_tiled_bytes(T, K) reports, each rounded up to 256, must fit the array (e.g.
 *     T <= 1088 at K = 14336, T <= 544 at K = 28672); beyond it the call returns DUQPP_ERR_TOO_LARGE and
 *     launches nothing.
 *   - Every call on a GPU uses that GPU's one array: calls that may overlap on a GPU (different streams, several
 *     host threads) race and must be ordered by the caller.  Nothing of an earlier call's contents is read.
 *   - The array's device address is looked up once per device (at duqpp_init, else at the first call there).
 */
size_t duqpp_noalloc_scratch_bytes(void);   /* host, pure */
int duqpp_rotq_gemm_tiled_noalloc(const void* x_bf16, int64_t ldx, const float* R, int64_t n_rblocks,
                                  const uint8_t* b_codes_t, const uint8_t* b_scales_t,
                                  int64_t T, int64_t N, int64_t K,
                                  void* y, int out_dtype, int64_t ldy, void* stream);

/*
 * Smoothing (Sec. 4.2, Eq. 3) merged into the rotation blocks, offline.  Eq. 5 in full is
 * Y = Q(X Lambda^-1 R^) . Q(R^T Lambda W) with a diagonal Lambda over the reduction axis.  A diagonal times a
 * block-diagonal matrix is block-diagonal, so with
 *     R_act[j][r][c] = R[j][r][c] / lambda[32 j + r],      R_wgt[j][r][c] = R[j][r][c] * lambda[32 j + r]
 * duqpp_rotate_quantize(x, R_act) produces Q(X Lambda^-1 R^) and duqpp_quantize_weights(w, R_wgt) produces
 * Q(R^T Lambda W): the online path is unchanged and costs nothing extra.
 *   R       in   [n_rblocks, 32, 32] fp32, n_rblocks == K/32 or 1 (a shared block expands to K/32 blocks)
 *   lambda  in   [K] fp32, finite and positive (not checked: it lives on the device)
 *   R_act, R_wgt  out  [K/32, 32, 32] fp32 each; must not alias R
 */
int duqpp_fold_smoothing(const float* R, int64_t n_rblocks, const float* lambda, int64_t K,
                         float* R_act, float* R_wgt, void* stream);

/*
 * Offline: greedy outlier-aware construction of the rotation block that all groups share (Sec. 4.2, paragraph
 * "Fine-grained Block-diagonal Rotation", steps (1)-(3)).  The paper sketches the construction; the reading built
 * here: take the block of 32 channels holding the largest |x| of the calibration activations; repeat max_steps
 * times: find the channel with the largest magnitude, multiply by  E_d . H . diag(1, Q'_t) . E_d  (E_d exchanges
 * that channel with channel 0, H is the normalised 32 x 32 Sylvester-Hadamard matrix, Q'_t the caller's t-th
 * orthogonal 31 x 31 draw); keep the product after the step count with the smallest peak |value| (0 steps = the
 * identity if nothing lowers it).  fp64 in a fixed operation order: the result does not depend on the launch shape.
 *   x_bf16     in   [T, K] bf16 calibration activations, row stride ldx (elements, multiple of 8), 16-byte aligned
 *   q_steps    in   [max_steps, 31, 31] fp64, each orthogonal (not checked: it lives on the device)
 *   max_steps       0 .. 4096 (the paper uses 128)
 *   R_out      out  [32, 32] fp32, R[r][c] with r the input channel: pass it with n_rblocks = 1
 *   info       out  2 x int32 on the device: index of the block the matrix was built from, steps kept
 *   peaks      out  nullable, [max_steps + 1] fp64 on the device: peak |value| after 0, 1, ... steps
 *   workspace       at least duqpp_construct_rotation_workspace_bytes(T, max_steps) bytes, 256-byte aligned
 * Enqueues max_steps + 4 kernels on the stream.  Errors as for the other calls.
 */
size_t duqpp_construct_rotation_workspace_bytes(int64_t T, int max_steps);   /* host, pure; 0 for invalid arguments */
int duqpp_construct_rotation(const void* x_bf16, int64_t T, int64_t K, int64_t ldx,
                             const double* q_steps, int max_steps,
                             float* R_out, int32_t* info, double* peaks,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Host, pure: scratch bytes duqpp_mxfp4_gemm (fused = 0) can use or duqpp_rotq_gemm (fused = 1) needs:
 * room for both operands in the tiled layout.  0 for invalid shapes. */
size_t duqpp_gemm_workspace_bytes(int64_t T, int64_t N, int64_t K, int fused);

/*
 * Host-only argument checks, exactly the ones the entry points run before launching.
 * They never touch the device, so they can be called without a GPU.
 */
int duqpp_validate_rotate_quantize(const void* x_bf16, int64_t T, int64_t K, int64_t ldx,
                                   const float* R, int64_t n_rblocks,
                                   const uint8_t* codes, const uint8_t* scales);
int duqpp_validate_mxfp4_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                              const uint8_t* b_codes, const uint8_t* b_scales,
                              int64_t T, int64_t N, int64_t K,
                              const void* y, int out_dtype, int64_t ldy,
                              const void* workspace, size_t workspace_bytes,
                              int fused /* 0 separate, 1 fused, 2 tiled operands (no workspace) */);

/* Static strings. */
const char* duqpp_status_string(int status);
const char* duqpp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DUQPP_H */
