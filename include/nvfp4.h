/*
 * nvfp4.h -- C ABI of the MI355X (gfx950) FP4 quantized linear layer.
 *
 * Implements the hot path of "FP4 All the Way: Fully Quantized Training of
 * LLMs": the block quantization operation Q (Sec. 3: E2M1 elements in blocks
 * that share one E4M3 or E8M0 scale; Sec. 3.2: round-to-nearest or stochastic
 * rounding) and the three GEMMs of every linear layer (Eqs. 4-6).
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or keeps them.  Scratch memory comes in through a
 *     `workspace` argument whose size the matching *_workspace_bytes() call
 *     returns; the workspace may be reused by the next call on the same stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued asynchronously; no call synchronizes.
 *   - Arguments are validated on the host before anything is launched; a bad
 *     argument returns an error code and enqueues nothing.
 *   - Tensor pointers must be 16-byte aligned, leading dimensions must keep
 *     every row 16-byte aligned.
 *   - Non-finite inputs give unspecified codes (no error).
 *   - Row-major everywhere.  "codes" hold two 4-bit E2M1 codes per byte, the
 *     element with the even index along the blocked axis in the low nibble.
 *     Code bits: sign | exponent(2) | mantissa(1); magnitudes
 *     {0, .5, 1, 1.5, 2, 3, 4, 6}.  "scales" hold one byte per block: E4M3
 *     (bias 7, finite-only, sign bit never set) or E8M0 (2^(byte-127)).
 *   - Value of a quantized element: (-1)^sign * magnitude * scale * g, where g
 *     is the per-tensor fp32 scale (1 when the format has none).
 */
#ifndef NVFP4_H
#define NVFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NVFP4_OK = 0,
    NVFP4_EINVAL = 1,       /* null pointer, unknown enum value, bad axis or flag */
    NVFP4_ESHAPE = 2,       /* non-positive size, or blocked axis not a multiple of the block */
    NVFP4_EALIGN = 3,       /* pointer or leading dimension breaks 16-byte alignment */
    NVFP4_EUNSUPPORTED = 4, /* format combination the library does not implement */
    NVFP4_EWORKSPACE = 5,   /* workspace missing or too small */
    NVFP4_EHIP = 6          /* the HIP runtime reported a launch error */
} nvfp4_status;

typedef enum { NVFP4_RTN = 0, NVFP4_SR = 1 } nvfp4_rounding;
typedef enum { NVFP4_F32 = 0, NVFP4_BF16 = 1 } nvfp4_dtype;
typedef enum { NVFP4_SCALE_E4M3 = 0, NVFP4_SCALE_E8M0 = 1 } nvfp4_scale_fmt;

/* Block format (Sec. 3, Table 1).  NVFP4 = {16, E4M3, 1}; MXFP4 = {32, E8M0, 0};
 * the block-size study of Sec. 3.1 / Fig. 2 adds {32|64|128, E4M3, 1}.
 * block must be 16, 32, 64 or 128.  E8M0 scales take no tensor scale. */
typedef struct {
    int32_t block;
    int32_t scale;        /* nvfp4_scale_fmt */
    int32_t tensor_scale; /* 1: per-tensor fp32 scale g; 0: g = 1 */
} nvfp4_format;

/*
 * Three switches exist for cross-checking; the first two change no result bit.  They are taken from the environment once,
 * by the first call that needs them, and stay fixed for the process unless nvfp4_cross_check_switches replaces them:
 *   bit 0 / NVFP4_SOFT_CONVERT=1    round elements and block scales with integer/fp32 arithmetic instead of the
 *                                   gfx950 convert instructions (then nvfp4_quantize_dual runs as two kernels, no slabs);
 *   bit 1 / NVFP4_PLAIN_OPERANDS=1  the fused linear entries keep their internal operands row-major (no slabs);
 *   bit 2 / NVFP4_FP4_WIDE_BLOCKS=1 GEMMs with E4M3 scales at blocks of 64 / 128 (K a multiple of 128) run on the FP4 matrix
 *                                   instruction with unit scales and rescale each block's partial sum in binary32, instead
 *                                   of expanding their operands to fp16 like NVFP4 (this one changes the accumulation
 *                                   order, within the 1e-5 bound; measured 1.8x / 3x slower, so it is off by default).
 * nvfp4_cross_check_switches(set, value) returns the switches in force and, with set != 0, replaces them by
 * `value` (bits 0-2) for every later call of the process.  It is a test hook: call it only while no other thread is
 * inside the library, and not between a forward call that fills a `saved` buffer and its backward call
 * (nvfp4_linear_bwd refuses such a buffer with NVFP4_EINVAL).
 */
#define NVFP4_SWITCH_SOFT_CONVERT 1u
#define NVFP4_SWITCH_PLAIN_OPERANDS 2u
#define NVFP4_SWITCH_FP4_WIDE_BLOCKS 4u
uint32_t nvfp4_cross_check_switches(int set, uint32_t value);

/* nvfp4_quantize flags */
#define NVFP4_PRESET_TSCALE 1u /* read g from *tensor_scale instead of computing it */
/* nvfp4_quantize_dual only: write the row-blocked / the column-blocked output in the slab layout (below) */
#define NVFP4_SLAB_ROWS 2u
#define NVFP4_SLAB_COLS 4u

const char *nvfp4_status_string(nvfp4_status s);

/* Output sizes in bytes for a logical [rows, cols] tensor. */
size_t nvfp4_codes_bytes(int64_t rows, int64_t cols);
size_t nvfp4_scales_bytes(int64_t rows, int64_t cols, int axis, const nvfp4_format *f);

/* Scratch sizes in bytes. */
size_t nvfp4_quantize_workspace_bytes(int64_t rows, int64_t cols);
size_t nvfp4_linear_fwd_workspace_bytes(int64_t M, int64_t N, int64_t K, const nvfp4_format *f);
size_t nvfp4_linear_bwd_workspace_bytes(int64_t M, int64_t N, int64_t K, const nvfp4_format *f);
/* Size of the buffer through which nvfp4_linear_fwd hands Q(X^T), Q(W^T) and the tensor scales to nvfp4_linear_bwd. */
size_t nvfp4_linear_saved_bytes(int64_t M, int64_t N, int64_t K, const nvfp4_format *f);

/*
 * Per-tensor scale g (not in the paper; it fixes only the element and block
 * scale formats): g = max|x| / (6 * 448), so that the block holding the
 * largest element gets the largest E4M3 scale.  g = 1 for an all-zero tensor;
 * g is never below 2^-117.  Writes g to tensor_scale[0] (device fp32).
 * x: [rows, cols] with leading dimension ld (elements), dtype dt.
 * workspace: >= nvfp4_quantize_workspace_bytes(rows, cols).
 */
nvfp4_status nvfp4_tensor_scale(const void *x, nvfp4_dtype dt, int64_t rows, int64_t cols,
                                int64_t ld, float *tensor_scale, void *workspace,
                                size_t workspace_bytes, void *stream);

/*
 * Q of Eqs. 1-6: block-quantize x [rows, cols] (leading dimension ld).
 * Blocks of f->block elements run along `axis`, which must be the contraction
 * axis of the GEMM the result feeds:
 *   axis 1 (along a row):    codes [rows, cols/2], scales [rows, cols/block]
 *   axis 0 (down a column):  codes [cols, rows/2], scales [cols, rows/block]
 *                            -- the output is the quantized TRANSPOSE, which is
 *                            how Eqs. 2-3 consume W^T and a^T.
 * The blocked length (cols for axis 1, rows for axis 0) must be a multiple of
 * the block size.
 *
 * Per block (E4M3 scales): a = max|x|; scale byte = E4M3_RNE_sat(a * (1/(6g)));
 * with s its value and d = s*g, element magnitudes are min(|x * (1/d)|, 6)
 * rounded to the E2M1 grid; a zero scale byte gives zero magnitudes.
 * Per block (E8M0 scales): byte = clamp(floor(log2 a) - 2 + 127, 0, 254),
 * elements x * 2^(127-byte), same clamp and rounding.
 * All of this in fp32, one rounding per operation.
 *
 * rounding (Sec. 3.2, Eqs. 4-6): NVFP4_RTN = nearest grid value, ties to the
 * even code; NVFP4_SR = round up with probability equal to the relative
 * distance t from the lower neighbour (exactly: up iff u + 1/2 <= 65536 t for
 * the element's 16-bit draw u), drawn from 16 bits of Philox4x32-10 with
 * key = seed and counter = (row-major index of the element in x) >> 3; the
 * draw does not depend on `axis`.  `seed` is ignored for RTN.
 *
 * tensor_scale: device fp32[1].  With f->tensor_scale == 0 it is written with
 * 1.  Otherwise it is computed from x and written, unless flags has
 * NVFP4_PRESET_TSCALE, in which case it is read (and used as max(g, 2^-117)).
 * workspace: >= nvfp4_quantize_workspace_bytes(rows, cols); may be NULL with
 * NVFP4_PRESET_TSCALE or a format without tensor scale.
 */
nvfp4_status nvfp4_quantize(const void *x, nvfp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                            int axis, nvfp4_rounding rounding, uint64_t seed,
                            const nvfp4_format *f, uint8_t *codes, uint8_t *scales,
                            float *tensor_scale, uint32_t flags, void *workspace,
                            size_t workspace_bytes, void *stream);

/*
 * nvfp4_quantize for callers that cannot allocate device memory or carry a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * nvfp4_quantize without `workspace`: the scratch (header + per-workgroup partial maxima of the tensor-maximum
 * pass) is a 65792-byte array inside the library's device image, one per GPU, held until the process ends.  The
 * call allocates nothing.  Limit: any dense tensor (ld == cols) fits; a strided one needs one partial maximum per
 * 8192-element span of a row and at most 16384 of them (e.g. 16384 rows of up to 8192 columns) -- beyond that the
 * call returns NVFP4_EWORKSPACE and enqueues nothing.  With NVFP4_PRESET_TSCALE or a format without tensor scale
 * the array is not touched.  Every call on a GPU shares that GPU's array: calls whose kernels may overlap on one
 * GPU (different streams, or threads) race on it and must be ordered by the caller; calls on one stream are safe.
 * Nothing in the array has to start at zero (every partial maximum is written before it is read).
 * NVFP4_EHIP if the runtime cannot report the array's address on the current device.
 */
nvfp4_status nvfp4_quantize_static(const void *x, nvfp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                   int axis, nvfp4_rounding rounding, uint64_t seed,
                                   const nvfp4_format *f, uint8_t *codes, uint8_t *scales,
                                   float *tensor_scale, uint32_t flags, void *stream);

/*
 * Both orientations of one tensor in one pass over it: Eqs. 5-6 use the output
 * gradient blocked along N (for dX) and along M (for dW), Eqs. 4-5 use W blocked
 * along K and along N.  The results are exactly those of
 *   nvfp4_quantize(x, ..., axis 1, rounding_rows, seed_rows, ...) -> codes_rows [rows, cols/2], scales_rows [rows, cols/block]
 *   nvfp4_quantize(x, ..., axis 0, rounding_cols, seed_cols, ...) -> codes_cols [cols, rows/2], scales_cols [cols, rows/block]
 * with one shared per-tensor scale (same rule, flags and workspace as
 * nvfp4_quantize).  rows and cols must both be multiples of the block size.
 * Blocks of 16 and 32 with 16-byte aligned rows of x run as one fused kernel
 * (x is read once), except SR rows with RtN columns; other cases run the two
 * single-orientation kernels.
 * All output pointers device memory, 16-byte aligned, owned by the caller.
 */
nvfp4_status nvfp4_quantize_dual(const void *x, nvfp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                                 nvfp4_rounding rounding_rows, uint64_t seed_rows,
                                 nvfp4_rounding rounding_cols, uint64_t seed_cols,
                                 const nvfp4_format *f, uint8_t *codes_rows, uint8_t *scales_rows,
                                 uint8_t *codes_cols, uint8_t *scales_cols, float *tensor_scale,
                                 uint32_t flags, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Block-scaled GEMM shared by Eqs. 4-6, operands stored with the contraction
 * axis contiguous ("NT"):
 *   out[i, j] = gA * gB * sum_k a[i, k] * b[j, k],   a = magnitude*scale of A, same for B
 * A_codes [M, K/2], A_scales [M, K/block]; B_codes [N, K/2], B_scales [N, K/block].
 * tensor_scales: device fp32[2] = {gA, gB}.
 * out: [M, N] of out_dt with leading dimension ldc.  Products are exact;
 * accumulation is fp32.
 * K must be a multiple of the block and of 32, at most 2^23; M, N >= 1.
 * Formats: E4M3 scales with blocks 16/32/64/128 (operands expanded exactly to
 * fp16 for the matrix instruction; blocks 64/128 have a second, slower route on
 * the FP4 matrix instruction behind a cross-check switch), and E8M0 scales with
 * block 32 (MXFP4, run on the FP4 matrix instruction as stored); other pairs:
 * NVFP4_EUNSUPPORTED.
 */
nvfp4_status nvfp4_gemm(int64_t M, int64_t N, int64_t K, const nvfp4_format *f,
                        const uint8_t *A_codes, const uint8_t *A_scales, const uint8_t *B_codes,
                        const uint8_t *B_scales, const float *tensor_scales, void *out,
                        nvfp4_dtype out_dt, int64_t ldc, void *stream);

/*
 * Slab layout of an NVFP4 operand (block 16, E4M3 scales) or an MXFP4 operand
 * (block 32, E8M0 scales), an alternative to the row-major [rows, K/2] codes
 * and [rows, K/block] scales above.  It holds the same bytes (same
 * quantization, Sec. 3), arranged the way the large GEMM kernels fetch them: K
 * must be a multiple of 128; the rows are padded to a multiple of 256; codes
 * are [rows/256][K/128] slabs of 16 KB, scales the same grid of slabs of 2 KB
 * (NVFP4: 8 scale bytes per row and K tile) or 1 KB (MXFP4: 4).  Inside a slab,
 * row r (0..255) of the tile sits at position
 * p(r) = (r & ~63) | ((r & 7) << 3) | ((r >> 3) & 7) and owns 64 code bytes
 * (its 128 elements of that K tile, even element in the low nibble) or its 8
 * resp. 4 scale bytes.  Padding rows are never written and never reach a
 * stored output.
 * nvfp4_quantize_dual writes it on request (NVFP4_SLAB_ROWS / NVFP4_SLAB_COLS:
 * the one-pass kernel must apply, i.e. 16-byte aligned rows of x and not SR rows
 * with RtN columns, else NVFP4_EUNSUPPORTED; cols resp. rows a multiple of 128,
 * else NVFP4_ESHAPE); the output
 * buffers then need nvfp4_slab_codes_bytes / nvfp4_slab_scales_bytes (rows =
 * rows of the OPERAND: cols of x for the column-blocked side;
 * nvfp4_slab_scales_bytes is stated for NVFP4, an MXFP4 operand uses the first
 * half of it).  nvfp4_gemm_slab is nvfp4_gemm with either operand in this
 * layout (a_slab, b_slab non-zero: codes AND scales of that operand); it
 * applies where nvfp4_gemm_takes_slabs returns 1 (NVFP4: K a multiple of 128
 * and at least 128 output tiles of 256 x 256; MXFP4: K a multiple of 128 and at
 * least 512), otherwise NVFP4_EUNSUPPORTED.  The fused linear entries below use
 * the layout internally wherever it applies; results are bit-identical either
 * way.
 */
size_t nvfp4_slab_codes_bytes(int64_t rows, int64_t K);
size_t nvfp4_slab_scales_bytes(int64_t rows, int64_t K);
int nvfp4_gemm_takes_slabs(int64_t M, int64_t N, int64_t K, const nvfp4_format *f);
nvfp4_status nvfp4_gemm_slab(int64_t M, int64_t N, int64_t K, const nvfp4_format *f,
                             const uint8_t *A_codes, const uint8_t *A_scales, const uint8_t *B_codes,
                             const uint8_t *B_scales, const float *tensor_scales, void *out,
                             nvfp4_dtype out_dt, int64_t ldc, int a_slab, int b_slab, void *stream);

/*
 * Forward GEMM, Eq. 4:  Y[M, N] = Q_RtN(X[M, K]) * Q_RtN(W[N, K])^T, blocks along K.
 * X, W dense row-major of in_dt; Y dense row-major of out_dt.
 * xw_scales_out: NULL, or device fp32[2] that receives the per-tensor scales
 * {gX, gW} this call derived from max|X| and max|W| (1, 1 for a format without
 * tensor scale), to be handed to nvfp4_linear_bwd for the same X and W.
 * saved: NULL, or device memory of >= nvfp4_linear_saved_bytes(M, N, K, f)
 * bytes, 256-byte aligned, owned by the caller and kept until the backward call:
 * the passes that quantize X and W for Eq. 4 then also write what Eqs. 5-6 need
 * of them -- Q_SR(X^T) (blocks along M, SR stream bwd_seed + 2), Q_RtN(W^T)
 * (blocks along N) and {gX, gW} -- so that nvfp4_linear_bwd, given the same
 * `saved` and seed == bwd_seed, reads neither X nor W.  Requires M and N to be
 * multiples of the block size and of 32 (NVFP4_ESHAPE otherwise).  Y is the
 * same with and without `saved`.  bwd_seed is ignored when saved is NULL.
 * The buffer's contents are private to the library (row-major or slab layout
 * per operand, whichever the consuming GEMM of the backward call will read):
 * pass it to nvfp4_linear_bwd in the same process and leave it alone.  Its
 * header carries a tag (M, N, K, format, bwd_seed, operand layouts) that the
 * backward call checks.
 */
nvfp4_status nvfp4_linear_fwd(const void *X, const void *W, void *Y, int64_t M, int64_t N,
                              int64_t K, nvfp4_dtype in_dt, nvfp4_dtype out_dt,
                              const nvfp4_format *f, void *workspace, size_t workspace_bytes,
                              void *stream, float *xw_scales_out, void *saved, uint64_t bwd_seed);

/*
 * Backward and update GEMMs, Eqs. 5-6, for upstream gradient dY[M, N]:
 *   dX[M, K] = Q_SR(dY) * Q_RtN(W^T)^T     blocks along N; SR stream `seed`
 *   dW[N, K] = Q_SR(dY^T) * Q_SR(X^T)^T    blocks along M; SR streams seed+1 (dY), seed+2 (X)
 * Either of dX, dW may be NULL to skip that GEMM.
 * xw_scales: NULL, or device fp32[2] = {gX, gW} as nvfp4_linear_fwd returned
 * them for these X and W: the two tensor-maximum passes over X and W are then
 * skipped (the per-tensor scale is a function of the tensor alone, so the
 * results are identical).  Ignored for a format without tensor scale.
 * saved: NULL, or what nvfp4_linear_fwd wrote for the same M, N, K, format and
 * bwd_seed == seed: X, W and xw_scales are then not read (they may be NULL) and
 * the results are identical to those of the call without `saved`.  A buffer
 * that one of the last 256 forward calls of this process wrote for different
 * shapes, format, seed or cross-check switches is refused with NVFP4_EINVAL
 * before anything is launched; for a buffer the library has no host record of,
 * the tag in the buffer itself is compared on the device and a mismatch turns
 * dX and dW into NaN.
 * With both dX and dW requested, dY is read once for its two quantizations.
 */
nvfp4_status nvfp4_linear_bwd(const void *dY, const void *X, const void *W, void *dX, void *dW,
                              int64_t M, int64_t N, int64_t K, nvfp4_dtype in_dt,
                              nvfp4_dtype out_dt, const nvfp4_format *f, uint64_t seed,
                              void *workspace, size_t workspace_bytes, void *stream,
                              const float *xw_scales, const void *saved);

/*
 * The weight operand of Eqs. 4-5 quantized once for every micro-batch of an
 * optimizer step: with a global batch of several micro-batches per device
 * (Sec. 5 trains with 4M tokens per step on 256 devices) W does not change
 * between them, and Eqs. 4 and 5 use the same Q_RtN(W) / Q_RtN(W^T) each time.
 * nvfp4_quantize_weight runs the tensor-maximum pass and one dual-orientation
 * pass over W[N, K] (dense row-major of dt) and leaves, in the caller-owned
 * device buffer w_operands (>= nvfp4_weight_operands_bytes(N, K, f) bytes,
 * 256-byte aligned): gW, Q_RtN(W) blocked along K and Q_RtN(W^T) blocked along
 * N, each in the layout (row-major or slabs) that the GEMMs of micro-batches of
 * M tokens will read -- so M here must be the M of the later calls.  N and K
 * must be multiples of the block size and of 32.  workspace: >=
 * nvfp4_quantize_workspace_bytes(N, K) (not needed without tensor scale).
 * The buffer's contents are private to the library; it carries a tag (M, N, K,
 * format, layouts) that the calls below check (NVFP4_EINVAL on a mismatch).
 *
 * nvfp4_linear_fwd_wq / nvfp4_linear_bwd_wq are nvfp4_linear_fwd /
 * nvfp4_linear_bwd with w_operands in place of W: no pass over W is made (no
 * maximum, no quantizer), everything else -- arguments, `saved` hand-over of
 * Q_SR(X^T), results bit for bit -- is the same.  A `saved` buffer filled by
 * nvfp4_linear_fwd_wq holds only the X part and must go to nvfp4_linear_bwd_wq.
 * Since W's operands depend on nothing but W, nvfp4_quantize_weight can run on
 * another stream, under the GEMMs of another layer.
 */
size_t nvfp4_weight_operands_bytes(int64_t N, int64_t K, const nvfp4_format *f);
nvfp4_status nvfp4_quantize_weight(const void *W, nvfp4_dtype dt, int64_t M, int64_t N, int64_t K,
                                   const nvfp4_format *f, void *w_operands, void *workspace,
                                   size_t workspace_bytes, void *stream);
nvfp4_status nvfp4_linear_fwd_wq(const void *X, const void *w_operands, void *Y, int64_t M, int64_t N,
                                 int64_t K, nvfp4_dtype in_dt, nvfp4_dtype out_dt,
                                 const nvfp4_format *f, void *workspace, size_t workspace_bytes,
                                 void *stream, float *xw_scales_out, void *saved, uint64_t bwd_seed);
nvfp4_status nvfp4_linear_bwd_wq(const void *dY, const void *X, const void *w_operands, void *dX, void *dW,
                                 int64_t M, int64_t N, int64_t K, nvfp4_dtype in_dt,
                                 nvfp4_dtype out_dt, const nvfp4_format *f, uint64_t seed,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 const float *xw_scales, const void *saved);

/*
 * A tensor quantized along both axes, as nvfp4_quantize_dual writes it: the operand pair a backward call needs of
 * its upstream gradient (Eq. 5 uses it blocked along N, Eq. 6 along M).  All pointers are device memory owned by
 * the caller; layout = NVFP4_SLAB_ROWS / NVFP4_SLAB_COLS bits for a side stored in the slab layout; g = device
 * fp32[1], the per-tensor scale shared by both sides (written as 1 for a format without tensor scale).
 */
typedef struct {
    uint8_t *codes_rows, *scales_rows; /* [rows, cols/2], [rows, cols/block] */
    uint8_t *codes_cols, *scales_cols; /* [cols, rows/2], [cols, rows/block] */
    float *g;
    uint32_t layout;
} nvfp4_dual_operands;

/*
 * SwiGLU backward fused with the quantizers of its results.  In the SwiGLU MLP of the Sec. 5 model the gate and
 * up layers' upstream gradients are dG = dH u sigma(g) (1 + g (1 - sigma(g))) and dU = dH g sigma(g), g and u the
 * two layers' forward outputs and dH the down layer's input gradient; Eqs. 5-6 then need Q_SR(dG), Q_SR(dU)
 * blocked along both axes.  This call produces those four operands from dH, G, U [M, F] (dense row-major of dt)
 * with the tensor-maximum pass of both quantizers folded into the elementwise pass (one pass over dH, G, U leaves the
 * maxima of dG and dU; then one dual-orientation pass per result), and optionally without dG or dU ever being stored.  The paper gives no arithmetic for the elementwise step; it is fixed in binary32
 * (one rounding per operation): e = exp(-|g|) by k = rint(t log2 e), r = t - k ln2 (two fused steps, ln2 = 0.693145751953125
 * + 1.42860677e-6), degree-6 Taylor polynomial in Horner form with fused multiply-adds, exact scaling by 2^k, t clamped
 * at -87; sigma = (g >= 0 ? 1 : e) / (1 + e); dG = (dH u)(sigma (1 + g (1 - sigma))); dU = dH (g sigma); each result
 * rounded to dt (bf16: nearest even) before it is quantized -- i.e. the results equal nvfp4_quantize_dual of the
 * tensors an elementwise kernel with this arithmetic would have stored.
 *   seed_gate, seed_up   SR streams: rows side seed, columns side seed + 1 (what nvfp4_linear_bwd uses for dY)
 *   dG, dU               outputs; layout bits choose row-major or slabs per side (slabs: F resp. M a multiple of 128)
 *   dG_store, dU_store   both NULL: nothing but the operands is written (each result is evaluated in the maxima
 *                        pass and again in its quantizer pass); both given (device, [M, F] of dt, 16-byte aligned):
 *                        the maxima pass also stores the two results and the quantizer passes read them back -- the
 *                        same bits out, the tensors available to the caller, and the faster form on this GPU, where
 *                        the quantizer passes are bound by vector-ALU work rather than by memory
 *   workspace            >= nvfp4_swiglu_bwd_workspace_bytes(M, F), 16-byte aligned (not needed without tensor scale
 *                        unless the results are stored)
 * Formats: NVFP4 {16, E4M3, 1} and MXFP4 {32, E8M0, 0}; M and F multiples of the block size; not with the
 * software-convert cross-check switch (NVFP4_EUNSUPPORTED).  Other errors as nvfp4_quantize_dual.
 * nvfp4_linear_bwd_dyq is nvfp4_linear_bwd for an upstream gradient that is already quantized (such a pair, with
 * the streams `seed`, `seed + 1`): no pass over dY is made; X, W / xw_scales / saved as in nvfp4_linear_bwd, and
 * w_operands (may be NULL) as in nvfp4_linear_bwd_wq.  A side given in the slab layout must be one the consuming
 * GEMM takes (nvfp4_gemm_takes_slabs(M, K, N) for rows, (N, K, M) for columns), else NVFP4_EUNSUPPORTED.
 */
size_t nvfp4_swiglu_bwd_workspace_bytes(int64_t M, int64_t F);
nvfp4_status nvfp4_swiglu_bwd_quantize(const void *dH, const void *G, const void *U, nvfp4_dtype dt, int64_t M,
                                       int64_t F, uint64_t seed_gate, uint64_t seed_up, const nvfp4_format *f,
                                       const nvfp4_dual_operands *dG, const nvfp4_dual_operands *dU,
                                       void *dG_store, void *dU_store,
                                       void *workspace, size_t workspace_bytes, void *stream);
nvfp4_status nvfp4_linear_bwd_dyq(const nvfp4_dual_operands *dY, const void *X, const void *W,
                                  const void *w_operands, void *dX, void *dW, int64_t M, int64_t N, int64_t K,
                                  nvfp4_dtype in_dt, nvfp4_dtype out_dt, const nvfp4_format *f, uint64_t seed,
                                  void *workspace, size_t workspace_bytes, void *stream,
                                  const float *xw_scales, const void *saved);
/* The elementwise step alone, results stored: dG, dU of dt, n elements each (n a multiple of 8; all pointers device,
 * 16-byte aligned, dense).  nvfp4_quantize_dual of these two tensors equals what nvfp4_swiglu_bwd_quantize writes. */
nvfp4_status nvfp4_swiglu_bwd(const void *dH, const void *G, const void *U, nvfp4_dtype dt, int64_t n, void *dG,
                              void *dU, void *stream);
/* host evaluation of the elementwise step (the kernels' own inline function), n elements, host pointers */
void nvfp4_host_swiglu_bwd(const float *dH, const float *G, const float *U, int64_t n, float *dG, float *dU);

/*
 * Quantization-noise statistics of a quantized tensor against its source
 * (noise-threshold section, Sec. 4: with eps = Q(x) - x the quantization error
 * of a d-element gradient and sigma_q^2 its mean square, the paper monitors
 * ||x|| / (sigma_q sqrt(d)) = sqrt(sum x^2 / sum eps^2) against sqrt(3); the
 * same quotient inverted is the relative quantization MSE of a format):
 *   sums[0] = sum x^2,   sums[1] = sum (Q(x) - x)^2     over all rows * cols elements,
 * Q(x) = (-1)^sign * E2M1 magnitude * block scale * tensor scale of the stored element.
 *   x, dt, rows, cols, ld, axis, f   as in nvfp4_quantize (device pointer)
 *   codes, scales   device, the operand nvfp4_quantize wrote for this x, axis and format
 *   tensor_scale    device fp32 scalar (read only when f->tensor_scale is 1)
 *   sums            device double[2], 8-byte aligned
 *   workspace       device, >= nvfp4_quant_noise_workspace_bytes(rows, cols, axis), 16-byte aligned
 * Squares are summed in fp32 over 8 elements, everything above that in fp64 in
 * a fixed order: the result is deterministic and agrees with an fp64 evaluation
 * to about 1e-6 relative.  Asynchronous on `stream`.  An empty tensor gives {0, 0}.
 * Errors: as nvfp4_quantize (NVFP4_EINVAL / ESHAPE / EALIGN / EUNSUPPORTED / EWORKSPACE / EHIP).
 */
size_t nvfp4_quant_noise_workspace_bytes(int64_t rows, int64_t cols, int axis);
nvfp4_status nvfp4_quant_noise(const void *x, nvfp4_dtype dt, int64_t rows, int64_t cols, int64_t ld,
                               int axis, const nvfp4_format *f, const uint8_t *codes,
                               const uint8_t *scales, const float *tensor_scale, double *sums,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * Diagnostic, not part of the method: the sustained rate of the matrix
 * instruction a GEMM kernel issues, measured on the current device from a
 * register-only loop (no LDS or global traffic) in that kernel's register-tile
 * pattern, one workgroup per compute unit.  The published MFMA peaks assume the
 * top clock; under a chip-wide matrix load the clock is power-managed and
 * depends on how many operand bits toggle, so this is the practical ceiling a
 * GEMM's achieved rate can be compared with.
 *   kind             0: v_mfma_f32_32x32x16_f16 (exact NVFP4 / E4M3 GEMM)
 *                    1: v_mfma_scale_f32_32x32x64_f8f6f4 on FP4 (MXFP4 GEMM)
 *   random_operands  0: all-zero operand registers; 1: pseudo-random operand
 *                    bits that change every step
 *   iters            loop trips per wave, 1 .. 2^22
 *   scratch          device memory, >= 4 * 512 * (number of compute units) bytes
 *                    (the kernels write one float per thread there)
 *   tflops           host pointer, receives TFLOP/s
 * Blocks the calling thread until the measurement is done.  NVFP4_EINVAL for a
 * bad kind / iters / null pointer, NVFP4_EWORKSPACE for a short scratch,
 * NVFP4_EHIP if the runtime reports an error.
 */
nvfp4_status nvfp4_probe_mfma_rate(int kind, int random_operands, int iters, void *scratch,
                                   size_t scratch_bytes, double *tflops, void *stream);

/*
 * Host-side evaluations of the scalar steps the kernels use (the same inline
 * functions, compiled for the host).  They let a CPU-only test sweep the
 * rounding logic against an independent implementation; they touch no GPU.
 */
uint8_t nvfp4_host_e4m3_encode(float r);            /* r >= 0 -> scale byte */
float nvfp4_host_e4m3_decode(uint8_t byte);
uint8_t nvfp4_host_round_rtn(float m);              /* m in [0, 6] -> magnitude code */
uint8_t nvfp4_host_round_sr(float m, uint32_t u16); /* m in [0, 6], 16 random bits */
void nvfp4_host_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
uint32_t nvfp4_host_sr_bits(uint64_t seed, uint64_t element_index);
uint8_t nvfp4_host_e8m0_encode(float a);            /* a > 0 -> shared-exponent byte */
/* array forms: n inputs -> n outputs (host pointers) */
void nvfp4_host_e4m3_encode_n(const float *r, int64_t n, uint8_t *out);
void nvfp4_host_round_rtn_n(const float *m, int64_t n, uint8_t *out);
void nvfp4_host_round_sr_n(const float *m, const uint32_t *u16, int64_t n, uint8_t *out);

#ifdef __cplusplus
}
#endif
#endif /* NVFP4_H */
