/*
 * nvfp4_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, single-purpose CPU statement of what the FP4 quantized linear
 * layer of "FP4 All the Way: Fully Quantized Training of LLMs" computes:
 *
 *   - the number formats of Sec. 3 / Table 1 (E2M1 elements; E4M3 or E8M0
 *     block scales; block 16 = NVFP4, block 32 + E8M0 = MXFP4),
 *   - the quantization operation Q of Eqs. 1-3 in its two rounding modes
 *     (round-to-nearest and stochastic rounding, Sec. 1 / Sec. 3.2),
 *   - the three GEMMs of Eqs. 4-6 on dequantized operands, accumulated in fp64,
 *   - the elementwise SwiGLU backward that produces the gate/up layers' upstream
 *     gradients (Sec. 5 model), in a fixed binary32 evaluation.
 *
 * It shares no code with the HIP library.  Only tests, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  Every lookup is a brute-force scan
 * over the representable values so that each function can be read against the
 * definition it cites; nothing here is blocked, fused, tabulated or reordered.
 *
 * Where the paper is silent (how a block scale is derived, the per-tensor
 * scale, tie-breaking, saturation, the random-number source) the readings are
 * the ones stated next to each function.
 *
 * Arithmetic contract: all scale arithmetic is IEEE-754 binary32 with
 * round-to-nearest-even, one rounding per written operation, no fused
 * multiply-add (build with -ffp-contract=off, never -ffast-math).  bf16 inputs
 * are widened exactly to binary32 first.
 *
 * Pins (tests/test_oracle_*.py): E2M1 grid, E4M3 against an independent
 * library cast, Philox known-answer vectors, brute-force nearest value,
 * idempotence on representable tensors, power-of-two covariance, sign
 * symmetry, SR support and unbiasedness, hand-worked blocks, exact integer
 * GEMM; the SwiGLU backward against a library exponential, finite differences
 * and the closed form in fp64.  No function in this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_F32 0
#define ORC_BF16 1
#define ORC_RTN 0
#define ORC_SR 1
#define ORC_SCALE_E4M3 0
#define ORC_SCALE_E8M0 1

typedef struct {
    int32_t block;        /* elements sharing one scale: 16 (NVFP4), 32 (MXFP4), ... */
    int32_t scale_fmt;    /* ORC_SCALE_E4M3 or ORC_SCALE_E8M0 */
    int32_t tensor_scale; /* 1: a per-tensor fp32 scale g multiplies every block scale */
} orc_format;

/* ------------------------------------------------------------------ formats */

/* E2M1 (Sec. 3): 1 sign, 2 exponent (bias 1), 1 mantissa bit.  Exponent field
 * 0 is the subnormal binade: value = m * 2^-1.  Otherwise 2^(e-1) * (1 + m/2).
 * Magnitudes are therefore {0, .5, 1, 1.5, 2, 3, 4, 6}. */
float orc_e2m1_decode(uint8_t code)
{
    int s = (code >> 3) & 1, e = (code >> 1) & 3, m = code & 1;
    float mag = (e == 0) ? 0.5f * (float)m : ldexpf(1.0f + 0.5f * (float)m, e - 1);
    return s ? -mag : mag;
}

/* E4M3 used as an unsigned block scale (Sec. 3, Table 1; Sec. 3.1 notes the
 * sign bit is unused): 4 exponent bits (bias 7), 3 mantissa bits, finite-only
 * variant: E=15,M=7 is not a number, so the largest value is 448 (byte 0x7E). */
float orc_e4m3_decode(uint8_t byte)
{
    int e = (byte >> 3) & 15, m = byte & 7;
    if (e == 0) return ldexpf((float)m / 8.0f, -6);
    return ldexpf(1.0f + (float)m / 8.0f, e - 7);
}

/* Nearest E4M3 value to r >= 0, ties to the even byte, values above 448 go to
 * 448 (reading: the scale is cast like any fp32 -> fp8 conversion that
 * saturates).  Brute force over the 127 finite non-negative bytes. */
uint8_t orc_e4m3_encode(float r)
{
    uint8_t best = 0;
    double bestd = INFINITY;
    for (int b = 0; b <= 0x7E; ++b) {
        double d = fabs((double)r - (double)orc_e4m3_decode((uint8_t)b));
        if (d < bestd || (d == bestd && (b & 1) == 0)) {
            bestd = d;
            best = (uint8_t)b;
        }
    }
    return best;
}

/* E8M0 (Sec. 3): exponent-only byte, value 2^(byte-127), no sign, no mantissa. */
float orc_e8m0_decode(uint8_t byte) { return ldexpf(1.0f, (int)byte - 127); }

/* ------------------------------------------------------------- random bits */

/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  One round:
 * the two 32x32->64 products of counter words 0 and 2 with the two round
 * multipliers are split in high and low halves; the new counter is
 * (hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0); the key is then bumped by the two
 * Weyl constants. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The 16 random bits of the element whose row-major index in the logical
 * input tensor is e (independent of the quantization axis).  Key = the seed's
 * two halves; counter = (e>>3, 0, 0) so one 128-bit draw serves 8 consecutive
 * elements: word (e>>1)&3, low half for even e, high half for odd e. */
uint32_t orc_sr_bits(uint64_t seed, uint64_t e)
{
    uint64_t c = e >> 3;
    uint32_t ctr[4] = {(uint32_t)c, (uint32_t)(c >> 32), 0u, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    uint32_t w = out[(e >> 1) & 3];
    return (e & 1) ? (w >> 16) : (w & 0xFFFFu);
}

/* --------------------------------------------------------- element rounding */

/* Round-to-nearest as Sec. 1 defines it (the grid value nearest to the input):
 * m in [0, 6] -> magnitude code 0..7.  Ties go to the even code (reading; the
 * IEEE default). */
uint8_t orc_round_rtn(float m)
{
    uint8_t best = 0;
    double bestd = INFINITY;
    for (int c = 0; c < 8; ++c) {
        double d = fabs((double)m - (double)orc_e2m1_decode((uint8_t)c));
        if (d < bestd || (d == bestd && (c & 1) == 0)) {
            bestd = d;
            best = (uint8_t)c;
        }
    }
    return best;
}

/* Stochastic rounding as Sec. 1 defines it (one of the two neighbouring grid
 * values, chosen at random by how close each is): with lo <= m < hi the
 * neighbouring grid values and t = (m - lo)/(hi - lo), the result is hi with probability t (to 2^-17) and lo
 * otherwise, so that the expected result is m (the E[eps] = 0 property used in
 * Sec. 4).  The draw is a 16-bit uniform u: round up iff u + 1/2 <= 65536 t,
 * which is the classic formulation (add uniformly random bits below the kept
 * digit, then truncate) with the draw centred on the 16-bit grid (reading: the
 * paper fixes neither the number of random bits nor which way the one exact
 * tie u + 1/2 = 65536 t goes).  A value on the grid (t = 0) and the saturated
 * value 6 never move. */
uint8_t orc_round_sr(float m, uint32_t u16)
{
    int lo = 0;
    for (int c = 0; c < 8; ++c)
        if (orc_e2m1_decode((uint8_t)c) <= m) lo = c;
    if (lo == 7) return 7;
    float vlo = orc_e2m1_decode((uint8_t)lo), vhi = orc_e2m1_decode((uint8_t)(lo + 1));
    float t = (m - vlo) / (vhi - vlo); /* both operations exact in binary32 */
    int up = ((float)u16 + 0.5f) <= t * 65536.0f;
    return (uint8_t)(lo + up);
}

/* ------------------------------------------------------------ tensor scale */

static float load_elem(const void *x, int dtype, int64_t idx)
{
    if (dtype == ORC_F32) return ((const float *)x)[idx];
    uint32_t bits = (uint32_t)((const uint16_t *)x)[idx] << 16; /* bf16 = top half of binary32 */
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* T = max |x| over the logical [rows, cols] tensor with leading dimension ld. */
float orc_tensor_amax(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld)
{
    float T = 0.0f;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            float a = fabsf(load_elem(x, dtype, i * ld + j));
            if (a > T) T = a;
        }
    return T;
}

/* Per-tensor scale (not in the paper; reading): g = T / (6 * 448), so the
 * block holding the tensor maximum receives the largest E4M3 scale.  g = 1 for
 * an all-zero tensor.  g is never below 2^-117, which keeps every decoded
 * block scale s*g (s >= 2^-9) a normal binary32 number with a finite
 * reciprocal. */
float orc_tensor_scale_from_amax(float T)
{
    if (T == 0.0f) return 1.0f;
    float g = T / 2688.0f;
    float floor_g = ldexpf(1.0f, -117);
    return g < floor_g ? floor_g : g;
}

/* ---------------------------------------------------------------- quantize */

static float ipow2f(int e) { return ldexpf(1.0f, e); }

/*
 * Q of Eqs. 1-6 for one tensor.  x is the logical row-major [rows, cols]
 * tensor (leading dimension ld elements).  Blocks of f->block elements run
 * along `axis` (1: along a row; 0: down a column), i.e. along the contraction
 * axis of the GEMM the result feeds (reading of Q(W^T), Q(a^T) in Eqs. 2-3: a
 * transposed operand is quantized again with blocks along its new contraction
 * axis).  The output always has the blocked axis contiguous:
 *   axis 1: codes [rows, cols/2], scales [rows, cols/block]
 *   axis 0: codes [cols, rows/2], scales [cols, rows/block]   (transposed)
 * Two 4-bit codes per byte, even position in the low nibble.
 *
 * E4M3 block scales (NVFP4 and its block-size variants), per block:
 *   a = max|x_i|;  r = a * k with k = 1/(6 g);  s8 = E4M3(r);  s = decode(s8)
 *   s8 == 0 -> all magnitudes 0;  else d = s*g, q = 1/d, y_i = x_i * q,
 *   m_i = min(|y_i|, 6), magnitude code by RtN or SR.
 * E8M0 block scales (MXFP4): shared exponent e = floor(log2 a) - 2 (2 is the
 *   exponent of E2M1's largest binade), byte = clamp(e+127, 0, 254),
 *   y_i = x_i * 2^-(byte-127) (exact), then the same clamp and rounding.
 *   a == 0 -> byte 0 and zero magnitudes.
 * The sign bit of a code is the sign bit of x_i, also on a zero magnitude.
 *
 * *g_io: with f->tensor_scale == 0 it is set to 1.  Otherwise, preset != 0
 * reads it (raised to 2^-117 if smaller), preset == 0 computes it from the
 * tensor maximum; the value used is written back.
 * Returns 0, or -1 on a shape the format cannot hold.
 */
int orc_quantize(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld, int axis,
                 int rounding, uint64_t seed, const orc_format *f, uint8_t *codes,
                 uint8_t *scales, float *g_io, int preset)
{
    const int64_t B = f->block;
    const int64_t outer = axis == 1 ? rows : cols;
    const int64_t inner = axis == 1 ? cols : rows;
    if (B <= 0 || (B & 1) || inner % B != 0 || ld < cols) return -1;
    if (f->scale_fmt == ORC_SCALE_E8M0 && f->tensor_scale) return -1;

    float g = 1.0f;
    if (f->tensor_scale) {
        if (preset) {
            g = *g_io;
            float floor_g = ldexpf(1.0f, -117);
            if (g < floor_g) g = floor_g;
        } else {
            g = orc_tensor_scale_from_amax(orc_tensor_amax(x, dtype, rows, cols, ld));
        }
    }
    *g_io = g;
    const float k = 1.0f / (6.0f * g);

    memset(codes, 0, (size_t)(outer * (inner / 2)));
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o) {
        for (int64_t b = 0; b < inner / B; ++b) {
            /* block maximum */
            float a = 0.0f;
            for (int64_t t = 0; t < B; ++t) {
                int64_t n = b * B + t;
                int64_t i = axis == 1 ? o : n, j = axis == 1 ? n : o;
                float ax = fabsf(load_elem(x, dtype, i * ld + j));
                if (ax > a) a = ax;
            }
            /* block scale and the multiplier that maps x onto the E2M1 grid */
            uint8_t sbyte;
            float q;
            int zero_block;
            if (f->scale_fmt == ORC_SCALE_E4M3) {
                float r = a * k;
                sbyte = orc_e4m3_encode(r);
                zero_block = (sbyte == 0);
                float d = orc_e4m3_decode(sbyte) * g;
                q = zero_block ? 0.0f : 1.0f / d;
            } else {
                zero_block = (a == 0.0f);
                if (zero_block) {
                    sbyte = 0;
                    q = 0.0f;
                } else {
                    int ex;
                    (void)frexpf(a, &ex); /* a = fr * 2^ex, fr in [.5,1) => floor(log2 a) = ex-1 */
                    int e = (ex - 1) - 2;
                    int biased = e + 127;
                    if (biased < 0) biased = 0;
                    if (biased > 254) biased = 254;
                    sbyte = (uint8_t)biased;
                    q = ipow2f(127 - biased);
                }
            }
            scales[o * (inner / B) + b] = sbyte;
            /* elements */
            for (int64_t t = 0; t < B; ++t) {
                int64_t n = b * B + t;
                int64_t i = axis == 1 ? o : n, j = axis == 1 ? n : o;
                float xv = load_elem(x, dtype, i * ld + j);
                uint8_t mag = 0;
                if (!zero_block) {
                    float y = xv * q;
                    float m = fabsf(y);
                    if (m > 6.0f) m = 6.0f;
                    if (rounding == ORC_RTN)
                        mag = orc_round_rtn(m);
                    else
                        mag = orc_round_sr(m, orc_sr_bits(seed, (uint64_t)(i * cols + j)));
                }
                uint8_t code = (uint8_t)((signbit(xv) ? 8 : 0) | mag);
                codes[o * (inner / 2) + n / 2] |= (uint8_t)(code << (4 * (n & 1)));
            }
        }
    }
    return 0;
}

/* -------------------------------------------------------------- dequantize */

static double scale_value(uint8_t byte, const orc_format *f)
{
    return f->scale_fmt == ORC_SCALE_E4M3 ? (double)orc_e4m3_decode(byte)
                                          : (double)orc_e8m0_decode(byte);
}

/* Value of a quantized operand stored [outer, K/2] + [outer, K/block]:
 * v = (-1)^sign * grid[code] * s * g, every factor widened to fp64 (the
 * product has at most 2 + 4 + 24 significant bits, so it is exact). */
void orc_dequantize(const uint8_t *codes, const uint8_t *scales, float g, int64_t outer,
                    int64_t K, const orc_format *f, double *out)
{
    const int64_t B = f->block;
#pragma omp parallel for schedule(static)
    for (int64_t o = 0; o < outer; ++o)
        for (int64_t n = 0; n < K; ++n) {
            uint8_t code = (codes[o * (K / 2) + n / 2] >> (4 * (n & 1))) & 15;
            double s = scale_value(scales[o * (K / B) + n / B], f);
            out[o * K + n] = (double)orc_e2m1_decode(code) * s * (double)g;
        }
}

/*
 * Quantization-noise statistics behind the gradient-to-noise monitor of the
 * noise-threshold section (Sec. 4): with eps = Q(x) - x the quantization
 * error of a tensor of d elements, sigma_q^2 is its mean square, and the
 * monitored ratio ||x|| / (sigma_q sqrt(d)) = sqrt(sum x^2 / sum eps^2) is
 * compared with sqrt(3).  out[0] = sum x^2, out[1] = sum (Q(x) - x)^2, both
 * accumulated in fp64 in row-major order of x; Q(x) is the exact value of the
 * stored element (orc_dequantize's definition).  axis as in orc_quantize:
 * axis 1 -> operand stored [rows, cols/2]; axis 0 -> stored [cols, rows/2].
 */
void orc_quant_noise(const void *x, int dtype, int64_t rows, int64_t cols, int64_t ld, int axis,
                     const orc_format *f, const uint8_t *codes, const uint8_t *scales, float g,
                     double out[2])
{
    const int64_t B = f->block;
    const int64_t inner = axis == 1 ? cols : rows;
    double sx = 0.0, se = 0.0;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            const int64_t o = axis == 1 ? i : j, n = axis == 1 ? j : i;
            const uint8_t code = (codes[o * (inner / 2) + n / 2] >> (4 * (n & 1))) & 15;
            const double q = (double)orc_e2m1_decode(code) * scale_value(scales[o * (inner / B) + n / B], f) *
                             (f->tensor_scale ? (double)g : 1.0);
            const double xv = (double)load_elem(x, dtype, i * ld + j);
            sx += xv * xv;
            se += (q - xv) * (q - xv);
        }
    out[0] = sx;
    out[1] = se;
}

/* -------------------------------------------------------------------- GEMM */

/*
 * The GEMM of Eqs. 4-6 in "NT" storage: A is [M, K], B is [N, K], both
 * quantized with blocks along K;  out[i, j] = sum_k vA[i, k] * vB[j, k]
 * accumulated in fp64 in index order.  take_abs != 0 sums |vA||vB| instead
 * (the magnitude that the floating-point tolerance is stated against).
 */
void orc_gemm_nt(int64_t M, int64_t N, int64_t K, const orc_format *f, const uint8_t *A_codes,
                 const uint8_t *A_scales, float gA, const uint8_t *B_codes,
                 const uint8_t *B_scales, float gB, int take_abs, double *out)
{
    double *vA = (double *)malloc(sizeof(double) * (size_t)(M * K));
    double *vB = (double *)malloc(sizeof(double) * (size_t)(N * K));
    orc_dequantize(A_codes, A_scales, gA, M, K, f, vA);
    orc_dequantize(B_codes, B_scales, gB, N, K, f, vB);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i)
        for (int64_t j = 0; j < N; ++j) {
            double acc = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double p = vA[i * K + k] * vB[j * K + k];
                acc += take_abs ? fabs(p) : p;
            }
            out[i * N + j] = acc;
        }
    free(vA);
    free(vB);
}

/* The same sum for a list of n output positions (ii[t], jj[t]) only: lets a
 * test check sampled entries of a full-size product one by one. */
void orc_gemm_nt_sample(int64_t M, int64_t N, int64_t K, const orc_format *f,
                        const uint8_t *A_codes, const uint8_t *A_scales, float gA,
                        const uint8_t *B_codes, const uint8_t *B_scales, float gB, int take_abs,
                        const int64_t *ii, const int64_t *jj, int64_t n, double *out)
{
    (void)M;
    (void)N;
    const int64_t B = f->block;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) {
        int64_t i = ii[t], j = jj[t];
        double acc = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            uint8_t ca = (A_codes[i * (K / 2) + k / 2] >> (4 * (k & 1))) & 15;
            uint8_t cb = (B_codes[j * (K / 2) + k / 2] >> (4 * (k & 1))) & 15;
            double va = (double)orc_e2m1_decode(ca) * scale_value(A_scales[i * (K / B) + k / B], f) *
                        (double)gA;
            double vb = (double)orc_e2m1_decode(cb) * scale_value(B_scales[j * (K / B) + k / B], f) *
                        (double)gB;
            double p = va * vb;
            acc += take_abs ? fabs(p) : p;
        }
        out[t] = acc;
    }
}

/* ------------------------------------------------- SwiGLU backward (glue) */

/*
 * The gate/up layers of the 7B model (Sec. 5 setup: SwiGLU MLP) receive, as the
 * upstream gradient of Eqs. 5-6, the elementwise backward of h = silu(g) * u:
 *     dG = dH * u * sigma(g) * (1 + g * (1 - sigma(g))),    dU = dH * g * sigma(g),
 * sigma(g) = 1 / (1 + exp(-g)).  The paper gives no arithmetic for it.  Because
 * the results are quantized next (a floating-point value decides an integer
 * code), the evaluation is FIXED here, in binary32 with one rounding per
 * written operation, so that any implementation can reproduce it bit for bit:
 *   e   = exp(-|g|) by orc_exp_nonpos (below);
 *   sig = g >= 0 ? 1 / (1 + e) : e / (1 + e)            (one add, one division)
 *   dG  = (dH * u) * (sig * (1 + g * (1 - sig)));   dU = dH * (g * sig)
 * and the results are rounded to the element type of the inputs (bf16: round
 * to nearest even), which is the value the quantizer then sees.
 *
 * orc_exp_nonpos(t), t <= 0 (clamped at -87 so that every intermediate is a
 * normal number): k = rint(t * log2(e)); r = t - k ln2 in two fused steps with
 * ln2 split into a 12-bit head and a tail; exp(r) by the degree-6 Taylor
 * polynomial in Horner form with fused multiply-adds (|r| <= 0.347: truncation
 * below 1.3e-7 relative); the factor 2^k is applied exactly.
 */
float orc_exp_nonpos(float t)
{
    if (t < -87.0f) t = -87.0f;
    const float k = rintf(t * 1.44269504f);
    float r = fmaf(-k, 0.693145751953125f, t);
    r = fmaf(-k, 1.42860677e-6f, r);
    float p = 1.0f / 720.0f;
    p = fmaf(p, r, 1.0f / 120.0f);
    p = fmaf(p, r, 1.0f / 24.0f);
    p = fmaf(p, r, 1.0f / 6.0f);
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    return ldexpf(p, (int)k); /* exact: p in [0.70, 1.42], k >= -126, result normal */
}

static void store_elem(void *x, int dtype, int64_t idx, float v)
{
    if (dtype == ORC_F32) {
        ((float *)x)[idx] = v;
        return;
    }
    uint32_t bits;
    memcpy(&bits, &v, 4);
    bits += 0x7FFFu + ((bits >> 16) & 1u); /* round to nearest even on the 16 dropped bits (finite inputs) */
    ((uint16_t *)x)[idx] = (uint16_t)(bits >> 16);
}

void orc_swiglu_bwd(const void *dH, const void *G, const void *U, int dtype, int64_t n, void *dG, void *dU)
{
    for (int64_t i = 0; i < n; ++i) {
        const float h = load_elem(dH, dtype, i), g = load_elem(G, dtype, i), u = load_elem(U, dtype, i);
        const float e = orc_exp_nonpos(-fabsf(g));
        const float den = 1.0f + e;
        const float sig = g >= 0.0f ? 1.0f / den : e / den;
        const float a = 1.0f - sig;
        const float b = g * a;
        const float c = 1.0f + b;
        const float d = sig * c;
        const float hu = h * u;
        const float q = g * sig;
        store_elem(dG, dtype, i, hu * d);
        store_elem(dU, dtype, i, h * q);
    }
}

/* ------------------------------------------- array forms of the scalar steps
 * (so that a test can sweep millions of inputs without a Python loop) */
void orc_e4m3_encode_array(const float *r, int64_t n, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) out[t] = orc_e4m3_encode(r[t]);
}

void orc_round_rtn_array(const float *m, int64_t n, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) out[t] = orc_round_rtn(m[t]);
}

void orc_round_sr_array(const float *m, const uint32_t *u16, int64_t n, uint8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) out[t] = orc_round_sr(m[t], u16[t]);
}

void orc_sr_bits_array(uint64_t seed, uint64_t e0, int64_t n, uint32_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n; ++t) out[t] = orc_sr_bits(seed, e0 + (uint64_t)t);
}
