// Scalar steps of the FP4 block quantizer, shared by the HIP kernels and (compiled for the
// host) by the nvfp4_host_* probes of the C ABI.  Formats: Sec. 3 / Table 1 of "FP4 All the
// Way"; rounding modes: Sec. 3.2.  Every function is branch-light integer/fp32 arithmetic whose
// result is fully determined by IEEE binary32 (no contraction: this header must be compiled
// with -ffp-contract=off).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define NVFP4_HD __host__ __device__ __forceinline__

namespace nvfp4 {

NVFP4_HD uint32_t f2u(float f) { return __builtin_bit_cast(uint32_t, f); }
NVFP4_HD float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }
NVFP4_HD uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Smallest per-tensor scale: keeps s*g (s >= 2^-9) a normal number with a finite reciprocal.
NVFP4_HD float tensor_scale_floor() { return u2f((127u - 117u) << 23); }

// g from the tensor maximum T (reading, not in the paper): T/(6*448); 1 for T == 0.
NVFP4_HD float tensor_scale_from_amax(float T)
{
    if (T == 0.0f) return 1.0f;
    float g = T / 2688.0f;
    return g < tensor_scale_floor() ? tensor_scale_floor() : g;
}

// E4M3 (bias 7, 3 mantissa bits, finite-only, max 448) of r >= 0: round to nearest even,
// saturate.  Returns the byte; *s receives the decoded value.
//   normal range (r >= 2^-6): round the binary32 mantissa to 3 bits by integer add;
//   below 2^-6 the step is 2^-9: adding 2^14 (whose ulp is 2^-9) lets the fp32 adder round.
NVFP4_HD uint32_t e4m3_encode(float r, float *s)
{
    r = r < 448.0f ? r : 448.0f;
    if (r < 0.015625f) {
        float t = r + 16384.0f;
        *s = t - 16384.0f;
        return f2u(t) & 0xFu;
    }
    uint32_t b = f2u(r);
    b += 0x7FFFFu + ((b >> 20) & 1u);
    b &= 0xFFF00000u;
    *s = u2f(b);
    return (b >> 20) - (120u << 3);
}

NVFP4_HD float e4m3_decode(uint32_t byte)
{
    uint32_t e = (byte >> 3) & 15u, m = byte & 7u;
    if (e == 0) return (float)m * 0.001953125f;  // m * 2^-9
    return u2f(((e + 120u) << 23) | (m << 20));
}

// E8M0 shared exponent of a block with maximum a >= 0, finite (MXFP4, Sec. 3): byte =
// clamp(floor(log2 a) - 2 + 127, 0, 254); *q = 2^(127 - byte) maps the block onto E2M1's range.
// With ex the biased binary32 exponent of a, floor(log2 a) = ex - 127 for a normal a, so the byte is ex - 2;
// ex <= 2 (which includes every subnormal a, whose logarithm is below -126, and a = 0) clamps to byte 0, and the
// upper clamp is never reached (ex <= 254).  No branch, no leading-zero count.  q is at least 2^-125: normal.
NVFP4_HD uint32_t e8m0_encode(float a, float *q)
{
    const uint32_t ex = f2u(a) >> 23;
    const uint32_t byte = (ex > 2u ? ex : 2u) - 2u;
    *q = u2f((254u - byte) << 23);
    return byte;
}

// Round-to-nearest-even of m in [0, 6] onto the E2M1 magnitudes {0,.5,1,1.5,2,3,4,6}.
// The grid step is 2^(e-1) with e = 0 for m < 2, 1 for [2,4), 2 for [4,6]; adding 2^(23+e-1)
// makes the fp32 adder round m to a multiple of the step, ties to even, and leaves the
// multiple in the low mantissa bits.  Even multiples are even codes, so this is ties-to-even
// on codes as well.
NVFP4_HD uint32_t round_rtn(float m)
{
    uint32_t e = umax(f2u(m) >> 23, 127u) - 127u;
    uint32_t n = f2u(m + u2f((149u + e) << 23)) & 7u;
    return n + (e << 1);
}

// Stochastic rounding of m in [0, 6] with a 16-bit uniform u: with lo <= m < hi the grid
// neighbours and t = (m - lo)/(hi - lo), round up iff u + 1/2 <= 65536 t ("add the random bits
// below the kept digit, then truncate", draw centred on the 16-bit grid).
// fx = 65536 m/step is exact; with n = floor(m/step): 65536 t = fx - 65536 n, so the rule is
// 65536 n + u <= fx - 1/2, i.e. 65536 n + u <= R with R = floor(fx - 1/2), and the rounded
// multiple of the step is floor((R + 65536 - u) / 65536)  (R = -1 for fx < 1/2: never up).
// This is the integer/fp32 formulation; the kernels use the gfx950 stochastic convert, which
// computes the same function when given the seed word sr_seed_lo/hi below (checked on every
// path by the tests).
NVFP4_HD uint32_t round_sr(float m, uint32_t u16)
{
    uint32_t e = umax(f2u(m) >> 23, 127u) - 127u;
    float fx = m * u2f((144u - e) << 23);
    int R = (int)floorf(fx - 0.5f);
    uint32_t k = (uint32_t)(R + 65536 - (int)u16) >> 16;
    return k + (e << 1);
}

// v_cvt_scalef32_sr_pk_fp4_f32 rounds |y| (saturated at 6) up iff floor(2^22 frac) + r >= 2^22,
// frac = the position of |y| between its grid neighbours and r = seed[31:10] for the first
// element of the pair, seed[30:9] for the second.  With r = 64 (65535 - u) + 32 that is
// floor(2^22 frac) >= 64 u + 32, i.e. 65536 frac >= u + 1/2: the rule above.
NVFP4_HD uint32_t sr_seed_first(uint32_t u16) { return ((~u16 & 0xFFFFu) << 16) | 0x8000u; }
NVFP4_HD uint32_t sr_seed_second(uint32_t u16) { return ((~u16 & 0xFFFFu) << 15) | 0x4000u; }

// Elementwise backward of h = silu(g) * u (the SwiGLU of the Sec. 5 model), whose results are the upstream
// gradients of the gate and up layers in Eqs. 5-6.  The values are quantized next, so the evaluation is fixed in
// binary32, one rounding per written operation (fused where written as fmaf), and is the same on every machine:
//   exp(t), t <= 0 (clamped at -87): k = rint(t log2 e), r = t - k ln2 in two fused steps (12-bit head, tail),
//   degree-6 Taylor polynomial of exp(r) in Horner form, times 2^k by an exponent-field add (exact: the result is normal);
//   sigma = g >= 0 ? 1 / (1 + e) : e / (1 + e) with e = exp(-|g|);
//   dG = (dH u) (sigma (1 + g (1 - sigma))),  dU = dH (g sigma).
NVFP4_HD float exp_nonpos(float t)
{
    t = t < -87.0f ? -87.0f : t;
    const float k = __builtin_rintf(t * 1.44269504f);
    float r = __builtin_fmaf(-k, 0.693145751953125f, t);
    r = __builtin_fmaf(-k, 1.42860677e-6f, r);
    float p = 1.0f / 720.0f;
    p = __builtin_fmaf(p, r, 1.0f / 120.0f);
    p = __builtin_fmaf(p, r, 1.0f / 24.0f);
    p = __builtin_fmaf(p, r, 1.0f / 6.0f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    return u2f(f2u(p) + ((uint32_t)(int)k << 23));
}

NVFP4_HD void swiglu_bwd_elem(float h, float g, float u, float *dg, float *du)
{
    const float e = exp_nonpos(-__builtin_fabsf(g));
    const float den = 1.0f + e;
    const float sig = (g >= 0.0f ? 1.0f : e) / den;
    const float a = 1.0f - sig;
    const float b = g * a;
    const float c = 1.0f + b;
    const float d = sig * c;
    const float hu = h * u;
    const float q = g * sig;
    *dg = hu * d;
    *du = h * q;
}

// binary32 -> bf16 bit pattern, round to nearest even (finite inputs)
NVFP4_HD uint32_t bf16_rne_bits(float f)
{
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// Philox4x32-10 (Salmon et al., SC'11).
struct u32x4 {
    uint32_t x, y, z, w;
};

NVFP4_HD uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);  // one three-input bit operation (truth table of a ^ b ^ c)
#else
    return a ^ b ^ c;
#endif
}

NVFP4_HD u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                             uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
        uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
        c1 = (uint32_t)p1;
        c3 = (uint32_t)p0;
        c0 = n0;
        c2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return u32x4{c0, c1, c2, c3};
}

// Philox4x32-10 of the counter (c0, c1, 0, 0): the first round written out, since with the upper counter
// words zero one of its two products is zero and two of its xor operands vanish.
NVFP4_HD u32x4 philox4x32_10_low(uint32_t c0, uint32_t c1, uint32_t k0, uint32_t k1)
{
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    uint32_t a0 = c1 ^ k0, a1 = 0u, a2 = (uint32_t)(p0 >> 32) ^ k1, a3 = (uint32_t)p0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
#pragma unroll
    for (int r = 1; r < 10; ++r) {
        uint64_t q0 = (uint64_t)0xD2511F53u * a0;
        uint64_t q1 = (uint64_t)0xCD9E8D57u * a2;
        uint32_t n0 = xor3((uint32_t)(q1 >> 32), a1, k0);
        uint32_t n2 = xor3((uint32_t)(q0 >> 32), a3, k1);
        a1 = (uint32_t)q1;
        a3 = (uint32_t)q0;
        a0 = n0;
        a2 = n2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return u32x4{a0, a1, a2, a3};
}

// The 128 random bits shared by the 8 elements whose row-major indices are 8c .. 8c+7.
NVFP4_HD u32x4 sr_draw(uint64_t seed, uint64_t c)
{
    return philox4x32_10_low((uint32_t)c, (uint32_t)(c >> 32), (uint32_t)seed, (uint32_t)(seed >> 32));
}

// 16 bits of element e & 7 out of its group's draw.
NVFP4_HD uint32_t sr_bits_of(const u32x4 &d, uint32_t e_low3)
{
    uint32_t w = (e_low3 >> 1) == 0 ? d.x : (e_low3 >> 1) == 1 ? d.y : (e_low3 >> 1) == 2 ? d.z : d.w;
    return (e_low3 & 1u) ? (w >> 16) : (w & 0xFFFFu);
}

}  // namespace nvfp4
