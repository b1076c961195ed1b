// Block quantizer kernels for gfx950: tensor maximum, row-blocked quantizer, column-blocked
// (transposed-output) quantizer.  Implements the operation Q of Eqs. 1-6 of "FP4 All the Way"
// for the formats of Sec. 3 / Table 1 and the two rounding modes of Sec. 3.2.
//
// Memory plan (the kernels are HBM-bound, so everything is about 16-byte coalesced access):
//   rows kernel   : one lane = 8 consecutive elements of a row (one 16 B load for bf16), a
//                   block of B elements = B/8 adjacent lanes, block maximum by DPP max across
//                   those lanes, one 4 B store of 8 packed codes per lane.
//   columns kernel: one lane = 16 consecutive rows x 8 consecutive columns held in registers.
//                   Lanes that are adjacent in the wave hold vertically adjacent row groups of
//                   the same 8 columns, so the four waves of a workgroup read 512 B (bf16)
//                   contiguous per row and a wave writes 64 B contiguous per output row of the
//                   transposed code matrix, without staging through LDS.
#include "kernels.h"
#include "nvfp4_math.h"

namespace nvfp4 {

// ------------------------------------------------------------------ small device helpers

template <int CTRL>
__device__ __forceinline__ float dpp_max(float a)
{
    // a >= 0: unsigned order of the bit patterns is the float order
    int o = __builtin_amdgcn_update_dpp(0, (int)f2u(a), CTRL, 0xF, 0xF, false);
    uint32_t ou = (uint32_t)o;
    return u2f(umax(f2u(a), ou));
}

// Maximum over groups of L adjacent lanes (L = 1, 2, 4, 8, 16; groups aligned to L).
template <int L>
__device__ __forceinline__ float group_max(float a)
{
    if (L >= 2) a = dpp_max<0xB1>(a);   // quad_perm [1,0,3,2]  : lane ^ 1
    if (L >= 4) a = dpp_max<0x4E>(a);   // quad_perm [2,3,0,1]  : lane ^ 2
    if (L >= 8) a = dpp_max<0x141>(a);  // row_half_mirror      : swaps the two quads of 8 lanes
    if (L >= 16) a = dpp_max<0x140>(a); // row_mirror           : swaps the two halves of 16 lanes
    return a;
}

// The quantizer streams: every input byte is read once and every output byte written once, so
// loads and stores carry the nontemporal hint (measured on gfx950 with the quantizer's 16 B in /
// 4 B out shape: 6.1-6.2 TB/s with the hint against 5.4 TB/s without).  STREAM = false keeps a
// tensor in the last-level cache for a second pass.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
template <bool STREAM>
__device__ __forceinline__ uint4 load16(const void *p)
{
    if (STREAM) {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    }
    return *reinterpret_cast<const uint4 *>(p);
}
__device__ __forceinline__ void store4_stream(void *p, uint32_t v) { __builtin_nontemporal_store(v, reinterpret_cast<uint32_t *>(p)); }
__device__ __forceinline__ void store8_stream(void *p, uint32_t a, uint32_t b)
{
    const u32x2_t v = {a, b};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2_t *>(p));
}

template <int DT>
struct Chunk;  // 8 consecutive elements as loaded from memory

template <>
struct Chunk<NVFP4_BF16> {
    uint4 raw;
    template <bool STREAM = true>
    __device__ __forceinline__ void load(const void *x, int64_t off)
    {
        raw = load16<STREAM>(reinterpret_cast<const uint16_t *>(x) + off);
    }
    __device__ __forceinline__ void load_partial(const void *x, int64_t off, int n)
    {
        const uint16_t *p = reinterpret_cast<const uint16_t *>(x) + off;
        uint32_t w[4] = {0, 0, 0, 0};
        for (int t = 0; t < n; ++t) w[t >> 1] |= (uint32_t)p[t] << (16 * (t & 1));
        raw = make_uint4(w[0], w[1], w[2], w[3]);
    }
    __device__ __forceinline__ void zero() { raw = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void store(void *x, int64_t off) const
    {
        *reinterpret_cast<uint4 *>(reinterpret_cast<uint16_t *>(x) + off) = raw;
    }
    // 8 binary32 values rounded to bf16 (nearest even) and packed
    __device__ __forceinline__ void set(const float (&f)[8])
    {
        typedef float f2_t __attribute__((ext_vector_type(2)));
        typedef __bf16 b2_t __attribute__((ext_vector_type(2)));
        uint32_t w[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const f2_t p = {f[2 * t], f[2 * t + 1]};
            const b2_t b = __builtin_convertvector(p, b2_t);
            w[t] = __builtin_bit_cast(uint32_t, b);
        }
        raw = make_uint4(w[0], w[1], w[2], w[3]);
    }
    __device__ __forceinline__ void launder() { asm volatile("" : "+v"(raw.x), "+v"(raw.y), "+v"(raw.z), "+v"(raw.w)); }
    // elements 2i (low half) and 2i + 1 (high half) as stored
    __device__ __forceinline__ uint32_t word(int i) const { return i == 0 ? raw.x : i == 1 ? raw.y : i == 2 ? raw.z : raw.w; }
    __device__ __forceinline__ float get(int t) const
    {
        uint32_t w = t < 2 ? raw.x : t < 4 ? raw.y : t < 6 ? raw.z : raw.w;
        return (t & 1) ? u2f(w & 0xFFFF0000u) : u2f(w << 16);
    }
};

template <>
struct Chunk<NVFP4_F32> {
    float4 lo, hi;
    template <bool STREAM = true>
    __device__ __forceinline__ void load(const void *x, int64_t off)
    {
        const float *p = reinterpret_cast<const float *>(x) + off;
        const uint4 a = load16<STREAM>(p), b = load16<STREAM>(p + 4);
        lo = make_float4(u2f(a.x), u2f(a.y), u2f(a.z), u2f(a.w));
        hi = make_float4(u2f(b.x), u2f(b.y), u2f(b.z), u2f(b.w));
    }
    __device__ __forceinline__ void load_partial(const void *x, int64_t off, int n)
    {
        const float *p = reinterpret_cast<const float *>(x) + off;
        float v[8];
        for (int t = 0; t < 8; ++t) v[t] = t < n ? p[t] : 0.0f;
        lo = make_float4(v[0], v[1], v[2], v[3]);
        hi = make_float4(v[4], v[5], v[6], v[7]);
    }
    __device__ __forceinline__ void zero()
    {
        lo = make_float4(0, 0, 0, 0);
        hi = lo;
    }
    __device__ __forceinline__ void set(const float (&f)[8])
    {
        lo = make_float4(f[0], f[1], f[2], f[3]);
        hi = make_float4(f[4], f[5], f[6], f[7]);
    }
    __device__ __forceinline__ void store(void *x, int64_t off) const
    {
        float *p = reinterpret_cast<float *>(x) + off;
        *reinterpret_cast<float4 *>(p) = lo;
        *reinterpret_cast<float4 *>(p + 4) = hi;
    }
    __device__ __forceinline__ void launder() {}
    __device__ __forceinline__ uint32_t word(int) const { return 0; }  // (bf16 chunks only)
    __device__ __forceinline__ float get(int t) const
    {
        switch (t) {
        case 0: return lo.x;
        case 1: return lo.y;
        case 2: return lo.z;
        case 3: return lo.w;
        case 4: return hi.x;
        case 5: return hi.y;
        case 6: return hi.z;
        default: return hi.w;
        }
    }
};

template <int DT>
__device__ __forceinline__ float chunk_amax(const Chunk<DT> &c)
{
    float a = 0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t) a = fmaxf(a, fabsf(c.get(t)));
    return a;
}

// The same on a bf16 chunk as stored: magnitudes of finite bf16 values order like their bit patterns, so the
// maximum is taken on packed 16-bit integers, two elements per instruction, and widened once at the end.
typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pk_umax16(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, a), __builtin_bit_cast(u16x2_t, b)));
}
// the two halves of a packed maximum as binary32 (even element, odd element)
__device__ __forceinline__ float pk_even(uint32_t m) { return u2f(m << 16); }
__device__ __forceinline__ float pk_odd(uint32_t m) { return u2f(m & 0xFFFF0000u); }
template <int DT>
__device__ __forceinline__ float chunk_amax_packed(const Chunk<DT> &c)
{
    if constexpr (DT == NVFP4_BF16) {
        const uint32_t m = pk_umax16(pk_umax16(c.word(0) & 0x7FFF7FFFu, c.word(1) & 0x7FFF7FFFu),
                                     pk_umax16(c.word(2) & 0x7FFF7FFFu, c.word(3) & 0x7FFF7FFFu));
        return u2f(umax(m << 16, m & 0xFFFF0000u));
    } else {
        return chunk_amax(c);
    }
}

// Per-tensor scale as the kernels see it: none, preset in memory, or the bit pattern of the
// tensor maximum left by the amax kernel.
// With n_partials > 0 the tensor maximum arrives as that many per-workgroup maxima and every
// workgroup (256 threads, all of them must call this) folds them for itself: 2 KB from the L2 per
// workgroup instead of a separate one-workgroup kernel between the maximum pass and the quantizer.
__device__ __forceinline__ float resolve_g(const QuantArgs &P)
{
    if (P.g_mode == G_NONE) return 1.0f;
    if (P.g_mode == G_PRESET) {
        float g = *P.g_src;
        return g < tensor_scale_floor() ? tensor_scale_floor() : g;
    }
    const uint32_t *bits = reinterpret_cast<const uint32_t *>(P.g_src);
    if (P.n_partials == 0) return tensor_scale_from_amax(u2f(*bits));
    __shared__ uint32_t fold[16];
    uint32_t m = 0;
    for (int i = threadIdx.x; i < P.n_partials; i += 256) m = umax(m, bits[i]);
    m = f2u(group_max<16>(u2f(m)));
    if ((threadIdx.x & 15) == 0) fold[threadIdx.x >> 4] = m;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 16; ++t) m = umax(m, fold[t]);
    return tensor_scale_from_amax(u2f(m));
}

// Block scale byte and the multiplier q that maps the block onto the E2M1 range.
// With E4M3 scales q = 0 for a block whose magnitudes are all zero.
// HW: the E4M3 byte and its value come from the gfx950 FP8 converts (OCP E4M3, round to nearest
// even; the input is clamped to 448 first, as in the software encode, so the convert never sees
// an out-of-range value).  Checked against e4m3_encode / e4m3_decode on every non-negative fp32
// up to 512: identical bytes and values.  The software formulation costs ~15 instructions per block.
// With E4M3 scales and a per-tensor g the multiplier q = 1 / (s * g) is a function of the scale byte alone: a
// workgroup evaluates it once for each of the 127 finite bytes (the same multiply and correctly rounded division
// every block would do) and the blocks then look it up, which takes ~12 instructions out of every block's path.
// All 256 threads of the workgroup must call this (it ends in a barrier).  Returns false where no table applies.
__shared__ float qtab[128];
template <int SF, bool HW>
__device__ __forceinline__ bool build_qtab(float g)
{
    if (SF != NVFP4_SCALE_E4M3 || !HW) return false;
    if (threadIdx.x < 128) {
        const uint32_t byte = threadIdx.x;
        const float s = __builtin_amdgcn_cvt_f32_fp8((int)byte, 0);
        const float d = byte == 0 ? 1.0f : s * g;
        const float r = 1.0f / d;
        qtab[byte] = byte == 0 ? 0.0f : r;
    }
    __syncthreads();
    return true;
}

// TAB: look q up in the workgroup's table (build_qtab() must have run) instead of dividing.
template <int SF, bool HW = false, bool TAB = false>
__device__ __forceinline__ uint32_t block_scale(float a, float g, float k, float *q)
{
    if (SF == NVFP4_SCALE_E4M3) {
        float s;
        uint32_t byte;
        if (HW) {
            const float r = a * k;
            const float rc = r < 448.0f ? r : 448.0f;
            byte = (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(rc, 0.0f, 0, false) & 0xFFu;
            if (TAB) {
                *q = qtab[byte];
                return byte;
            }
            s = __builtin_amdgcn_cvt_f32_fp8((int)byte, 0);
        } else {
            byte = e4m3_encode(a * k, &s);
        }
        // (no branch around the division: a zero scale byte divides by 1 and is then replaced)
        const bool zero = byte == 0;
        const float d = zero ? 1.0f : s * g;
        const float r = 1.0f / d;
        *q = zero ? 0.0f : r;
        return byte;
    } else {
        // (an all-zero block: byte 0, and its zeros times any finite q are zeros of the same sign)
        return e8m0_encode(a, q);
    }
}

// One element: sign | magnitude code.
template <int RND>
__device__ __forceinline__ uint32_t quant_elem(float x, float q, uint32_t u16)
{
    float m = fabsf(x * q);
    m = m < 6.0f ? m : 6.0f;
    uint32_t mag = RND == NVFP4_RTN ? round_rtn(m) : round_sr(m, u16);
    return mag | ((f2u(x) >> 28) & 8u);
}

// Two adjacent elements -> one byte via the gfx950 convert (RNE, saturating at +-6, sign
// kept on zero), low nibble = first element; the byte replaces byte BYTE of acc, the others stay.
template <int BYTE>
__device__ __forceinline__ uint32_t quant_pair_hw(uint32_t acc, float x0, float x1, float q)
{
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(acc, x0 * q, x1 * q, 1.0f, BYTE);
}

// Stochastic rounding of one element through the gfx950 convert, which takes a pair: the
// element sits in slot SLOT (0: low nibble, random bits seed[31:10]; 1: high nibble, seed[30:9]),
// the other slot holds +0 (never rounded up: code 0).  Byte BYTE of acc is replaced and the
// other bytes kept, so two accumulators (one per slot) are filled and OR-ed.  Saturation at
// +-6 and the sign (also of a zero) are the convert's own.
// Written as inline assembly with the accumulator tied to the destination: the compiler's
// builtin for this instruction does not tie its "old" operand, which loses the other bytes.
template <int SLOT, int BYTE>
__device__ __forceinline__ uint32_t sr_elem_hw(uint32_t acc, float y, uint32_t u16)
{
    typedef float float2_t __attribute__((ext_vector_type(2)));
    const float2_t v = SLOT == 0 ? float2_t{y, 0.0f} : float2_t{0.0f, y};
    const uint32_t seed = SLOT == 0 ? sr_seed_first(u16) : sr_seed_second(u16);
    if (BYTE == 0) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0" : "+v"(acc) : "v"(v), "v"(seed));
    if (BYTE == 1) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,1,0]" : "+v"(acc) : "v"(v), "v"(seed));
    if (BYTE == 2) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,0,1]" : "+v"(acc) : "v"(v), "v"(seed));
    if (BYTE == 3) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,1,1]" : "+v"(acc) : "v"(v), "v"(seed));
    return acc;
}

// The same through slot 0 only, with the seed word taken straight from a draw word: nw is the COMPLEMENT of the
// Philox word that holds the element's 16 bits in its low (HALF 0) or high (HALF 1) half, and
// sr_seed_first(u16) = ((~u16 & 0xFFFF) << 16) | 0x8000 becomes one shift-or or one and-or.  An element that
// belongs in the high nibble of its byte is converted into the low nibble of a second accumulator, which the
// caller shifts by 4 once per word.
__device__ __forceinline__ uint32_t sr_seed0(uint32_t nw, int half)
{
    return half ? ((nw & 0xFFFF0000u) | 0x8000u) : ((nw << 16) | 0x8000u);
}
template <int BYTE>
__device__ __forceinline__ uint32_t sr_elem0(uint32_t acc, float y, uint32_t seed)
{
    typedef float float2_t __attribute__((ext_vector_type(2)));
    const float2_t v = float2_t{y, 0.0f};
    if (BYTE == 0) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0" : "+v"(acc) : "v"(v), "v"(seed));
    if (BYTE == 1) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,1,0]" : "+v"(acc) : "v"(v), "v"(seed));
    if (BYTE == 2) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,0,1]" : "+v"(acc) : "v"(v), "v"(seed));
    if (BYTE == 3) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, 1.0 op_sel:[0,0,1,1]" : "+v"(acc) : "v"(v), "v"(seed));
    return acc;
}
// 8 consecutive elements of a row (chunk v, multiplier q, their draw d) -> 8 codes in one word
template <int DT>
__device__ __forceinline__ uint32_t sr_chunk_hw(const Chunk<DT> &v, float q, const u32x4 &d)
{
    const uint32_t n0 = ~d.x, n1 = ~d.y, n2 = ~d.z, n3 = ~d.w;
    uint32_t lo = 0, hi = 0;
    lo = sr_elem0<0>(lo, v.get(0) * q, sr_seed0(n0, 0));
    hi = sr_elem0<0>(hi, v.get(1) * q, sr_seed0(n0, 1));
    lo = sr_elem0<1>(lo, v.get(2) * q, sr_seed0(n1, 0));
    hi = sr_elem0<1>(hi, v.get(3) * q, sr_seed0(n1, 1));
    lo = sr_elem0<2>(lo, v.get(4) * q, sr_seed0(n2, 0));
    hi = sr_elem0<2>(hi, v.get(5) * q, sr_seed0(n2, 1));
    lo = sr_elem0<3>(lo, v.get(6) * q, sr_seed0(n3, 0));
    hi = sr_elem0<3>(hi, v.get(7) * q, sr_seed0(n3, 1));
    return lo | (hi << 4);
}

// ---- MXFP4 through the converts' own scale operand.
// The gfx950 FP4 converts divide the source by a power of two taken from the exponent field of a binary32 "scale"
// operand before rounding.  An E8M0 block scale byte b is exactly such a power (2^(b - 127), also for b = 0), so
// the operand is b << 23 and the element needs no multiply; a bf16 source goes in as stored, two elements per
// register, with no unpacking either.  (With E4M3 block scales the multiplier 1 / (s g) is no power of two and
// the elements are multiplied in binary32 first, as above.)
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float mx_scale_operand(uint32_t byte) { return u2f(byte << 23); }

template <int BYTE>
__device__ __forceinline__ uint32_t mx_pair_bf16(uint32_t acc, uint32_t w, float sc)
{
    return __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(acc, __builtin_bit_cast(bf16x2_t, w), sc, BYTE);
}
// elements 2 BYTE and 2 BYTE + 1 of a chunk -> byte BYTE of acc, round to nearest
template <int DT, int BYTE>
__device__ __forceinline__ uint32_t mx_rtn_pair(uint32_t acc, const Chunk<DT> &v, float sc)
{
    if constexpr (DT == NVFP4_BF16)
        return mx_pair_bf16<BYTE>(acc, v.word(BYTE), sc);
    else
        return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(acc, v.get(2 * BYTE), v.get(2 * BYTE + 1), sc, BYTE);
}
// rows R and R + 1 of column c of a lane tile -> byte BYTE of acc, round to nearest
template <int DT, int BYTE>
__device__ __forceinline__ uint32_t mx_rtn_rows(uint32_t acc, const Chunk<DT> &top, const Chunk<DT> &bot, int c, float sc)
{
    if constexpr (DT == NVFP4_BF16) {
        const uint32_t w = __builtin_amdgcn_perm(bot.word(c >> 1), top.word(c >> 1), (c & 1) ? 0x07060302u : 0x05040100u);
        return mx_pair_bf16<BYTE>(acc, w, sc);
    } else {
        return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(acc, top.get(c), bot.get(c), sc, BYTE);
    }
}
// Stochastic rounding of element t of a chunk through slot 0 of the convert (see sr_elem0) -> low nibble of byte
// BYTE of acc.  (Inline assembly for the same reason as above: the accumulator must be tied to the destination.)
// Always the binary32-source convert: the bf16-source form of the stochastic convert does not consume the 16
// random bits the way the binary32 form does (measured: 0.6 % of the codes of a bf16 tensor differ, all of them
// elements that land between 0 and 0.5), so a bf16 element is widened first; only the multiply is saved.
template <int DT, int BYTE>
__device__ __forceinline__ uint32_t mx_sr_elem0(uint32_t acc, const Chunk<DT> &v, int t, uint32_t seed, float sc)
{
    typedef float float2_t __attribute__((ext_vector_type(2)));
    const float2_t p = float2_t{v.get(t), 0.0f};
    if (BYTE == 0) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, %3" : "+v"(acc) : "v"(p), "v"(seed), "v"(sc));
    if (BYTE == 1) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, %3 op_sel:[0,0,1,0]" : "+v"(acc) : "v"(p), "v"(seed), "v"(sc));
    if (BYTE == 2) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, %3 op_sel:[0,0,0,1]" : "+v"(acc) : "v"(p), "v"(seed), "v"(sc));
    if (BYTE == 3) asm("v_cvt_scalef32_sr_pk_fp4_f32 %0, %1, %2, %3 op_sel:[0,0,1,1]" : "+v"(acc) : "v"(p), "v"(seed), "v"(sc));
    return acc;
}
template <int DT>
__device__ __forceinline__ uint32_t mx_sr_chunk(const Chunk<DT> &v, float sc, const u32x4 &d)
{
    const uint32_t n0 = ~d.x, n1 = ~d.y, n2 = ~d.z, n3 = ~d.w;
    uint32_t lo = 0, hi = 0;
    lo = mx_sr_elem0<DT, 0>(lo, v, 0, sr_seed0(n0, 0), sc);
    hi = mx_sr_elem0<DT, 0>(hi, v, 1, sr_seed0(n0, 1), sc);
    lo = mx_sr_elem0<DT, 1>(lo, v, 2, sr_seed0(n1, 0), sc);
    hi = mx_sr_elem0<DT, 1>(hi, v, 3, sr_seed0(n1, 1), sc);
    lo = mx_sr_elem0<DT, 2>(lo, v, 4, sr_seed0(n2, 0), sc);
    hi = mx_sr_elem0<DT, 2>(hi, v, 5, sr_seed0(n2, 1), sc);
    lo = mx_sr_elem0<DT, 3>(lo, v, 6, sr_seed0(n3, 0), sc);
    hi = mx_sr_elem0<DT, 3>(hi, v, 7, sr_seed0(n3, 1), sc);
    return lo | (hi << 4);
}
// 8 elements of a row, rounding RND, MX (scale operand) or multiplier form
template <int DT, int RND, bool MXS>
__device__ __forceinline__ uint32_t chunk_codes_hw(const Chunk<DT> &v, float q, uint32_t seed, uint64_t ctr)
{
    uint32_t packed = 0;
    if constexpr (RND == NVFP4_RTN && MXS) {
        packed = mx_rtn_pair<DT, 0>(packed, v, q);
        packed = mx_rtn_pair<DT, 1>(packed, v, q);
        packed = mx_rtn_pair<DT, 2>(packed, v, q);
        packed = mx_rtn_pair<DT, 3>(packed, v, q);
    } else if constexpr (RND == NVFP4_RTN) {
        packed = quant_pair_hw<0>(packed, v.get(0), v.get(1), q);
        packed = quant_pair_hw<1>(packed, v.get(2), v.get(3), q);
        packed = quant_pair_hw<2>(packed, v.get(4), v.get(5), q);
        packed = quant_pair_hw<3>(packed, v.get(6), v.get(7), q);
    } else if constexpr (MXS) {
        packed = mx_sr_chunk(v, q, sr_draw(seed, ctr));
    } else {
        packed = sr_chunk_hw(v, q, sr_draw(seed, ctr));
    }
    return packed;
}

// ------------------------------------------------------------------ tensor maximum (Q0)

// max|x| over a [rows, cols] tensor: one partial maximum (bit pattern) per workgroup into
// part_out[blockIdx.y * gridDim.x + blockIdx.x]; a single small workgroup folds them afterwards.
// (One atomic max per workgroup on a single address serializes: 8192 of them cost ~80 us.)
// grid.x covers the 8-element chunks of a row span (4 per thread, all four loads in flight
// before the first use), grid.y the row spans; for a dense tensor the host passes one span of
// rows*cols elements.  Loads are ordinary (cacheable): the quantizer reads the tensor again
// right after, and up to 256 MB of it are then still in the last-level cache.
constexpr int AMAX_UNROLL = 4;
template <int DT>
__global__ __launch_bounds__(256) void amax_kernel(const void *x, int64_t cols, int64_t ld,
                                                   uint32_t *part_out)
{
    const int64_t row = blockIdx.y;
    const int64_t nchunk = cols >> 3;
    const int64_t base = (int64_t)blockIdx.x * (256 * AMAX_UNROLL) + threadIdx.x;
    Chunk<DT> v[AMAX_UNROLL];
#pragma unroll
    for (int u = 0; u < AMAX_UNROLL; ++u) {
        const int64_t c = base + u * 256;
        if (c < nchunk)
            v[u].template load<false>(x, row * ld + c * 8);
        else
            v[u].zero();
    }
    float a = 0.0f;
#pragma unroll
    for (int u = 0; u < AMAX_UNROLL; ++u) a = fmaxf(a, chunk_amax(v[u]));
    if (blockIdx.x == 0 && threadIdx.x == 0 && (cols & 7)) {
        Chunk<DT> t;
        t.load_partial(x, row * ld + nchunk * 8, (int)(cols & 7));
        a = fmaxf(a, chunk_amax(t));
    }
    a = group_max<16>(a);
    // 4 rows of 16 lanes per wave, 4 waves: finish through LDS
    __shared__ uint32_t part[16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((lane & 15) == 0) part[wave * 4 + (lane >> 4)] = f2u(a);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = 0;
#pragma unroll
        for (int t = 0; t < 16; ++t) m = umax(m, part[t]);
        part_out[(int64_t)blockIdx.y * gridDim.x + blockIdx.x] = m;
    }
}

// Dense tensors: a fixed grid of large workgroups strides over the chunks, one partial each.
constexpr int AMAX_DENSE_THREADS = 1024;
template <int DT>
__global__ __launch_bounds__(AMAX_DENSE_THREADS) void amax_dense_kernel(const void *x, int64_t n, uint32_t *part_out)
{
    const int64_t nchunk = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * (AMAX_DENSE_THREADS * AMAX_UNROLL);
    float a = 0.0f;
    for (int64_t base = (int64_t)blockIdx.x * (AMAX_DENSE_THREADS * AMAX_UNROLL) + threadIdx.x; base < nchunk; base += stride) {
        Chunk<DT> v[AMAX_UNROLL];
#pragma unroll
        for (int u = 0; u < AMAX_UNROLL; ++u) {
            const int64_t c = base + u * AMAX_DENSE_THREADS;
            if (c < nchunk)
                v[u].template load<false>(x, c * 8);
            else
                v[u].zero();
        }
#pragma unroll
        for (int u = 0; u < AMAX_UNROLL; ++u) a = fmaxf(a, chunk_amax(v[u]));
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && (n & 7)) {
        Chunk<DT> t;
        t.load_partial(x, nchunk * 8, (int)(n & 7));
        a = fmaxf(a, chunk_amax(t));
    }
    a = group_max<16>(a);
    __shared__ uint32_t part[AMAX_DENSE_THREADS / 16];
    if ((threadIdx.x & 15) == 0) part[threadIdx.x >> 4] = f2u(a);
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t m = 0;
#pragma unroll
        for (int t = 0; t < AMAX_DENSE_THREADS / 16; ++t) m = umax(m, part[t]);
        part_out[blockIdx.x] = m;
    }
}

// Folds n partial maxima into amax_bits[0]; with g_out != nullptr also writes the tensor scale.
__global__ __launch_bounds__(1024) void fold_amax_kernel(const uint32_t *partials, int64_t n,
                                                         uint32_t *amax_bits, float *g_out)
{
    uint32_t m = 0;
    for (int64_t i = threadIdx.x; i < n; i += 1024) m = umax(m, partials[i]);
    m = f2u(group_max<16>(u2f(m)));
    __shared__ uint32_t part[64];
    if ((threadIdx.x & 15) == 0) part[threadIdx.x >> 4] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t r = 0;
#pragma unroll
        for (int t = 0; t < 64; ++t) r = umax(r, part[t]);
        *amax_bits = r;
        if (g_out) *g_out = tensor_scale_from_amax(u2f(r));
    }
}

// ------------------------------------------------------------------ row-blocked quantizer

constexpr int ROWS_UNROLL = 4;  // chunks per thread

template <int DT, int B, int SF, int RND, bool HW>
__global__ __launch_bounds__(256) void quantize_rows_kernel(QuantArgs P)
{
    constexpr int LPB = B / 8;  // lanes per block
    constexpr bool MXS = HW && SF == NVFP4_SCALE_E8M0;  // block scale as the convert's scale operand
    const int64_t cpr = P.cols >> 3;
    const int64_t total = P.rows * cpr;
    const int64_t base = (int64_t)blockIdx.x * (256 * ROWS_UNROLL) + threadIdx.x;
    const bool dense = P.ld == P.cols;
    Chunk<DT> v[ROWS_UNROLL];
#pragma unroll
    for (int u = 0; u < ROWS_UNROLL; ++u) {
        const int64_t id = base + u * 256;
        if (id < total) {
            int64_t off = id * 8;
            if (!dense) {
                const int64_t i = id / cpr;
                off = i * P.ld + (id - i * cpr) * 8;
            }
            v[u].template load<true>(P.x, off);
        } else {
            v[u].zero();
        }
    }
    // (after the loads are issued: folding the partial maxima then overlaps their latency)
    const float g = resolve_g(P);
    const float k = 1.0f / (6.0f * g);
    build_qtab<SF, HW>(g);
    if (blockIdx.x == 0 && threadIdx.x == 0) *P.g_out = g;
#pragma unroll
    for (int u = 0; u < ROWS_UNROLL; ++u) {
        const int64_t id = base + u * 256;
        // a whole block is in or out of range together, so the lanes exchanged below are
        // either all live or all holding zeros
        const float a = group_max<LPB>(MXS ? chunk_amax_packed(v[u]) : chunk_amax(v[u]));
        float q;
        const uint32_t sbyte = block_scale<SF, HW, HW && SF == NVFP4_SCALE_E4M3>(a, g, k, &q);
        uint32_t packed = 0;
        if (HW) {
            if (MXS) q = mx_scale_operand(sbyte);
            packed = chunk_codes_hw<DT, RND, MXS>(v[u], q, P.seed, (uint64_t)id);  // element index = 8*id + t
        } else {
            u32x4 d = {0, 0, 0, 0};
            if (RND == NVFP4_SR) d = sr_draw(P.seed, (uint64_t)id);  // element index = 8*id + t
#pragma unroll
            for (int t = 0; t < 8; ++t)
                packed |= quant_elem<RND>(v[u].get(t), q, sr_bits_of(d, t)) << (4 * t);
        }
        // scale bytes: lanes that start a block hold them; up to four neighbouring blocks are
        // merged into one 4-byte store
        constexpr int GATHER = LPB <= 4 ? 4 : 1;  // blocks merged per store
        uint32_t sw = sbyte;
        if (GATHER == 4) {
            sw |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)sw, 0x100 + LPB, 0xF, 0xF, true) << 8;       // lane + LPB
            sw |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)sw, 0x100 + 2 * LPB, 0xF, 0xF, true) << 16;  // lane + 2 LPB
        }
        if (id < total) {
            store4_stream(reinterpret_cast<uint32_t *>(P.codes) + id, packed);
            const int64_t blk = id / LPB;
            if (GATHER == 4 && blk + 4 <= total / LPB) {
                if ((threadIdx.x & (4 * LPB - 1)) == 0) store4_stream(P.scales + blk, sw);
            } else if ((threadIdx.x & (LPB - 1)) == 0) {
                P.scales[blk] = (uint8_t)sbyte;  // last (partial) group of four, or wide blocks
            }
        }
    }
}

// ------------------------------------------------------------------ column-blocked quantizer

// Lane tile: 16 rows x 8 columns.  Wave tile: (16 LV) rows x (8 * 64 / LV) columns, lanes with
// consecutive ids stacked vertically; workgroup: 4 waves side by side.  LV = 8 gives 64-byte
// runs per output row; measured on [8192, 8192] bf16: LV = 4 (32-byte runs) is 45 % slower,
// LV = 16 (128-byte runs, 64-byte reads) no faster.
template <int DT, int LV = 8>
struct ColGeom {
    static constexpr int RPL = 16;
    static constexpr int LANES_V = LV;                 // lanes stacked vertically
    static constexpr int LANES_H = 64 / LANES_V;       // column groups per wave
    static constexpr int WAVE_COLS = 8 * LANES_H;
    static constexpr int WG_COLS = 4 * WAVE_COLS;
    static constexpr int WG_ROWS = RPL * LANES_V;
};

// 16 bits of the column c of a lane's 8 in row-major element order: from draw d0 when the 8
// columns are aligned to a draw (shift = 0), else from d0 or d1.
template <bool ALIGNED>
__device__ __forceinline__ uint32_t col_bits(const u32x4 &d0, const u32x4 &d1, uint32_t shift, int c)
{
    if (ALIGNED) return sr_bits_of(d0, c);
    const uint32_t pos = shift + c;
    return pos < 8 ? sr_bits_of(d0, pos) : sr_bits_of(d1, pos - 8);
}

// Stochastic rounding of a lane's 16 x 8 tile through the hardware convert, two rows at a time
// (the byte select of the convert must be a constant, hence the recursion over row pairs).
// ALIGNED (every row holds a whole number of draws and the lane's 8 columns are one of them): ctr is the draw
// counter of row row0 + R at the lane's columns and cstep = cols / 8 the distance to the next row's, both carried
// along instead of being recomputed from 64-bit element indices for every row.
// MXS: q holds the converts' scale operands instead of multipliers.
template <int DT, int RND, bool ALIGNED, int BL, int R, bool MXS>
__device__ __forceinline__ void col_sr_hw(const QuantArgs &P, Chunk<DT> (&v)[16], float (&q)[8][16 / BL],
                                          int64_t row0, int64_t col0, uint32_t (&weven)[8][2],
                                          uint32_t (&wodd)[8][2], uint64_t ctr, uint64_t cstep)
{
    if constexpr (R < 16) {
        const uint64_t e0 = (uint64_t)(row0 + R) * (uint64_t)P.cols + (uint64_t)col0;
        const uint64_t e1 = e0 + (uint64_t)P.cols;
        const u32x4 z = {0, 0, 0, 0};
        const u32x4 a0 = sr_draw(P.seed, ALIGNED ? ctr : e0 >> 3), b0 = sr_draw(P.seed, ALIGNED ? ctr + cstep : e1 >> 3);
        const u32x4 a1 = ALIGNED ? z : sr_draw(P.seed, (e0 >> 3) + 1);
        const u32x4 b1 = ALIGNED ? z : sr_draw(P.seed, (e1 >> 3) + 1);
        const uint32_t sa = (uint32_t)e0 & 7u, sb = (uint32_t)e1 & 7u;
        if constexpr (ALIGNED) {
            // (odd rows are converted into the low nibbles of wodd; the caller shifts them up)
            const uint32_t na[4] = {~a0.x, ~a0.y, ~a0.z, ~a0.w}, nb[4] = {~b0.x, ~b0.y, ~b0.z, ~b0.w};
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                if constexpr (MXS) {
                    weven[c][R / 8] = mx_sr_elem0<DT, (R % 8) / 2>(weven[c][R / 8], v[R], c, sr_seed0(na[c / 2], c & 1), q[c][R / BL]);
                    wodd[c][R / 8] = mx_sr_elem0<DT, (R % 8) / 2>(wodd[c][R / 8], v[R + 1], c, sr_seed0(nb[c / 2], c & 1), q[c][(R + 1) / BL]);
                } else {
                    weven[c][R / 8] = sr_elem0<(R % 8) / 2>(weven[c][R / 8], v[R].get(c) * q[c][R / BL], sr_seed0(na[c / 2], c & 1));
                    wodd[c][R / 8] = sr_elem0<(R % 8) / 2>(wodd[c][R / 8], v[R + 1].get(c) * q[c][(R + 1) / BL], sr_seed0(nb[c / 2], c & 1));
                }
            }
        } else {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                weven[c][R / 8] = sr_elem_hw<0, (R % 8) / 2>(weven[c][R / 8], v[R].get(c) * q[c][R / BL],
                                                             col_bits<ALIGNED>(a0, a1, sa, c));
                wodd[c][R / 8] = sr_elem_hw<1, (R % 8) / 2>(wodd[c][R / 8], v[R + 1].get(c) * q[c][(R + 1) / BL],
                                                            col_bits<ALIGNED>(b0, b1, sb, c));
            }
        }
        col_sr_hw<DT, RND, ALIGNED, BL, R + 2, MXS>(P, v, q, row0, col0, weven, wodd, ctr + 2 * cstep, cstep);
    }
}

// Round-to-nearest of a lane's 16 x 8 tile through the hardware convert: rows R and R + 1 of a column share a
// byte, which the convert writes in place (its byte select must be a constant, hence the recursion over row pairs).
template <int DT, int BL, int R, bool MXS>
__device__ __forceinline__ void col_rtn_hw(Chunk<DT> (&v)[16], float (&q)[8][16 / BL], uint32_t (&words)[8][2])
{
    if constexpr (R < 16) {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            if constexpr (MXS)
                words[c][R / 8] = mx_rtn_rows<DT, (R % 8) / 2>(words[c][R / 8], v[R], v[R + 1], c, q[c][R / BL]);
            else
                words[c][R / 8] = quant_pair_hw<(R % 8) / 2>(words[c][R / 8], v[R].get(c), v[R + 1].get(c), q[c][R / BL]);
        }
        col_rtn_hw<DT, BL, R + 2, MXS>(v, q, words);
    }
}

// Where a lane's column-blocked outputs go in the slab layout: column c of the lane stores its 8 code bytes at
// codes + 512 c and its scale byte at scales + 64 c (blocks of 16) or, from the lowest of the eight stacked lanes,
// the column's four scale bytes at scales + 32 c (blocks of 32); the lane index is folded into the two pointers.
struct ColSlab {
    uint8_t *codes, *scales;
};

template <int DT, int B, int SF, int RND, bool HW, bool ALIGNED, int LV>
__device__ __forceinline__ void cols_tile(const QuantArgs &P, Chunk<DT> (&v)[16], float g, float k, int64_t row0,
                                          int64_t col0, int ncol, int lv, const ColSlab *slab = nullptr);

// ALIGNED: cols is a multiple of 8, so the 8 columns of a lane share one random draw per row.
template <int DT, int B, int SF, int RND, bool HW, bool ALIGNED, int LV = 8>
__global__ __launch_bounds__(256) void quantize_cols_kernel(QuantArgs P)
{
    using G = ColGeom<DT, LV>;
    constexpr int RPL = G::RPL;
    constexpr int BL = B < RPL ? B : RPL;        // rows of one block held by this lane
    constexpr int NB = RPL / BL;                 // blocks (or block parts) per lane per column
    constexpr int LPB = B / BL;                  // lanes sharing one block

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lv = lane % G::LANES_V, lh = lane / G::LANES_V;
    const int64_t row0 = (int64_t)blockIdx.y * G::WG_ROWS + lv * RPL;
    const int64_t col0 = (int64_t)blockIdx.x * G::WG_COLS + wave * G::WAVE_COLS + lh * 8;
    const int ncol = col0 >= P.cols ? 0 : (P.cols - col0 >= 8 ? 8 : (int)(P.cols - col0));

    Chunk<DT> v[RPL];
#pragma unroll
    for (int r = 0; r < RPL; ++r) {
        const int64_t i = row0 + r;
        if (i < P.rows && ncol == 8)
            v[r].template load<true>(P.x, i * P.ld + col0);
        else if (i < P.rows && ncol > 0)
            v[r].load_partial(P.x, i * P.ld + col0, ncol);
        else
            v[r].zero();
    }
    const float g = resolve_g(P);
    const float k = 1.0f / (6.0f * g);
    build_qtab<SF, HW>(g);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *P.g_out = g;
    cols_tile<DT, B, SF, RND, HW, ALIGNED, LV>(P, v, g, k, row0, col0, ncol, lv);
}

// The column-blocked quantization of one lane tile (16 rows x 8 columns in v): block maxima,
// scale bytes, codes, and the stores into the transposed outputs.
template <int DT, int B, int SF, int RND, bool HW, bool ALIGNED, int LV>
__device__ __forceinline__ void cols_tile(const QuantArgs &P, Chunk<DT> (&v)[16], float g, float k, int64_t row0,
                                          int64_t col0, int ncol, int lv, const ColSlab *slab)
{
    using G = ColGeom<DT, LV>;
    constexpr int RPL = G::RPL;
    constexpr int BL = B < RPL ? B : RPL;
    constexpr int NB = RPL / BL;
    constexpr int LPB = B / BL;
    const int64_t rows_half = P.rows >> 1;
    const int64_t nblk = P.rows / B;

    // pass 1: block maxima -> scale bytes and multipliers, per column and per block part
    // MXS: the multipliers are replaced by the converts' scale operands, and an unaligned tile (whose stochastic
    // rounding goes through the two-slot form) keeps multipliers.
    constexpr bool MXS = HW && SF == NVFP4_SCALE_E8M0 && (ALIGNED || RND == NVFP4_RTN);
    float q[8][NB];
    uint32_t sbytes[8][NB];
    if constexpr (MXS && DT == NVFP4_BF16) {
        // maxima on the packed bf16 magnitudes, two columns per instruction
#pragma unroll
        for (int cp = 0; cp < 4; ++cp) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                uint32_t m = 0;
#pragma unroll
                for (int r = 0; r < BL; ++r) m = pk_umax16(m, v[nb * BL + r].word(cp) & 0x7FFF7FFFu);
                const float a0 = group_max<LPB>(pk_even(m)), a1 = group_max<LPB>(pk_odd(m));
                sbytes[2 * cp][nb] = block_scale<SF, HW, false>(a0, g, k, &q[2 * cp][nb]);
                sbytes[2 * cp + 1][nb] = block_scale<SF, HW, false>(a1, g, k, &q[2 * cp + 1][nb]);
            }
        }
    } else {
#pragma unroll
        for (int c = 0; c < 8; ++c) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                float a = 0.0f;
#pragma unroll
                for (int r = 0; r < BL; ++r) a = fmaxf(a, fabsf(v[nb * BL + r].get(c)));
                a = group_max<LPB>(a);
                sbytes[c][nb] = block_scale<SF, HW, HW && SF == NVFP4_SCALE_E4M3>(a, g, k, &q[c][nb]);
            }
        }
    }
    if constexpr (MXS) {
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) q[c][nb] = mx_scale_operand(sbytes[c][nb]);
    }

    // (the empty asm makes the compiler unpack the raw registers again in pass 2 instead of
    // keeping 128 unpacked floats alive across the passes)
#pragma unroll
    for (int r = 0; r < RPL; ++r) v[r].launder();

    // pass 2: codes.  words[c][w] collects rows 8w..8w+7 of column c, one nibble per row.
    uint32_t words[8][RPL / 8];
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int w = 0; w < RPL / 8; ++w) words[c][w] = 0;

    if (RND == NVFP4_RTN && HW) {
        col_rtn_hw<DT, BL, 0, MXS>(v, q, words);
    } else if (RND == NVFP4_SR && HW) {
        // rows 2p and 2p+1 of a column share a byte: even rows go through slot 0, odd rows
        // through slot 1 of the convert, into two sets of words that are OR-ed at the end
        uint32_t wodd[8][RPL / 8];
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int w = 0; w < RPL / 8; ++w) wodd[c][w] = 0;
        const uint64_t cstep = (uint64_t)P.cols >> 3;
        col_sr_hw<DT, RND, ALIGNED, BL, 0, MXS>(P, v, q, row0, col0, words, wodd, (uint64_t)row0 * cstep + ((uint64_t)col0 >> 3), cstep);
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int w = 0; w < RPL / 8; ++w) words[c][w] |= ALIGNED ? wodd[c][w] << 4 : wodd[c][w];
    } else {
        // the 8 columns of a lane are 8 consecutive elements of a row; their random bits come
        // from one draw when that group is aligned in the row-major numbering, else from two
#pragma clang loop unroll(full)
        for (int r = 0; r < RPL; ++r) {
            u32x4 d0 = {0, 0, 0, 0}, d1 = {0, 0, 0, 0};
            uint32_t shift = 0;
            if (RND == NVFP4_SR) {
                const uint64_t e0 = (uint64_t)(row0 + r) * (uint64_t)P.cols + (uint64_t)col0;
                d0 = sr_draw(P.seed, e0 >> 3);
                shift = (uint32_t)e0 & 7u;
                if (!ALIGNED) d1 = sr_draw(P.seed, (e0 >> 3) + 1);
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                uint32_t u16 = 0;
                if (RND == NVFP4_SR) {
                    if (ALIGNED) {
                        u16 = sr_bits_of(d0, c);
                    } else {
                        const uint32_t pos = shift + c;
                        u16 = pos < 8 ? sr_bits_of(d0, pos) : sr_bits_of(d1, pos - 8);
                    }
                }
                words[c][r / 8] |= quant_elem<RND>(v[r].get(c), q[c][r / BL], u16) << (4 * (r % 8));
            }
        }
    }

    // Scale bytes, row-major [cols, rows / B]: the eight lanes stacked vertically hold consecutive bytes of a column's
    // row (blocks of 16: one per lane, 8 per workgroup tile; blocks of 32: one per pair of lanes, 4 per tile).  Where
    // the rows allow, four bytes are gathered into the lowest of their lanes through DPP row shifts (lane + n; every
    // lane takes part) and leave as one aligned dword instead of single bytes.
    constexpr bool GATHER = RPL == 16 && LV == 8 && NB == 1 && (B == 16 || B == 32);
    constexpr int GSTEP = B == 16 ? 1 : 2;  // lanes between consecutive bytes
    uint32_t sw[8];
    bool wide = false, owner = false;
    if constexpr (GATHER) {
        // (the whole 128-row tile inside the tensor, whole dwords per tile, aligned rows of the scale matrix)
        wide = (nblk & 3) == 0 && (reinterpret_cast<uintptr_t>(P.scales) & 3) == 0 && (row0 - lv * RPL) + G::WG_ROWS <= P.rows;
        owner = (lv & (4 * GSTEP - 1)) == 0;  // blocks of 16: lanes 0 and 4 of the eight; blocks of 32: lane 0
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            sw[c] = sbytes[c][0];
            sw[c] |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)sw[c], 0x100 + GSTEP, 0xF, 0xF, true) << 8;       // lane + GSTEP
            sw[c] |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)sw[c], 0x100 + 2 * GSTEP, 0xF, 0xF, true) << 16;  // lanes + 2, + 3 GSTEP
        }
    }

    if (RPL == 16 && slab != nullptr) {
        // slab layout (the caller guarantees a lane tile entirely inside the tensor or entirely outside, blocks of
        // 16 or 32): a store instruction of the wave writes 512 contiguous code bytes and 64 contiguous scale bytes
        // (blocks of 16) or 32 contiguous scale bytes from its eight owner lanes (blocks of 32)
        if (ncol == 8) {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                store8_stream(slab->codes + 512 * c, words[c][0], words[c][1]);
                if (B == 16) {
                    slab->scales[64 * c] = (uint8_t)sbytes[c][0];
                } else if (GATHER) {
                    // blocks of 32: the lowest of the eight stacked lanes holds the column's four bytes of this K tile
                    if (owner) *reinterpret_cast<uint32_t *>(slab->scales + 32 * c) = sw[c];
                }
            }
        }
        return;
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        if (c < ncol) {
            const int64_t col = col0 + c;
            uint8_t *crow = P.codes + col * rows_half + (row0 >> 1);
#pragma unroll
            for (int h = 0; h < RPL / 16; ++h)
                if (row0 + 16 * h < P.rows)
                    store8_stream(crow + 8 * h, words[c][2 * h], words[c][2 * h + 1]);
            if (GATHER && wide) {
                if (owner) *reinterpret_cast<uint32_t *>(P.scales + col * nblk + row0 / B) = sw[c];
            } else if (lv % LPB == 0) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    if (row0 + nb * BL < P.rows)
                        P.scales[col * nblk + (row0 + nb * BL) / B] = (uint8_t)sbytes[c][nb];
            }
        }
    }
}

// ------------------------------------------------------------------ SwiGLU backward as a tile source

// Where the dual quantizer's tile comes from: a tensor in memory, or dG / dU of the SwiGLU backward evaluated from
// dH, G, U while loading (nvfp4_math.h: swiglu_bwd_elem), rounded to the element type like a stored tensor would be.
enum { SRC_TENSOR = 0, SRC_SWIGLU_DG = 1, SRC_SWIGLU_DU = 2 };

// 8 consecutive elements of dG (WHICH = SRC_SWIGLU_DG), of dU (SRC_SWIGLU_DU), or both (0: og and ou)
template <int DT, int WHICH>
__device__ __forceinline__ void swiglu_chunk(const void *dH, const void *G, const void *U, int64_t off, Chunk<DT> *og, Chunk<DT> *ou)
{
    Chunk<DT> h, g, u;
    // (cacheable loads: the three tensors are read by the maximum pass and by both quantizer passes)
    h.template load<false>(dH, off);
    g.template load<false>(G, off);
    u.template load<false>(U, off);
    float rg[8], ru[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) swiglu_bwd_elem(h.get(t), g.get(t), u.get(t), &rg[t], &ru[t]);
    if (WHICH != SRC_SWIGLU_DU) og->set(rg);
    if (WHICH != SRC_SWIGLU_DG) ou->set(ru);
}

// max|dG| and max|dU| (of the values as rounded to the element type) over n = 8 * nchunk elements: one partial
// maximum of each per workgroup, as amax_dense_kernel leaves them for a tensor in memory.
// STORE: the two results are also written out as tensors (dG_out, dU_out), for quantizer passes that read them back
// instead of evaluating them again.
template <int DT, bool STORE>
__global__ __launch_bounds__(1024) void swiglu_amax_kernel(const void *dH, const void *G, const void *U, int64_t n,
                                                           uint32_t *part_g, uint32_t *part_u, void *dG_out, void *dU_out)
{
    const int64_t nchunk = n >> 3;
    const int64_t stride = (int64_t)gridDim.x * (1024 * 2);
    float ag = 0.0f, au = 0.0f;
    for (int64_t base = (int64_t)blockIdx.x * (1024 * 2) + threadIdx.x; base < nchunk; base += stride) {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int64_t c = base + k * 1024;
            if (c < nchunk) {
                Chunk<DT> cg, cu;
                swiglu_chunk<DT, 0>(dH, G, U, c * 8, &cg, &cu);
                if (STORE) {
                    cg.store(dG_out, c * 8);
                    cu.store(dU_out, c * 8);
                }
                ag = fmaxf(ag, chunk_amax(cg));
                au = fmaxf(au, chunk_amax(cu));
            }
        }
    }
    ag = group_max<16>(ag);
    au = group_max<16>(au);
    __shared__ uint32_t pg[64], pu[64];
    if ((threadIdx.x & 15) == 0) {
        pg[threadIdx.x >> 4] = f2u(ag);
        pu[threadIdx.x >> 4] = f2u(au);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t mg = 0, mu = 0;
#pragma unroll
        for (int t = 0; t < 64; ++t) {
            mg = umax(mg, pg[t]);
            mu = umax(mu, pu[t]);
        }
        part_g[blockIdx.x] = mg;
        part_u[blockIdx.x] = mu;
    }
}

// dG and dU stored as tensors (the unfused form of the same step): n = 8 * nchunk elements.
template <int DT>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const void *dH, const void *G, const void *U, int64_t n, void *dG, void *dU)
{
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= (n >> 3)) return;
    Chunk<DT> cg, cu;
    swiglu_chunk<DT, 0>(dH, G, U, c * 8, &cg, &cu);
    cg.store(dG, c * 8);
    cu.store(dU, c * 8);
}

hipError_t launch_swiglu_bwd(const void *dH, const void *G, const void *U, int dt, int64_t n, void *dG, void *dU, hipStream_t st)
{
    const unsigned grid = (unsigned)(((n >> 3) + 255) / 256);
    if (grid == 0) return hipSuccess;
    if (dt == NVFP4_BF16)
        hipLaunchKernelGGL(swiglu_bwd_kernel<NVFP4_BF16>, dim3(grid), dim3(256), 0, st, dH, G, U, n, dG, dU);
    else
        hipLaunchKernelGGL(swiglu_bwd_kernel<NVFP4_F32>, dim3(grid), dim3(256), 0, st, dH, G, U, n, dG, dU);
    return hipGetLastError();
}

// ------------------------------------------------------------------ both orientations in one pass

// Eqs. 5-6 use the output gradient twice, blocked along N for dX and along M for dW; Eqs. 4-5
// do the same with W.  This kernel reads the tensor once and writes both quantizations, each
// identical to what the single-orientation kernels produce (same scale rule, same convert, same
// draws: seed_r for the row-blocked output, P.seed for the column-blocked one), each with its
// own rounding mode (X is needed round-to-nearest along K for Eq. 4 and stochastically rounded
// along M for Eq. 6).
// Geometry of the columns kernel (lane = 16 rows x 8 columns, workgroup = 128 rows x 256
// columns).  A row block of B = 16 or 32 columns spans 2 or 4 lanes that are 8 apart in the wave
// (DPP row rotate / swizzle for the maximum).  The row-blocked codes of the tile (128 rows x 128
// bytes) and its scale bytes are staged in LDS and written out 16 bytes per lane, so both outputs
// leave in full lines although the lanes hold the data column-wise.
// Host guarantees: rows % B == 0, cols % B == 0 (so a lane's 16 x 8 tile is entirely inside or
// outside the tensor), 16-byte aligned rows of x.
// One workgroup tile (128 rows x 256 columns at tile coordinates tx, ty; the lane's 16 x 8 part of it in v) through
// both quantizers and out to memory.  Every thread of the workgroup must call it (barriers inside).
template <int DT, int B, int SF, int RND_R, int RND_C>
__device__ __forceinline__ void dual_tile(const DualArgs &D, Chunk<DT> (&v)[16], float g, float k, int tx, int ty,
                                          uint32_t *lds_codes, uint8_t *lds_scales)
{
    using G = ColGeom<DT, 8>;
    constexpr int LPBR = B / 8;                  // lanes sharing one row block
    constexpr bool MXS = SF == NVFP4_SCALE_E8M0;  // block scale as the convert's scale operand
    constexpr int ROW_BYTES = G::WG_COLS / 2;    // 128 code bytes per tile row
    constexpr int ROW_SC = G::WG_COLS / B;       // scale bytes per tile row
    const QuantArgs &P = D.c;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lv = lane % G::LANES_V, lh = lane / G::LANES_V;
    const int64_t wrow0 = (int64_t)ty * G::WG_ROWS, wcol0 = (int64_t)tx * G::WG_COLS;
    const int64_t row0 = wrow0 + lv * 16;
    const int64_t col0 = wcol0 + wave * G::WAVE_COLS + lh * 8;
    const bool inside = row0 < P.rows && col0 < P.cols;

    // row-blocked side: one block scale and 8 codes per row of the lane tile
    const uint64_t cstep_r = (uint64_t)P.cols >> 3;
    uint64_t ctr_r = (uint64_t)row0 * cstep_r + ((uint64_t)col0 >> 3);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        float a = MXS ? chunk_amax_packed(v[r]) : chunk_amax(v[r]);
        a = dpp_max<0x128>(a);  // row_ror:8 : lane ^ 8, the neighbouring column group
        if (LPBR == 4) {
            const uint32_t o = (uint32_t)__builtin_amdgcn_ds_swizzle((int)f2u(a), 0x401F);  // lane ^ 16
            a = u2f(umax(f2u(a), o));
        }
        float q;
        const uint32_t sbyte = block_scale<SF, true, SF == NVFP4_SCALE_E4M3>(a, g, k, &q);
        if (MXS) q = mx_scale_operand(sbyte);
        // (cols is a multiple of the block, col0 of 8: the lane's 8 columns are one draw, cols / 8 draws per row)
        const uint32_t packed = chunk_codes_hw<DT, RND_R, MXS>(v[r], q, D.seed_r, ctr_r);
        ctr_r += cstep_r;
        // tile row R = 16 lv + r holds 32 dwords; dword w is stored at w ^ (4 lv): the 16-byte
        // chunk c of the row sits at chunk c ^ lv, which spreads the 8 rows a wave writes at a
        // time over the banks
        const int R = lv * 16 + r;
        lds_codes[R * (ROW_BYTES / 4) + ((wave * 8 + lh) ^ (lv << 2))] = packed;
        if ((lh & (LPBR - 1)) == 0) lds_scales[R * 16 + (wave * G::WAVE_COLS + lh * 8) / B] = (uint8_t)sbyte;
    }

    // (unpack the raw registers again below instead of keeping 128 floats alive)
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r].launder();

    // column-blocked side: exactly the columns kernel's tile.  In the slab layout the workgroup's 256 columns are
    // one tile of operand rows and its 128 rows one K tile: it fills exactly one slab.
    ColSlab cs;
    if (D.slab_c) {
        const int64_t slab = (int64_t)tx * (P.rows / SLAB_K) + ty;
        cs.codes = P.codes + slab * SLAB_CODE_BYTES + wave * 4096 + lane * 8;
        // (tile column 64 wave + 8 lh + c sits at position 64 wave + 8 c + lh)
        cs.scales = B == 16 ? P.scales + slab * SLAB_SCALE_BYTES + wave * 512 + lane
                            : P.scales + slab * SLAB_MX_SCALE_BYTES + wave * 256 + lh * 4;
    }
    cols_tile<DT, B, SF, RND_C, true, true, 8>(P, v, g, k, row0, col0, inside ? 8 : 0, lv, D.slab_c ? &cs : nullptr);

    __syncthreads();
    if (D.slab_r) {
        // slab layout: the tile is rows (wrow0 % 256) .. + 127 of two slabs (K tiles 2 tx and + 1 of row
        // tile wrow0 / 256).  Threads walk the slab positions q; position q holds tile row slab_row(q).
        const int64_t nkt = P.cols / SLAB_K;
        const int64_t slab0 = (wrow0 / SLAB_ROWS) * nkt + 2 * (int64_t)tx;
        const int half = (int)(wrow0 & 128);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = threadIdx.x + 256 * i, q = id >> 3, c = id & 7, R = slab_row(q);
            if (wrow0 + R < P.rows && wcol0 + c * 32 < P.cols) {
                const uint4 w = *reinterpret_cast<const uint4 *>(&lds_codes[R * (ROW_BYTES / 4) + ((c ^ (R >> 4)) << 2)]);
                const u32x4_t o = {w.x, w.y, w.z, w.w};
                __builtin_nontemporal_store(o, reinterpret_cast<u32x4_t *>(D.codes_r + (slab0 + (c >> 2)) * SLAB_CODE_BYTES + (half + q) * 64 + (c & 3) * 16));
            }
        }
        if (threadIdx.x < G::WG_ROWS) {
            const int q = threadIdx.x, R = slab_row(q);
            if (wrow0 + R < P.rows) {
                const uint32_t *src = reinterpret_cast<const uint32_t *>(&lds_scales[R * 16]);
                if (B == 16) {
                    uint8_t *dst = D.scales_r + slab0 * SLAB_SCALE_BYTES + (half + q) * 8;
                    store8_stream(dst, src[0], src[1]);
                    if (wcol0 + 128 < P.cols) store8_stream(dst + SLAB_SCALE_BYTES, src[2], src[3]);
                } else {
                    // blocks of 32: four bytes per row and K tile
                    uint8_t *dst = D.scales_r + slab0 * SLAB_MX_SCALE_BYTES + (half + q) * 4;
                    store4_stream(dst, src[0]);
                    if (wcol0 + 128 < P.cols) store4_stream(dst + SLAB_MX_SCALE_BYTES, src[1]);
                }
            }
        }
        return;
    }
    const int64_t cpr = P.cols >> 1;
    const bool wide = (cpr & 15) == 0;  // rows of the code matrix are 16-byte aligned
    if (!D.slab_r) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int id = threadIdx.x + 256 * i, R = id >> 3, c = id & 7;
            const int64_t row = wrow0 + R, col = wcol0 + c * 32;
            if (row < P.rows && col < P.cols) {
                const uint4 w = *reinterpret_cast<const uint4 *>(&lds_codes[R * (ROW_BYTES / 4) + ((c ^ (R >> 4)) << 2)]);
                uint8_t *dst = D.codes_r + row * cpr + (col >> 1);
                if (col + 32 <= P.cols && wide) {
                    const u32x4_t o = {w.x, w.y, w.z, w.w};
                    __builtin_nontemporal_store(o, reinterpret_cast<u32x4_t *>(dst));
                } else {
                    store8_stream(dst, w.x, w.y);
                    if (col + 32 <= P.cols) store8_stream(dst + 8, w.z, w.w);
                }
            }
        }
    }
    if (threadIdx.x < G::WG_ROWS) {
        const int R = threadIdx.x;
        const int64_t row = wrow0 + R, nsc = P.cols / B, s0 = wcol0 / B;
        if (row < P.rows && s0 < nsc) {
            uint8_t *dst = D.scales_r + row * nsc + s0;
            const uint32_t *src = reinterpret_cast<const uint32_t *>(&lds_scales[R * 16]);
            if (s0 + ROW_SC <= nsc && nsc % ROW_SC == 0) {
                store8_stream(dst, src[0], src[1]);
                if (ROW_SC == 16) store8_stream(dst + 8, src[2], src[3]);
            } else {
                const int n = (int)(nsc - s0 < ROW_SC ? nsc - s0 : ROW_SC);
                for (int j = 0; j < n; ++j) dst[j] = lds_scales[R * 16 + j];
            }
        }
    }
}

template <int DT, int B, int SF, int RND_R, int RND_C, int SRC = SRC_TENSOR>
__global__ __launch_bounds__(256) void quantize_dual_kernel(DualArgs D)
{
    using G = ColGeom<DT, 8>;
    static_assert(B == 16 || B == 32, "row blocks must fit the 8 column groups of a wave");
    __shared__ __align__(16) uint32_t lds_codes[G::WG_ROWS * (G::WG_COLS / 2) / 4];
    __shared__ __align__(16) uint8_t lds_scales[G::WG_ROWS * 16];

    const QuantArgs &P = D.c;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lv = lane % G::LANES_V, lh = lane / G::LANES_V;
    const int64_t row0 = (int64_t)blockIdx.y * G::WG_ROWS + lv * 16;
    const int64_t col0 = (int64_t)blockIdx.x * G::WG_COLS + wave * G::WAVE_COLS + lh * 8;
    const bool inside = row0 < P.rows && col0 < P.cols;

    Chunk<DT> v[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if (!inside)
            v[r].zero();
        else if (SRC == SRC_TENSOR)
            v[r].template load<true>(P.x, (row0 + r) * P.ld + col0);
        else
            swiglu_chunk<DT, SRC>(P.x, D.src_g, D.src_u, (row0 + r) * P.ld + col0, &v[r], &v[r]);
    }

    const float g = resolve_g(P);
    const float k = 1.0f / (6.0f * g);
    build_qtab<SF, true>(g);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        // (a `saved` buffer that is not the one this call expects poisons the scale the GEMMs will multiply by)
        const float g_gemm = tag_apply(D.tag) ? g : __builtin_nanf("");
        *P.g_out = g_gemm;
        if (D.g_out2) *D.g_out2 = g_gemm;
    }
    dual_tile<DT, B, SF, RND_R, RND_C>(D, v, g, k, (int)blockIdx.x, (int)blockIdx.y, lds_codes, lds_scales);
}

__global__ void saved_tag_kernel(TagArgs t, float *g1, float *g2)
{
    if (!tag_apply(t)) {
        if (g1) *g1 = __builtin_nanf("");
        if (g2) *g2 = __builtin_nanf("");
    }
}

// ------------------------------------------------------------------ host-side launchers

static inline hipError_t launch_status() { return hipGetLastError(); }

int64_t tensor_amax_partials(int64_t rows, int64_t cols, int64_t ld)
{
    int64_t span_rows = rows, span_cols = cols;
    if (ld == cols) {
        span_cols = rows * cols;
        span_rows = 1;
    }
    int64_t gx = ((span_cols >> 3) + 256 * AMAX_UNROLL - 1) / (256 * AMAX_UNROLL);
    if (gx < 1) gx = 1;
    return gx * (span_rows < 1 ? 1 : span_rows);
}

hipError_t launch_tensor_amax(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld,
                              uint32_t *amax_bits, uint32_t *partials, float *g_out, hipStream_t st)
{
    if (rows <= 0 || cols <= 0) {
        // an empty tensor has no partial maxima: the fold alone leaves max = 0, scale = 1
        hipLaunchKernelGGL(fold_amax_kernel, dim3(1), dim3(1024), 0, st, partials, (int64_t)0, amax_bits, g_out);
        return launch_status();
    }
    int64_t span_rows = rows, span_cols = cols;
    if (ld == cols) {
        span_cols = rows * cols;
        span_rows = 1;
    }
    int64_t gx = ((span_cols >> 3) + 256 * AMAX_UNROLL - 1) / (256 * AMAX_UNROLL);
    if (gx < 1) gx = 1;
    // grid.y is limited to 65535: walk taller tensors in slabs
    for (int64_t r0 = 0; r0 < span_rows; r0 += 65535) {
        const int64_t nr = span_rows - r0 < 65535 ? span_rows - r0 : 65535;
        const char *base = reinterpret_cast<const char *>(x) + r0 * ld * (dt == NVFP4_BF16 ? 2 : 4);
        if (dt == NVFP4_BF16)
            hipLaunchKernelGGL(amax_kernel<NVFP4_BF16>, dim3((unsigned)gx, (unsigned)nr), dim3(256), 0, st,
                               base, span_cols, ld, partials + r0 * gx);
        else
            hipLaunchKernelGGL(amax_kernel<NVFP4_F32>, dim3((unsigned)gx, (unsigned)nr), dim3(256), 0, st,
                               base, span_cols, ld, partials + r0 * gx);
    }
    hipLaunchKernelGGL(fold_amax_kernel, dim3(1), dim3(1024), 0, st, partials, gx * span_rows, amax_bits, g_out);
    return launch_status();
}

hipError_t launch_tensor_amax_dense(const void *x, int dt, int64_t n_elements, uint32_t *partials, int *n, hipStream_t st)
{
    int64_t gx = ((n_elements >> 3) + AMAX_DENSE_THREADS * AMAX_UNROLL - 1) / (AMAX_DENSE_THREADS * AMAX_UNROLL);
    gx = gx < 1 ? 1 : (gx > AMAX_DENSE_PARTIALS ? AMAX_DENSE_PARTIALS : gx);
    if (dt == NVFP4_BF16)
        hipLaunchKernelGGL(amax_dense_kernel<NVFP4_BF16>, dim3((unsigned)gx), dim3(AMAX_DENSE_THREADS), 0, st, x, n_elements, partials);
    else
        hipLaunchKernelGGL(amax_dense_kernel<NVFP4_F32>, dim3((unsigned)gx), dim3(AMAX_DENSE_THREADS), 0, st, x, n_elements, partials);
    *n = (int)gx;
    return launch_status();
}

template <int DT, int B, int SF, int RND, bool HW>
static void launch_q(const QuantArgs &P, int axis, hipStream_t st)
{
    if (axis == 1) {
        const int64_t total = P.rows * (P.cols >> 3);
        const int64_t per = 256 * ROWS_UNROLL;
        hipLaunchKernelGGL((quantize_rows_kernel<DT, B, SF, RND, HW>), dim3((unsigned)((total + per - 1) / per)),
                           dim3(256), 0, st, P);
    } else {
        using G = ColGeom<DT>;
        dim3 grid((unsigned)((P.cols + G::WG_COLS - 1) / G::WG_COLS),
                  (unsigned)((P.rows + G::WG_ROWS - 1) / G::WG_ROWS));
        if (RND == NVFP4_SR && (P.cols & 7) != 0)
            hipLaunchKernelGGL((quantize_cols_kernel<DT, B, SF, RND, HW, RND == NVFP4_RTN>), grid, dim3(256), 0, st, P);
        else
            hipLaunchKernelGGL((quantize_cols_kernel<DT, B, SF, RND, HW, true>), grid, dim3(256), 0, st, P);
    }
}

template <int DT, int B, int SF>
static void launch_q_rnd(const QuantArgs &P, int axis, int rounding, bool hw, hipStream_t st)
{
    if (rounding == NVFP4_SR && hw)
        launch_q<DT, B, SF, NVFP4_SR, true>(P, axis, st);
    else if (rounding == NVFP4_SR)
        launch_q<DT, B, SF, NVFP4_SR, false>(P, axis, st);
    else if (hw)
        launch_q<DT, B, SF, NVFP4_RTN, true>(P, axis, st);
    else
        launch_q<DT, B, SF, NVFP4_RTN, false>(P, axis, st);
}

template <int DT>
static void launch_q_fmt(const QuantArgs &P, int axis, int rounding, int block, int sf, bool hw,
                         hipStream_t st)
{
#define NVFP4_CASE(BB)                                                                   \
    case BB:                                                                             \
        if (sf == NVFP4_SCALE_E4M3)                                                      \
            launch_q_rnd<DT, BB, NVFP4_SCALE_E4M3>(P, axis, rounding, hw, st);           \
        else                                                                             \
            launch_q_rnd<DT, BB, NVFP4_SCALE_E8M0>(P, axis, rounding, hw, st);           \
        break;
    switch (block) {
        NVFP4_CASE(16)
        NVFP4_CASE(32)
        NVFP4_CASE(64)
        NVFP4_CASE(128)
    default: break;
    }
#undef NVFP4_CASE
}

hipError_t launch_quantize(const QuantArgs &P, int dt, int axis, int rounding, int block, int sf,
                           bool hw_convert, hipStream_t st)
{
    if (dt == NVFP4_BF16)
        launch_q_fmt<NVFP4_BF16>(P, axis, rounding, block, sf, hw_convert, st);
    else
        launch_q_fmt<NVFP4_F32>(P, axis, rounding, block, sf, hw_convert, st);
    return launch_status();
}

template <int DT, int B, int SF>
static void launch_dual_rnd(const DualArgs &D, int rnd_r, int rnd_c, hipStream_t st)
{
    using G = ColGeom<DT>;
    dim3 grid((unsigned)((D.c.cols + G::WG_COLS - 1) / G::WG_COLS), (unsigned)((D.c.rows + G::WG_ROWS - 1) / G::WG_ROWS));
    if (rnd_r == NVFP4_SR && rnd_c == NVFP4_SR)
        hipLaunchKernelGGL((quantize_dual_kernel<DT, B, SF, NVFP4_SR, NVFP4_SR>), grid, dim3(256), 0, st, D);
    else if (rnd_r == NVFP4_RTN && rnd_c == NVFP4_SR)
        hipLaunchKernelGGL((quantize_dual_kernel<DT, B, SF, NVFP4_RTN, NVFP4_SR>), grid, dim3(256), 0, st, D);
    else
        hipLaunchKernelGGL((quantize_dual_kernel<DT, B, SF, NVFP4_RTN, NVFP4_RTN>), grid, dim3(256), 0, st, D);
}

template <int DT>
static void launch_dual_fmt(const DualArgs &D, int rnd_r, int rnd_c, int block, int sf, hipStream_t st)
{
    if (block == 16 && sf == NVFP4_SCALE_E4M3) launch_dual_rnd<DT, 16, NVFP4_SCALE_E4M3>(D, rnd_r, rnd_c, st);
    else if (block == 16) launch_dual_rnd<DT, 16, NVFP4_SCALE_E8M0>(D, rnd_r, rnd_c, st);
    else if (sf == NVFP4_SCALE_E4M3) launch_dual_rnd<DT, 32, NVFP4_SCALE_E4M3>(D, rnd_r, rnd_c, st);
    else launch_dual_rnd<DT, 32, NVFP4_SCALE_E8M0>(D, rnd_r, rnd_c, st);
}

template <int DT, int B, int SF>
static void launch_swiglu_dual_fmt(const DualArgs &g, const DualArgs &u, hipStream_t st)
{
    using G = ColGeom<DT>;
    dim3 grid((unsigned)((g.c.cols + G::WG_COLS - 1) / G::WG_COLS), (unsigned)((g.c.rows + G::WG_ROWS - 1) / G::WG_ROWS));
    hipLaunchKernelGGL((quantize_dual_kernel<DT, B, SF, NVFP4_SR, NVFP4_SR, SRC_SWIGLU_DG>), grid, dim3(256), 0, st, g);
    hipLaunchKernelGGL((quantize_dual_kernel<DT, B, SF, NVFP4_SR, NVFP4_SR, SRC_SWIGLU_DU>), grid, dim3(256), 0, st, u);
}

hipError_t launch_swiglu_bwd_dual(DualArgs &g, DualArgs &u, int dt, int block, int sf, uint32_t *partials_g,
                                  uint32_t *partials_u, void *dG_store, void *dU_store, hipStream_t st)
{
    const int64_t n = g.c.rows * g.c.cols;
    const bool nv = block == 16 && sf == NVFP4_SCALE_E4M3, mxf = block == 32 && sf == NVFP4_SCALE_E8M0;
    if (!nv && !mxf) return hipErrorInvalidValue;
    const bool store = dG_store != nullptr;
    if (g.c.g_mode == G_FROM_AMAX || store) {
        int64_t gx = ((n >> 3) + 2047) / 2048;
        gx = gx < 1 ? 1 : (gx > AMAX_DENSE_PARTIALS ? AMAX_DENSE_PARTIALS : gx);
        const dim3 grid((unsigned)gx), wg(1024);
        if (dt == NVFP4_BF16 && store)
            hipLaunchKernelGGL((swiglu_amax_kernel<NVFP4_BF16, true>), grid, wg, 0, st, g.c.x, g.src_g, g.src_u, n, partials_g, partials_u, dG_store, dU_store);
        else if (dt == NVFP4_BF16)
            hipLaunchKernelGGL((swiglu_amax_kernel<NVFP4_BF16, false>), grid, wg, 0, st, g.c.x, g.src_g, g.src_u, n, partials_g, partials_u, dG_store, dU_store);
        else if (store)
            hipLaunchKernelGGL((swiglu_amax_kernel<NVFP4_F32, true>), grid, wg, 0, st, g.c.x, g.src_g, g.src_u, n, partials_g, partials_u, dG_store, dU_store);
        else
            hipLaunchKernelGGL((swiglu_amax_kernel<NVFP4_F32, false>), grid, wg, 0, st, g.c.x, g.src_g, g.src_u, n, partials_g, partials_u, dG_store, dU_store);
        if (g.c.g_mode == G_FROM_AMAX) {
            g.c.g_src = reinterpret_cast<const float *>(partials_g);
            u.c.g_src = reinterpret_cast<const float *>(partials_u);
            g.c.n_partials = u.c.n_partials = (int)gx;
        }
    }
    if (store) {
        // the quantizers read the stored results (the ordinary dual kernel), not dH, G, U again
        g.c.x = dG_store;
        u.c.x = dU_store;
        g.src_g = g.src_u = u.src_g = u.src_u = nullptr;
        hipError_t e = launch_quantize_dual(g, dt, NVFP4_SR, NVFP4_SR, block, sf, true, st);
        if (e != hipSuccess) return e;
        return launch_quantize_dual(u, dt, NVFP4_SR, NVFP4_SR, block, sf, true, st);
    }
    if (dt == NVFP4_BF16) {
        if (nv) launch_swiglu_dual_fmt<NVFP4_BF16, 16, NVFP4_SCALE_E4M3>(g, u, st);
        else launch_swiglu_dual_fmt<NVFP4_BF16, 32, NVFP4_SCALE_E8M0>(g, u, st);
    } else {
        if (nv) launch_swiglu_dual_fmt<NVFP4_F32, 16, NVFP4_SCALE_E4M3>(g, u, st);
        else launch_swiglu_dual_fmt<NVFP4_F32, 32, NVFP4_SCALE_E8M0>(g, u, st);
    }
    return launch_status();
}

bool quantize_dual_fused(int dt, int64_t rows, int64_t cols, int64_t ld, int block, bool hw_convert)
{
    const int64_t esz = dt == NVFP4_BF16 ? 2 : 4;
    return hw_convert && (block == 16 || block == 32) && rows % block == 0 && cols % block == 0 &&
           (ld * esz) % 16 == 0 && cols < (int64_t(1) << 31) && rows < (int64_t(1) << 31);
}

hipError_t launch_quantize_dual(const DualArgs &D, int dt, int rnd_r, int rnd_c, int block, int sf, bool hw_convert,
                                hipStream_t st)
{
    // (SR rows with RtN columns is a combination no equation asks for: two kernels)
    if (quantize_dual_fused(dt, D.c.rows, D.c.cols, D.c.ld, block, hw_convert) && !(rnd_r == NVFP4_SR && rnd_c == NVFP4_RTN)) {
        if (dt == NVFP4_BF16)
            launch_dual_fmt<NVFP4_BF16>(D, rnd_r, rnd_c, block, sf, st);
        else
            launch_dual_fmt<NVFP4_F32>(D, rnd_r, rnd_c, block, sf, st);
        return launch_status();
    }
    // other block sizes and ragged shapes: the two single-orientation kernels (they write the plain layout only)
    if (D.slab_r || D.slab_c) return hipErrorInvalidValue;
    QuantArgs r = D.c;
    r.codes = D.codes_r;
    r.scales = D.scales_r;
    r.seed = D.seed_r;
    r.g_out = D.c.g_out;
    hipError_t e = launch_quantize(r, dt, 1, rnd_r, block, sf, hw_convert, st);
    if (e != hipSuccess) return e;
    e = launch_quantize(D.c, dt, 0, rnd_c, block, sf, hw_convert, st);
    if (e != hipSuccess) return e;
    if (D.g_out2) {
        e = hipMemcpyAsync(D.g_out2, D.c.g_out, sizeof(float), hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return e;
    }
    return launch_saved_tag(D.tag, D.c.g_out, D.g_out2, st);
}

hipError_t launch_saved_tag(const TagArgs &t, float *g1, float *g2, hipStream_t st)
{
    if (!t.dst && !t.chk) return hipSuccess;
    hipLaunchKernelGGL(saved_tag_kernel, dim3(1), dim3(1), 0, st, t, g1, g2);
    return launch_status();
}

}  // namespace nvfp4
