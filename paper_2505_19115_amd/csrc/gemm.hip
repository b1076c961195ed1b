// Block-scaled FP4 GEMM for gfx950 ("NT": both operands stored with the contraction axis
// contiguous), the matrix product shared by Eqs. 4-6 of "FP4 All the Way":
//     out[i, j] = gA gB sum_k cA[i,k] sA[i,k/B] cB[j,k] sB[j,k/B].
//
// E4M3 block scales (NVFP4 and its wider-block variants).  The CDNA4 scaled FP4 MFMA applies
// one power-of-two (E8M0) scale per 32 contraction elements, so it cannot apply a 16-wide
// E4M3 scale, and an E2M1 x E4M3 product needs up to 6 significant bits, more than FP8 or FP6
// hold.  The product is exact in fp16 (11 bits; magnitudes 2^-10 .. 2688), so operands travel
// through HBM and LDS as packed 4-bit codes plus scale bytes and are expanded in registers:
//     v_cvt_scalef32_pk_f16_fp4 (code pair -> fp16 pair, times 2^8)  and
//     v_pk_mul_f16 by the block scale written as fp16(scale * 2^-8),
// which is exact for every E4M3 byte, including its subnormals; the MFMA operands themselves
// are always normal fp16 numbers or zero.  The contraction runs on v_mfma_f32_32x32x16_f16 with
// fp32 accumulation; the tensor scales multiply once in the epilogue.
#include "kernels.h"
#include "nvfp4_math.h"

namespace nvfp4 {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int KT = 128;      // contraction elements per LDS tile
constexpr int KTB = KT / 2;  // bytes of codes per row per tile
constexpr int SROW = 8;      // LDS bytes reserved per row for the tile's scale bytes

// 16-byte chunk c (0..3) of tile row r lives at chunk slot c ^ ((r >> 1) & 3): 8 consecutive
// rows reading the same logical chunk then hit 8 different 16-byte bank groups.
__device__ __forceinline__ int swz(int r, int c) { return r * KTB + ((c ^ ((r >> 1) & 3)) << 4); }

// 8 codes (one dword) of one block -> 8 fp16 values times the block scale.
// s2 = fp16 pair holding scale * 2^-8 twice.
__device__ __forceinline__ half8_t dequant8(uint32_t w, half2_t s2)
{
    half2_t h0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 0) * s2;
    half2_t h1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 1) * s2;
    half2_t h2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 2) * s2;
    half2_t h3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 3) * s2;
    half8_t r;
    r[0] = h0[0]; r[1] = h0[1]; r[2] = h1[0]; r[3] = h1[1];
    r[4] = h2[0]; r[5] = h2[1]; r[6] = h3[0]; r[7] = h3[1];
    return r;
}

// E4M3 byte -> fp16 pair of scale * 2^-8: the byte shifted into fp16's exponent/mantissa
// fields is that value for normal and subnormal bytes alike (fp16 bias 15 = E4M3 bias 7 + 8).
__device__ __forceinline__ half2_t scale_pair(uint32_t byte)
{
    uint32_t b = byte << 7;
    return __builtin_bit_cast(half2_t, b | (b << 16));
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Workgroup: 256 threads = 2 x 2 waves; a wave owns (32 TA) x (32 TB) outputs as TA x TB MFMA
// tiles.  Per 128-wide K tile the 64 code bytes of each operand row sit in LDS as four
// 16-byte chunks; lane (r = lane % 32, h = lane / 32) expands chunk 2p + h (p = 0, 1), and
// its dword t feeds the t-th MFMA of that half tile.  A and B use the same assignment of
// contraction indices to (lane half, slot), which is all the instruction requires.
template <int B, int TA, int TB, int OUT_DT>
__global__ __launch_bounds__(256) void gemm_nt_f16_kernel(GemmArgs P)
{
    constexpr int BM = 64 * TA, BN = 64 * TB;
    constexpr int SPT = KT / B;  // scale bytes per row per tile
    __shared__ __attribute__((aligned(16))) uint8_t sA[BM * KTB];
    __shared__ __attribute__((aligned(16))) uint8_t sB[BN * KTB];
    __shared__ __attribute__((aligned(16))) uint8_t sSA[BM * SROW];
    __shared__ __attribute__((aligned(16))) uint8_t sSB[BN * SROW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, h = lane >> 5;
    const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * BN;
    const int64_t Kb = P.K >> 1;          // code bytes per row
    const int64_t Ks = P.K / B;           // scale bytes per row
    const int nkt = (int)((P.K + KT - 1) / KT);
    const bool vec_scales = (P.K % KT) == 0;

    float16_t acc[TA][TB];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    uint4 ga[TA], gb[TB];
    uint64_t gsa = 0, gsb = 0;

    auto fetch = [&](int kt) {
#pragma unroll
        for (int u = 0; u < TA; ++u) {
            const int qd = tid + 256 * u, row = qd >> 2, ch = qd & 3;
            const int64_t kb = (int64_t)kt * KTB + ch * 16;
            ga[u] = (m0 + row < P.M && kb < Kb)
                        ? *reinterpret_cast<const uint4 *>(P.A_codes + (m0 + row) * Kb + kb)
                        : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int qd = tid + 256 * u, row = qd >> 2, ch = qd & 3;
            const int64_t kb = (int64_t)kt * KTB + ch * 16;
            gb[u] = (n0 + row < P.N && kb < Kb)
                        ? *reinterpret_cast<const uint4 *>(P.B_codes + (n0 + row) * Kb + kb)
                        : make_uint4(0, 0, 0, 0);
        }
        auto fetch_scales = [&](const uint8_t *base, int64_t row_g, int64_t nrows) -> uint64_t {
            uint64_t s = 0;
            if (row_g < nrows) {
                const uint8_t *p = base + row_g * Ks + (int64_t)kt * SPT;
                if (vec_scales) {
                    if (SPT == 8) s = *reinterpret_cast<const uint64_t *>(p);
                    else if (SPT == 4) s = *reinterpret_cast<const uint32_t *>(p);
                    else if (SPT == 2) s = *reinterpret_cast<const uint16_t *>(p);
                    else s = *p;
                } else {
                    const int64_t left = Ks - (int64_t)kt * SPT;
#pragma unroll
                    for (int t = 0; t < SPT; ++t)
                        if (t < left) s |= (uint64_t)p[t] << (8 * t);
                }
            }
            return s;
        };
        if (tid < BM) gsa = fetch_scales(P.A_scales, m0 + tid, P.M);
        if (tid < BN) gsb = fetch_scales(P.B_scales, n0 + tid, P.N);
    };

    auto stash = [&]() {
#pragma unroll
        for (int u = 0; u < TA; ++u) {
            const int qd = tid + 256 * u;
            *reinterpret_cast<uint4 *>(sA + swz(qd >> 2, qd & 3)) = ga[u];
        }
#pragma unroll
        for (int u = 0; u < TB; ++u) {
            const int qd = tid + 256 * u;
            *reinterpret_cast<uint4 *>(sB + swz(qd >> 2, qd & 3)) = gb[u];
        }
        if (tid < BM) *reinterpret_cast<uint64_t *>(sSA + tid * SROW) = gsa;
        if (tid < BN) *reinterpret_cast<uint64_t *>(sSB + tid * SROW) = gsb;
    };

    fetch(0);
    for (int kt = 0; kt < nkt; ++kt) {
        __syncthreads();
        stash();
        __syncthreads();
        if (kt + 1 < nkt) fetch(kt + 1);

#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int ch = 2 * p + h;  // this lane's chunk: tile elements 32 ch .. 32 ch + 31
            uint4 ca[TA], cb[TB];
            uint32_t sca[TA], scb[TB];  // the chunk's scale bytes (two for B = 16, else one)
#pragma unroll
            for (int a = 0; a < TA; ++a) {
                const int row = wm * 32 * TA + 32 * a + r;
                ca[a] = *reinterpret_cast<const uint4 *>(sA + swz(row, ch));
                if (B == 16)
                    sca[a] = *reinterpret_cast<const uint16_t *>(sSA + row * SROW + 2 * ch);
                else
                    sca[a] = sSA[row * SROW + (32 * ch) / B];
            }
#pragma unroll
            for (int b = 0; b < TB; ++b) {
                const int row = wn * 32 * TB + 32 * b + r;
                cb[b] = *reinterpret_cast<const uint4 *>(sB + swz(row, ch));
                if (B == 16)
                    scb[b] = *reinterpret_cast<const uint16_t *>(sSB + row * SROW + 2 * ch);
                else
                    scb[b] = sSB[row * SROW + (32 * ch) / B];
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                half8_t fa[TA], fb[TB];
#pragma unroll
                for (int a = 0; a < TA; ++a) {
                    const uint32_t w = t == 0 ? ca[a].x : t == 1 ? ca[a].y : t == 2 ? ca[a].z : ca[a].w;
                    const uint32_t sb = (B == 16 && t >= 2) ? (sca[a] >> 8) : (sca[a] & 0xFFu);
                    fa[a] = dequant8(w, scale_pair(sb));
                }
#pragma unroll
                for (int b = 0; b < TB; ++b) {
                    const uint32_t w = t == 0 ? cb[b].x : t == 1 ? cb[b].y : t == 2 ? cb[b].z : cb[b].w;
                    const uint32_t sb = (B == 16 && t >= 2) ? (scb[b] >> 8) : (scb[b] & 0xFFu);
                    fb[b] = dequant8(w, scale_pair(sb));
                }
#pragma unroll
                for (int a = 0; a < TA; ++a)
#pragma unroll
                    for (int b = 0; b < TB; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[a], fb[b], acc[a][b], 0, 0, 0);
            }
        }
    }

    // epilogue: accumulator register v of lane (r, h) is row 8 (v / 4) + 4 h + v % 4, column r
    const float gg = P.tensor_scales[0] * P.tensor_scales[1];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            const int64_t col = n0 + wn * 32 * TB + 32 * b + r;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wm * 32 * TA + 32 * a + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < P.M && col < P.N) {
                    const float y = acc[a][b][v] * gg;
                    if (OUT_DT == NVFP4_F32)
                        reinterpret_cast<float *>(P.out)[row * P.ldc + col] = y;
                    else
                        reinterpret_cast<uint16_t *>(P.out)[row * P.ldc + col] = f32_to_bf16_rne(y);
                }
            }
        }
}

template <int B, int TA, int TB>
static void launch_f16(const GemmArgs &P, int out_dt, hipStream_t st)
{
    constexpr int BM = 64 * TA, BN = 64 * TB;
    dim3 grid((unsigned)((P.N + BN - 1) / BN), (unsigned)((P.M + BM - 1) / BM));
    if (out_dt == NVFP4_F32)
        hipLaunchKernelGGL((gemm_nt_f16_kernel<B, TA, TB, NVFP4_F32>), grid, dim3(256), 0, st, P);
    else
        hipLaunchKernelGGL((gemm_nt_f16_kernel<B, TA, TB, NVFP4_BF16>), grid, dim3(256), 0, st, P);
}

hipError_t launch_gemm(const GemmArgs &P, int block, int sf, int out_dt, hipStream_t st)
{
    if (sf != NVFP4_SCALE_E4M3) return hipErrorNotSupported;
    switch (block) {
    case 16: launch_f16<16, 2, 2>(P, out_dt, st); break;
    case 32: launch_f16<32, 2, 2>(P, out_dt, st); break;
    case 64: launch_f16<64, 2, 2>(P, out_dt, st); break;
    case 128: launch_f16<128, 2, 2>(P, out_dt, st); break;
    default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

}  // namespace nvfp4
