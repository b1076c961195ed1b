// MXFP4 GEMM on the CDNA4 scaled FP4 MFMA ("NT": both operands stored with the contraction
// axis contiguous).  MXFP4 (Sec. 3 / Table 1 of "FP4 All the Way": E2M1 elements, blocks of 32,
// E8M0 power-of-two scales) is exactly what v_mfma_scale_f32_32x32x64_f8f6f4 consumes: each
// lane supplies 32 consecutive contraction elements (16 bytes of packed codes) of one row plus
// one E8M0 byte for them, so the packed operands go from LDS straight into the instruction with
// no expansion arithmetic at all:
//     out[i, j] = gA gB sum_b 2^(eA[i,b] - 127) 2^(eB[j,b] - 127) sum_{k in b} cA[i,k] cB[j,k].
// Products and the power-of-two scaling are exact; accumulation is fp32.
//
// Geometry of both kernels: 256 threads = 2 x 2 waves, wave tile 128 x 128 (4 x 4 MFMA tiles, all
// 256 accumulator registers, one wave per SIMD), workgroup tile 256 x 256: with no VALU work in
// the loop what matters is bytes moved per MFMA (a 4 x 4 register tile reads 8 KB of LDS per 16
// MFMAs), hence the largest register tile that fits.  The MFMA's first operand is the B (N-side)
// tile, so a lane's accumulator holds four consecutive output COLUMNS of one row.
#include "kernels.h"
#include "nvfp4_math.h"

namespace nvfp4 {

typedef int int8v_t __attribute__((ext_vector_type(8)));
typedef float float16v_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2v_t __attribute__((ext_vector_type(2)));

namespace mx {
constexpr int NT = 256, BM = 256, BN = 256, TA = 4, TB = 4;
}

__device__ __forceinline__ uint16_t mx_bf16_rne(float f)
{
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Epilogue of both kernels: accumulator register v of lane (r, g) of tile (a, b) is output row
// 32 a + r, column 32 b + 8 (v / 4) + 4 g + v % 4.  Full tiles with a suitably aligned output get
// one packed convert pair and one 8-byte (bf16) or 16-byte (fp32) store per four outputs; edge
// tiles store element by element.  The lane coordinates are re-derived from an opaque copy so
// that none of the output addressing is computed before the K loop and kept in registers across it.
// lds_lines: 64 KB of LDS (32 KB suffice for bf16) that no wave reads and no load writes any more (the caller has waited and
// synchronized), or nullptr.  With it, bf16 output goes out in complete lines: per accumulator row
// of tiles a wave transposes its 32 rows x 128 columns through a private 8 KB piece (16-byte chunks
// XOR-swizzled by row) and stores 4 rows of 256 contiguous bytes per instruction.
template <int OUT_DT>
__device__ __forceinline__ void mx_store_tile(const GemmArgs &P, float16v_t (&acc)[mx::TA][mx::TB], int64_t m0, int64_t n0,
                                              int lane, int wave, uint8_t *lds_lines = nullptr)
{
    using namespace mx;
    int lane_e = lane, wave_e = wave;
    asm volatile("" : "+v"(lane_e), "+v"(wave_e));
    const int re = lane_e & 31, ge = lane_e >> 5, wme = wave_e >> 1, wne = wave_e & 1;
    const float gg = P.gA[0] * P.gB[0];
    constexpr int ESZ = OUT_DT == NVFP4_F32 ? 4 : 2;
    const int64_t row0 = m0 + wme * 128 + re, col0 = n0 + wne * 128 + 4 * ge;
    uint8_t *const out = reinterpret_cast<uint8_t *>(P.out);
    const bool fast = m0 + BM <= P.M && n0 + BN <= P.N && (P.ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(P.out) & 15) == 0;
    if (OUT_DT == NVFP4_F32 && lds_lines != nullptr && fast) {
        // fp32: 32 rows x 512 bytes at a time (16 KB per wave), two complete rows per store
        uint8_t *const mine = lds_lines + __builtin_amdgcn_readfirstlane(wave_e) * 16384;
#pragma unroll
        for (int a = 0; a < TA; ++a) {
#pragma unroll
            for (int b = 0; b < TB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int chunk = 8 * b + 2 * q + ge;  // columns 4 chunk .. 4 chunk + 3 of the wave's 128
                    *reinterpret_cast<float4 *>(mine + re * 512 + ((chunk ^ (re & 15)) << 4)) =
                        make_float4(acc[a][b][4 * q] * gg, acc[a][b][4 * q + 1] * gg, acc[a][b][4 * q + 2] * gg, acc[a][b][4 * q + 3] * gg);
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int rowl = 2 * i + (lane_e >> 5), chunk = lane_e & 31;
                const uint4 v = *reinterpret_cast<const uint4 *>(mine + rowl * 512 + ((chunk ^ (rowl & 15)) << 4));
                const int64_t grow = m0 + wme * 128 + 32 * a + rowl, gcol = n0 + wne * 128 + 4 * chunk;
                *reinterpret_cast<uint4 *>(out + (grow * P.ldc + gcol) * 4) = v;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    } else if (OUT_DT == NVFP4_BF16 && lds_lines != nullptr && fast && (P.ldc & 7) == 0) {
        uint8_t *const mine = lds_lines + __builtin_amdgcn_readfirstlane(wave_e) * 8192;
#pragma unroll
        for (int a = 0; a < TA; ++a) {
#pragma unroll
            for (int b = 0; b < TB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float2v_t lo = {acc[a][b][4 * q] * gg, acc[a][b][4 * q + 1] * gg};
                    const float2v_t hi = {acc[a][b][4 * q + 2] * gg, acc[a][b][4 * q + 3] * gg};
                    const bf16x2_t blo = __builtin_convertvector(lo, bf16x2_t), bhi = __builtin_convertvector(hi, bf16x2_t);
                    uint2 w;
                    w.x = *reinterpret_cast<const uint32_t *>(&blo);
                    w.y = *reinterpret_cast<const uint32_t *>(&bhi);
                    const int chunk = 4 * b + q;  // columns 8 chunk .. 8 chunk + 7 of the wave's 128
                    *reinterpret_cast<uint2 *>(mine + re * 256 + ((chunk ^ (re & 15)) << 4) + 8 * ge) = w;
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int rowl = 4 * i + (lane_e >> 4), chunk = lane_e & 15;
                const uint4 v = *reinterpret_cast<const uint4 *>(mine + rowl * 256 + ((chunk ^ (rowl & 15)) << 4));
                const int64_t grow = m0 + wme * 128 + 32 * a + rowl, gcol = n0 + wne * 128 + 8 * chunk;
                *reinterpret_cast<uint4 *>(out + (grow * P.ldc + gcol) * 2) = v;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    } else if (fast) {
#pragma unroll
        for (int a = 0; a < TA; ++a) {
            uint8_t *prow = out + ((row0 + 32 * a) * P.ldc + col0) * ESZ;
#pragma unroll
            for (int b = 0; b < TB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float y0 = acc[a][b][4 * q] * gg, y1 = acc[a][b][4 * q + 1] * gg;
                    const float y2 = acc[a][b][4 * q + 2] * gg, y3 = acc[a][b][4 * q + 3] * gg;
                    uint8_t *dst = prow + (32 * b + 8 * q) * ESZ;
                    if (OUT_DT == NVFP4_F32) {
                        *reinterpret_cast<float4 *>(dst) = make_float4(y0, y1, y2, y3);
                    } else {
                        const float2v_t lo = {y0, y1}, hi = {y2, y3};
                        const bf16x2_t blo = __builtin_convertvector(lo, bf16x2_t), bhi = __builtin_convertvector(hi, bf16x2_t);
                        uint2 w;
                        w.x = *reinterpret_cast<const uint32_t *>(&blo);
                        w.y = *reinterpret_cast<const uint32_t *>(&bhi);
                        *reinterpret_cast<uint2 *>(dst) = w;
                    }
                }
            __builtin_amdgcn_sched_barrier(0);  // one accumulator row of tiles at a time keeps the register peak low
        }
    } else {
#pragma unroll
        for (int a = 0; a < TA; ++a)
#pragma unroll
            for (int b = 0; b < TB; ++b) {
                const int64_t row = row0 + 32 * a;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t col = col0 + 32 * b + 8 * (v >> 2) + (v & 3);
                    if (row < P.M && col < P.N) {
                        const float y = acc[a][b][v] * gg;
                        if (OUT_DT == NVFP4_F32)
                            reinterpret_cast<float *>(P.out)[row * P.ldc + col] = y;
                        else
                            reinterpret_cast<uint16_t *>(P.out)[row * P.ldc + col] = mx_bf16_rne(y);
                    }
                }
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Fallback kernel: any K that is a multiple of 32, any operand alignment.  K tile 64 = one MFMA
// step, two LDS stages, everything staged through registers (chunks past K are zero-filled, rows
// past the edge clamped to the last row: their products land in outputs that are never stored).
// LDS stage: codes [512 rows][32 bytes], the two 16-byte chunks of row r swapped when r is odd;
// scales as dwords [2 lane halves][512 rows], byte 0 = the E8M0 byte of the lane half's block.
namespace mxf {
constexpr int KT = 64, ROWB = 32;
constexpr int CODES = (mx::BM + mx::BN) * ROWB;
constexpr int STAGE = CODES + 2 * (mx::BM + mx::BN) * 4;
constexpr int LDS_BYTES = 2 * STAGE;
}  // namespace mxf

template <int OUT_DT>
__global__ __launch_bounds__(256) void gemm_nt_mxfp4_kernel(GemmArgs P)
{
    using namespace mx;
    using namespace mxf;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, g = lane >> 5;
    const int ntx = (int)((P.N + BN - 1) / BN), nty = (int)((P.M + BM - 1) / BM);
    int ty, tx;
    tile_coords((int)blockIdx.x, ntx, nty, ty, tx);
    const int64_t m0 = (int64_t)ty * BM, n0 = (int64_t)tx * BN;
    const int64_t Kb = P.K >> 1, Ks = P.K >> 5;
    const int nkt = (int)((P.K + KT - 1) / KT);

    float16v_t acc[TA][TB];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // ---- global -> registers -> LDS: thread t stages chunks t and t + 256 (row = chunk / 2) of each operand
    uint4 ga[2], gb[2];
    uint32_t gsa = 0, gsb = 0;
    const uint8_t *pA[2], *pB[2];
    int ldsW[2], chunk[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int qd = tid + NT * u, row = qd >> 1, c = qd & 1;
        const int64_t ar = m0 + row < P.M ? m0 + row : P.M - 1, br = n0 + row < P.N ? n0 + row : P.N - 1;
        pA[u] = P.A_codes + ar * Kb + c * 16;
        pB[u] = P.B_codes + br * Kb + c * 16;
        chunk[u] = c;
        ldsW[u] = row * ROWB + ((c ^ (row & 1)) << 4);
    }
    const int64_t sar = m0 + tid < P.M ? m0 + tid : P.M - 1, sbr = n0 + tid < P.N ? n0 + tid : P.N - 1;
    auto load16u = [](const uint8_t *p) -> uint4 {  // any alignment
        uint4 v;
        __builtin_memcpy(&v, p, 16);
        return v;
    };
    auto fetch = [&](int kt) {
        const int64_t kb = (int64_t)kt * ROWB;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const bool in = kb + chunk[u] * 16 < Kb;  // zero codes past K
            ga[u] = in ? load16u(pA[u] + kb) : make_uint4(0, 0, 0, 0);
            gb[u] = in ? load16u(pB[u] + kb) : make_uint4(0, 0, 0, 0);
        }
        const uint8_t *sa = P.A_scales + sar * Ks + (int64_t)kt * 2, *sb = P.B_scales + sbr * Ks + (int64_t)kt * 2;
        const bool two = (int64_t)kt * 2 + 1 < Ks;
        gsa = (uint32_t)sa[0] | (two ? (uint32_t)sa[1] << 8 : 0u);
        gsb = (uint32_t)sb[0] | (two ? (uint32_t)sb[1] << 8 : 0u);
    };
    auto stash = [&](int stage) {
        uint8_t *base = lds + stage * STAGE;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            *reinterpret_cast<uint4 *>(base + ldsW[u]) = ga[u];
            *reinterpret_cast<uint4 *>(base + BM * ROWB + ldsW[u]) = gb[u];
        }
        uint32_t *sS = reinterpret_cast<uint32_t *>(base + CODES);
        sS[tid] = gsa & 0xFFu;
        sS[(BM + BN) + tid] = gsa >> 8;
        sS[BM + tid] = gsb & 0xFFu;
        sS[(BM + BN) + BM + tid] = gsb >> 8;
    };

    // ---- LDS -> registers -> MFMA: lane (r, g) multiplies chunk g of its rows
    struct Frags {
        uint4 a[TA], b[TB];
        uint32_t sa[TA], sb[TB];
    };
    const int rd = r * ROWB + ((g ^ (r & 1)) << 4);
    auto load_frags = [&](int stage, Frags &F) {
        const uint8_t *p = lds + stage * STAGE + rd;
        const uint32_t *q = reinterpret_cast<const uint32_t *>(lds + stage * STAGE + CODES) + g * (BM + BN) + r;
#pragma unroll
        for (int a = 0; a < TA; ++a) {
            F.a[a] = *reinterpret_cast<const uint4 *>(p + (wm * 128 + 32 * a) * ROWB);
            F.sa[a] = q[wm * 128 + 32 * a];
        }
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            F.b[b] = *reinterpret_cast<const uint4 *>(p + (BM + wn * 128 + 32 * b) * ROWB);
            F.sb[b] = q[BM + wn * 128 + 32 * b];
        }
    };
    auto mma = [&](const Frags &F) {
#pragma unroll
        for (int a = 0; a < TA; ++a)
#pragma unroll
            for (int b = 0; b < TB; ++b) {
                const int8v_t va = {(int)F.a[a].x, (int)F.a[a].y, (int)F.a[a].z, (int)F.a[a].w, 0, 0, 0, 0};
                const int8v_t vb = {(int)F.b[b].x, (int)F.b[b].y, (int)F.b[b].z, (int)F.b[b].w, 0, 0, 0, 0};
                acc[a][b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vb, va, acc[a][b], 4, 4, 0, (int)F.sb[b], 0, (int)F.sa[a]);
            }
    };

    Frags F;
    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
        const int stage = kt & 1;
        const bool more = kt + 1 < nkt;
        if (more) fetch(kt + 1);
        load_frags(stage, F);
        if (more) stash(stage ^ 1);  // the other stage: last read before the previous barrier
        mma(F);
        __syncthreads();
    }
    mx_store_tile<OUT_DT>(P, acc, m0, n0, lane, wave);
}

// ---------------------------------------------------------------------------------------------
// E4M3 block scales at blocks of 64 and 128 on the FP4 matrix instruction (the block-size study of Sec. 3.1 / Fig. 2):
// an E4M3 scale has a mantissa, which the instruction's power-of-two scale operand cannot carry, so the blocks are
// multiplied with unit scales and the partial sum of each block is rescaled in binary32:
//     acc[i, j] += P_b[i, j] * (sA[i, b] * sB[j, b]),      P_b = sum_{k in b} cA[i, k] cB[j, k].
// P_b is exact (a multiple of 1/4 below 2^13), the product of two E4M3 values is exact (8 significant bits), and so is
// their product with P_b (<= 23 bits): every term enters the accumulator with the one rounding of the addition, as in
// the other kernels.  One 32 x 32 x 64 MFMA is exactly one block of 64; two chained ones are one block of 128.  The
// cost is on the vector ALU: 16 scale products and 16 multiply-adds per 32 x 32 tile and block.
// K tile 128 = two MFMA steps; step s of lane half g multiplies chunk 2 s + g, so a step covers elements 64 s .. 64 s + 63
// of the tile (one block of 64, half a block of 128).  Two LDS stages, everything staged through registers; the block
// scales are decoded to binary32 when they are staged.  K must be a multiple of 128; rows past the edge are clamped.
namespace mxr {
constexpr int KT = 128, ROWB = 64;
constexpr int CODES = (mx::BM + mx::BN) * ROWB;              // 32 KB
constexpr int STAGE = CODES + 2 * (mx::BM + mx::BN) * 4;     // + decoded scales [2 blocks][512 rows]
constexpr int LDS_BYTES = 2 * STAGE;                         // 72 KB (>= the 64 KB the fp32 epilogue borrows)
}  // namespace mxr

template <int OUT_DT, int B>
__global__ __launch_bounds__(256) void gemm_nt_fp4_rescale_kernel(GemmArgs P)
{
    using namespace mx;
    using namespace mxr;
    static_assert(B == 64 || B == 128, "blocks that are whole MFMA steps");
    constexpr int NBLK = KT / B;  // blocks per K tile
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, g = lane >> 5;
    const int ntx = (int)((P.N + BN - 1) / BN), nty = (int)((P.M + BM - 1) / BM);
    int ty, tx;
    tile_coords((int)blockIdx.x, ntx, nty, ty, tx);
    const int64_t m0 = (int64_t)ty * BM, n0 = (int64_t)tx * BN;
    const int64_t Kb = P.K >> 1, Ks = P.K / B;
    const int nkt = (int)(P.K / KT);

    float16v_t acc[TA][TB];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // ---- global -> registers -> LDS: thread t stages chunks t, t + 256, t + 512, t + 768 (row = chunk / 4) of each operand
    uint4 ga[4], gb[4];
    float gsa[NBLK], gsb[NBLK];
    const uint8_t *pA[4], *pB[4];
    int ldsW[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int qd = tid + NT * u, row = qd >> 2, c = qd & 3;
        const int64_t ar = m0 + row < P.M ? m0 + row : P.M - 1, br = n0 + row < P.N ? n0 + row : P.N - 1;
        pA[u] = P.A_codes + ar * Kb + c * 16;
        pB[u] = P.B_codes + br * Kb + c * 16;
        ldsW[u] = row * ROWB + ((c ^ ((row >> 2) & 3)) << 4);
    }
    const int64_t sar = m0 + tid < P.M ? m0 + tid : P.M - 1, sbr = n0 + tid < P.N ? n0 + tid : P.N - 1;
    auto fetch = [&](int kt) {
        const int64_t kb = (int64_t)kt * ROWB;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ga[u] = *reinterpret_cast<const uint4 *>(pA[u] + kb);
            gb[u] = *reinterpret_cast<const uint4 *>(pB[u] + kb);
        }
#pragma unroll
        for (int q = 0; q < NBLK; ++q) {
            gsa[q] = e4m3_decode(P.A_scales[sar * Ks + (int64_t)kt * NBLK + q]);
            gsb[q] = e4m3_decode(P.B_scales[sbr * Ks + (int64_t)kt * NBLK + q]);
        }
    };
    auto stash = [&](int stage) {
        uint8_t *base = lds + stage * STAGE;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            *reinterpret_cast<uint4 *>(base + ldsW[u]) = ga[u];
            *reinterpret_cast<uint4 *>(base + BM * ROWB + ldsW[u]) = gb[u];
        }
        float *sS = reinterpret_cast<float *>(base + CODES);
#pragma unroll
        for (int q = 0; q < NBLK; ++q) {
            sS[q * (BM + BN) + tid] = gsa[q];
            sS[q * (BM + BN) + BM + tid] = gsb[q];
        }
    };

    const int sw = (r >> 2) & 3;
    // one K tile: per step the 8 fragments, per block the lane's scales (its row of each A fragment, its 16 columns of
    // each B fragment), then 16 tiles of MFMA (+ MFMA) and rescale
    auto tile = [&](int stage) {
        const uint8_t *cbase = lds + stage * STAGE;
        const float *sS = reinterpret_cast<const float *>(cbase + CODES);
        // the A fragments of both steps stay in registers; B fragments and B scales are fetched per column of tiles
        uint4 fa[2][TA];
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int a = 0; a < TA; ++a)
                fa[s][a] = *reinterpret_cast<const uint4 *>(cbase + (((2 * s + g) ^ sw) << 4) + (wm * 128 + 32 * a + r) * ROWB);
#pragma unroll
        for (int q = 0; q < NBLK; ++q) {
            float sa[TA];
#pragma unroll
            for (int a = 0; a < TA; ++a) sa[a] = sS[q * (BM + BN) + wm * 128 + 32 * a + r];
#pragma unroll
            for (int b = 0; b < TB; ++b) {
                float4 sb[4];
#pragma unroll
                for (int c4 = 0; c4 < 4; ++c4)
                    sb[c4] = *reinterpret_cast<const float4 *>(&sS[q * (BM + BN) + BM + wn * 128 + 32 * b + 8 * c4 + 4 * g]);
                uint4 fb[2];
#pragma unroll
                for (int s = 0; s < 2; ++s)
                    fb[s] = *reinterpret_cast<const uint4 *>(cbase + (((2 * s + g) ^ sw) << 4) + (BM + wn * 128 + 32 * b + r) * ROWB);
#pragma unroll
                for (int a = 0; a < TA; ++a) {
                    float16v_t t;
#pragma unroll
                    for (int v = 0; v < 16; ++v) t[v] = 0.0f;
                    // B = 128: both steps belong to the one block; B = 64: step q is block q
#pragma unroll
                    for (int s = (B == 128 ? 0 : q); s < (B == 128 ? 2 : q + 1); ++s) {
                        const int8v_t va = {(int)fa[s][a].x, (int)fa[s][a].y, (int)fa[s][a].z, (int)fa[s][a].w, 0, 0, 0, 0};
                        const int8v_t vb = {(int)fb[s].x, (int)fb[s].y, (int)fb[s].z, (int)fb[s].w, 0, 0, 0, 0};
                        t = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vb, va, t, 4, 4, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
                    }
#pragma unroll
                    for (int c4 = 0; c4 < 4; ++c4) {
                        acc[a][b][4 * c4 + 0] = __builtin_fmaf(t[4 * c4 + 0], sa[a] * sb[c4].x, acc[a][b][4 * c4 + 0]);
                        acc[a][b][4 * c4 + 1] = __builtin_fmaf(t[4 * c4 + 1], sa[a] * sb[c4].y, acc[a][b][4 * c4 + 1]);
                        acc[a][b][4 * c4 + 2] = __builtin_fmaf(t[4 * c4 + 2], sa[a] * sb[c4].z, acc[a][b][4 * c4 + 2]);
                        acc[a][b][4 * c4 + 3] = __builtin_fmaf(t[4 * c4 + 3], sa[a] * sb[c4].w, acc[a][b][4 * c4 + 3]);
                    }
                }
            }
        }
    };

    fetch(0);
    stash(0);
    __syncthreads();
    for (int kt = 0; kt < nkt; ++kt) {
        const int stage = kt & 1;
        const bool more = kt + 1 < nkt;
        if (more) fetch(kt + 1);
        tile(stage);
        if (more) stash(stage ^ 1);  // the other stage: every wave finished reading it before the previous barrier
        __syncthreads();
    }
    mx_store_tile<OUT_DT>(P, acc, m0, n0, lane, wave, lds);
}

// ---------------------------------------------------------------------------------------------
// Main kernel (K a multiple of 128 and at least 512, 16-byte aligned codes): four LDS stages of
// 128 contraction elements, every byte written by direct global -> LDS loads, three K tiles in
// flight, one barrier per tile, no VALU work in the loop except eight scale shifts per tile.
//
// What bounds the loop besides the MFMA pipe is the vector L1: it takes one request (at most 64
// bytes) per clock, and a lane-per-row load costs one request per lane however few bytes it
// fetches.  The codes need 512 requests per tile (64 bytes per row); the scales are therefore
// fetched 16 bytes per row at a time = FOUR tiles' worth in one request, into a double-buffered
// scale area, instead of one dword per row per tile.
//
// LDS: four code stages [512 rows][64 bytes] with the 16-byte chunk c of row r at slot
// c ^ ((r >> 2) & 3) (sixteen consecutive rows reading one logical chunk cover all sixteen 16-byte
// slots of the 256-byte bank period); two scale buffers [512 rows][16 bytes] (a group of four K
// tiles each); 4 KB that absorbs the filler loads.  MFMA step s (0, 1) of lane half g multiplies
// chunk 2 g + s of the tile: the lane shifts the tile's scale dword right by 16 g once and the
// instruction's byte select is the compile-time s.
//
// An operand in the slab layout (A_SLAB / B_SLAB) brings its scales as slabs too: 256 positions x 4 bytes per K
// tile, contiguous, so ONE instruction of one wave fetches the scales of a whole K tile (wave 0: A, wave 1: B), they
// travel with the codes of their tile through four 1 KB stages (which take the place of that operand's part of the
// first scale buffer), and a lane reads its row's dword at position slab_row(row): 32 consecutive rows are 32
// different banks.  (Row-major scales lie 16 bytes apart in LDS, so 32 rows share 16 banks and those reads conflict.)
//
// Every wave issues the same ten direct-to-LDS instructions per K tile, which the counted waits rely on: 4 + 4
// codes, one slot for a row-major scale group and one for a scale slab; a slot with nothing to fetch issues a
// one-request filler.
//
// The MFMA's first operand is the B (N-side) tile, so a lane's accumulator holds four consecutive
// output COLUMNS of one row: the epilogue is one packed convert pair and one 8-byte (bf16) or
// 16-byte (fp32) store per four outputs.
namespace mxd {
constexpr int KT = 128, ROWB = 64, NS = 4;
constexpr int STAGE = (mx::BM + mx::BN) * ROWB;        // 32 KB of codes
constexpr int SBUF = (mx::BM + mx::BN) * 16;           // 8 KB: the scales of four K tiles
constexpr int SCALES0 = NS * STAGE, DUMP0 = SCALES0 + 2 * SBUF;
constexpr int LDS_BYTES = DUMP0 + 4096;
constexpr int PER_TILE = 10;  // direct-to-LDS instructions per wave per K tile: 4 + 4 codes, 2 scale slots
}  // namespace mxd

template <int OUT_DT, bool A_SLAB, bool B_SLAB>
__global__ __launch_bounds__(256) void gemm_nt_mxfp4_dma_kernel(GemmArgs P)
{
    using namespace mx;
    using namespace mxd;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, g = lane >> 5;
    const int ntx = (int)((P.N + BN - 1) / BN), nty = (int)((P.M + BM - 1) / BM);
    int ty, tx;
    tile_coords((int)blockIdx.x, ntx, nty, ty, tx);
    const int64_t m0 = (int64_t)ty * BM, n0 = (int64_t)tx * BN;
    const int64_t Kb = P.K >> 1, Ks = P.K >> 5;
    const int nkt = (int)(P.K / KT);

    float16v_t acc[TA][TB];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // ---- global -> LDS.  A code instruction fills 1 KB = 16 consecutive tile rows, lane i landing
    // at byte 16 i (row i / 4, slot i % 4), so the swizzle is applied by choosing WHICH global chunk
    // the lane fetches.  Rows past the edge are clamped to the last row (their products land in
    // outputs that are never stored).  Lane offsets are relative to the tile's first row, the
    // 64-bit part of the address is wave-uniform.
    const int64_t mrows = P.M - m0 < BM ? P.M - m0 : BM, nrows = P.N - n0 < BN ? P.N - n0 : BN;
    uint32_t offA[4], offB[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int row = (wave * 4 + u) * 16 + (lane >> 2);
        const int c = (lane & 3) ^ ((lane >> 4) & 3);
        // (an operand in the slab layout has all 256 rows of the tile, 64 bytes apart, in slab order)
        offA[u] = A_SLAB ? (uint32_t)(slab_row(row) * 64 + c * 16) : (uint32_t)((row < mrows ? row : mrows - 1) * Kb + c * 16);
        offB[u] = B_SLAB ? (uint32_t)(slab_row(row) * 64 + c * 16) : (uint32_t)((row < nrows ? row : nrows - 1) * Kb + c * 16);
    }
    const int srow = wave * 64 + lane;
    const uint32_t offSA = (uint32_t)((srow < mrows ? srow : mrows - 1) * Ks);
    const uint32_t offSB = (uint32_t)((srow < nrows ? srow : nrows - 1) * Ks);
    typedef __attribute__((address_space(3))) void *lds_ptr_t;
    auto uniform_ptr = [](const uint8_t *p) -> const uint8_t * {
        const uint64_t v = reinterpret_cast<uint64_t>(p);
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
    };
    // Issued through inline assembly on purpose: the compiler's wait-count pass treats a
    // direct-to-LDS load as a possible writer of every LDS location and would wait for ALL of them
    // before the next LDS read.  Here a stage is never read before the explicit counted wait and
    // the barrier that follow its loads.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    const uint32_t code_dst = __builtin_amdgcn_readfirstlane(lds0 + wave * 4096);
    const uint32_t scale_dst = __builtin_amdgcn_readfirstlane(lds0 + SCALES0 + wave * 1024);
    const uint32_t dump_dst = __builtin_amdgcn_readfirstlane(lds0 + DUMP0 + wave * 1024);
    auto dma16 = [&](uint32_t lds_addr, uint32_t voff, const uint8_t *base) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(voff), "s"(base) : "memory");
    };
    // codes of K tile kt: tile + kt * step (row-major: 64 bytes further along every row; slabs: the next 16 KB slab)
    const uint8_t *tileA = A_SLAB ? P.A_codes + (int64_t)ty * nkt * SLAB_CODE_BYTES : P.A_codes + m0 * Kb;
    const uint8_t *tileB = B_SLAB ? P.B_codes + (int64_t)tx * nkt * SLAB_CODE_BYTES : P.B_codes + n0 * Kb;
    constexpr int64_t stepA = A_SLAB ? SLAB_CODE_BYTES : ROWB, stepB = B_SLAB ? SLAB_CODE_BYTES : ROWB;
    // scales: the tile's rows in the row-major matrix, or the tile row's scale slabs (one per K tile)
    const uint8_t *tileSA = A_SLAB ? P.A_scales + (int64_t)ty * nkt * SLAB_MX_SCALE_BYTES : P.A_scales + m0 * Ks;
    const uint8_t *tileSB = B_SLAB ? P.B_scales + (int64_t)tx * nkt * SLAB_MX_SCALE_BYTES : P.B_scales + n0 * Ks;
    auto dma_codes = [&](int kt) {
        const uint32_t st = (uint32_t)(kt & (NS - 1)) * STAGE;
        const uint8_t *pa = uniform_ptr(tileA + kt * stepA), *pb = uniform_ptr(tileB + kt * stepB);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            dma16(code_dst + st + u * 1024, offA[u], pa);
            dma16(code_dst + st + BM * ROWB + u * 1024, offB[u], pb);
        }
    };
    // Scale group G = the 16 scale bytes of a row that cover K tiles 4 G .. 4 G + 3; the window of the
    // last group is moved back to end with the row (Ks >= 16), so no load passes the end of a row.
    auto group_start = [&](int G) -> int { return 16 * G + 16 <= Ks ? 16 * G : (int)Ks - 16; };
    // keeps the number of loads per tile constant (the counted waits rely on it): one request, lands in the dump
    // (the first bytes of A's codes: a valid address in both layouts)
    auto dma_filler = [&]() { dma16(dump_dst, 0u, uniform_ptr(tileA)); };
    // row-major scales, group G.  part 0: this wave's 64 A rows, part 1: its 64 B rows
    auto dma_scales = [&](int G, int part) {
        if ((part == 0 && A_SLAB) || (part == 1 && B_SLAB)) {
            dma_filler();
            return;
        }
        const uint8_t *base = (part ? tileSB : tileSA) + group_start(G);
        dma16(scale_dst + (G & 1) * SBUF + part * (BM * 16), part ? offSB : offSA, uniform_ptr(base));
    };
    // scale slabs of K tile kt (real: kt < nkt): wave 0 fetches A's, wave 1 B's, 16 bytes per lane, into stage
    // kt % 4 of that operand's part of the first scale buffer; the other waves (and a wave whose operand is
    // row-major) fill in
    const uint32_t slab_scale_dst = __builtin_amdgcn_readfirstlane(lds0 + SCALES0 + (wave == 1 ? BM * 16 : 0));
    const bool slab_loader = __builtin_amdgcn_readfirstlane((wave == 0 && A_SLAB) || (wave == 1 && B_SLAB));
    auto dma_scale_slab = [&](int kt, bool real) {
        const bool go = slab_loader && real;
        const uint8_t *base = go ? (wave == 0 ? tileSA : tileSB) + (int64_t)kt * SLAB_MX_SCALE_BYTES : tileA;
        dma16(go ? slab_scale_dst + (uint32_t)(kt & (NS - 1)) * 1024 : dump_dst, go ? (uint32_t)lane * 16 : 0u, uniform_ptr(base));
    };

    // ---- LDS -> registers
    struct Frags {
        uint4 a[TA], b[TB];
    };
    struct Scales {
        uint32_t a[TA], b[TB];
    };
    const int sw = (r >> 2) & 3;
    const int rdA = (wm * 128 + r) * ROWB, rdB = (BM + wn * 128 + r) * ROWB;
    // scale dword of fragment i (rows 32 i + r of the wave's part): row-major image [row][16 bytes], or the slab
    // image [position][4 bytes] with the row at position slab_row(row) (for row 128 w + 32 i + r that is
    // 128 w + 64 (i / 2) + 8 (r % 8) + 4 (i % 2) + r / 8: a lane part plus a constant per fragment)
    const int rdS = SCALES0 + (A_SLAB ? slab_row(wm * 128 + r) * 4 : (wm * 128 + r) * 16);
    const int rdT = SCALES0 + BM * 16 + (B_SLAB ? slab_row(wn * 128 + r) * 4 : (wn * 128 + r) * 16);
    auto frag_off = [](bool slab, int i) -> int { return slab ? 256 * (i >> 1) + 16 * (i & 1) : 512 * i; };
    // where in the scale area the dwords of K tile kt start
    auto tile_off = [&](bool slab, int kt) -> int {
        const int G = kt >> 2;
        return slab ? (kt & (NS - 1)) * 1024 : (G & 1) * SBUF + (4 * kt - group_start(G));
    };
    const int sh = 16 * g;
    // fragment i of both operands (rows 32 i + r of the wave's A and B parts) for MFMA step s of tile kt
    auto load_frag = [&](int kt, int s, Frags &F, int i) {
        const uint8_t *p = lds + (kt & (NS - 1)) * STAGE + (((2 * g + s) ^ sw) << 4);
        F.a[i] = *reinterpret_cast<const uint4 *>(p + rdA + 32 * i * ROWB);
        F.b[i] = *reinterpret_cast<const uint4 *>(p + rdB + 32 * i * ROWB);
    };
    // raw scale dwords of a tile (all four E8M0 bytes of the row); shifted into place when the tile starts
    auto load_scale = [&](int kt, Scales &R, int i) {
        R.a[i] = *reinterpret_cast<const uint32_t *>(lds + tile_off(A_SLAB, kt) + rdS + frag_off(A_SLAB, i));
        R.b[i] = *reinterpret_cast<const uint32_t *>(lds + tile_off(B_SLAB, kt) + rdT + frag_off(B_SLAB, i));
    };
    auto shift_scales = [&](const Scales &R, Scales &S) {
#pragma unroll
        for (int a = 0; a < TA; ++a) S.a[a] = R.a[a] >> sh;
#pragma unroll
        for (int b = 0; b < TB; ++b) S.b[b] = R.b[b] >> sh;
    };
    // one MFMA: output rows of A fragment ia against B fragment ib.  The first MFMA operand is the
    // B tile (its rows become accumulator rows), the second the A tile.
#define NVFP4_MXD_MMA(F, S, s, ia, ib)                                                                    \
    {                                                                                                     \
        const int8v_t va = {(int)F.a[ia].x, (int)F.a[ia].y, (int)F.a[ia].z, (int)F.a[ia].w, 0, 0, 0, 0};  \
        const int8v_t vb = {(int)F.b[ib].x, (int)F.b[ib].y, (int)F.b[ib].z, (int)F.b[ib].w, 0, 0, 0, 0};  \
        acc[ia][ib] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(vb, va, acc[ia][ib], 4, 4, s, (int)S.b[ib], s, \
                                                                      (int)S.a[ia]);                      \
        __builtin_amdgcn_sched_barrier(0);                                                                \
    }
    // wait until at most n direct-to-LDS instructions of this wave are still in flight
#define NVFP4_MXD_WAIT(n) asm volatile("s_waitcnt vmcnt(%0)" : : "n"(n) : "memory");
    // pins the software pipeline: the compiler's scheduler, left alone, sinks every LDS read down to
    // its first use
#define NVFP4_MXD_FENCE __builtin_amdgcn_sched_barrier(0);

    Frags F0, F1;
    Scales S, R;
    // ten loads per batch, three batches: scale group 0 rides with tile 0 (eleven loads)
    dma_scales(0, 0);
    dma_scales(0, 1);
    dma_codes(0);
    dma_scale_slab(0, true);
    dma_codes(1);
    dma_filler();
    dma_scale_slab(1, true);
    dma_codes(2);
    dma_filler();
    dma_scale_slab(2, true);
    NVFP4_MXD_WAIT(2 * PER_TILE)  // batch 0 has landed
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        load_frag(0, 0, F0, i);
        load_scale(0, R, i);
    }

    // K tile kt (stage kt % 4).  With one wave per SIMD nothing hides an instruction that takes long
    // to issue, so exactly one LDS read or one load follows each MFMA and issues in its shadow
    // (scheduling fences pin that order).  Step 0 multiplies while step 1's fragments are read
    // and the codes of tile kt + 3 are requested (into the stage tile kt - 1 occupied: every wave
    // finished reading it before the barrier it passed during tile kt - 1), then one half of the
    // next scale group (tiles 0 and 1 of a group) or a filler.  This wave's loads of tile kt + 1
    // (issued two tiles ago; the two newest batches stay in flight) are waited for, ONE barrier,
    // and step 1 multiplies while the first fragments and the scales of tile kt + 1 are read.
    // Every tile runs the same code: past the end the loads become one-request fillers (lane
    // offsets masked to zero, landing in the free stage) that keep the counted wait exact, and
    // the barrier / reads of the tile after the last one are harmless.
    for (int kt = 0; kt < nkt; ++kt) {
        const bool more = kt + 3 < nkt;
        const uint32_t lanes = more ? ~0u : 0u;
        const uint32_t dst3 = code_dst + (uint32_t)((kt + 3) & (NS - 1)) * STAGE;
        const uint8_t *pa = uniform_ptr(more ? tileA + (kt + 3) * stepA : tileA);
        const uint8_t *pb = uniform_ptr(more ? tileB + (kt + 3) * stepB : tileA);
        shift_scales(R, S);
        NVFP4_MXD_FENCE
        // step 0: MFMAs 0-7 each shadow one fragment read of step 1 (B fragments first: every row of
        // MFMAs needs all four), MFMAs 8-15 each shadow one load of tile kt + 3; by the barrier the
        // reads of this stage are long complete
        {
            const uint8_t *p = lds + (kt & (NS - 1)) * STAGE + (((2 * g + 1) ^ sw) << 4);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                NVFP4_MXD_MMA(F0, S, 0, j >> 2, j & 3)
                if (j < 4)
                    F1.b[j] = *reinterpret_cast<const uint4 *>(p + rdB + 32 * j * ROWB);
                else if (j < 8)
                    F1.a[j - 4] = *reinterpret_cast<const uint4 *>(p + rdA + 32 * (j - 4) * ROWB);
                else if (j & 1)
                    dma16(dst3 + BM * ROWB + ((j - 8) >> 1) * 1024, offB[(j - 8) >> 1] & lanes, pb);
                else
                    dma16(dst3 + ((j - 8) >> 1) * 1024, offA[(j - 8) >> 1] & lanes, pa);
                NVFP4_MXD_FENCE
            }
        }
        {
            // slot of the row-major scale groups: halves of the next group ride with tiles 0 and 1 of this one
            const int Gn = (kt >> 2) + 1, part = kt & 1;
            const bool real = (kt & 3) < 2 && 4 * Gn < nkt && !(part ? B_SLAB : A_SLAB);
            const uint8_t *base = real ? (part ? tileSB : tileSA) + group_start(Gn) : tileA;
            dma16(real ? scale_dst + (Gn & 1) * SBUF + part * (BM * 16) : dump_dst, real ? (part ? offSB : offSA) : 0u, uniform_ptr(base));
            // slot of the scale slabs: those of tile kt + 3, next to its codes
            dma_scale_slab(kt + 3, more);
        }
        NVFP4_MXD_WAIT(2 * PER_TILE)
        __syncthreads();
        NVFP4_MXD_FENCE
        // step 1: MFMAs 0-7 shadow the scale reads of tile kt + 1, MFMAs 8-15 its first fragments
        {
            const uint8_t *p = lds + ((kt + 1) & (NS - 1)) * STAGE + (((2 * g) ^ sw) << 4);
            const uint8_t *qa = lds + tile_off(A_SLAB, kt + 1) + rdS, *qb = lds + tile_off(B_SLAB, kt + 1) + rdT;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                NVFP4_MXD_MMA(F1, S, 1, j >> 2, j & 3)
                if (j < 4)
                    R.a[j] = *reinterpret_cast<const uint32_t *>(qa + frag_off(A_SLAB, j));
                else if (j < 8)
                    R.b[j - 4] = *reinterpret_cast<const uint32_t *>(qb + frag_off(B_SLAB, j - 4));
                else if (j < 12)
                    F0.b[j - 8] = *reinterpret_cast<const uint4 *>(p + rdB + 32 * (j - 8) * ROWB);
                else
                    F0.a[j - 12] = *reinterpret_cast<const uint4 *>(p + rdA + 32 * (j - 12) * ROWB);
                NVFP4_MXD_FENCE
            }
        }
    }
#undef NVFP4_MXD_FENCE
#undef NVFP4_MXD_WAIT
#undef NVFP4_MXD_MMA

    // every load of every wave has landed and every fragment has been read: stage 0 is free for
    // the epilogue's line buffers
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    mx_store_tile<OUT_DT>(P, acc, m0, n0, lane, wave, lds);
}

template <int OUT_DT, bool A_SLAB, bool B_SLAB>
static void launch_mx_dma_as(const GemmArgs &P, hipStream_t st)
{
    const unsigned ntiles = (unsigned)(((P.N + mx::BN - 1) / mx::BN) * ((P.M + mx::BM - 1) / mx::BM));
    auto k = gemm_nt_mxfp4_dma_kernel<OUT_DT, A_SLAB, B_SLAB>;
    static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, mxd::LDS_BYTES), true);
    (void)once;
    hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), mxd::LDS_BYTES, st, P);
}

template <int OUT_DT>
static void launch_mx_dma_out(const GemmArgs &P, hipStream_t st)
{
    if (P.a_slab && P.b_slab) launch_mx_dma_as<OUT_DT, true, true>(P, st);
    else if (P.a_slab) launch_mx_dma_as<OUT_DT, true, false>(P, st);
    else if (P.b_slab) launch_mx_dma_as<OUT_DT, false, true>(P, st);
    else launch_mx_dma_as<OUT_DT, false, false>(P, st);
}

static void launch_mx_dma(const GemmArgs &P, int out_dt, hipStream_t st)
{
    if (out_dt == NVFP4_F32)
        launch_mx_dma_out<NVFP4_F32>(P, st);
    else
        launch_mx_dma_out<NVFP4_BF16>(P, st);
}

static void launch_mx_fallback(const GemmArgs &P, int out_dt, hipStream_t st)
{
    const unsigned ntiles = (unsigned)(((P.N + mx::BN - 1) / mx::BN) * ((P.M + mx::BM - 1) / mx::BM));
    if (out_dt == NVFP4_F32) {
        auto k = gemm_nt_mxfp4_kernel<NVFP4_F32>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, mxf::LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), mxf::LDS_BYTES, st, P);
    } else {
        auto k = gemm_nt_mxfp4_kernel<NVFP4_BF16>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, mxf::LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), mxf::LDS_BYTES, st, P);
    }
}

template <int B>
static void launch_rescale(const GemmArgs &P, int out_dt, hipStream_t st)
{
    const unsigned ntiles = (unsigned)(((P.N + mx::BN - 1) / mx::BN) * ((P.M + mx::BM - 1) / mx::BM));
    if (out_dt == NVFP4_F32) {
        auto k = gemm_nt_fp4_rescale_kernel<NVFP4_F32, B>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, mxr::LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), mxr::LDS_BYTES, st, P);
    } else {
        auto k = gemm_nt_fp4_rescale_kernel<NVFP4_BF16, B>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, mxr::LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), mxr::LDS_BYTES, st, P);
    }
}

// E4M3 scales at blocks of 64 / 128 on the FP4 matrix instruction with binary32 rescaling of the block sums.
bool fp4_rescale_gemm_applies(int64_t K, int block, const GemmArgs &P)
{
    const uintptr_t codes = reinterpret_cast<uintptr_t>(P.A_codes) | reinterpret_cast<uintptr_t>(P.B_codes);
    return (block == 64 || block == 128) && K % 128 == 0 && (codes & 15) == 0 && !P.a_slab && !P.b_slab;
}

hipError_t launch_gemm_fp4_rescale(const GemmArgs &P, int block, int out_dt, hipStream_t st)
{
    if (block == 64)
        launch_rescale<64>(P, out_dt, st);
    else
        launch_rescale<128>(P, out_dt, st);
    return hipGetLastError();
}

// The shapes the direct-to-LDS kernel serves (given 16-byte aligned codes and 4-byte aligned scales); it is also the
// kernel that can read the codes of an operand from slabs.
bool mxfp4_gemm_takes_slabs(int64_t K)
{
    // lane offsets of the direct-to-LDS loads are 32-bit and relative to the tile's first row
    const bool offsets_fit = (K >> 1) * 256 < ((int64_t)1 << 31);
    return K % 128 == 0 && K >= 512 && offsets_fit;
}

hipError_t launch_gemm_mxfp4(const GemmArgs &P, int out_dt, hipStream_t st)
{
    const uintptr_t codes = reinterpret_cast<uintptr_t>(P.A_codes) | reinterpret_cast<uintptr_t>(P.B_codes);
    const uintptr_t scales = reinterpret_cast<uintptr_t>(P.A_scales) | reinterpret_cast<uintptr_t>(P.B_scales);
    if (mxfp4_gemm_takes_slabs(P.K) && (codes & 15) == 0 && (scales & 3) == 0)
        launch_mx_dma(P, out_dt, st);
    else if (P.a_slab || P.b_slab)
        return hipErrorInvalidValue;  // (the fallback kernel reads row-major operands only)
    else
        launch_mx_fallback(P, out_dt, st);
    return hipGetLastError();
}

}  // namespace nvfp4
