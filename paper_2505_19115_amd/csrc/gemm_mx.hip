// MXFP4 GEMM on the CDNA4 scaled FP4 MFMA ("NT": both operands stored with the contraction
// axis contiguous).  MXFP4 (Sec. 3 / Table 1 of "FP4 All the Way": E2M1 elements, blocks of 32,
// E8M0 power-of-two scales) is exactly what v_mfma_scale_f32_32x32x64_f8f6f4 consumes: each
// lane supplies 32 consecutive contraction elements (16 bytes of packed codes) of one row plus
// one E8M0 byte for them, so the packed operands go from LDS straight into the instruction with
// no expansion arithmetic at all:
//     out[i, j] = gA gB sum_b 2^(eA[i,b] - 127) 2^(eB[j,b] - 127) sum_{k in b} cA[i,k] cB[j,k].
// Products and the power-of-two scaling are exact; accumulation is fp32.
//
// Geometry: 256 threads = 2 x 2 waves, wave tile 128 x 128 (4 x 4 MFMA tiles, 256 accumulator
// registers, one wave per SIMD), workgroup tile 256 x 256.  With no VALU work in the loop the
// single-wave issue limit does not matter; what matters is LDS bandwidth (a 4 x 4 register tile
// reads 8 KB per 16 MFMAs = 128 B/clk/CU at full MFMA rate, the LDS peak), hence the largest
// register tile that fits.
#include "kernels.h"
#include "nvfp4_math.h"

namespace nvfp4 {

typedef int int8v_t __attribute__((ext_vector_type(8)));
typedef float float16v_t __attribute__((ext_vector_type(16)));

namespace mx {
constexpr int NT = 256, BM = 256, BN = 256, TA = 4, TB = 4;
}

__device__ __forceinline__ uint16_t mx_bf16_rne(float f)
{
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// KT = contraction elements per LDS stage (256: four MFMA steps per barrier; 64: one step, any
// K that is a multiple of 32, chunks past K are zero-filled).
// LDS stage: codes [BM + BN rows][KT/2 bytes], 16-byte chunk c of row r at slot c ^ (r & (NCH-1))
// (8 consecutive rows reading one logical chunk hit 8 different 16-byte bank groups); scales as
// dwords [2 lane halves][BM + BN rows], byte s of a dword = the E8M0 byte of MFMA step s for that
// lane half, so the instruction's byte select is a compile-time constant.
template <int KT, int OUT_DT>
__global__ __launch_bounds__(256) void gemm_nt_mxfp4_kernel(GemmArgs P)
{
    using namespace mx;
    constexpr int ROWB = KT / 2;          // code bytes per row per stage
    constexpr int NCH = ROWB / 16;        // 16-byte chunks per row (8 or 2)
    constexpr int STEPS = KT / 64;        // MFMA steps per stage (4 or 1)
    constexpr int CPT = (BM * NCH) / NT;  // chunks per thread per operand (8 or 2)
    constexpr int CODES = (BM + BN) * ROWB;
    constexpr int STAGE = CODES + 2 * (BM + BN) * 4;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r = lane & 31, g = lane >> 5;
    const int ntx = (int)((P.N + BN - 1) / BN), nty = (int)((P.M + BM - 1) / BM);
    int ty, tx;
    tile_coords(blockIdx.x, ntx, nty, ty, tx);
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

    // ---- global -> registers -> LDS.  Rows past the edge are clamped to the last row (their
    // products land in outputs that are never stored).
    // KT = 256: the codes go from global memory straight into LDS (global_load_lds, 16 bytes per
    // lane): a wave instruction fills 1 KB = 8 consecutive tile rows, lane i landing at byte 16 i,
    // so the XOR swizzle is applied by choosing WHICH global chunk lane i fetches.  No staging
    // registers, no LDS store instructions.  KT = 64 stages through registers (it must be able
    // to zero-fill past K).
    constexpr bool DMA = KT == 256;
    uint4 ga[DMA ? 1 : CPT], gb[DMA ? 1 : CPT];
    uint64_t gsa = 0, gsb = 0;
    uint32_t offA[CPT], offB[CPT];
    int ldsW[CPT];
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
        int row, c;
        if (DMA) {
            row = (wave * CPT + u) * 8 + (lane >> 3);
            c = (lane & 7) ^ (row & 7);
            ldsW[u] = (wave * CPT + u) * 1024;  // wave-uniform base of this instruction's 1 KB
        } else {
            const int qd = tid + NT * u;
            row = qd / NCH;
            c = qd % NCH;
            ldsW[u] = row * ROWB + ((c ^ (row & (NCH - 1))) << 4);
        }
        const int64_t ar = m0 + row < P.M ? m0 + row : P.M - 1;
        const int64_t br = n0 + row < P.N ? n0 + row : P.N - 1;
        offA[u] = (uint32_t)(ar * Kb + c * 16);
        offB[u] = (uint32_t)(br * Kb + c * 16);
    }
    typedef __attribute__((address_space(3))) void *lds_ptr_t;
    typedef const __attribute__((address_space(1))) void *glb_ptr_t;
    // wave-uniform 64-bit value -> scalar registers (keeps "uniform base + 32-bit lane offset"
    // addressing instead of one 64-bit vector pointer per load)
    auto uniform_ptr = [](const uint8_t *p) -> const uint8_t * {
        const uint64_t v = reinterpret_cast<uint64_t>(p);
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
    };
    // The loads are issued through inline assembly on purpose: the compiler's wait-count pass
    // treats a direct-to-LDS load as a possible writer of every LDS location and would put
    // s_waitcnt vmcnt(0) in front of the next LDS read, i.e. expose the full global latency once
    // per tile.  Here the destination stage is never read before the explicit wait + barrier below.
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    const uint32_t dma_base = __builtin_amdgcn_readfirstlane(lds0 + wave * CPT * 1024);
    auto dma_one = [&](uint32_t lds_addr, uint32_t voff, const uint8_t *base) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :
                     : "s"(lds_addr), "v"(voff), "s"(base)
                     : "memory");
    };
    auto dma_codes = [&](int kt, int stage) {
        const uint8_t *pa = uniform_ptr(P.A_codes + (int64_t)kt * ROWB);
        const uint8_t *pb = uniform_ptr(P.B_codes + (int64_t)kt * ROWB);
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const uint32_t dst = dma_base + stage * STAGE + u * 1024;
            dma_one(dst, offA[u], pa);
            dma_one(dst + BM * ROWB, offB[u], pb);
        }
    };
    const int64_t sar = m0 + tid < P.M ? m0 + tid : P.M - 1;
    const int64_t sbr = n0 + tid < P.N ? n0 + tid : P.N - 1;
    auto fetch = [&](int kt) {
        const int64_t kb = (int64_t)kt * ROWB;
        if (!DMA) {
#pragma unroll
            for (int u = 0; u < CPT; ++u) {
                const bool in = kb + ((tid + NT * u) % NCH) * 16 < Kb;  // zero codes past K
                ga[u] = in ? *reinterpret_cast<const uint4 *>(P.A_codes + kb + offA[u]) : make_uint4(0, 0, 0, 0);
                gb[u] = in ? *reinterpret_cast<const uint4 *>(P.B_codes + kb + offB[u]) : make_uint4(0, 0, 0, 0);
            }
        }
        const uint8_t *pa = P.A_scales + sar * Ks + (int64_t)kt * (KT / 32);
        const uint8_t *pb = P.B_scales + sbr * Ks + (int64_t)kt * (KT / 32);
        if (KT == 256) {
            gsa = *reinterpret_cast<const uint64_t *>(pa);
            gsb = *reinterpret_cast<const uint64_t *>(pb);
        } else {
            const bool two = (int64_t)kt * 2 + 1 < Ks;
            gsa = (uint64_t)pa[0] | (two ? (uint64_t)pa[1] << 8 : 0);
            gsb = (uint64_t)pb[0] | (two ? (uint64_t)pb[1] << 8 : 0);
        }
    };
    // scale bytes of a row, in block order b0 b1 ... -> dword of lane half 0 (blocks 0, 2, 4, 6)
    // and dword of lane half 1 (blocks 1, 3, 5, 7)
    auto split_scales = [&](uint64_t s, uint32_t &even, uint32_t &odd) {
        const uint32_t lo = (uint32_t)s, hi = (uint32_t)(s >> 32);
        even = __builtin_amdgcn_perm(hi, lo, 0x06040200u);
        odd = __builtin_amdgcn_perm(hi, lo, 0x07050301u);
    };
    auto stash = [&](int stage) {
        uint8_t *base = lds + stage * STAGE;
        if (!DMA) {
#pragma unroll
            for (int u = 0; u < CPT; ++u) {
                *reinterpret_cast<uint4 *>(base + ldsW[u]) = ga[u];
                *reinterpret_cast<uint4 *>(base + BM * ROWB + ldsW[u]) = gb[u];
            }
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's direct-to-LDS loads have landed
        }
        uint32_t *sS = reinterpret_cast<uint32_t *>(base + CODES);
        uint32_t e, o;
        split_scales(gsa, e, o);
        sS[tid] = e;
        sS[(BM + BN) + tid] = o;
        split_scales(gsb, e, o);
        sS[BM + tid] = e;
        sS[(BM + BN) + BM + tid] = o;
    };

    // ---- LDS -> registers
    struct Frags {
        uint4 a[TA], b[TB];
    };
    struct Scales {
        uint32_t a[TA], b[TB];
    };
    int rd[STEPS];  // byte offset of this lane's chunk of MFMA step s inside its row
#pragma unroll
    for (int s = 0; s < STEPS; ++s) rd[s] = r * ROWB + (((2 * s + g) ^ (r & (NCH - 1))) << 4);
    auto load_frags = [&](int stage, int s, Frags &F) {
        const uint8_t *p = lds + stage * STAGE + rd[s];
#pragma unroll
        for (int a = 0; a < TA; ++a) F.a[a] = *reinterpret_cast<const uint4 *>(p + (wm * 128 + 32 * a) * ROWB);
#pragma unroll
        for (int b = 0; b < TB; ++b) F.b[b] = *reinterpret_cast<const uint4 *>(p + (BM + wn * 128 + 32 * b) * ROWB);
    };
    auto load_scales = [&](int stage, Scales &S) {
        const uint32_t *p = reinterpret_cast<const uint32_t *>(lds + stage * STAGE + CODES) + g * (BM + BN) + r;
#pragma unroll
        for (int a = 0; a < TA; ++a) S.a[a] = p[wm * 128 + 32 * a];
#pragma unroll
        for (int b = 0; b < TB; ++b) S.b[b] = p[BM + wn * 128 + 32 * b];
    };
#define NVFP4_MX_MMA(F, S, s)                                                                              \
    _Pragma("unroll") for (int a = 0; a < TA; ++a) _Pragma("unroll") for (int b = 0; b < TB; ++b)          \
    {                                                                                                      \
        const int8v_t va = {(int)F.a[a].x, (int)F.a[a].y, (int)F.a[a].z, (int)F.a[a].w, 0, 0, 0, 0};       \
        const int8v_t vb = {(int)F.b[b].x, (int)F.b[b].y, (int)F.b[b].z, (int)F.b[b].w, 0, 0, 0, 0};       \
        acc[a][b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vb, acc[a][b], 4, 4, s, (int)S.a[a], s, \
                                                                    (int)S.b[b]);                          \
    }

    Frags F0, F1;
    Scales S0, S1;
    if (DMA) dma_codes(0, 0);
    fetch(0);
    stash(0);
    __syncthreads();
    load_frags(0, 0, F0);
    load_scales(0, S0);

    // One K tile: steps 0..STEPS-1 multiply while the fragments of the next step are read; the
    // next tile goes to the other LDS stage before the last step, ONE barrier, and the first
    // fragments / scales of the next tile are already in flight during the last step.
    // Sc = scales of this tile, Sn = registers for the next tile's.
    // The compiler's scheduler, left alone, sinks every LDS read down to its first use (and the
    // scale loads down to the wait), which exposes the LDS latency once per four MFMAs.  Fences
    // pin the software pipeline; inside a step the eight fragment reads of the NEXT step are
    // spread between the sixteen MFMAs of this one.
#define NVFP4_MX_FENCE __builtin_amdgcn_sched_barrier(0);
#define NVFP4_MX_MIX                                            \
    _Pragma("unroll") for (int i_ = 0; i_ < 8; ++i_)            \
    {                                                           \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);      \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      \
    }
#define NVFP4_MX_TILE(stage, kt, more, Sc, Sn)                  \
    {                                                           \
        if (more) {                                             \
            if (DMA) dma_codes((kt) + 1, (stage) ^ 1);          \
            fetch((kt) + 1);                                    \
        }                                                       \
        NVFP4_MX_FENCE                                          \
        if (STEPS == 4) {                                       \
            load_frags(stage, 1, F1);                           \
            NVFP4_MX_MMA(F0, Sc, 0)                             \
            NVFP4_MX_MIX                                        \
            NVFP4_MX_FENCE                                      \
            load_frags(stage, 2, F0);                           \
            NVFP4_MX_MMA(F1, Sc, 1)                             \
            NVFP4_MX_MIX                                        \
            NVFP4_MX_FENCE                                      \
            load_frags(stage, 3, F1);                           \
            NVFP4_MX_MMA(F0, Sc, 2)                             \
            NVFP4_MX_MIX                                        \
            NVFP4_MX_FENCE                                      \
            if (more) {                                         \
                stash((stage) ^ 1);                             \
                __syncthreads();                                \
                NVFP4_MX_FENCE                                  \
                load_frags((stage) ^ 1, 0, F0);                 \
                load_scales((stage) ^ 1, Sn);                   \
                NVFP4_MX_FENCE                                  \
            }                                                   \
            NVFP4_MX_MMA(F1, Sc, 3)                             \
            NVFP4_MX_FENCE                                      \
        } else {                                                \
            if (more) stash((stage) ^ 1);                       \
            NVFP4_MX_MMA(F0, Sc, 0)                             \
            if (more) {                                         \
                __syncthreads();                                \
                load_frags((stage) ^ 1, 0, F0);                 \
                load_scales((stage) ^ 1, Sn);                   \
            }                                                   \
        }                                                       \
    }
    int kt = 0;
    for (; kt + 2 < nkt; kt += 2) {
        NVFP4_MX_TILE(0, kt, true, S0, S1)
        NVFP4_MX_TILE(1, kt + 1, true, S1, S0)
    }
    if (kt + 1 < nkt) {
        NVFP4_MX_TILE(0, kt, true, S0, S1)
        ++kt;
        NVFP4_MX_TILE(1, kt, false, S1, S0)
    } else {
        NVFP4_MX_TILE(0, kt, false, S0, S1)
    }
#undef NVFP4_MX_TILE
#undef NVFP4_MX_MIX
#undef NVFP4_MX_FENCE
#undef NVFP4_MX_MMA

    // epilogue: accumulator register v of lane (r, g) is row 8 (v / 4) + 4 g + v % 4, column r
    // The lane coordinates are re-derived from an opaque copy so that none of the output
    // addressing is computed before the K loop and kept in registers across it.
    int lane_e = lane, wave_e = wave;
    asm volatile("" : "+v"(lane_e), "+v"(wave_e));
    const int re = lane_e & 31, ge = lane_e >> 5, wme = wave_e >> 1, wne = wave_e & 1;
    const float gg = P.tensor_scales[0] * P.tensor_scales[1];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            const int64_t col = n0 + wne * 128 + 32 * b + re;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t row = m0 + wme * 128 + 32 * a + 8 * (v >> 2) + 4 * ge + (v & 3);
                if (row < P.M && col < P.N) {
                    const float y = acc[a][b][v] * gg;
                    if (OUT_DT == NVFP4_F32)
                        reinterpret_cast<float *>(P.out)[row * P.ldc + col] = y;
                    else
                        reinterpret_cast<uint16_t *>(P.out)[row * P.ldc + col] = mx_bf16_rne(y);
                }
            }
            __builtin_amdgcn_sched_barrier(0);  // one accumulator tile at a time: keeps the register peak low
        }
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
// The MFMA's first operand is the B (N-side) tile, so a lane's accumulator holds four consecutive
// output COLUMNS of one row: the epilogue is one packed convert pair and one 8-byte (bf16) or
// 16-byte (fp32) store per four outputs.
namespace mxd {
constexpr int KT = 128, ROWB = 64, NS = 4;
constexpr int STAGE = (mx::BM + mx::BN) * ROWB;        // 32 KB of codes
constexpr int SBUF = (mx::BM + mx::BN) * 16;           // 8 KB: the scales of four K tiles
constexpr int SCALES0 = NS * STAGE, DUMP0 = SCALES0 + 2 * SBUF;
constexpr int LDS_BYTES = DUMP0 + 4096;
constexpr int PER_TILE = 9;  // direct-to-LDS instructions per wave per K tile: 4 + 4 codes, 1 scales or filler
}  // namespace mxd

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2v_t __attribute__((ext_vector_type(2)));

template <int OUT_DT>
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
        offA[u] = (uint32_t)((row < mrows ? row : mrows - 1) * Kb + c * 16);
        offB[u] = (uint32_t)((row < nrows ? row : nrows - 1) * Kb + c * 16);
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
    const uint8_t *tileA = P.A_codes + m0 * Kb, *tileB = P.B_codes + n0 * Kb;
    const uint8_t *tileSA = P.A_scales + m0 * Ks, *tileSB = P.B_scales + n0 * Ks;
    auto dma_codes = [&](int kt) {
        const uint32_t st = (uint32_t)(kt & (NS - 1)) * STAGE;
        const uint8_t *pa = uniform_ptr(tileA + (int64_t)kt * ROWB), *pb = uniform_ptr(tileB + (int64_t)kt * ROWB);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            dma16(code_dst + st + u * 1024, offA[u], pa);
            dma16(code_dst + st + BM * ROWB + u * 1024, offB[u], pb);
        }
    };
    // Scale group G = the 16 scale bytes of a row that cover K tiles 4 G .. 4 G + 3; the window of the
    // last group is moved back to end with the row (Ks >= 16), so no load passes the end of a row.
    auto group_start = [&](int G) -> int { return 16 * G + 16 <= Ks ? 16 * G : (int)Ks - 16; };
    // part 0: this wave's 64 A rows, part 1: its 64 B rows
    auto dma_scales = [&](int G, int part) {
        const uint8_t *base = (part ? tileSB : tileSA) + group_start(G);
        dma16(scale_dst + (G & 1) * SBUF + part * (BM * 16), part ? offSB : offSA, uniform_ptr(base));
    };
    // keeps the number of loads per tile constant (the counted waits rely on it): one request, lands in the dump
    auto dma_filler = [&]() { dma16(dump_dst, 0u, uniform_ptr(tileSA)); };

    // ---- LDS -> registers
    struct Frags {
        uint4 a[TA], b[TB];
    };
    struct Scales {
        uint32_t a[TA], b[TB];
    };
    const int sw = (r >> 2) & 3;
    const int rdA = (wm * 128 + r) * ROWB, rdB = (BM + wn * 128 + r) * ROWB;
    const int rdS = SCALES0 + (wm * 128 + r) * 16, rdT = SCALES0 + (BM + wn * 128 + r) * 16;
    const int sh = 16 * g;
    // fragment i of both operands (rows 32 i + r of the wave's A and B parts) for MFMA step s of tile kt
    auto load_frag = [&](int kt, int s, Frags &F, int i) {
        const uint8_t *p = lds + (kt & (NS - 1)) * STAGE + (((2 * g + s) ^ sw) << 4);
        F.a[i] = *reinterpret_cast<const uint4 *>(p + rdA + 32 * i * ROWB);
        F.b[i] = *reinterpret_cast<const uint4 *>(p + rdB + 32 * i * ROWB);
    };
    // raw scale dwords of a tile (all four E8M0 bytes of the row); shifted into place when the tile starts
    auto load_scale = [&](int kt, Scales &R, int i) {
        const int G = kt >> 2;
        const uint8_t *p = lds + (G & 1) * SBUF + (4 * kt - group_start(G));
        R.a[i] = *reinterpret_cast<const uint32_t *>(p + rdS + 512 * i);
        R.b[i] = *reinterpret_cast<const uint32_t *>(p + rdT + 512 * i);
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
    // nine loads per batch, three batches: scale group 0 rides with tile 0
    dma_scales(0, 0);
    dma_scales(0, 1);
    dma_codes(0);
    dma_codes(1);
    dma_filler();
    dma_codes(2);
    dma_filler();
    NVFP4_MXD_WAIT(2 * PER_TILE)  // batch 0 (ten loads) has landed
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
        const uint8_t *pa = uniform_ptr(more ? tileA + (int64_t)(kt + 3) * ROWB : tileSA);
        const uint8_t *pb = uniform_ptr(more ? tileB + (int64_t)(kt + 3) * ROWB : tileSA);
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
            const int Gn = (kt >> 2) + 1, part = kt & 1;
            const bool real = (kt & 3) < 2 && 4 * Gn < nkt;
            const uint8_t *base = real ? (part ? tileSB : tileSA) + group_start(Gn) : tileSA;
            dma16(real ? scale_dst + (Gn & 1) * SBUF + part * (BM * 16) : dump_dst, real ? (part ? offSB : offSA) : 0u, uniform_ptr(base));
        }
        NVFP4_MXD_WAIT(2 * PER_TILE)
        __syncthreads();
        NVFP4_MXD_FENCE
        // step 1: MFMAs 0-7 shadow the scale reads of tile kt + 1, MFMAs 8-15 its first fragments
        {
            const uint8_t *p = lds + ((kt + 1) & (NS - 1)) * STAGE + (((2 * g) ^ sw) << 4);
            const int G = (kt + 1) >> 2;
            const uint8_t *q = lds + (G & 1) * SBUF + (4 * (kt + 1) - group_start(G));
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                NVFP4_MXD_MMA(F1, S, 1, j >> 2, j & 3)
                if (j < 4)
                    R.a[j] = *reinterpret_cast<const uint32_t *>(q + rdS + 512 * j);
                else if (j < 8)
                    R.b[j - 4] = *reinterpret_cast<const uint32_t *>(q + rdT + 512 * (j - 4));
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

    // ---- epilogue: accumulator register v of lane (r, g) of tile (a, b) is output row 32 a + r,
    // column 32 b + 8 (v / 4) + 4 g + v % 4.  The lane coordinates are re-derived from an opaque
    // copy so that none of the output addressing is computed before the K loop and kept in
    // registers across it.
    int lane_e = lane, wave_e = wave;
    asm volatile("" : "+v"(lane_e), "+v"(wave_e));
    const int re = lane_e & 31, ge = lane_e >> 5, wme = wave_e >> 1, wne = wave_e & 1;
    const float gg = P.tensor_scales[0] * P.tensor_scales[1];
    constexpr int ESZ = OUT_DT == NVFP4_F32 ? 4 : 2;
    const int64_t row0 = m0 + wme * 128 + re, col0 = n0 + wne * 128 + 4 * ge;
    uint8_t *const out = reinterpret_cast<uint8_t *>(P.out);
    const bool fast = m0 + BM <= P.M && n0 + BN <= P.N && (P.ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(P.out) & 15) == 0;
    if (fast) {
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

static void launch_mx_dma(const GemmArgs &P, int out_dt, hipStream_t st)
{
    const unsigned ntiles = (unsigned)(((P.N + mx::BN - 1) / mx::BN) * ((P.M + mx::BM - 1) / mx::BM));
    if (out_dt == NVFP4_F32) {
        auto k = gemm_nt_mxfp4_dma_kernel<NVFP4_F32>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, mxd::LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), mxd::LDS_BYTES, st, P);
    } else {
        auto k = gemm_nt_mxfp4_dma_kernel<NVFP4_BF16>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, mxd::LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), mxd::LDS_BYTES, st, P);
    }
}

template <int KT>
static void launch_mx(const GemmArgs &P, int out_dt, hipStream_t st)
{
    constexpr int LDS_BYTES = 2 * ((mx::BM + mx::BN) * (KT / 2) + 2 * (mx::BM + mx::BN) * 4);
    const unsigned ntiles = (unsigned)(((P.N + mx::BN - 1) / mx::BN) * ((P.M + mx::BM - 1) / mx::BM));
    if (out_dt == NVFP4_F32) {
        auto k = gemm_nt_mxfp4_kernel<KT, NVFP4_F32>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), LDS_BYTES, st, P);
    } else {
        auto k = gemm_nt_mxfp4_kernel<KT, NVFP4_BF16>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(256), LDS_BYTES, st, P);
    }
}

hipError_t launch_gemm_mxfp4(const GemmArgs &P, int out_dt, hipStream_t st)
{
    const uintptr_t codes = reinterpret_cast<uintptr_t>(P.A_codes) | reinterpret_cast<uintptr_t>(P.B_codes);
    const uintptr_t scales = reinterpret_cast<uintptr_t>(P.A_scales) | reinterpret_cast<uintptr_t>(P.B_scales);
    // lane offsets of the direct-to-LDS loads are 32-bit and relative to the tile's first row
    const bool offsets_fit = (P.K >> 1) * 256 < ((int64_t)1 << 31);
    if (P.K % 128 == 0 && P.K >= 512 && (codes & 15) == 0 && (scales & 3) == 0 && offsets_fit)
        launch_mx_dma(P, out_dt, st);
    else if (P.K % 256 == 0)
        launch_mx<256>(P, out_dt, st);
    else
        launch_mx<64>(P, out_dt, st);
    return hipGetLastError();
}

}  // namespace nvfp4
