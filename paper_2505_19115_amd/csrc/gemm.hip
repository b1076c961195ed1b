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
//
// Operand storage: row-major ([rows, K/2] codes, [rows, K/B] scale bytes), or, for blocks of 16 in the 256 x 256
// kernel, the slab layout of kernels.h, in which the 256 rows x 64 code bytes (and 256 x 8 scale bytes) that a
// workgroup fetches per K tile are one contiguous piece.  Only addresses differ: per-lane offsets, two base
// pointers and their step per K tile.
#include "kernels.h"
#include "nvfp4_math.h"

namespace nvfp4 {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float float2v_t __attribute__((ext_vector_type(2)));

constexpr int KT = 128;      // contraction elements per LDS tile
constexpr int KTB = KT / 2;  // bytes of codes per row per tile
constexpr int SROW = 16;     // LDS bytes per row for the tile's scales: 8 fp16 values, one per 16 elements

// LDS placement of the codes of one tile row r (64 bytes = 4 chunks of 16): chunk c sits in
// chunk slot c ^ ((r >> 2) & 3).  Rows are 64 bytes apart, so 16 consecutive rows reading the same
// logical chunk (one ds_read_b128 wavefront pass) cover all sixteen 16-byte slots of the 256-byte
// bank period, and a 16-byte store of a whole chunk by 4 consecutive threads per row covers
// contiguous bytes: no conflicts either way.
__device__ __forceinline__ int swz(int r, int c) { return r * KTB + ((c ^ ((r >> 2) & 3)) << 4); }

// 8 codes (one dword) of one block -> 8 fp16 values times the block scale.
// s = fp16 holding scale * 2^-8; the convert multiplies the codes by 2^8.
__device__ __forceinline__ half8_t dequant8(uint32_t w, _Float16 s)
{
    const half2_t s2 = {s, s};
    half2_t h0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 0) * s2;
    half2_t h1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 1) * s2;
    half2_t h2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 2) * s2;
    half2_t h3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(w, 256.0f, 3) * s2;
    half8_t r;
    r[0] = h0[0]; r[1] = h0[1]; r[2] = h1[0]; r[3] = h1[1];
    r[4] = h2[0]; r[5] = h2[1]; r[6] = h3[0]; r[7] = h3[1];
    return r;
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = f2u(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Tile geometry.  A workgroup is WM x WN waves; a wave owns (32 TA) x (32 TB) outputs as
// TA x TB MFMA tiles.  The production shape is 2 x 4 waves of 4 x 2 tiles: 256 x 256 per
// workgroup, 128 accumulator registers per wave, so TWO waves fit on every SIMD.  That is
// the point of the shape: measured on gfx950, one wave alone issues a VALU instruction only
// every ~8 cycles, two waves per SIMD reach the full rate of one per 4 cycles, and the
// operand expansion costs 8 (TA + TB) / (TA TB) = 6 VALU instructions per 32-cycle MFMA.
//
// Per 128-wide K tile the 64 code bytes of each operand row sit in LDS as four 16-byte chunks
// and its 8 block scales as fp16 values (scale * 2^-8; for blocks wider than 16 the value is
// repeated).  Lane (r = lane % 32, h = lane / 32) owns chunk 2p + h (p = 0, 1) of its row:
// 32 codes = two 16-element blocks; dword t (0..3) of the chunk feeds one MFMA step and
// belongs to block t / 2.  A and B use the same assignment of contraction indices to (lane
// half, step), which is all the instruction requires.
template <int B, int WM, int WN, int TA, int TB, int OUT_DT, bool KTAIL>
__global__ __launch_bounds__(64 * WM * WN) void gemm_nt_f16_kernel(GemmArgs P)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int BM = 32 * TA * WM, BN = 32 * TB * WN;
    constexpr int SPT = KT / B;  // scale bytes per row per tile in global memory
    constexpr int VALU_PER_MFMA = (8 * (TA + TB) + TA * TB - 1) / (TA * TB);
    constexpr int A_BYTES = BM * KTB, B_BYTES = BN * KTB, SA_BYTES = BM * SROW, SB_BYTES = BN * SROW;
    constexpr int STAGE = A_BYTES + B_BYTES + SA_BYTES + SB_BYTES;
    constexpr int CA = BM * 4 / NT, CB = BN * 4 / NT;  // 16-byte chunks per thread per tile
    static_assert(BM * 4 % NT == 0 && BN * 4 % NT == 0 && BM + BN <= NT * 2, "tile/thread mismatch");
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int r = lane & 31, h = lane >> 5;
    const int ntx = (int)((P.N + BN - 1) / BN), nty = (int)((P.M + BM - 1) / BM);
    int ty, tx;
    tile_coords(blockIdx.x, ntx, nty, ty, tx);
    const int64_t m0 = (int64_t)ty * BM, n0 = (int64_t)tx * BN;
    const int64_t Kb = P.K >> 1;          // code bytes per row
    const int64_t Ks = P.K / B;           // scale bytes per row
    const int nkt = (int)((P.K + KT - 1) / KT);

    float16_t acc[TA][TB];
#pragma unroll
    for (int a = 0; a < TA; ++a)
#pragma unroll
        for (int b = 0; b < TB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // ---- global -> registers -> LDS staging of one K tile.
    // Rows past the matrix edge are clamped to the last row (their products land in outputs
    // that are never stored), so the code loads carry no predicate.  A K tail (K not a
    // multiple of 128) is handled through the scales alone: chunks past K are read from a
    // clamped address and meet zero scales.
    // Without a K tail the codes go from global memory straight into LDS (global_load_lds, 16
    // bytes per lane): a wave instruction fills 1 KB = 16 consecutive tile rows, lane i landing at
    // byte 16 i (row i / 4, slot i % 4), so the swizzle is applied by choosing WHICH global chunk
    // the lane fetches.  No staging registers, no LDS store instructions for the codes.
    constexpr bool DMA = !KTAIL;
    constexpr int NSR = (BM + BN + NT - 1) / NT;  // scale rows per thread
    uint4 ga[DMA ? 1 : CA], gb[DMA ? 1 : CB];
    uint64_t gs[NSR];
    uint32_t offA[CA], offB[CB];  // byte offset of this thread's chunks inside a K tile column
    int ldsA[CA], ldsB[CB];
#pragma unroll
    for (int u = 0; u < CA; ++u) {
        const int qd = tid + NT * u;
        const int row = DMA ? (wave * CA + u) * 16 + (lane >> 2) : qd >> 2;
        const int ch = DMA ? (lane & 3) ^ ((lane >> 4) & 3) : qd & 3;
        const int64_t lr = m0 + row < P.M ? row : P.M - 1 - m0;  // row inside the tile, clamped
        offA[u] = P.a_slab ? (uint32_t)(slab_row(row) * 64 + ch * 16)  // (a slab holds all 256 rows: nothing to clamp)
                           : (uint32_t)(lr * Kb + ch * 16);       // (relative to the tile's first row: 32 bits suffice)
        ldsA[u] = DMA ? __builtin_amdgcn_readfirstlane((wave * CA + u) * 1024) : swz(row, ch);
    }
#pragma unroll
    for (int u = 0; u < CB; ++u) {
        const int qd = tid + NT * u;
        const int row = DMA ? (wave * CB + u) * 16 + (lane >> 2) : qd >> 2;
        const int ch = DMA ? (lane & 3) ^ ((lane >> 4) & 3) : qd & 3;
        const int64_t lr = n0 + row < P.N ? row : P.N - 1 - n0;
        offB[u] = P.b_slab ? (uint32_t)(slab_row(row) * 64 + ch * 16) : (uint32_t)(lr * Kb + ch * 16);
        ldsB[u] = DMA ? __builtin_amdgcn_readfirstlane(A_BYTES + (wave * CB + u) * 1024) : A_BYTES + swz(row, ch);
    }
    typedef __attribute__((address_space(3))) void *lds_ptr_t;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_ptr_t)lds;
    // wave-uniform 64-bit value -> scalar registers
    auto uniform_ptr = [](const uint8_t *p) -> const uint8_t * {
        const uint64_t v = reinterpret_cast<uint64_t>(p);
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return reinterpret_cast<const uint8_t *>(((uint64_t)hi << 32) | lo);
    };
    // Issued through inline assembly on purpose: the compiler's wait-count pass treats a
    // direct-to-LDS load as a possible writer of every LDS location and would wait for it before
    // the next LDS read.  Here the destination stage is not read before the explicit wait and the
    // barrier in stash().
    auto dma16 = [&](uint32_t lds_addr, uint32_t voff, const uint8_t *base) {
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(voff), "s"(base) : "memory");
    };
    const uint8_t *srow_ptr[NSR];
    int srow_step[NSR];  // bytes from one K tile's scales of the row to the next
    bool srow_on[NSR];
#pragma unroll
    for (int u = 0; u < NSR; ++u) {
        const int srow = tid + NT * u;
        const bool isA = srow < BM;
        int64_t gr = isA ? m0 + srow : n0 + (srow - BM);
        const int64_t nrows = isA ? P.M : P.N;
        gr = gr < nrows ? gr : nrows - 1;
        srow_on[u] = srow < BM + BN;
        srow_ptr[u] = (isA ? P.A_scales : P.B_scales) + gr * Ks;
        srow_step[u] = SPT;
        if (DMA && (isA ? P.a_slab : P.b_slab) && srow_on[u]) {
            const int64_t tile = isA ? ty : tx;
            const int lrow = isA ? srow : srow - BM;
            srow_ptr[u] = (isA ? P.A_scales : P.B_scales) + tile * nkt * SLAB_SCALE_BYTES + slab_row(lrow) * 8;
            srow_step[u] = (int)SLAB_SCALE_BYTES;
        }
    }
    // codes of K tile kt: base + kt * step (+ the lane offsets above)
    const uint8_t *baseA = P.a_slab ? P.A_codes + (int64_t)ty * nkt * SLAB_CODE_BYTES : P.A_codes + m0 * Kb;
    const uint8_t *baseB = P.b_slab ? P.B_codes + (int64_t)tx * nkt * SLAB_CODE_BYTES : P.B_codes + n0 * Kb;
    const int64_t stepA = P.a_slab ? SLAB_CODE_BYTES : KTB, stepB = P.b_slab ? SLAB_CODE_BYTES : KTB;
    const int64_t last_chunk = Kb - 16;
    // tile kt: codes -> LDS stage `stage` (direct) or staging registers; scale bytes -> registers
    auto fetch = [&](int kt, int stage) {
        const int64_t kb = (int64_t)kt * KTB;
        const uint8_t *pa = baseA + kt * stepA, *pb = baseB + kt * stepB;
        if (!KTAIL) {
            const uint8_t *ua = uniform_ptr(pa), *ub = uniform_ptr(pb);
            const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + stage * STAGE);
#pragma unroll
            for (int u = 0; u < CA; ++u) dma16(dst + ldsA[u], offA[u], ua);
#pragma unroll
            for (int u = 0; u < CB; ++u) dma16(dst + ldsB[u], offB[u], ub);
#pragma unroll
            for (int u = 0; u < NSR; ++u) {
                if (!srow_on[u]) continue;
                const uint8_t *sp = srow_ptr[u] + (int64_t)kt * srow_step[u];
                if (SPT == 8) gs[u] = *reinterpret_cast<const uint64_t *>(sp);
                else if (SPT == 4) gs[u] = *reinterpret_cast<const uint32_t *>(sp);
                else if (SPT == 2) gs[u] = *reinterpret_cast<const uint16_t *>(sp);
                else gs[u] = *sp;
            }
        } else {
            // K tail present: clamp chunk addresses, assemble scale bytes one by one, zero past K
#pragma unroll
            for (int u = 0; u < CA; ++u) {
                const int64_t c = kb + ((tid + NT * u) & 3) * 16;
                ga[u] = *reinterpret_cast<const uint4 *>(pa + offA[u] - (c > last_chunk ? c - last_chunk : 0));
            }
#pragma unroll
            for (int u = 0; u < CB; ++u) {
                const int64_t c = kb + ((tid + NT * u) & 3) * 16;
                gb[u] = *reinterpret_cast<const uint4 *>(pb + offB[u] - (c > last_chunk ? c - last_chunk : 0));
            }
            const int64_t left = Ks - (int64_t)kt * SPT;
#pragma unroll
            for (int u = 0; u < NSR; ++u) {
                if (!srow_on[u]) continue;
                const uint8_t *sp = srow_ptr[u] + (int64_t)kt * SPT;
                uint64_t sv = 0;
#pragma unroll
                for (int t = 0; t < SPT; ++t)
                    if (t < left) sv |= (uint64_t)sp[t] << (8 * t);
                gs[u] = sv;
            }
        }
    };
    // LDS scale layout: [4 chunks of 32 elements][BM + BN rows] dwords, each dword = the fp16
    // scales (byte << 7 = fp16(scale * 2^-8), exact for normal and subnormal E4M3 bytes alike
    // because fp16's bias is E4M3's plus 8) of the chunk's two 16-element blocks; a wave reads
    // 32 consecutive rows of one chunk.  For blocks wider than 16 the value is repeated.
    auto stash = [&](int stage) {
        uint8_t *base = lds + stage * STAGE;
        if (DMA) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's direct-to-LDS loads have landed
        } else {
#pragma unroll
            for (int u = 0; u < CA; ++u) *reinterpret_cast<uint4 *>(base + ldsA[u]) = ga[u];
#pragma unroll
            for (int u = 0; u < CB; ++u) *reinterpret_cast<uint4 *>(base + ldsB[u]) = gb[u];
        }
        uint32_t *sS = reinterpret_cast<uint32_t *>(base + A_BYTES + B_BYTES);
#pragma unroll
        for (int u = 0; u < NSR; ++u) {
            if (!srow_on[u]) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                // bytes i0, i1 of the staged scale bytes -> (b0 << 7) | (b1 << 23): one byte permute
                // (b0 into byte 0, b1 into byte 2, zeros between) and one shift
                const int i0 = (32 * j) / B, i1 = (32 * j + 16) / B;  // (constants after unrolling)
                const uint32_t lo = (uint32_t)gs[u], hi = (uint32_t)(gs[u] >> 32);
                const uint32_t sel = 0x0C000C00u | (uint32_t)i0 | ((uint32_t)i1 << 16);
                sS[j * (BM + BN) + tid + NT * u] = __builtin_amdgcn_perm(hi, lo, sel) << 7;
            }
        }
    };

    // ---- LDS -> registers.  A lane reads chunk 2 p + h (16 bytes = 32 codes = two blocks of 16,
    // four MFMA steps) of rows (frag base + r): its byte offset inside a row is one of two lane
    // constants, the rest are immediates.
    struct Codes {
        uint4 ca[TA], cb[TB];
    };
    struct Scales {  // two fp16 scales (first and second block of the lane's 32-element chunk)
        uint32_t sa[TA], sb[TB];
    };
    int coff[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) coff[p] = swz(r, 2 * p + h);
    const int soff = (h * (BM + BN) + r) * 4;
    auto load_codes = [&](int stage, int p, Codes &Q) {
        const uint8_t *sA = lds + stage * STAGE + coff[p], *sB = sA + A_BYTES;
#pragma unroll
        for (int a = 0; a < TA; ++a)
            Q.ca[a] = *reinterpret_cast<const uint4 *>(sA + (wm * 32 * TA + 32 * a) * KTB);
#pragma unroll
        for (int b = 0; b < TB; ++b)
            Q.cb[b] = *reinterpret_cast<const uint4 *>(sB + (wn * 32 * TB + 32 * b) * KTB);
    };
    auto load_scales = [&](int stage, int p, Scales &S) {
        const uint8_t *sS = lds + stage * STAGE + A_BYTES + B_BYTES + soff + 2 * p * (BM + BN) * 4;
#pragma unroll
        for (int a = 0; a < TA; ++a) S.sa[a] = *reinterpret_cast<const uint32_t *>(sS + (wm * 32 * TA + 32 * a) * 4);
#pragma unroll
        for (int b = 0; b < TB; ++b) S.sb[b] = *reinterpret_cast<const uint32_t *>(sS + (BM + wn * 32 * TB + 32 * b) * 4);
    };
    struct Frags {
        half8_t a[TA], b[TB];
    };
    // operands of MFMA step t (0..3) of a chunk: its dword t, scaled by the scale of the block
    // (t / 2) that dword belongs to
    auto expand = [&](const Codes &Q, const Scales &S, int t, Frags &F) {
        auto dword = [&](const uint4 &v) { return t == 0 ? v.x : t == 1 ? v.y : t == 2 ? v.z : v.w; };
#pragma unroll
        for (int a = 0; a < TA; ++a) {
            const half2_t sp = __builtin_bit_cast(half2_t, S.sa[a]);
            F.a[a] = dequant8(dword(Q.ca[a]), t >= 2 ? sp[1] : sp[0]);
        }
#pragma unroll
        for (int b = 0; b < TB; ++b) {
            const half2_t sp = __builtin_bit_cast(half2_t, S.sb[b]);
            F.b[b] = dequant8(dword(Q.cb[b]), t >= 2 ? sp[1] : sp[0]);
        }
    };
    auto mma = [&](const Frags &F) {
#pragma unroll
        for (int a = 0; a < TA; ++a)
#pragma unroll
            for (int b = 0; b < TB; ++b)
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(F.b[b], F.a[a], acc[a][b], 0, 0, 0);
    };

    // Software pipeline, continuous across K tiles (8 MFMA steps of TA*TB MFMAs per tile; the
    // operands of step s+1 are expanded under the MFMAs of step s).  On entry to iteration kt
    // the LDS stage kt & 1 holds tile kt; Ca holds the lanes' chunk of its first half, S0 the
    // scales of that half, F0 the operands of its first step.  Within the iteration:
    //   top      global loads of tile kt+1 -> registers; LDS loads of the second half (Cb, S1)
    //   step 6   tile kt+1 -> other LDS stage, ONE barrier, LDS loads of its first half
    //   step 7   already expands the first operands of tile kt+1.
    // After the barrier nobody reads stage kt & 1 again (both halves are in registers), so the
    // next iteration may overwrite it.
    // The scheduling hints pin "one MFMA, then its share of the expansion work" so that VALU
    // work is always queued behind an MFMA that holds the matrix pipe for 32 cycles.
#define NVFP4_INTERLEAVE()                                                  \
    _Pragma("unroll") for (int i = 0; i < TA * TB; ++i) {                   \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                  \
        __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);      \
    }                                                                       \
    __builtin_amdgcn_sched_barrier(0);
#define NVFP4_STEP(Qn, Sn, tn, Fn, Fc) \
    expand(Qn, Sn, tn, Fn);            \
    mma(Fc);                           \
    NVFP4_INTERLEAVE()

    Codes Ca, Cb;
    Scales S0, S1;
    Frags F0, F1;
    fetch(0, 0);
    stash(0);
    __syncthreads();
    load_codes(0, 0, Ca);
    load_scales(0, 0, S0);
    expand(Ca, S0, 0, F0);
#define NVFP4_TILE(stage, kt)                     \
    {                                             \
        fetch((kt) + 1, (stage) ^ 1);             \
        load_codes(stage, 1, Cb);                 \
        load_scales(stage, 1, S1);                \
        __builtin_amdgcn_sched_barrier(0);        \
        NVFP4_STEP(Ca, S0, 1, F1, F0)             \
        NVFP4_STEP(Ca, S0, 2, F0, F1)             \
        NVFP4_STEP(Ca, S0, 3, F1, F0)             \
        NVFP4_STEP(Cb, S1, 0, F0, F1)             \
        NVFP4_STEP(Cb, S1, 1, F1, F0)             \
        NVFP4_STEP(Cb, S1, 2, F0, F1)             \
        stash((stage) ^ 1);                       \
        __syncthreads();                          \
        load_codes((stage) ^ 1, 0, Ca);           \
        load_scales((stage) ^ 1, 0, S0);          \
        __builtin_amdgcn_sched_barrier(0);        \
        NVFP4_STEP(Cb, S1, 3, F1, F0)             \
        NVFP4_STEP(Ca, S0, 0, F0, F1)             \
    }
    // two tiles per trip so that the LDS stage (and with it every LDS offset) is a constant
    int kt = 0;
    for (; kt + 2 < nkt; kt += 2) {
        NVFP4_TILE(0, kt)
        NVFP4_TILE(1, kt + 1)
    }
    if (kt + 1 < nkt) {
        NVFP4_TILE(0, kt)
        ++kt;
    }
#undef NVFP4_TILE
    {
        const int stage = kt & 1;  // the last tile
        load_codes(stage, 1, Cb);
        load_scales(stage, 1, S1);
        __builtin_amdgcn_sched_barrier(0);
        NVFP4_STEP(Ca, S0, 1, F1, F0)
        NVFP4_STEP(Ca, S0, 2, F0, F1)
        NVFP4_STEP(Ca, S0, 3, F1, F0)
        NVFP4_STEP(Cb, S1, 0, F0, F1)
        NVFP4_STEP(Cb, S1, 1, F1, F0)
        NVFP4_STEP(Cb, S1, 2, F0, F1)
        NVFP4_STEP(Cb, S1, 3, F1, F0)
        mma(F1);
    }
#undef NVFP4_STEP
#undef NVFP4_INTERLEAVE

    // epilogue.  The MFMA's first operand is the B (N-side) fragment, so accumulator register v of
    // lane (r, h) of tile (a, b) is output row 32 a + r, column 32 b + 8 (v / 4) + 4 h + v % 4: four
    // consecutive columns of one row = one packed convert pair and one 8-byte (bf16) or 16-byte
    // (fp32) store.  Full tiles with a suitably aligned output take that path; edge tiles store
    // element by element.  bf16 output of the 8-wave shape goes through LDS first (below): measured
    // 2.5-5 % faster per GEMM than 16-byte pieces that the L2 has to merge into lines, while
    // nontemporal 8-byte stores that bypass the merging were 30 % slower.
    const float gg = P.gA[0] * P.gB[0];
    constexpr int ESZ = OUT_DT == NVFP4_F32 ? 4 : 2;
    const int64_t row0 = m0 + wm * 32 * TA + r, col0 = n0 + wn * 32 * TB + 4 * h;
    const bool fast = m0 + BM <= P.M && n0 + BN <= P.N && (P.ldc & 3) == 0 && (reinterpret_cast<uintptr_t>(P.out) & 15) == 0;
    constexpr bool LINES = TA == 4 && TB == 2 && !KTAIL;  // 128 x 64 per wave: 128-byte (bf16) or 256-byte (fp32) rows
    if (LINES && OUT_DT == NVFP4_F32 && fast) {
        // fp32: 32 rows x 256 bytes at a time through the wave's 8 KB, four complete rows per store
        __syncthreads();
        uint8_t *const out = reinterpret_cast<uint8_t *>(P.out);
        uint8_t *const mine = lds + wave * 8192;
#pragma unroll
        for (int a = 0; a < TA; ++a) {
#pragma unroll
            for (int b = 0; b < TB; ++b)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int chunk = 8 * b + 2 * q + h;  // columns 4 chunk .. 4 chunk + 3 of the wave's 64
                    *reinterpret_cast<float4 *>(mine + r * 256 + ((chunk ^ (r & 15)) << 4)) =
                        make_float4(acc[a][b][4 * q] * gg, acc[a][b][4 * q + 1] * gg, acc[a][b][4 * q + 2] * gg, acc[a][b][4 * q + 3] * gg);
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int rowl = 4 * i + (lane >> 4), chunk = lane & 15;
                const uint4 v = *reinterpret_cast<const uint4 *>(mine + rowl * 256 + ((chunk ^ (rowl & 15)) << 4));
                const int64_t grow = m0 + wm * 128 + 32 * a + rowl, gcol = n0 + wn * 64 + 4 * chunk;
                *reinterpret_cast<uint4 *>(out + (grow * P.ldc + gcol) * 4) = v;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    } else if (LINES && OUT_DT == NVFP4_BF16 && fast && (P.ldc & 7) == 0) {
        // Full-line output: the wave transposes its accumulators through a private 8 KB piece of
        // LDS (64 rows x 128 bytes at a time, 16-byte chunks XOR-swizzled by row) so that a store
        // instruction writes 8 complete 128-byte rows instead of 32 pieces of 16 bytes.
        __syncthreads();  // every wave has read the last K tile: the stages may be overwritten
        uint8_t *const out = reinterpret_cast<uint8_t *>(P.out);
        uint8_t *const mine = lds + wave * 8192;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
#pragma unroll
            for (int a2 = 0; a2 < 2; ++a2) {
                const int a = 2 * half + a2, rowl = 32 * a2 + r;
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
                        const int chunk = 4 * b + q;  // columns 8 chunk .. 8 chunk + 7 of the wave's 64
                        *reinterpret_cast<uint2 *>(mine + rowl * 128 + ((chunk ^ (rowl & 7)) << 4) + 8 * h) = w;
                    }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int rowl = 8 * i + (lane >> 3), chunk = lane & 7;
                const uint4 v = *reinterpret_cast<const uint4 *>(mine + rowl * 128 + ((chunk ^ (rowl & 7)) << 4));
                const int64_t grow = m0 + wm * 128 + 64 * half + rowl, gcol = n0 + wn * 64 + 8 * chunk;
                *reinterpret_cast<uint4 *>(out + (grow * P.ldc + gcol) * 2) = v;
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
    } else if (fast) {
        uint8_t *const out = reinterpret_cast<uint8_t *>(P.out);
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
                            reinterpret_cast<uint16_t *>(P.out)[row * P.ldc + col] = f32_to_bf16_rne(y);
                    }
                }
            }
    }
}

template <int B, int WM, int WN, int TA, int TB, bool KTAIL>
static void launch_f16(const GemmArgs &P, int out_dt, hipStream_t st)
{
    constexpr int BM = 32 * TA * WM, BN = 32 * TB * WN;
    constexpr int LDS_BYTES = 2 * ((BM + BN) * KTB + (BM + BN) * SROW);
    const unsigned ntiles = (unsigned)(((P.N + BN - 1) / BN) * ((P.M + BM - 1) / BM));
    if (out_dt == NVFP4_F32) {
        auto k = gemm_nt_f16_kernel<B, WM, WN, TA, TB, NVFP4_F32, KTAIL>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(64 * WM * WN), LDS_BYTES, st, P);
    } else {
        auto k = gemm_nt_f16_kernel<B, WM, WN, TA, TB, NVFP4_BF16, KTAIL>;
        static bool once = ((void)hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES), true);
        (void)once;
        hipLaunchKernelGGL(k, dim3(ntiles), dim3(64 * WM * WN), LDS_BYTES, st, P);
    }
}

// Tile choice: 256 x 256 (8 waves) when the output has enough such tiles to occupy the 256
// CUs, else 128 x 128 (4 waves, several workgroups per CU).
static bool large_tile(int64_t M, int64_t N, int64_t K)
{
    const int64_t big = ((M + 255) / 256) * ((N + 255) / 256);
    return big >= 128 && K % KT == 0;  // the large tile is built for K % 128 == 0 only
}

bool gemm_takes_slabs(int64_t M, int64_t N, int64_t K, int block, int sf)
{
    if (sf == NVFP4_SCALE_E8M0) return block == 32 && mxfp4_gemm_takes_slabs(K);
    return sf == NVFP4_SCALE_E4M3 && block == 16 && large_tile(M, N, K);
}

template <int B>
static void launch_f16_auto(const GemmArgs &P, int out_dt, hipStream_t st)
{
    const bool ktail = (P.K % KT) != 0;
    if (large_tile(P.M, P.N, P.K))
        launch_f16<B, 2, 4, 4, 2, false>(P, out_dt, st);
    else if (!ktail)
        launch_f16<B, 2, 2, 2, 2, false>(P, out_dt, st);
    else
        launch_f16<B, 2, 2, 2, 2, true>(P, out_dt, st);
}

static int g_fp4_rescale_route = 0;  // (measured slower than the fp16 route: opt-in)
void set_fp4_rescale_route(int on) { g_fp4_rescale_route = on; }
int fp4_rescale_route() { return g_fp4_rescale_route; }

hipError_t launch_gemm(const GemmArgs &P, int block, int sf, int out_dt, hipStream_t st)
{
    // lane offsets inside a 256-row tile are 32-bit
    if ((P.K >> 1) * 256 >= ((int64_t)1 << 31)) return hipErrorInvalidValue;
    if ((P.a_slab || P.b_slab) && !gemm_takes_slabs(P.M, P.N, P.K, block, sf)) return hipErrorInvalidValue;
    if (sf == NVFP4_SCALE_E8M0) return block == 32 ? launch_gemm_mxfp4(P, out_dt, st) : hipErrorNotSupported;
    if (g_fp4_rescale_route && fp4_rescale_gemm_applies(P.K, block, P)) return launch_gemm_fp4_rescale(P, block, out_dt, st);
    switch (block) {
    case 16: launch_f16_auto<16>(P, out_dt, st); break;
    case 32: launch_f16_auto<32>(P, out_dt, st); break;
    case 64: launch_f16_auto<64>(P, out_dt, st); break;
    case 128: launch_f16_auto<128>(P, out_dt, st); break;
    default: return hipErrorNotSupported;
    }
    return hipGetLastError();
}

}  // namespace nvfp4
