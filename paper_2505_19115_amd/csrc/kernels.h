// Internal interface between the C ABI (api.hip) and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/nvfp4.h"

namespace nvfp4 {

enum { G_NONE = 0, G_PRESET = 1, G_FROM_AMAX = 2 };

struct QuantArgs {
    const void *x;        // [rows, cols], leading dimension ld
    int64_t rows, cols, ld;
    uint8_t *codes;       // axis 1: [rows, cols/2]; axis 0: [cols, rows/2]
    uint8_t *scales;      // axis 1: [rows, cols/B]; axis 0: [cols, rows/B]
    const float *g_src;   // G_PRESET: the scale; G_FROM_AMAX: bit pattern of max|x| (n_partials == 0) or
                          // n_partials per-workgroup maxima that every workgroup folds for itself
    float *g_out;         // receives the scale actually used
    int g_mode;
    uint64_t seed;
    int n_partials = 0;
};

// Identity of what nvfp4_linear_fwd left in a `saved` buffer (shapes, format, seed, layout of each operand): the
// forward call's quantizer writes the words to dst; the backward call's quantizer compares them with chk and, on a
// mismatch, replaces the tensor scale it hands to the GEMMs by NaN, so that a backward call on the wrong buffer
// gives NaN outputs instead of plausible wrong numbers.
struct TagArgs {
    uint32_t *dst = nullptr;
    const uint32_t *chk = nullptr;
    uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
};
// (one thread) writes / checks the tag; returns false on a mismatch
__device__ __forceinline__ bool tag_apply(const TagArgs &t)
{
    bool ok = true;
    if (t.dst)
        for (int i = 0; i < 8; ++i) t.dst[i] = t.w[i];
    if (t.chk)
        for (int i = 0; i < 8; ++i) ok = ok && t.chk[i] == t.w[i];
    return ok;
}
// The same from a one-thread kernel, for the paths that do not run the one-pass dual quantizer; g1 / g2 (either may
// be null) are overwritten with NaN on a mismatch.
hipError_t launch_saved_tag(const TagArgs &t, float *g1, float *g2, hipStream_t st);

// Both orientations of one tensor: c describes the tensor and the column-blocked outputs
// (codes [cols, rows/2], scales [cols, rows/B], seed); the row-blocked outputs come beside it.
struct DualArgs {
    QuantArgs c;
    uint8_t *codes_r;   // [rows, cols/2]
    uint8_t *scales_r;  // [rows, cols/B]
    uint64_t seed_r;
    float *g_out2;      // optional second destination of the tensor scale
    int slab_r = 0;     // write the row-blocked / column-blocked output in the slab layout (below) instead
    int slab_c = 0;
    TagArgs tag;        // optional: identity of a `saved` buffer to write or to check (fused linear entries)
    // With a SwiGLU source (launch_swiglu_bwd_dual) the tensor being quantized is never in memory: c.x is dH and
    // these are G and U, all dense [rows, cols]; the kernel evaluates dG or dU per element as it loads.
    const void *src_g = nullptr, *src_u = nullptr;
};

// Slab layout of a packed operand (used inside the workspaces and the saved buffer of the fused linear entries,
// and documented in include/nvfp4.h for nvfp4_quantize_dual's slab outputs and nvfp4_gemm_slab).  For an operand of R rows and contraction length K
// (K a multiple of 128) the codes are stored as [ceil(R / 256)][K / 128] slabs of 16 KB: one slab is
// what one GEMM workgroup fetches per K tile, 256 rows x 64 bytes, contiguous.  Inside a slab row r (0..255) sits
// at position slab_row(r), which swaps the two 3-bit fields of r below bit 6: the column-blocked quantizer holds
// rows 8 cx + j (lane group cx, column j of the lane) and with this order each of its store instructions writes
// 512 contiguous bytes.  The scales follow the same scheme with 8 bytes per row (slabs of 2 KB).
// MXFP4 operands (block 32, E8M0) use the same slabs for their codes, and scale slabs of 256 positions x 4 bytes
// (the four E8M0 bytes of a row's K tile; 1 KB, same position rule): one direct-to-LDS instruction of the FP4 GEMM
// fetches a whole one, and its image in LDS is read 4 bytes per lane at a 4-byte stride, free of bank conflicts.
constexpr int64_t SLAB_ROWS = 256, SLAB_K = 128, SLAB_CODE_BYTES = 16384, SLAB_SCALE_BYTES = 2048, SLAB_MX_SCALE_BYTES = 1024;
__host__ __device__ inline int slab_row(int r) { return (r & ~63) | ((r & 7) << 3) | ((r >> 3) & 7); }
inline int64_t slab_rows_padded(int64_t rows) { return (rows + SLAB_ROWS - 1) / SLAB_ROWS * SLAB_ROWS; }

struct GemmArgs {
    int64_t M, N, K;
    const uint8_t *A_codes, *A_scales, *B_codes, *B_scales;
    const float *gA, *gB;  // per-tensor scales of the two operands (device)
    void *out;
    int64_t ldc;
    int a_slab = 0, b_slab = 0;  // operand stored in the slab layout (only where gemm_takes_slabs() holds)
};
// True when launch_gemm() runs the 256 x 256 direct-to-LDS kernel for this problem, the one that can read operands
// in the slab layout.
bool gemm_takes_slabs(int64_t M, int64_t N, int64_t K, int block, int sf);

// Tensor maximum: one partial per workgroup into `partials` (tensor_amax_partials() entries),
// then folded into amax_bits[0] (bit pattern of max|x|) and, if g_out is given, into the scale.
int64_t tensor_amax_partials(int64_t rows, int64_t cols, int64_t ld);
// Workgroup id -> output tile (ty, tx) of an nty x ntx tile grid.
// Consecutive workgroup ids land on different XCDs (8 of them, each with its own 4 MB L2), so
// XCD x = id % 8 is given a contiguous band of a walk over the grid, and the walk itself goes
// down panels of 4 tile rows column by column: the ~32 workgroups an XCD runs at a time then
// cover about 4 x 8 tiles and share 12 operand strips in its L2 instead of 33.
__device__ __forceinline__ void tile_coords(int wg, int ntx, int nty, int &ty, int &tx)
{
    const int ntiles = ntx * nty;
    const int per = (ntiles + 7) / 8, xcd = wg & 7, slot = wg >> 3;
    const int full = ntiles - (per - 1) * 8;  // XCDs that receive `per` tiles (the others per-1)
    const int t = xcd < full ? xcd * per + slot : full * per + (xcd - full) * (per - 1) + slot;
    constexpr int GH = 4;
    const int panel = t / (GH * ntx), in_panel = t - panel * (GH * ntx);
    const int rows = nty - panel * GH < GH ? nty - panel * GH : GH;  // the last panel may be short
    tx = in_panel / rows;
    ty = panel * GH + in_panel - tx * rows;
}

hipError_t launch_tensor_amax(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld,
                              uint32_t *amax_bits, uint32_t *partials, float *g_out, hipStream_t st);
// Dense tensors only: at most AMAX_DENSE_PARTIALS partial maxima into `partials`, no fold kernel
// (the consuming quantizer folds them: QuantArgs::n_partials).  Returns their number in *n.
constexpr int AMAX_DENSE_PARTIALS = 512;
hipError_t launch_tensor_amax_dense(const void *x, int dt, int64_t n_elements, uint32_t *partials, int *n, hipStream_t st);
hipError_t launch_quantize(const QuantArgs &P, int dt, int axis, int rounding, int block, int sf,
                           bool hw_convert, hipStream_t st);
// Row-blocked and column-blocked quantization of one tensor; one fused kernel when
// quantize_dual_fused() holds, else the two single-orientation kernels.
bool quantize_dual_fused(int dt, int64_t rows, int64_t cols, int64_t ld, int block, bool hw_convert);
hipError_t launch_quantize_dual(const DualArgs &D, int dt, int rnd_rows, int rnd_cols, int block, int sf,
                                bool hw_convert, hipStream_t st);
// SwiGLU backward fused with the quantizers of its two results: one pass over dH, G, U leaves the partial maxima of
// dG and dU (AMAX_DENSE_PARTIALS slots each, the counts come back in n_g / n_u; skipped without tensor scale), then one
// dual-orientation pass per result re-evaluates it while loading.  g / u describe the outputs as for
// launch_quantize_dual (c.x = dH, src_g, src_u set; stochastic rounding on both sides).  Formats: the ones the
// one-pass dual kernel serves with slabs (block 16 + E4M3, block 32 + E8M0); the caller checks quantize_dual_fused().
// With dG_store / dU_store (both or neither) the first pass also stores the two results and the quantizer passes read
// them back through the ordinary dual kernel instead of evaluating them again.
hipError_t launch_swiglu_bwd_dual(DualArgs &g, DualArgs &u, int dt, int block, int sf, uint32_t *partials_g,
                                  uint32_t *partials_u, void *dG_store, void *dU_store, hipStream_t st);
// The same elementwise step with dG and dU stored as tensors of dt (n a multiple of 8).
hipError_t launch_swiglu_bwd(const void *dH, const void *G, const void *U, int dt, int64_t n, void *dG, void *dU, hipStream_t st);
hipError_t launch_gemm(const GemmArgs &P, int block, int sf, int out_dt, hipStream_t st);
hipError_t launch_gemm_mxfp4(const GemmArgs &P, int out_dt, hipStream_t st);  // block 32, E8M0
// E4M3 scales at blocks of 64 / 128 as unit-scale FP4 MFMAs per block + binary32 rescale (row-major operands, K % 128 == 0)
bool fp4_rescale_gemm_applies(int64_t K, int block, const GemmArgs &P);
hipError_t launch_gemm_fp4_rescale(const GemmArgs &P, int block, int out_dt, hipStream_t st);
// Which of the two exact routes launch_gemm() takes for those formats: 0 = expanded to fp16 (the NVFP4 kernel), 1 = this one
void set_fp4_rescale_route(int on);
int fp4_rescale_route();
bool mxfp4_gemm_takes_slabs(int64_t K);  // MXFP4: the codes of an operand may come as slabs (its scales stay row-major)
// Noise statistics: per-workgroup partial pairs (quant_noise_partials() of them), folded into sums[2].
int64_t quant_noise_partials(int64_t rows, int64_t cols, int axis);
hipError_t launch_quant_noise(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld, int axis, int block, int sf,
                              const uint8_t *codes, const uint8_t *scales, const float *g, double *partials, double *sums,
                              hipStream_t st);

}  // namespace nvfp4
