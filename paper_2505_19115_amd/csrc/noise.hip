// Quantization-noise statistics of a quantized tensor against its source: sum x^2 and
// sum (Q(x) - x)^2.  With eps = Q(x) - x the quantization error of a d-element gradient, the
// noise-threshold section (Sec. 4) of "FP4 All the Way" monitors ||x|| / (sigma_q sqrt(d)) =
// sqrt(sum x^2 / sum eps^2) against sqrt(3); the same two sums give the relative quantization
// MSE of a format.  One pass over x (2 or 4 B/elt) plus the packed operand (0.5 B + 1/block B):
// HBM-bound.
//
// A lane takes 8 consecutive elements of one stored operand row (4 bytes of codes, one scale byte):
// squares are summed in fp32 over those 8 and then accumulated in fp64, lanes / waves / workgroups
// are combined in fp64 in a fixed order, so the result does not depend on timing.
//   axis 1 (blocks along rows of x):  the 8 elements are 16 contiguous bytes of x (bf16);
//   axis 0 (blocks down columns):     the operand row is a column of x; a lane owns 4 adjacent
//                                     columns (1 for shapes that do not allow vector loads) and a
//                                     wave 256 consecutive ones, so each of its 8 row loads is 512
//                                     contiguous bytes (bf16) and each lane reads 32 contiguous
//                                     code bytes (64 elements) of each of its columns.
#include "kernels.h"
#include "nvfp4_math.h"

namespace nvfp4 {

constexpr int NOISE_THREADS = 256;
constexpr int NOISE_ROWS_CHUNKS = 4;  // axis 1: 8-element chunks per thread
constexpr int NOISE_COLS_SPAN = 64;   // axis 0: elements of its column per thread

typedef float float2n_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float scale_of(uint32_t byte, int sf)
{
    if (sf == NVFP4_SCALE_E4M3) return e4m3_decode(byte);
    return byte == 0 ? u2f(0x00400000u) : u2f(byte << 23);  // E8M0: 2^(byte - 127)
}

template <int DT>
__device__ __forceinline__ float load_x(const void *x, int64_t idx)
{
    if (DT == NVFP4_F32) return reinterpret_cast<const float *>(x)[idx];
    return u2f((uint32_t)reinterpret_cast<const uint16_t *>(x)[idx] << 16);
}

// 8 consecutive elements (16-byte aligned: the leading dimension and the base are)
template <int DT>
__device__ __forceinline__ void load_x8(const void *x, int64_t idx, float *xs)
{
    if (DT == NVFP4_F32) {
        const float4 a = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(x) + idx);
        const float4 b = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(x) + idx + 4);
        xs[0] = a.x; xs[1] = a.y; xs[2] = a.z; xs[3] = a.w;
        xs[4] = b.x; xs[5] = b.y; xs[6] = b.z; xs[7] = b.w;
    } else {
        const uint4 r = *reinterpret_cast<const uint4 *>(reinterpret_cast<const uint16_t *>(x) + idx);
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            xs[2 * t] = u2f(w[t] << 16);
            xs[2 * t + 1] = u2f(w[t] & 0xFFFF0000u);
        }
    }
}

// 8 codes (one dword, element 2 t in the low nibble of byte t) times d against xs[0..7]
__device__ __forceinline__ void accumulate8(uint32_t w, float d, const float *xs, double &sx, double &se)
{
    float px = 0.0f, pe = 0.0f;
#define NVFP4_NOISE_PAIR(t)                                                             \
    {                                                                                   \
        const float2n_t c = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, 1.0f, t);       \
        const float e0 = c[0] * d - xs[2 * t], e1 = c[1] * d - xs[2 * t + 1];           \
        px = fmaf(xs[2 * t], xs[2 * t], px);                                            \
        px = fmaf(xs[2 * t + 1], xs[2 * t + 1], px);                                    \
        pe = fmaf(e0, e0, pe);                                                          \
        pe = fmaf(e1, e1, pe);                                                          \
    }
    NVFP4_NOISE_PAIR(0)
    NVFP4_NOISE_PAIR(1)
    NVFP4_NOISE_PAIR(2)
    NVFP4_NOISE_PAIR(3)
#undef NVFP4_NOISE_PAIR
    sx += (double)px;
    se += (double)pe;
}

// fixed-order fp64 sum over the workgroup -> partials[2 wg], partials[2 wg + 1]
__device__ __forceinline__ void reduce_and_store(double sx, double se, double *partials)
{
    __shared__ double red[2][NOISE_THREADS / 64];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        sx += __shfl_down(sx, o, 64);
        se += __shfl_down(se, o, 64);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) {
        red[0][wave] = sx;
        red[1][wave] = se;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0, b = 0.0;
        for (int w = 0; w < NOISE_THREADS / 64; ++w) {
            a += red[0][w];
            b += red[1][w];
        }
        partials[2 * (int64_t)blockIdx.x] = a;
        partials[2 * (int64_t)blockIdx.x + 1] = b;
    }
}

struct NoiseArgs {
    const void *x;
    int64_t rows, cols, ld;
    const uint8_t *codes, *scales;
    const float *g;  // device scalar or null (no tensor scale)
    int block, sf;
    double *partials;
};

template <int DT>
__global__ __launch_bounds__(NOISE_THREADS) void noise_rows_kernel(NoiseArgs P)
{
    const float g = P.g ? *P.g : 1.0f;
    // 8-element chunks, numbered row-major; a load instruction of a wave covers 64 consecutive chunks
    const uint32_t cpr = (uint32_t)(P.cols >> 3);
    const int64_t total = P.rows * (int64_t)cpr;
    const int64_t first = (int64_t)blockIdx.x * (NOISE_THREADS * NOISE_ROWS_CHUNKS) + threadIdx.x;
    float xs[NOISE_ROWS_CHUNKS][8];
    uint32_t w[NOISE_ROWS_CHUNKS], sb[NOISE_ROWS_CHUNKS];
    // all loads first, then the arithmetic
#pragma unroll
    for (int u = 0; u < NOISE_ROWS_CHUNKS; ++u) {
        const int64_t q = first + u * NOISE_THREADS;
        if (q < total) {
            const int64_t r = q / cpr;  // (one 64-bit division per 8 elements)
            const int64_t c8 = q - r * cpr;
            load_x8<DT>(P.x, r * P.ld + c8 * 8, xs[u]);
            w[u] = *reinterpret_cast<const uint32_t *>(P.codes + q * 4);
            sb[u] = P.scales[r * (P.cols / P.block) + (c8 * 8) / P.block];
        }
    }
    double sx = 0.0, se = 0.0;
#pragma unroll
    for (int u = 0; u < NOISE_ROWS_CHUNKS; ++u)
        if (first + u * NOISE_THREADS < total) accumulate8(w[u], scale_of(sb[u], P.sf) * g, xs[u], sx, se);
    reduce_and_store(sx, se, P.partials);
}

// CW = adjacent columns per lane: 4 (one 8-byte bf16 / 16-byte fp32 load per row; needs cols % 4 == 0 and
// 16-byte aligned rows) or 1 (any shape).  A wave covers 64 CW consecutive columns.
template <int DT, int CW>
__global__ __launch_bounds__(NOISE_THREADS) void noise_cols_kernel(NoiseArgs P)
{
    const float g = P.g ? *P.g : 1.0f;
    // workgroup = 64 CW columns x (4 waves x 64 rows); operand row o = column of x, position n = row of x
    constexpr int ESZ = DT == NVFP4_F32 ? 4 : 2;
    const int64_t ctiles = (P.cols + 64 * CW - 1) / (64 * CW);
    const int64_t tr = blockIdx.x / ctiles, tc = blockIdx.x - tr * ctiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t o = (tc * 64 + lane) * CW, n0 = (tr * 4 + wave) * NOISE_COLS_SPAN;
    double sx = 0.0, se = 0.0;
    if (o < P.cols && n0 < P.rows) {
        // rows is a multiple of the block, hence of 8: groups of 8 are all-or-nothing
        const int groups = (int)((P.rows - n0 < NOISE_COLS_SPAN ? P.rows - n0 : NOISE_COLS_SPAN) >> 3);
        const uint8_t *px = reinterpret_cast<const uint8_t *>(P.x) + (n0 * P.ld + o) * ESZ;
        const uint32_t stride = (uint32_t)P.ld * ESZ;  // bytes between rows (< 4 GB)
        const int64_t crow = P.rows >> 1, srow = P.rows / P.block;  // bytes per operand row
        const uint8_t *pc = P.codes + o * crow + (n0 >> 1);
        const uint8_t *ps = P.scales + o * srow;
        const int bshift = P.block == 16 ? 4 : P.block == 32 ? 5 : P.block == 64 ? 6 : 7;
        // the lane's codes (32 bytes per column) and scale bytes (one per 16 rows) first: a 4-byte read per
        // group of 8 rows would fetch the same line of every column eight times, and the lines of a wave's
        // columns do not all stay in the vector L1 in between
        uint32_t cw[CW][8], sb[CW][4];
#pragma unroll
        for (int j = 0; j < CW; ++j) {
            if (groups == 8) {
                const uint4 lo = *reinterpret_cast<const uint4 *>(pc + j * crow), hi = *reinterpret_cast<const uint4 *>(pc + j * crow + 16);
                cw[j][0] = lo.x; cw[j][1] = lo.y; cw[j][2] = lo.z; cw[j][3] = lo.w;
                cw[j][4] = hi.x; cw[j][5] = hi.y; cw[j][6] = hi.z; cw[j][7] = hi.w;
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) cw[j][k] = k < groups ? *reinterpret_cast<const uint32_t *>(pc + j * crow + k * 4) : 0u;
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) sb[j][i] = 2 * i < groups ? ps[j * srow + ((n0 + 16 * i) >> bshift)] : 0u;
        }
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            if (k >= groups) break;
            float xs[CW][8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const uint8_t *p = px + (uint32_t)(k * 8 + t) * stride;
                if (CW == 1) {
                    xs[0][t] = DT == NVFP4_F32 ? *reinterpret_cast<const float *>(p) : u2f((uint32_t)*reinterpret_cast<const uint16_t *>(p) << 16);
                } else if (DT == NVFP4_F32) {
                    const float4 v = *reinterpret_cast<const float4 *>(p);
                    xs[0][t] = v.x; xs[1 % CW][t] = v.y; xs[2 % CW][t] = v.z; xs[3 % CW][t] = v.w;
                } else {
                    const uint2 v = *reinterpret_cast<const uint2 *>(p);
                    xs[0][t] = u2f(v.x << 16); xs[1 % CW][t] = u2f(v.x & 0xFFFF0000u);
                    xs[2 % CW][t] = u2f(v.y << 16); xs[3 % CW][t] = u2f(v.y & 0xFFFF0000u);
                }
            }
#pragma unroll
            for (int j = 0; j < CW; ++j) accumulate8(cw[j][k], scale_of(sb[j][k >> 1], P.sf) * g, xs[j], sx, se);
        }
    }
    reduce_and_store(sx, se, P.partials);
}

// one workgroup: partial pairs summed thread-strided, then the fixed-order tree
__global__ __launch_bounds__(NOISE_THREADS) void noise_fold_kernel(const double *partials, int64_t n, double *sums)
{
    double sx = 0.0, se = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += NOISE_THREADS) {
        sx += partials[2 * i];
        se += partials[2 * i + 1];
    }
    __shared__ double out[2];
    reduce_and_store(sx, se, out);
    __syncthreads();
    if (threadIdx.x == 0) {
        sums[0] = out[0];
        sums[1] = out[1];
    }
}

int64_t quant_noise_partials(int64_t rows, int64_t cols, int axis)
{
    if (rows <= 0 || cols <= 0) return 1;
    if (axis == 1) {
        const int64_t per_wg = (int64_t)NOISE_THREADS * NOISE_ROWS_CHUNKS;
        return (rows * (cols >> 3) + per_wg - 1) / per_wg;
    }
    return ((cols + 63) >> 6) * ((rows + 4 * NOISE_COLS_SPAN - 1) / (4 * NOISE_COLS_SPAN));  // (an upper bound when 4 columns per lane are used)
}

// workgroups of the axis-0 kernel with CW columns per lane
static int64_t noise_cols_wgs(int64_t rows, int64_t cols, int cw)
{
    return ((cols + 64 * cw - 1) / (64 * cw)) * ((rows + 4 * NOISE_COLS_SPAN - 1) / (4 * NOISE_COLS_SPAN));
}

hipError_t launch_quant_noise(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld, int axis, int block, int sf,
                              const uint8_t *codes, const uint8_t *scales, const float *g, double *partials, double *sums,
                              hipStream_t st)
{
    int64_t nwg = quant_noise_partials(rows, cols, axis);
    if (rows > 0 && cols > 0) {
        NoiseArgs P{x, rows, cols, ld, codes, scales, g, block, sf, partials};
        if (axis == 1) {
            if (dt == NVFP4_F32)
                hipLaunchKernelGGL(noise_rows_kernel<NVFP4_F32>, dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
            else
                hipLaunchKernelGGL(noise_rows_kernel<NVFP4_BF16>, dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
        } else {
            const int64_t esz = dt == NVFP4_F32 ? 4 : 2;
            const bool wide = cols % 4 == 0 && (ld * esz) % 16 == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
            nwg = noise_cols_wgs(rows, cols, wide ? 4 : 1);
            if (wide && dt == NVFP4_F32)
                hipLaunchKernelGGL((noise_cols_kernel<NVFP4_F32, 4>), dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
            else if (wide)
                hipLaunchKernelGGL((noise_cols_kernel<NVFP4_BF16, 4>), dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
            else if (dt == NVFP4_F32)
                hipLaunchKernelGGL((noise_cols_kernel<NVFP4_F32, 1>), dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
            else
                hipLaunchKernelGGL((noise_cols_kernel<NVFP4_BF16, 1>), dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
        }
        hipLaunchKernelGGL(noise_fold_kernel, dim3(1), dim3(NOISE_THREADS), 0, st, partials, nwg, sums);
    } else {
        hipLaunchKernelGGL(noise_fold_kernel, dim3(1), dim3(NOISE_THREADS), 0, st, partials, (int64_t)0, sums);
    }
    return hipGetLastError();
}

}  // namespace nvfp4
