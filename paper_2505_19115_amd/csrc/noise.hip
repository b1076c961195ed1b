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
//   axis 0 (blocks down columns):     the operand row is a column of x; a wave covers 64
//                                     consecutive columns, so each of its 8 element loads is one
//                                     contiguous 128-byte (bf16) line and each lane reads 32
//                                     contiguous code bytes (64 elements) of its column.
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

template <int DT>
__global__ __launch_bounds__(NOISE_THREADS) void noise_cols_kernel(NoiseArgs P)
{
    const float g = P.g ? *P.g : 1.0f;
    // workgroup = 64 columns x (4 waves x 64 rows); operand row o = column of x, position n = row of x
    const int64_t ctiles = (P.cols + 63) >> 6;
    const int64_t tr = blockIdx.x / ctiles, tc = blockIdx.x - tr * ctiles;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t o = tc * 64 + lane, n0 = (tr * 4 + wave) * NOISE_COLS_SPAN;
    double sx = 0.0, se = 0.0;
    if (o < P.cols && n0 < P.rows) {
        // rows is a multiple of the block, hence of 8: groups of 8 are all-or-nothing
        const int groups = (int)((P.rows - n0 < NOISE_COLS_SPAN ? P.rows - n0 : NOISE_COLS_SPAN) >> 3);
        const uint8_t *px = reinterpret_cast<const uint8_t *>(P.x) + (n0 * P.ld + o) * (DT == NVFP4_F32 ? 4 : 2);
        const uint32_t stride = (uint32_t)P.ld * (DT == NVFP4_F32 ? 4 : 2);  // bytes between rows (< 4 GB)
        const uint8_t *pc = P.codes + o * (P.rows >> 1) + (n0 >> 1);
        const uint8_t *ps = P.scales + o * (P.rows / P.block);
        const int bshift = P.block == 16 ? 4 : P.block == 32 ? 5 : P.block == 64 ? 6 : 7;
        for (int k = 0; k < groups; ++k) {
            float xs[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const uint8_t *p = px + (uint32_t)(k * 8 + t) * stride;
                xs[t] = DT == NVFP4_F32 ? *reinterpret_cast<const float *>(p) : u2f((uint32_t)*reinterpret_cast<const uint16_t *>(p) << 16);
            }
            const uint32_t w = *reinterpret_cast<const uint32_t *>(pc + k * 4);
            const float d = scale_of(ps[(n0 + k * 8) >> bshift], P.sf) * g;
            accumulate8(w, d, xs, sx, se);
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
    return ((cols + 63) >> 6) * ((rows + 4 * NOISE_COLS_SPAN - 1) / (4 * NOISE_COLS_SPAN));
}

hipError_t launch_quant_noise(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld, int axis, int block, int sf,
                              const uint8_t *codes, const uint8_t *scales, const float *g, double *partials, double *sums,
                              hipStream_t st)
{
    const int64_t nwg = quant_noise_partials(rows, cols, axis);
    if (rows > 0 && cols > 0) {
        NoiseArgs P{x, rows, cols, ld, codes, scales, g, block, sf, partials};
        if (axis == 1) {
            if (dt == NVFP4_F32)
                hipLaunchKernelGGL(noise_rows_kernel<NVFP4_F32>, dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
            else
                hipLaunchKernelGGL(noise_rows_kernel<NVFP4_BF16>, dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
        } else {
            if (dt == NVFP4_F32)
                hipLaunchKernelGGL(noise_cols_kernel<NVFP4_F32>, dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
            else
                hipLaunchKernelGGL(noise_cols_kernel<NVFP4_BF16>, dim3((unsigned)nwg), dim3(NOISE_THREADS), 0, st, P);
        }
        hipLaunchKernelGGL(noise_fold_kernel, dim3(1), dim3(NOISE_THREADS), 0, st, partials, nwg, sums);
    } else {
        hipLaunchKernelGGL(noise_fold_kernel, dim3(1), dim3(NOISE_THREADS), 0, st, partials, (int64_t)0, sums);
    }
    return hipGetLastError();
}

}  // namespace nvfp4
