// Sustained MFMA rate of the GPU the library runs on: the two matrix instructions the GEMM kernels
// issue, in the register-tile pattern those kernels use, from registers only (no LDS, no global
// memory).  MI355X reaches its published matrix peaks only at its top clock; under a chip-wide MFMA
// load the clock is power-managed and depends on how many operand bits toggle, so a kernel's MFMA
// utilisation is best judged against this measured rate as well as against the published peak.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/nvfp4.h"

namespace nvfp4 {

typedef int int8v_t __attribute__((ext_vector_type(8)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16v_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ uint32_t xorshift(uint32_t &h)
{
    h ^= h << 13;
    h ^= h >> 17;
    h ^= h << 5;
    return h;
}

// v_mfma_f32_32x32x16_f16, 4 x 2 accumulator tiles per wave, two waves per SIMD
template <bool RANDOM>
__global__ __launch_bounds__(512) void probe_f16_kernel(float *out, int iters)
{
    float16v_t acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
    uint32_t h = (threadIdx.x + 1) * 2654435761u + blockIdx.x * 40503u;
    half8_t va[4], vb[2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int j = 0; j < 8; ++j) va[a][j] = RANDOM ? (_Float16)(int)((xorshift(h) >> 8) % 13 - 6) : (_Float16)0.0f;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int j = 0; j < 8; ++j) vb[b][j] = RANDOM ? (_Float16)(int)((xorshift(h) >> 8) % 13 - 6) : (_Float16)0.0f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va[a], vb[b], acc[a][b], 0, 0, 0);
        if (RANDOM) {  // new operand bits every step, as if freshly loaded
#pragma unroll
            for (int a = 0; a < 4; ++a) va[a] = __builtin_shufflevector(va[a], va[(a + 1) & 3], 1, 2, 3, 4, 5, 6, 7, 8);
        }
    }
    float sum = 0.0f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[a][b][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

// v_mfma_scale_f32_32x32x64_f8f6f4 on FP4 operands, 4 x 4 accumulator tiles per wave, one wave per SIMD
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_fp4_kernel(float *out, int iters)
{
    float16v_t acc[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;
    uint32_t h = (threadIdx.x + 1) * 2654435761u + blockIdx.x * 40503u;
    int8v_t va[2][4], vb[2][4];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            va[s][a] = int8v_t{0, 0, 0, 0, 0, 0, 0, 0};
            vb[s][a] = int8v_t{0, 0, 0, 0, 0, 0, 0, 0};
            if (RANDOM) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    va[s][a][j] = (int)xorshift(h);
                    vb[s][a][j] = (int)xorshift(h);
                }
            }
        }
    const int unit = 0x7f7f7f7f;  // E8M0 127 = 2^0
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va[s][a], vb[s][b], acc[a][b], 4, 4, 0, unit, 0, unit);
            if (RANDOM) {
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    va[s][a][0] ^= va[s ^ 1][a][1];
                    vb[s][a][0] ^= vb[s ^ 1][a][1];
                }
            }
        }
    }
    float sum = 0.0f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) sum += acc[a][b][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

}  // namespace nvfp4

extern "C" nvfp4_status nvfp4_probe_mfma_rate(int kind, int random_operands, int iters, void *scratch, size_t scratch_bytes,
                                              double *tflops, void *stream)
{
    using namespace nvfp4;
    if ((kind != 0 && kind != 1) || iters <= 0 || iters > (1 << 22) || !scratch || !tflops) return NVFP4_EINVAL;
    hipDeviceProp_t prop;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return NVFP4_EHIP;
    const int wgs = prop.multiProcessorCount;  // one workgroup per compute unit
    const int threads = kind == 0 ? 512 : 256;
    if (scratch_bytes < (size_t)wgs * threads * sizeof(float)) return NVFP4_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    float *out = static_cast<float *>(scratch);
    auto launch = [&](int n) {
        if (kind == 0) {
            if (random_operands)
                hipLaunchKernelGGL(probe_f16_kernel<true>, dim3(wgs), dim3(threads), 0, st, out, n);
            else
                hipLaunchKernelGGL(probe_f16_kernel<false>, dim3(wgs), dim3(threads), 0, st, out, n);
        } else {
            if (random_operands)
                hipLaunchKernelGGL(probe_fp4_kernel<true>, dim3(wgs), dim3(threads), 0, st, out, n);
            else
                hipLaunchKernelGGL(probe_fp4_kernel<false>, dim3(wgs), dim3(threads), 0, st, out, n);
        }
    };
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return NVFP4_EHIP;
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return NVFP4_EHIP;
    }
    launch(16);  // warm-up: code object load, clocks
    hipError_t err = hipEventRecord(e0, st);
    launch(iters);
    if (err == hipSuccess) err = hipEventRecord(e1, st);
    if (err == hipSuccess) err = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    if (err == hipSuccess) err = hipGetLastError();
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (err != hipSuccess || ms <= 0.0f) return NVFP4_EHIP;
    // per wave and iteration: 8 MFMAs of 32 x 32 x 16 (f16) or 32 MFMAs of 32 x 32 x 64 (FP4)
    const double flop = kind == 0 ? (double)iters * 8 * (2.0 * 32 * 32 * 16) * (threads / 64) * wgs
                                  : (double)iters * 32 * (2.0 * 32 * 32 * 64) * (threads / 64) * wgs;
    *tflops = flop / (ms * 1e-3) / 1e12;
    return NVFP4_OK;
}
