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
    const float *g_src;   // G_PRESET: the scale; G_FROM_AMAX: bit pattern of max|x|
    float *g_out;         // receives the scale actually used
    int g_mode;
    uint64_t seed;
};

struct GemmArgs {
    int64_t M, N, K;
    const uint8_t *A_codes, *A_scales, *B_codes, *B_scales;
    const float *tensor_scales;  // {gA, gB}
    void *out;
    int64_t ldc;
};

// Tensor maximum: one partial per workgroup into `partials` (tensor_amax_partials() entries),
// then folded into amax_bits[0] (bit pattern of max|x|) and, if g_out is given, into the scale.
int64_t tensor_amax_partials(int64_t rows, int64_t cols, int64_t ld);
hipError_t launch_tensor_amax(const void *x, int dt, int64_t rows, int64_t cols, int64_t ld,
                              uint32_t *amax_bits, uint32_t *partials, float *g_out, hipStream_t st);
hipError_t launch_quantize(const QuantArgs &P, int dt, int axis, int rounding, int block, int sf,
                           bool hw_convert, hipStream_t st);
hipError_t launch_gemm(const GemmArgs &P, int block, int sf, int out_dt, hipStream_t st);
hipError_t launch_gemm_mxfp4(const GemmArgs &P, int out_dt, hipStream_t st);  // block 32, E8M0

}  // namespace nvfp4
