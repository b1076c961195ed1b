/* Sanitizer run of the CPU oracle (AddressSanitizer + UndefinedBehaviorSanitizer, host only): every entry of
 * nvfp4_oracle.c on small seeded inputs with exactly-sized heap buffers, both element types, both axes, both
 * roundings, every block format, so that an out-of-bounds index or undefined shift anywhere in it stops the run.
 * Built and run by tests/test_sanitizers.py; prints "sanitize-oracle ok" on success. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../oracle/nvfp4_oracle.c"

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s; }

int main(void)
{
    const orc_format fmts[5] = {{16, ORC_SCALE_E4M3, 1}, {32, ORC_SCALE_E8M0, 0}, {32, ORC_SCALE_E4M3, 1},
                                {64, ORC_SCALE_E4M3, 1}, {128, ORC_SCALE_E4M3, 1}};
    uint32_t s = 12345u;
    for (int fi = 0; fi < 5; ++fi) {
        const orc_format *f = &fmts[fi];
        const int64_t rows = 2 * f->block, cols = 3 * f->block, ld = cols + 8;
        for (int dtype = 0; dtype < 2; ++dtype) {
            const size_t esz = dtype == ORC_BF16 ? 2 : 4;
            void *x = malloc((size_t)(rows * ld) * esz);
            for (int64_t i = 0; i < rows * ld; ++i) {
                const float v = ((float)(lcg(&s) >> 8) / 8388608.0f - 1.0f) * (i % 37 == 0 ? 40.0f : 0.3f);
                if (dtype == ORC_BF16) {
                    uint32_t b;
                    memcpy(&b, &v, 4);
                    ((uint16_t *)x)[i] = (uint16_t)(b >> 16);
                } else {
                    ((float *)x)[i] = v;
                }
            }
            (void)orc_tensor_amax(x, dtype, rows, cols, ld);
            for (int axis = 0; axis < 2; ++axis)
                for (int rnd = 0; rnd < 2; ++rnd) {
                    const int64_t outer = axis ? rows : cols, inner = axis ? cols : rows;
                    uint8_t *codes = malloc((size_t)(outer * inner / 2));
                    uint8_t *scales = malloc((size_t)(outer * inner / f->block));
                    float g = 0.0f;
                    if (orc_quantize(x, dtype, rows, cols, ld, axis, rnd, 77u + (uint64_t)rnd, f, codes, scales, &g, 0) != 0) return 2;
                    double *deq = malloc(sizeof(double) * (size_t)(outer * inner));
                    orc_dequantize(codes, scales, g, outer, inner, f, deq);
                    double noise[2];
                    orc_quant_noise(x, dtype, rows, cols, ld, axis, f, codes, scales, g, noise);
                    if (!(noise[1] <= noise[0])) return 3;
                    double *out = malloc(sizeof(double) * (size_t)(outer * outer));
                    orc_gemm_nt(outer, outer, inner, f, codes, scales, g, codes, scales, g, axis, out);
                    const int64_t ii[3] = {0, outer - 1, outer / 2}, jj[3] = {outer - 1, 0, 1};
                    double smp[3];
                    orc_gemm_nt_sample(outer, outer, inner, f, codes, scales, g, codes, scales, g, 0, ii, jj, 3, smp);
                    if (axis == 0 && smp[0] != out[ii[0] * outer + jj[0]]) return 4;
                    free(out);
                    free(deq);
                    free(scales);
                    free(codes);
                }
            /* shapes the format cannot hold are refused, not overrun */
            uint8_t dummy[8];
            float g = 1.0f;
            if (orc_quantize(x, dtype, rows, f->block / 2, ld, 1, 0, 0, f, dummy, dummy, &g, 1) == 0) return 5;
            free(x);
        }
    }
    /* scalar entries over their whole input range */
    for (int b = 0; b < 256; ++b) {
        (void)orc_e2m1_decode((uint8_t)b);
        (void)orc_e4m3_decode((uint8_t)b);
        (void)orc_e8m0_decode((uint8_t)b);
    }
    float m[64];
    uint32_t u[64], bits[64];
    uint8_t o[64];
    for (int i = 0; i < 64; ++i) {
        m[i] = 6.0f * (float)i / 63.0f;
        u[i] = lcg(&s) & 0xFFFFu;
    }
    orc_e4m3_encode_array(m, 64, o);
    orc_round_rtn_array(m, 64, o);
    orc_round_sr_array(m, u, 64, o);
    orc_sr_bits_array(5u, (uint64_t)1 << 40, 64, bits);
    const uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6};
    uint32_t r4[4];
    orc_philox4x32_10(ctr, key, r4);
    (void)orc_tensor_scale_from_amax(0.0f);
    (void)orc_tensor_scale_from_amax(1e-44f);
    printf("sanitize-oracle ok\n");
    return 0;
}
