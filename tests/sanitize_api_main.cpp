// Sanitizer run of the HOST side of the C ABI (AddressSanitizer + UndefinedBehaviorSanitizer on the host pass
// only): size queries, every argument check that returns before a launch, the cross-check switch hook and the
// host evaluations of the kernels' scalar steps.  No GPU is touched: every call below is refused by validation or
// is a pure host function.  Built and run by tests/test_sanitizers.py; prints "sanitize-api ok" on success.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <initializer_list>

#include "../include/nvfp4.h"

#define EXPECT(call, code)                                                                         \
    do {                                                                                           \
        const int rc_ = (int)(call);                                                               \
        if (rc_ != (int)(code)) {                                                                  \
            fprintf(stderr, "%s:%d: %s returned %d, expected %d\n", __FILE__, __LINE__, #call, rc_, (int)(code)); \
            return 1;                                                                              \
        }                                                                                          \
    } while (0)

int main()
{
    const nvfp4_format nv = {16, NVFP4_SCALE_E4M3, 1}, mx = {32, NVFP4_SCALE_E8M0, 0}, bad = {8, NVFP4_SCALE_E4M3, 1};
    void *fake = reinterpret_cast<void *>(0x10000);  // non-null, aligned, never dereferenced: validation fails first
    uint8_t *fb = reinterpret_cast<uint8_t *>(fake);
    float *ff = reinterpret_cast<float *>(fake);
    for (int64_t r : {-1, 0, 1, 17, 4096, 1 << 20})
        for (int64_t c : {-1, 0, 16, 11008}) {
            (void)nvfp4_codes_bytes(r, c);
            (void)nvfp4_scales_bytes(r, c, 0, &nv);
            (void)nvfp4_scales_bytes(r, c, 1, &mx);
            (void)nvfp4_scales_bytes(r, c, 2, &bad);
            (void)nvfp4_quantize_workspace_bytes(r, c);
            (void)nvfp4_linear_fwd_workspace_bytes(r, c, 4096, &nv);
            (void)nvfp4_linear_bwd_workspace_bytes(r, c, 4096, &mx);
            (void)nvfp4_linear_saved_bytes(r, c, 4096, &nv);
            (void)nvfp4_weight_operands_bytes(r, c, &nv);
            (void)nvfp4_slab_codes_bytes(r, c);
            (void)nvfp4_slab_scales_bytes(r, c);
            (void)nvfp4_gemm_takes_slabs(r, c, 4096, &nv);
            (void)nvfp4_quant_noise_workspace_bytes(r, c, 0);
        }
    for (int s = -1; s < 9; ++s)
        if (!nvfp4_status_string((nvfp4_status)s)) return 1;
    EXPECT(nvfp4_quantize(nullptr, NVFP4_BF16, 64, 64, 64, 1, NVFP4_RTN, 0, &nv, fb, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quantize(fake, NVFP4_BF16, 64, 72, 72, 1, NVFP4_RTN, 0, &nv, fb, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_ESHAPE);
    EXPECT(nvfp4_quantize(fake, NVFP4_BF16, 64, 64, 64, 1, NVFP4_RTN, 0, &bad, fb, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_EUNSUPPORTED);
    EXPECT(nvfp4_quantize(fake, NVFP4_BF16, 64, 64, 64, 1, NVFP4_RTN, 0, &nv, fb, fb, ff, 0, nullptr, 0, nullptr), NVFP4_EWORKSPACE);
    EXPECT(nvfp4_quantize(fake, NVFP4_BF16, 64, 64, 64, 1, NVFP4_RTN, 0, nullptr, fb, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quantize_static(fake, NVFP4_BF16, 16385, 16, 24, 1, NVFP4_RTN, 0, &nv, fb, fb, ff, 0, nullptr), NVFP4_EWORKSPACE);
    EXPECT(nvfp4_quantize_dual(fake, NVFP4_BF16, 64, 64, 64, NVFP4_SR, 1, NVFP4_SR, 2, &nv, fb, fb, fb + 4, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_EALIGN);
    EXPECT(nvfp4_quantize_dual(fake, NVFP4_BF16, 64, 64, 64, NVFP4_SR, 1, NVFP4_SR, 2, &nv, fb, fb, fb, fb, ff, NVFP4_SLAB_ROWS, fake, 1 << 20, nullptr), NVFP4_ESHAPE);
    EXPECT(nvfp4_tensor_scale(fake, NVFP4_F32, 8, 8, 4, ff, fake, 1 << 20, nullptr), NVFP4_ESHAPE);
    EXPECT(nvfp4_gemm(64, 64, 48, &nv, fb, fb, fb, fb, ff, fake, NVFP4_F32, 64, nullptr), NVFP4_ESHAPE);
    EXPECT(nvfp4_gemm(64, 64, 64, &nv, fb, fb, fb, fb, ff, fake, NVFP4_F32, 8, nullptr), NVFP4_ESHAPE);
    EXPECT(nvfp4_gemm(0, 64, 64, &nv, fb, fb, fb, fb, ff, fake, NVFP4_F32, 64, nullptr), NVFP4_OK);
    EXPECT(nvfp4_gemm_slab(64, 64, 128, &nv, fb, fb, fb, fb, ff, fake, NVFP4_F32, 64, 1, 0, nullptr), NVFP4_EUNSUPPORTED);
    EXPECT(nvfp4_linear_fwd(fake, fake, fake, 64, 64, 64, NVFP4_BF16, NVFP4_BF16, &nv, nullptr, 0, nullptr, nullptr, nullptr, 0), NVFP4_EWORKSPACE);
    EXPECT(nvfp4_linear_fwd(fake, nullptr, fake, 64, 64, 64, NVFP4_BF16, NVFP4_BF16, &nv, fake, 1 << 30, nullptr, nullptr, nullptr, 0), NVFP4_EINVAL);
    EXPECT(nvfp4_linear_fwd(fake, fake, fake, 72, 64, 64, NVFP4_BF16, NVFP4_BF16, &nv, fake, 1 << 30, nullptr, nullptr, fake, 0), NVFP4_ESHAPE);
    EXPECT(nvfp4_linear_bwd(fake, nullptr, nullptr, fake, fake, 64, 64, 64, NVFP4_BF16, NVFP4_BF16, &nv, 0, fake, 1 << 30, nullptr, nullptr, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_linear_bwd(fake, fake, fake, fake, fake, 64, 72, 64, NVFP4_BF16, NVFP4_BF16, &nv, 0, fake, 1 << 30, nullptr, nullptr, nullptr), NVFP4_ESHAPE);
    EXPECT(nvfp4_quantize_weight(fake, NVFP4_BF16, 256, 72, 128, &nv, fake, fake, 1 << 20, nullptr), NVFP4_ESHAPE);
    EXPECT(nvfp4_linear_fwd_wq(fake, nullptr, fake, 64, 64, 64, NVFP4_BF16, NVFP4_BF16, &nv, fake, 1 << 30, nullptr, nullptr, nullptr, 0), NVFP4_EINVAL);
    EXPECT(nvfp4_linear_bwd_wq(fake, fake, nullptr, fake, fake, 64, 64, 64, NVFP4_BF16, NVFP4_BF16, &nv, 0, fake, 1 << 30, nullptr, nullptr, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quant_noise(fake, NVFP4_BF16, 64, 64, 64, 3, &nv, fb, fb, ff, reinterpret_cast<double *>(fake), fake, 1 << 20, nullptr), NVFP4_EINVAL);
    // enumeration arguments outside their enumerations, as a C caller or a foreign-function interface can pass them
    const nvfp4_dtype dt9 = static_cast<nvfp4_dtype>(9);
    const nvfp4_rounding rnd7 = static_cast<nvfp4_rounding>(7);
    EXPECT(nvfp4_quantize(fake, dt9, 64, 64, 64, 1, NVFP4_RTN, 0, &nv, fb, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quantize(fake, NVFP4_BF16, 64, 64, 64, 1, rnd7, 0, &nv, fb, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quantize_static(fake, dt9, 64, 64, 64, 1, NVFP4_RTN, 0, &nv, fb, fb, ff, NVFP4_PRESET_TSCALE, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quantize_dual(fake, NVFP4_BF16, 64, 64, 64, rnd7, 1, NVFP4_SR, 2, &nv, fb, fb, fb, fb, ff, 0, fake, 1 << 20, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_tensor_scale(fake, dt9, 8, 8, 8, ff, fake, 1 << 20, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_gemm(64, 64, 64, &nv, fb, fb, fb, fb, ff, fake, dt9, 64, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_linear_fwd(fake, fake, fake, 64, 64, 64, dt9, NVFP4_BF16, &nv, fake, 1 << 30, nullptr, nullptr, nullptr, 0), NVFP4_EINVAL);
    EXPECT(nvfp4_linear_bwd(fake, fake, fake, fake, fake, 64, 64, 64, NVFP4_BF16, dt9, &nv, 0, fake, 1 << 30, nullptr, nullptr, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quantize_weight(fake, dt9, 256, 128, 128, &nv, fake, fake, 1 << 20, nullptr), NVFP4_EINVAL);
    EXPECT(nvfp4_quant_noise(fake, dt9, 64, 64, 64, 1, &nv, fb, fb, ff, reinterpret_cast<double *>(fake), fake, 1 << 20, nullptr), NVFP4_EINVAL);
    double tf = 0.0;
    EXPECT(nvfp4_probe_mfma_rate(7, 0, 100, fake, 1 << 20, &tf, nullptr), NVFP4_EINVAL);
    const uint32_t before = nvfp4_cross_check_switches(0, 0);
    nvfp4_cross_check_switches(1, 0xFFFFFFFFu);
    if (nvfp4_cross_check_switches(1, before) != 7u) return 1;
    // host evaluations of the scalar steps, whole input ranges
    float m[97];
    uint32_t u[97];
    uint8_t o[97];
    for (int i = 0; i < 97; ++i) {
        m[i] = 6.0f * (float)i / 96.0f;
        u[i] = (uint32_t)(i * 677) & 0xFFFFu;
    }
    nvfp4_host_e4m3_encode_n(m, 97, o);
    nvfp4_host_round_rtn_n(m, 97, o);
    nvfp4_host_round_sr_n(m, u, 97, o);
    for (int b = 0; b < 256; ++b) (void)nvfp4_host_e4m3_decode((uint8_t)b);
    (void)nvfp4_host_e4m3_encode(1e30f);
    (void)nvfp4_host_e8m0_encode(1e-45f);
    (void)nvfp4_host_e8m0_encode(3e38f);
    (void)nvfp4_host_sr_bits(~0ull, ~0ull);
    const uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6};
    uint32_t r4[4];
    nvfp4_host_philox4x32_10(ctr, key, r4);
    printf("sanitize-api ok\n");
    return 0;
}
