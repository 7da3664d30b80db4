/* Driver for tests/test_oracle_sanitizers.py: calls every entry point of the CPU oracle on
 * heap buffers of EXACTLY the documented sizes, over many small and ragged shapes, so that a
 * build with -fsanitize=address,undefined reports any access outside a buffer, any signed
 * overflow, misaligned access or invalid shift in the oracle.  Prints "ok <calls>" on success. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int loco_ref_error_state_init(float *, size_t);
int loco_ref_compensate_quantize(const void *, int, float *, size_t, int, int, float, int, uint8_t *, float *);
int loco_ref_compensate_quantize_mt(const void *, int, float *, size_t, int, int, float, int, uint8_t *, float *, int);
int loco_ref_compensate_quantize_bf16_scales(const void *, int, float *, size_t, int, int, float, int, uint8_t *,
                                             uint16_t *);
int loco_ref_dequant_reduce(const uint8_t *, size_t, const float *, size_t, int, size_t, int, int, float *);
int loco_ref_dequant_reduce_mt(const uint8_t *, size_t, const float *, size_t, int, size_t, int, int, float *, int);
int loco_ref_dequant_reduce_bf16_scales(const uint8_t *, size_t, const uint16_t *, size_t, int, size_t, int, int,
                                        float *);
int loco_ref_fixed_compensate_quantize(const void *, int, int8_t *, size_t, int, int, int, float, int, uint8_t *);
int loco_ref_fixed_compensate_quantize_mt(const void *, int, int8_t *, size_t, int, int, int, float, int, uint8_t *,
                                          int);
int loco_ref_fixed_dequant_reduce(const uint8_t *, size_t, int, size_t, int, int, float *);
int loco_ref_fixed_dequant_reduce_mt(const uint8_t *, size_t, int, size_t, int, int, float *, int);
int loco_ref_clip_gradient(const void *, int, size_t, float, float *);
int loco_ref_sgd_update(float *, const float *, size_t, float);
int loco_ref_adam_update(float *, float *, float *, const float *, size_t, float, float, float, float);
int loco_ref_round_to_bf16(const float *, size_t, uint16_t *);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
static float rnd_float(void)
{   /* a spread of magnitudes, both signs, exact zeros, huge and subnormal values */
    uint32_t r = rnd();
    switch (r & 15u) {
    case 0: return 0.0f;
    case 1: return (r & 16u) ? 3.0e38f : -3.0e38f;
    case 2: return 1.0e-41f;
    default: return ((float)(int32_t)rnd() / 2147483648.0f) * (float)(1u << (r >> 28)) * 1.0e-4f;
    }
}
static void *exact(size_t bytes) { void *p = malloc(bytes ? bytes : 1); if (!p) abort(); memset(p, 0x5A, bytes); return p; }
#define CHECK(call) do { int rc_ = (call); if (rc_) { printf("FAILED %s -> %d (n=%zu bits=%d B=%d W=%d)\n", #call, rc_, n, bits, B, W); return 1; } ++calls; } while (0)

int main(void)
{
    static const size_t sizes[] = {1, 2, 3, 7, 8, 31, 32, 33, 63, 64, 65, 255, 256, 257, 511, 513, 1000, 1537, 4099};
    static const int blocks[] = {32, 64, 128, 256, 512};
    long calls = 0;
    for (size_t si = 0; si < sizeof sizes / sizeof *sizes; ++si)
        for (int bits = 4; bits <= 8; bits += 4)
            for (size_t bi = 0; bi < sizeof blocks / sizeof *blocks; ++bi)
                for (int dtype = 0; dtype <= 1; ++dtype) {
                    const size_t n = sizes[si];
                    const int B = blocks[bi];
                    const int W = 1 + (int)(rnd() % 5);
                    const size_t cb = (n * (size_t)bits + 7) / 8, nb = (n + (size_t)B - 1) / (size_t)B;
                    const size_t cstride = cb + (rnd() % 3), sstride = nb + (rnd() % 2);
                    void *grad = exact(n * (dtype ? 2 : 4));
                    for (size_t i = 0; i < n; ++i) {
                        float x = rnd_float();
                        if (dtype) { uint32_t u; memcpy(&u, &x, 4); ((uint16_t *)grad)[i] = (uint16_t)(u >> 16); }
                        else ((float *)grad)[i] = x;
                    }
                    float *err = exact(n * 4);
                    int8_t *err8 = exact(n);
                    uint8_t *codes = exact((size_t)(W - 1) * cstride + cb);
                    float *scales = exact(((size_t)(W - 1) * sstride + nb) * 4);
                    uint16_t *scales16 = exact(((size_t)(W - 1) * sstride + nb) * 2);
                    float *out = exact(n * 4), *clipped = exact(n * 4);
                    float *theta = exact(n * 4), *m = exact(n * 4), *v = exact(n * 4);
                    uint16_t *out16 = exact(n * 2);
                    for (size_t i = 0; i < n; ++i) { theta[i] = rnd_float(); m[i] = 0.0f; v[i] = 0.0f; err8[i] = (int8_t)rnd(); }
                    CHECK(loco_ref_error_state_init(err, n));
                    for (int w = 0; w < W; ++w) {
                        const int reset = (rnd() & 7u) == 0;
                        CHECK(loco_ref_compensate_quantize(grad, dtype, err, n, bits, B, 0.25f, reset,
                                                           codes + (size_t)w * cstride, scales + (size_t)w * sstride));
                        CHECK(loco_ref_compensate_quantize_mt(grad, dtype, err, n, bits, B, 0.3f, 0,
                                                              codes + (size_t)w * cstride, scales + (size_t)w * sstride, 3));
                    }
                    CHECK(loco_ref_dequant_reduce(codes, cstride, scales, sstride, W, n, bits, B, out));
                    CHECK(loco_ref_dequant_reduce_mt(codes, cstride, scales, sstride, W, n, bits, B, out, 3));
                    for (int w = 0; w < W; ++w)
                        CHECK(loco_ref_compensate_quantize_bf16_scales(grad, dtype, err, n, bits, B, 1.0f, 0,
                                                                       codes + (size_t)w * cstride,
                                                                       scales16 + (size_t)w * sstride));
                    CHECK(loco_ref_dequant_reduce_bf16_scales(codes, cstride, scales16, sstride, W, n, bits, B, out));
                    for (int w = 0; w < W; ++w) {
                        CHECK(loco_ref_fixed_compensate_quantize(grad, dtype, err8, n, bits, 19, 4 + 2 * (w & 1), 0.25f,
                                                                 (rnd() & 7u) == 0, codes + (size_t)w * cstride));
                        CHECK(loco_ref_fixed_compensate_quantize_mt(grad, dtype, err8, n, bits, -3, 6, 0.5f, 0,
                                                                    codes + (size_t)w * cstride, 3));
                    }
                    CHECK(loco_ref_fixed_dequant_reduce(codes, cstride, W, n, bits, 19, out));
                    CHECK(loco_ref_fixed_dequant_reduce_mt(codes, cstride, W, n, bits, 19, out, 3));
                    CHECK(loco_ref_clip_gradient(grad, dtype, n, 1.0e-3f, clipped));
                    CHECK(loco_ref_sgd_update(theta, clipped, n, 1.0e-2f));
                    CHECK(loco_ref_adam_update(theta, m, v, clipped, n, 1.0e-3f, 0.1f, 0.02f, 1.0e-8f));
                    CHECK(loco_ref_round_to_bf16(theta, n, out16));
                    free(grad); free(err); free(err8); free(codes); free(scales); free(scales16); free(out);
                    free(clipped); free(theta); free(m); free(v); free(out16);
                }
    printf("ok %ld\n", calls);
    return 0;
}
