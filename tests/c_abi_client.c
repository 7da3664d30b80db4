/* A plain C99 client of the C ABI (include/loco.h): no Python, no C++, no torch.  It allocates
 * with the HIP runtime's C API, runs three steps of compensate-quantize and one dequant-reduce
 * over W payloads through the library, runs the CPU oracle (oracle/loco_ref.c, linked in) on
 * the same inputs, and compares every output byte.  Built by tests/test_c_client_gpu.py.
 * Exit status 0 and a last line "c client ok" mean success. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "loco.h"

/* the oracle's entry points (test infrastructure) */
int loco_ref_compensate_quantize(const void *, int, float *, size_t, int, int, float, int, uint8_t *, float *);
int loco_ref_dequant_reduce(const uint8_t *, size_t, const float *, size_t, int, size_t, int, int, float *);

#define HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    printf("HIP error %d (%s) at line %d\n", (int)e_, hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define LOCO(call) do { loco_status_t s_ = (call); if (s_ != LOCO_OK) { \
    printf("%s -> %s (line %d)\n", #call, loco_status_string(s_), __LINE__); return 3; } } while (0)

static uint64_t lcg = 0x2407044802407044ull;
static float next_gauss_like(void)
{   /* sum of four uniforms, centred: bell shaped, deterministic, no libm */
    float s = 0.0f;
    int k;
    for (k = 0; k < 4; ++k) {
        lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
        s += (float)(uint32_t)(lcg >> 40) / 16777216.0f;
    }
    return (s - 2.0f) * 1.7e-3f;
}

static int run_case(size_t n, int bits, int B, int W, loco_dtype_t dtype)
{
    const float beta = 0.25f;
    const size_t cb = loco_code_bytes(n, bits), nb = loco_num_blocks(n, B);
    const size_t cstride = (cb + 15) / 16 * 16 + 32, sstride = nb + 3;
    const size_t gsz = dtype == LOCO_BF16 ? 2 : 4;
    void *g_h = malloc(n * gsz);
    float *e_h = calloc(n, 4), *e_back = malloc(n * 4), *out_h = malloc(n * 4), *out_back = malloc(n * 4);
    uint8_t *codes_h = calloc(W * cstride, 1), *codes_back = malloc(W * cstride);
    float *scales_h = calloc(W * sstride, 4), *scales_back = malloc(W * sstride * 4);
    void *g_d, *e_d, *codes_d, *scales_d, *out_d;
    int w, step;
    size_t i;
    if (!g_h || !e_h || !e_back || !out_h || !out_back || !codes_h || !codes_back || !scales_h || !scales_back) return 4;
    HIP(hipMalloc(&g_d, n * gsz));
    HIP(hipMalloc(&e_d, n * 4));
    HIP(hipMalloc(&codes_d, W * cstride));
    HIP(hipMalloc(&scales_d, W * sstride * 4));
    HIP(hipMalloc(&out_d, n * 4));
    HIP(hipMemset(codes_d, 0, W * cstride));
    HIP(hipMemset(scales_d, 0, W * sstride * 4));
    for (w = 0; w < W; ++w) {
        LOCO(loco_error_state_init((float *)e_d, n, NULL));
        memset(e_h, 0, n * 4);
        for (step = 0; step < (w == 0 ? 3 : 1); ++step) {
            for (i = 0; i < n; ++i) {
                float x = next_gauss_like();
                if (dtype == LOCO_BF16) { uint32_t u; memcpy(&u, &x, 4); ((uint16_t *)g_h)[i] = (uint16_t)(u >> 16); }
                else ((float *)g_h)[i] = x;
            }
            HIP(hipMemcpy(g_d, g_h, n * gsz, hipMemcpyHostToDevice));
            LOCO(loco_compensate_quantize(g_d, dtype, (float *)e_d, n, bits, B, beta, 0,
                                          (uint8_t *)codes_d + w * cstride, (float *)scales_d + w * sstride, NULL));
            if (loco_ref_compensate_quantize(g_h, dtype == LOCO_BF16, e_h, n, bits, B, beta, 0,
                                             codes_h + w * cstride, scales_h + w * sstride)) return 5;
            HIP(hipDeviceSynchronize());
            HIP(hipMemcpy(e_back, e_d, n * 4, hipMemcpyDeviceToHost));
            if (memcmp(e_back, e_h, n * 4)) { printf("state differs (worker %d step %d)\n", w, step); return 6; }
        }
    }
    HIP(hipMemcpy(codes_back, codes_d, W * cstride, hipMemcpyDeviceToHost));
    HIP(hipMemcpy(scales_back, scales_d, W * sstride * 4, hipMemcpyDeviceToHost));
    if (memcmp(codes_back, codes_h, W * cstride)) { printf("codes differ\n"); return 7; }
    if (memcmp(scales_back, scales_h, W * sstride * 4)) { printf("block steps differ\n"); return 8; }
    LOCO(loco_dequant_reduce((const uint8_t *)codes_d, cstride, (const float *)scales_d, sstride, W, n, bits, B,
                             (float *)out_d, NULL));
    if (loco_ref_dequant_reduce(codes_h, cstride, scales_h, sstride, W, n, bits, B, out_h)) return 9;
    HIP(hipDeviceSynchronize());
    HIP(hipMemcpy(out_back, out_d, n * 4, hipMemcpyDeviceToHost));
    if (memcmp(out_back, out_h, n * 4)) { printf("averaged gradient differs\n"); return 10; }
    /* the library refuses a host pointer instead of launching on it */
    if (loco_error_state_init(e_h, n, NULL) != LOCO_ERR_BAD_POINTER) { printf("host pointer was not refused\n"); return 11; }
    HIP(hipFree(g_d)); HIP(hipFree(e_d)); HIP(hipFree(codes_d)); HIP(hipFree(scales_d)); HIP(hipFree(out_d));
    free(g_h); free(e_h); free(e_back); free(out_h); free(out_back); free(codes_h); free(codes_back);
    free(scales_h); free(scales_back);
    printf("n=%zu bits=%d B=%d W=%d %s: identical\n", n, bits, B, W, dtype == LOCO_BF16 ? "bf16" : "fp32");
    return 0;
}

int main(void)
{
    int rc;
    if ((rc = run_case(7 * 2048 + 333, 4, 256, 3, LOCO_BF16))) return rc;
    if ((rc = run_case(100003, 8, 64, 5, LOCO_F32))) return rc;
    if ((rc = run_case(513, 4, 32, 1, LOCO_F32))) return rc;
    printf("c client ok\n");
    return 0;
}
