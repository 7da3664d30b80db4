/* loco_traffic_probe -- drives the C ABI (include/loco.h) over one workload shape from a plain
 * C99 process, so that hardware counters (rocprofv3 --pmc) can be collected for the library's
 * kernels at a benchmark shape with nothing else in the process: a few hundred dispatches, no
 * Python.  The bytes a kernel moves do not depend on the values, so the gradient is a cheap
 * deterministic bell-shaped pattern, every peer's payload comes from that same gradient, and
 * nothing is checked here (parity is the tests' business).
 *
 *   loco_traffic_probe N BITS BLOCK WORKERS GRAD FORM OPT OUT SCALES CLIP STEPS
 *     GRAD bf16|f32   FORM block|fixed|fixed_f32   OPT none|sgd|adam   OUT f32|bf16
 *     SCALES f32|bf16   CLIP 0 (off) or the threshold   STEPS timed-like steps to run
 * It also runs the library's plain copy of 2 GiB three times: the calibration of the counters.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "loco.h"

#define HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { \
    fprintf(stderr, "HIP error %d (%s) at line %d\n", (int)e_, hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define LOCO(call) do { loco_status_t s_ = (call); if (s_ != LOCO_OK) { \
    fprintf(stderr, "%s -> %s (line %d)\n", #call, loco_status_string(s_), __LINE__); return 3; } } while (0)

enum { LOG2_S = 19, SE_MULT = 4 };

int main(int argc, char **argv)
{
    if (argc != 12) {
        fprintf(stderr, "usage: %s N BITS BLOCK WORKERS bf16|f32 block|fixed|fixed_f32 none|sgd|adam f32|bf16 f32|bf16 CLIP STEPS\n", argv[0]);
        return 1;
    }
    const size_t n = (size_t)strtoull(argv[1], NULL, 10);
    const int bits = atoi(argv[2]), B = atoi(argv[3]), W = atoi(argv[4]);
    const loco_dtype_t dtype = strcmp(argv[5], "bf16") == 0 ? LOCO_BF16 : LOCO_F32;
    const int fixed = strncmp(argv[6], "fixed", 5) == 0, fixed_f32 = strcmp(argv[6], "fixed_f32") == 0;
    const int sgd = strcmp(argv[7], "sgd") == 0, adam = strcmp(argv[7], "adam") == 0;
    const int out_bf16 = strcmp(argv[8], "bf16") == 0, scales_bf16 = strcmp(argv[9], "bf16") == 0;
    const float clip = (float)atof(argv[10]);
    const int steps = atoi(argv[11]);
    const float beta = 0.25f, eta = 1e-4f;
    const size_t gsz = dtype == LOCO_BF16 ? 2 : 4;
    const size_t cb = loco_code_bytes(n, bits), nb = fixed ? 1 : loco_num_blocks(n, B);
    const size_t cstride = (cb + 15) / 16 * 16;
    if (n == 0 || cb == 0 || W < 1 || steps < 1) { fprintf(stderr, "bad arguments\n"); return 1; }

    /* gradient: a 16 Mi-element pattern made on the host, replicated on the device */
    const size_t pat = n < ((size_t)1 << 24) ? n : ((size_t)1 << 24);
    void *pat_h = malloc(pat * gsz), *g_d, *err_d, *codes_d, *scales_d, *out_d, *m_d = NULL, *v_d = NULL;
    uint64_t lcg = 0x2407044802407044ull;
    size_t i;
    if (!pat_h) return 4;
    for (i = 0; i < pat; ++i) {
        float s = 0.0f, x;
        uint32_t u;
        int k;
        for (k = 0; k < 4; ++k) {
            lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
            s += (float)(uint32_t)(lcg >> 40) / 16777216.0f;
        }
        x = (s - 2.0f) * 1.7e-3f;
        memcpy(&u, &x, 4);
        if (dtype == LOCO_BF16) ((uint16_t *)pat_h)[i] = (uint16_t)(u >> 16);
        else ((float *)pat_h)[i] = x;
    }
    HIP(hipMalloc(&g_d, n * gsz));
    HIP(hipMalloc(&err_d, n * 4));
    HIP(hipMalloc(&codes_d, (size_t)W * cstride));
    HIP(hipMalloc(&scales_d, (size_t)W * nb * 4));
    HIP(hipMalloc(&out_d, n * 4));
    if (adam) { HIP(hipMalloc(&m_d, n * 4)); HIP(hipMalloc(&v_d, n * 4)); HIP(hipMemset(m_d, 0, n * 4)); HIP(hipMemset(v_d, 0, n * 4)); }
    HIP(hipMemset(out_d, 0, n * 4));
    HIP(hipMemcpy(g_d, pat_h, pat * gsz, hipMemcpyHostToDevice));
    for (i = pat; i < n; i += pat) {
        const size_t take = n - i < pat ? n - i : pat;
        HIP(hipMemcpy((char *)g_d + i * gsz, g_d, take * gsz, hipMemcpyDeviceToDevice));
    }

    /* one compensate-quantize into payload slot w, from the state in err_d */
#define COMPRESS(w) do { \
        uint8_t *c_ = (uint8_t *)codes_d + (size_t)(w) * cstride; \
        if (fixed_f32) LOCO(loco_compensate_quantize_fixed_f32state(g_d, dtype, (float *)err_d, n, bits, LOG2_S, beta, 0, c_, NULL)); \
        else if (fixed && clip > 0) LOCO(loco_compensate_quantize_fixed_clip(g_d, dtype, clip, (int8_t *)err_d, n, bits, LOG2_S, SE_MULT, beta, 0, c_, NULL)); \
        else if (fixed) LOCO(loco_compensate_quantize_fixed(g_d, dtype, (int8_t *)err_d, n, bits, LOG2_S, SE_MULT, beta, 0, c_, NULL)); \
        else if (scales_bf16) LOCO(loco_compensate_quantize_bf16_scales(g_d, dtype, (float *)err_d, n, bits, B, beta, 0, c_, (uint16_t *)scales_d + (size_t)(w) * nb, NULL)); \
        else if (clip > 0) LOCO(loco_compensate_quantize_clip(g_d, dtype, clip, (float *)err_d, n, bits, B, beta, 0, c_, (float *)scales_d + (size_t)(w) * nb, NULL)); \
        else LOCO(loco_compensate_quantize(g_d, dtype, (float *)err_d, n, bits, B, beta, 0, c_, (float *)scales_d + (size_t)(w) * nb, NULL)); \
    } while (0)
#define STATE_INIT() do { \
        if (fixed && !fixed_f32) LOCO(loco_error_state8_init((int8_t *)err_d, n, NULL)); \
        else LOCO(loco_error_state_init((float *)err_d, n, NULL)); \
    } while (0)

    int w, k;
    for (w = W - 1; w >= 0; --w) {      /* peers first; slot 0 last, so that err_d ends as this worker's state */
        STATE_INIT();
        COMPRESS(w);
    }
    for (k = 0; k < steps; ++k) {
        const uint8_t *c = (const uint8_t *)codes_d;
        const float *s = (const float *)scales_d;
        COMPRESS(0);
        if (fixed) {
            if (adam) LOCO(loco_dequant_reduce_fixed_adam(c, cstride, W, n, bits, LOG2_S, eta, 0.1f, 0.02f, 1e-8f, (float *)m_d, (float *)v_d, (float *)out_d, NULL));
            else if (sgd) LOCO(loco_dequant_reduce_fixed_sgd(c, cstride, W, n, bits, LOG2_S, eta, (float *)out_d, NULL));
            else if (out_bf16) LOCO(loco_dequant_reduce_fixed_bf16(c, cstride, W, n, bits, LOG2_S, (uint16_t *)out_d, NULL));
            else LOCO(loco_dequant_reduce_fixed(c, cstride, W, n, bits, LOG2_S, (float *)out_d, NULL));
        } else {
            if (scales_bf16) LOCO(loco_dequant_reduce_bf16_scales(c, cstride, (const uint16_t *)scales_d, nb, W, n, bits, B, (float *)out_d, NULL));
            else if (adam) LOCO(loco_dequant_reduce_adam(c, cstride, s, nb, W, n, bits, B, eta, 0.1f, 0.02f, 1e-8f, (float *)m_d, (float *)v_d, (float *)out_d, NULL));
            else if (sgd) LOCO(loco_dequant_reduce_sgd(c, cstride, s, nb, W, n, bits, B, eta, (float *)out_d, NULL));
            else if (out_bf16) LOCO(loco_dequant_reduce_bf16(c, cstride, s, nb, W, n, bits, B, (uint16_t *)out_d, NULL));
            else LOCO(loco_dequant_reduce(c, cstride, s, nb, W, n, bits, B, (float *)out_d, NULL));
        }
    }
    HIP(hipDeviceSynchronize());
    HIP(hipFree(g_d)); HIP(hipFree(err_d)); HIP(hipFree(codes_d)); HIP(hipFree(scales_d)); HIP(hipFree(out_d));
    if (adam) { HIP(hipFree(m_d)); HIP(hipFree(v_d)); }

    {   /* calibration: what the counters read for 2 GiB read and 2 GiB written */
        const size_t bytes = (size_t)1 << 31;
        void *a, *b;
        HIP(hipMalloc(&a, bytes));
        HIP(hipMalloc(&b, bytes));
        HIP(hipMemset(a, 0, bytes));
        for (k = 0; k < 3; ++k) LOCO(loco_stream_copy(b, a, bytes, NULL));
        HIP(hipDeviceSynchronize());
        HIP(hipFree(a)); HIP(hipFree(b));
    }
    free(pat_h);
    printf("probe ok: n=%zu bits=%d block=%d W=%d steps=%d\n", n, bits, B, W, steps);
    return 0;
}
