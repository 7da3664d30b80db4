/*
 * loco_ref.c -- CPU oracle for LoCo's per-step local path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  Only the tests, the smoke check and the
 * cpu_baseline leg of the benchmark may build, load or call it; the product
 * library never does, and the two share no code.
 *
 * What it follows (LoCo, arXiv 2407.04480):
 *   Alg. 1 step 1 / Eq. 2   h = g + e~            (error state kept in fp32, so
 *                                                  decompressor(e) is the identity)
 *   Eq. 1 / Eq. 3           q = round_p-bit(h * s): nearest integer, clamped to
 *                           [-2^(p-1), 2^(p-1)-1]
 *   Alg. 1 step 2 / Eq. 1   d = float(q) / s
 *   Eq. 4                   delta = h - d
 *   Eq. 5                   e~' = (1-beta) e~ + beta delta,  e~_0 = 0
 *   Eq. 7                   periodic reset: the new state is 0
 *   Alg. 1 step 3 / Eq. 8   g~ = (1/N) sum_n decompressor(q^n)
 *
 * Readings taken where the paper is silent (each is listed in the design notes):
 *   - the scale is chosen per block of `block_size` consecutive elements:
 *     s_b = qmax / max|h| over the block, stored as the step D_b = max|h| / qmax;
 *     the compressor multiplies by r_b = 1 / D_b, the decompressor multiplies by D_b
 *     (the same D_b on the sender and on every receiver);
 *   - "nearest integer" ties go to the even integer (rintf in the default mode);
 *   - a block whose step would be zero or subnormal (D_b < FLT_MIN) stores
 *     D_b = +0 and all-zero codes, so the whole of h goes into the error;
 *   - 4-bit codes are two's complement nibbles, element 2j in the low nibble of
 *     byte j and element 2j+1 in the high nibble; a missing last nibble is 0;
 *     8-bit codes are int8;
 *   - all arithmetic is IEEE binary32, one rounding per written operation, the
 *     only fused operation being the fmaf of Eq. 5; the sum of Eq. 8 runs over
 *     the workers in index order and is multiplied by fl(1/N).
 * The precision is binary32, not binary64, because the codes are integers that
 * floating point decides and the error state feeds the next step's codes: both
 * sides have to take those decisions in the same precision.
 *
 * Pins (tests/test_oracle_pins.py): hand-worked dyadic example, exact
 * reconstruction d + delta = h, rounding bound of Lemma 5, closed form of the
 * Eq. 5 recurrence, beta = 1 (Eq. 4) and beta = 0, zero-error fixed point,
 * brute-force nearest level in binary64, the telescoping identity of Lemma 1,
 * the literal fixed-scale form of Eq. 1 at s = 2^19, reset, and Eq. 8 at N = 1.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC (see oracle/__init__.py).
 */
#include <float.h>
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

enum { LOCO_REF_OK = 0, LOCO_REF_BAD_ARG = 1 };
enum { LOCO_REF_F32 = 0, LOCO_REF_BF16 = 1 };

/* bf16 is the upper half of a binary32: widening is exact. */
static float grad_at(const void *grad, int dtype, size_t i)
{
    if (dtype == LOCO_REF_F32)
        return ((const float *)grad)[i];
    uint32_t bits = (uint32_t)((const uint16_t *)grad)[i] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

static int args_ok(size_t n, int bits, int block_size)
{
    (void)n;
    return (bits == 4 || bits == 8) && block_size >= 1;
}

/* e~_0 = 0 (below Eq. 5); also the hard form of the Eq. 7 reset. */
int loco_ref_error_state_init(float *err_state, size_t n)
{
    if (n && !err_state)
        return LOCO_REF_BAD_ARG;
    for (size_t i = 0; i < n; ++i)
        err_state[i] = 0.0f;
    return LOCO_REF_OK;
}

/*
 * Eq. 7 / Alg. 1 ("e_{k+1} = 0 if k % T_c = 0"): is step k one whose new state is zero?
 * The rule as printed fires at k = 0, T_c, 2 T_c, ...; a period of 0 or less never resets.
 */
int loco_ref_reset_due(long long step_index, long long reset_period)
{
    if (reset_period <= 0)
        return 0;
    long long remainder = step_index % reset_period;
    return remainder == 0;
}

/*
 * Alg. 1 steps 1-2 on the blocks [block_lo, block_hi) of one shard of n elements.
 * Blocks are independent, so any split into block ranges gives the same bytes;
 * with 4-bit codes a range must start at an even element index.
 */
static uint16_t bf16_nearest_even(float x);

/* scales_out (binary32 steps) or scales16_out (bf16 steps): exactly one is given. */
static int cq_blocks(const void *grad, int grad_dtype, float *err_state,
                     size_t n, int bits, int block_size, float beta, int reset,
                     uint8_t *codes_out, float *scales_out, uint16_t *scales16_out,
                     size_t block_lo, size_t block_hi)
{
    if (!args_ok(n, bits, block_size) || !(beta >= 0.0f && beta <= 1.0f))
        return LOCO_REF_BAD_ARG;
    if (grad_dtype != LOCO_REF_F32 && grad_dtype != LOCO_REF_BF16)
        return LOCO_REF_BAD_ARG;
    if (n && (!grad || !err_state || !codes_out || (!scales_out == !scales16_out)))
        return LOCO_REF_BAD_ARG;

    const int qmax = (1 << (bits - 1)) - 1; /* Eq. 1: range -2^(p-1) .. 2^(p-1)-1 */
    const int qmin = -(1 << (bits - 1));
    const size_t B = (size_t)block_size;
    const float one_minus_beta = 1.0f - beta;

    for (size_t b = block_lo; b < block_hi; ++b) {
        const size_t lo = b * B;
        const size_t hi = (lo + B < n) ? lo + B : n;
        if (lo >= n)
            break;

        /* block max of the compensated gradient h = g + e~ (Eq. 2) */
        float amax = 0.0f;
        for (size_t i = lo; i < hi; ++i) {
            float h = grad_at(grad, grad_dtype, i) + err_state[i];
            float ah = fabsf(h);
            if (ah > amax)
                amax = ah;
        }

        float D = amax / (float)qmax; /* the step 1/s_b */
        uint16_t D16 = 0;
        if (scales16_out) {           /* step kept in bf16: round it first, then use */
            D16 = bf16_nearest_even(D); /* the rounded value for everything below    */
            uint32_t wide = (uint32_t)D16 << 16;
            memcpy(&D, &wide, sizeof D);
        }
        float r = 0.0f;               /* s_b */
        int dead = D < FLT_MIN;       /* zero or subnormal step: nothing to encode */
        if (dead) {
            D = 0.0f;
            D16 = 0;
        } else {
            r = 1.0f / D;
        }
        if (scales16_out)
            scales16_out[b] = D16;
        else
            scales_out[b] = D;

        for (size_t i = lo; i < hi; ++i) {
            float e = err_state[i];
            float h = grad_at(grad, grad_dtype, i) + e; /* Eq. 2 */
            int q = 0;
            if (!dead) {
                q = (int)rintf(h * r); /* Eq. 1, 3: nearest integer ... */
                if (q > qmax)          /* ... within the p-bit range */
                    q = qmax;
                if (q < qmin)
                    q = qmin;
            }
            float d = (float)q * D;   /* decompressor, Eq. 1 */
            float delta = h - d;      /* Eq. 4 */
            float bd = beta * delta;
            err_state[i] = reset ? 0.0f : fmaf(one_minus_beta, e, bd); /* Eq. 5 / Eq. 7 */

            if (bits == 8) {
                codes_out[i] = (uint8_t)(int8_t)q;
            } else if ((i & 1) == 0) {
                codes_out[i >> 1] = (uint8_t)(q & 15);
            } else {
                codes_out[i >> 1] = (uint8_t)(codes_out[i >> 1] | ((q & 15) << 4));
            }
        }
    }
    return LOCO_REF_OK;
}

int loco_ref_compensate_quantize_blocks(const void *grad, int grad_dtype, float *err_state,
                                        size_t n, int bits, int block_size, float beta, int reset,
                                        uint8_t *codes_out, float *scales_out,
                                        size_t block_lo, size_t block_hi)
{
    return cq_blocks(grad, grad_dtype, err_state, n, bits, block_size, beta, reset, codes_out,
                     scales_out, 0, block_lo, block_hi);
}

/*
 * The same with the block steps stored in bf16 (2 bytes per block instead of 4).
 * D_b = max|h| / qmax is rounded to the nearest bf16 (ties to even) BEFORE it is
 * used: the compressor multiplies by 1 / D_b of the rounded step and the sender's
 * own decompressor uses the rounded step too, so sender and receivers still decode
 * with one and the same D_b (the premise of Lemma 1).  Rounding can shrink the step
 * by at most 2^-8 relative, so max|h| / D_b <= qmax / (1 - 2^-8) < qmax + 1/2 for
 * qmax <= 127: the largest element still rounds to qmax, nothing saturates.
 * The zero/subnormal test is made on the rounded step.
 */
int loco_ref_compensate_quantize_bf16_scales_blocks(const void *grad, int grad_dtype,
                                                    float *err_state, size_t n, int bits,
                                                    int block_size, float beta, int reset,
                                                    uint8_t *codes_out, uint16_t *scales16_out,
                                                    size_t block_lo, size_t block_hi)
{
    return cq_blocks(grad, grad_dtype, err_state, n, bits, block_size, beta, reset, codes_out,
                     0, scales16_out, block_lo, block_hi);
}

int loco_ref_compensate_quantize_bf16_scales(const void *grad, int grad_dtype, float *err_state,
                                             size_t n, int bits, int block_size, float beta,
                                             int reset, uint8_t *codes_out, uint16_t *scales16_out)
{
    if (!args_ok(n, bits, block_size))
        return LOCO_REF_BAD_ARG;
    size_t nb = (n + (size_t)block_size - 1) / (size_t)block_size;
    return cq_blocks(grad, grad_dtype, err_state, n, bits, block_size, beta, reset, codes_out,
                     0, scales16_out, 0, nb);
}

/* Alg. 1 steps 1-2 on a whole shard; err_state is read and overwritten. */
int loco_ref_compensate_quantize(const void *grad, int grad_dtype, float *err_state, size_t n,
                                 int bits, int block_size, float beta, int reset,
                                 uint8_t *codes_out, float *scales_out)
{
    if (!args_ok(n, bits, block_size))
        return LOCO_REF_BAD_ARG;
    size_t nb = (n + (size_t)block_size - 1) / (size_t)block_size;
    return loco_ref_compensate_quantize_blocks(grad, grad_dtype, err_state, n, bits, block_size,
                                               beta, reset, codes_out, scales_out, 0, nb);
}

static int code_at(const uint8_t *codes, int bits, size_t i)
{
    if (bits == 8)
        return (int)(int8_t)codes[i];
    int nib = (codes[i >> 1] >> (4 * (int)(i & 1))) & 15;
    return (nib ^ 8) - 8; /* two's complement nibble */
}

/*
 * Alg. 1 step 3 / Eq. 8 on the elements [elem_lo, elem_hi): decode every worker's
 * payload with that worker's block step and average in binary32.  Payload w is
 * codes + w*code_stride_bytes, scales + w*scale_stride_elems.
 */
static int dr_range(const uint8_t *codes, size_t code_stride_bytes,
                    const float *scales, const uint16_t *scales16, size_t scale_stride_elems,
                    int num_workers, size_t n, int bits, int block_size,
                    float *grad_out, size_t elem_lo, size_t elem_hi)
{
    if (!args_ok(n, bits, block_size) || num_workers < 1)
        return LOCO_REF_BAD_ARG;
    if (n && (!codes || (!scales == !scales16) || !grad_out))
        return LOCO_REF_BAD_ARG;
    if (elem_hi > n)
        elem_hi = n;
    const float inv = 1.0f / (float)num_workers;
    for (size_t i = elem_lo; i < elem_hi; ++i) {
        size_t b = i / (size_t)block_size;
        float acc = 0.0f;
        for (int w = 0; w < num_workers; ++w) {
            int q = code_at(codes + (size_t)w * code_stride_bytes, bits, i);
            float D;
            if (scales16) { /* bf16 step: widening is exact */
                uint32_t wide = (uint32_t)scales16[(size_t)w * scale_stride_elems + b] << 16;
                memcpy(&D, &wide, sizeof D);
            } else {
                D = scales[(size_t)w * scale_stride_elems + b];
            }
            float d = (float)q * D;
            acc = acc + d;
        }
        grad_out[i] = acc * inv;
    }
    return LOCO_REF_OK;
}

int loco_ref_dequant_reduce_range(const uint8_t *codes, size_t code_stride_bytes,
                                  const float *scales, size_t scale_stride_elems,
                                  int num_workers, size_t n, int bits, int block_size,
                                  float *grad_out, size_t elem_lo, size_t elem_hi)
{
    return dr_range(codes, code_stride_bytes, scales, 0, scale_stride_elems, num_workers, n, bits,
                    block_size, grad_out, elem_lo, elem_hi);
}

/* Eq. 8 over payloads whose block steps are bf16 (see the bf16-step compressor above). */
int loco_ref_dequant_reduce_bf16_scales_range(const uint8_t *codes, size_t code_stride_bytes,
                                              const uint16_t *scales16, size_t scale_stride_elems,
                                              int num_workers, size_t n, int bits, int block_size,
                                              float *grad_out, size_t elem_lo, size_t elem_hi)
{
    return dr_range(codes, code_stride_bytes, 0, scales16, scale_stride_elems, num_workers, n, bits,
                    block_size, grad_out, elem_lo, elem_hi);
}

int loco_ref_dequant_reduce_bf16_scales(const uint8_t *codes, size_t code_stride_bytes,
                                        const uint16_t *scales16, size_t scale_stride_elems,
                                        int num_workers, size_t n, int bits, int block_size,
                                        float *grad_out)
{
    return dr_range(codes, code_stride_bytes, 0, scales16, scale_stride_elems, num_workers, n, bits,
                    block_size, grad_out, 0, n);
}

int loco_ref_dequant_reduce(const uint8_t *codes, size_t code_stride_bytes, const float *scales,
                            size_t scale_stride_elems, int num_workers, size_t n, int bits,
                            int block_size, float *grad_out)
{
    return loco_ref_dequant_reduce_range(codes, code_stride_bytes, scales, scale_stride_elems,
                                         num_workers, n, bits, block_size, grad_out, 0, n);
}

/* ------------------------------------------------------------------------------------
 * The paper's literal form: one global scale s for the gradient codes and the error
 * state itself kept as 8-bit codes with scale s_e (Alg. 1 as printed; Eq. 1, 2, 3, 5, 7;
 * s = 2^19 or 2^17 and s_e = 4s or 6s in Sec. 3.1-3.2).
 *
 *   e^   = decompressor(e; s_e) = float(e) / s_e
 *   h    = g + e^                                              (Eq. 2)
 *   q    = round_p-bit(h * s), clamped to [-2^(p-1), 2^(p-1)-1] (Eq. 1, 3)
 *   d    = float(q) / s                                        (Alg. 1 step 2)
 *   e~'  = (1-beta) e^ + beta (h - d)                          (Eq. 5)
 *   e'   = 0 on a reset step, else round_8-bit(e~' * s_e)      (Eq. 7)
 *
 * Readings: s = 2^log2_s (the paper's values are powers of two, which makes h*s and
 * q/s exact); s_e = se_mult * s; only the 8-bit e is stored, so the "previous e~" of
 * Eq. 5 is its decoded value e^; the clamp is applied to the rounded float before the
 * conversion to an integer; ties to even; binary32 with one rounding per operation.
 * ---------------------------------------------------------------------------------- */
static int fixed_args_ok(int bits, int log2_s, int se_mult)
{
    return (bits == 4 || bits == 8) && log2_s >= -64 && log2_s <= 64 && se_mult >= 1 && se_mult <= 64;
}

static float clamp_round(float x, int lo, int hi)
{
    float t = rintf(x);
    if (t > (float)hi)
        t = (float)hi;
    if (t < (float)lo)
        t = (float)lo;
    return t;
}

int loco_ref_fixed_compensate_quantize_range(const void *grad, int grad_dtype, int8_t *err_state8,
                                             size_t n, int bits, int log2_s, int se_mult, float beta,
                                             int reset, uint8_t *codes_out, size_t elem_lo, size_t elem_hi)
{
    if (!fixed_args_ok(bits, log2_s, se_mult) || !(beta >= 0.0f && beta <= 1.0f))
        return LOCO_REF_BAD_ARG;
    if (grad_dtype != LOCO_REF_F32 && grad_dtype != LOCO_REF_BF16)
        return LOCO_REF_BAD_ARG;
    if (n && (!grad || !err_state8 || !codes_out))
        return LOCO_REF_BAD_ARG;
    if (elem_hi > n)
        elem_hi = n;
    const int qmax = (1 << (bits - 1)) - 1;
    const int qmin = -(1 << (bits - 1));
    const float s = ldexpf(1.0f, log2_s);
    const float s_e = (float)se_mult * s;
    const float one_minus_beta = 1.0f - beta;
    for (size_t i = elem_lo; i < elem_hi; ++i) {
        float e_hat = (float)err_state8[i] / s_e;            /* decompressor(e; s_e) */
        float h = grad_at(grad, grad_dtype, i) + e_hat;      /* Eq. 2 */
        int q = (int)clamp_round(h * s, qmin, qmax);         /* Eq. 1, 3 */
        float d = (float)q / s;                              /* decompressor(q; s) */
        float delta = h - d;                                 /* Eq. 4 */
        float bd = beta * delta;
        float e_new = fmaf(one_minus_beta, e_hat, bd);       /* Eq. 5 */
        int e8 = reset ? 0 : (int)clamp_round(e_new * s_e, -128, 127); /* Eq. 7 */
        err_state8[i] = (int8_t)e8;
        if (bits == 8) {
            codes_out[i] = (uint8_t)(int8_t)q;
        } else if ((i & 1) == 0) {
            codes_out[i >> 1] = (uint8_t)(q & 15);
        } else {
            codes_out[i >> 1] = (uint8_t)(codes_out[i >> 1] | ((q & 15) << 4));
        }
    }
    return LOCO_REF_OK;
}

int loco_ref_fixed_compensate_quantize(const void *grad, int grad_dtype, int8_t *err_state8, size_t n,
                                       int bits, int log2_s, int se_mult, float beta, int reset,
                                       uint8_t *codes_out)
{
    return loco_ref_fixed_compensate_quantize_range(grad, grad_dtype, err_state8, n, bits, log2_s,
                                                    se_mult, beta, reset, codes_out, 0, n);
}

/* ------------------------------------------------------------------------------------
 * The global scale s of Eq. 1 with the compensation error kept in high precision: the
 * ablation row without error compression (Table 9, Sec. 5.4 "Error compression").  Alg. 1
 * with decompressor(e; s_e) and compressor(.; s_e, 8) taken out:
 *   h    = g + e~                                              (Eq. 2)
 *   q    = round_p-bit(h * s), clamped                         (Eq. 1, 3)
 *   d    = float(q) / s
 *   e~'  = (1-beta) e~ + beta (h - d), or 0 on a reset step    (Eq. 5, Eq. 7)
 * Same readings as above (s a power of two, clamp on the rounded float, ties to even).
 * The payload is that of the 8-bit-state form, so Eq. 8 is loco_ref_fixed_dequant_reduce.
 * ---------------------------------------------------------------------------------- */
int loco_ref_fixed_compensate_quantize_f32state(const void *grad, int grad_dtype, float *err_state,
                                                size_t n, int bits, int log2_s, float beta, int reset,
                                                uint8_t *codes_out)
{
    if (!fixed_args_ok(bits, log2_s, 1) || !(beta >= 0.0f && beta <= 1.0f))
        return LOCO_REF_BAD_ARG;
    if (grad_dtype != LOCO_REF_F32 && grad_dtype != LOCO_REF_BF16)
        return LOCO_REF_BAD_ARG;
    if (n && (!grad || !err_state || !codes_out))
        return LOCO_REF_BAD_ARG;
    const int qmax = (1 << (bits - 1)) - 1;
    const int qmin = -(1 << (bits - 1));
    const float s = ldexpf(1.0f, log2_s);
    const float one_minus_beta = 1.0f - beta;
    for (size_t i = 0; i < n; ++i) {
        float e_old = err_state[i];                          /* high-precision e~_k, no decompression */
        float h = grad_at(grad, grad_dtype, i) + e_old;      /* Eq. 2 with the uncompressed state */
        int q = (int)clamp_round(h * s, qmin, qmax);         /* Eq. 1, 3 */
        float d_own = (float)q / s;                          /* own decompressor */
        float raw_err = h - d_own;                           /* Eq. 4 */
        float weighted = beta * raw_err;
        err_state[i] = reset ? 0.0f : fmaf(one_minus_beta, e_old, weighted);   /* Eq. 5, Eq. 7 */
        if (bits == 8) {
            codes_out[i] = (uint8_t)(int8_t)q;
        } else if ((i & 1) == 0) {
            codes_out[i >> 1] = (uint8_t)(q & 15);
        } else {
            codes_out[i >> 1] = (uint8_t)(codes_out[i >> 1] | ((q & 15) << 4));
        }
    }
    return LOCO_REF_OK;
}

/* Eq. 8 with the global scale: out = (sum_w float(q^w) / s) * (1/W), in worker order. */
int loco_ref_fixed_dequant_reduce_range(const uint8_t *codes, size_t code_stride_bytes, int num_workers,
                                        size_t n, int bits, int log2_s, float *grad_out,
                                        size_t elem_lo, size_t elem_hi)
{
    if (!fixed_args_ok(bits, log2_s, 1) || num_workers < 1)
        return LOCO_REF_BAD_ARG;
    if (n && (!codes || !grad_out))
        return LOCO_REF_BAD_ARG;
    if (elem_hi > n)
        elem_hi = n;
    const float s = ldexpf(1.0f, log2_s);
    const float inv = 1.0f / (float)num_workers;
    for (size_t i = elem_lo; i < elem_hi; ++i) {
        float acc = 0.0f;
        for (int w = 0; w < num_workers; ++w) {
            int q = code_at(codes + (size_t)w * code_stride_bytes, bits, i);
            float d = (float)q / s;
            acc = acc + d;
        }
        grad_out[i] = acc * inv;
    }
    return LOCO_REF_OK;
}

int loco_ref_fixed_dequant_reduce(const uint8_t *codes, size_t code_stride_bytes, int num_workers,
                                  size_t n, int bits, int log2_s, float *grad_out)
{
    return loco_ref_fixed_dequant_reduce_range(codes, code_stride_bytes, num_workers, n, bits, log2_s,
                                               grad_out, 0, n);
}

/* ------------------------------------------------------------------------------------
 * Element-wise clipping of the local gradient before step 1 (Sec. 5.2, MoE runs trained
 * from scratch; the threshold is the caller's, the paper states none):
 *   out_i = min(max(float(g_i), -c), c),  c > 0 (c = +inf leaves g unchanged).
 * The clipped gradient is fp32 (c need not be a bf16 value); feed it to the functions
 * above as an fp32 gradient.
 * ---------------------------------------------------------------------------------- */
int loco_ref_clip_gradient(const void *grad, int grad_dtype, size_t n, float clip_abs, float *out)
{
    if (grad_dtype != LOCO_REF_F32 && grad_dtype != LOCO_REF_BF16)
        return LOCO_REF_BAD_ARG;
    if (!(clip_abs > 0.0f) || (n && (!grad || !out)))
        return LOCO_REF_BAD_ARG;
    for (size_t i = 0; i < n; ++i) {
        float g = grad_at(grad, grad_dtype, i);
        if (g > clip_abs)
            g = clip_abs;
        if (g < -clip_abs)
            g = -clip_abs;
        out[i] = g;
    }
    return LOCO_REF_OK;
}

/* ------------------------------------------------------------------------------------
 * The optimizer steps that consume the averaged gradient g~ (Sec. 4).
 *   SGD (Eq. 9):           theta' = theta - eta g~
 *   Adam family (Eq. 10):  m'  = (1-beta1) m + beta1 g~
 *                          v'  = (1-beta2) v + beta2 g~^2        (Adam's second moment)
 *                          eta_k = eta / sqrt(v' + delta)         (the pre-conditioner v(.))
 *                          theta' = theta - eta_k m'
 * exactly as the paper writes them: no bias correction, delta inside the square root,
 * m_0 = v_0 = 0.  Binary32, one rounding per operation; the two moving averages are
 * written like Eq. 5, fmaf(1-beta, old, beta*new).
 * ---------------------------------------------------------------------------------- */
int loco_ref_sgd_update(float *theta, const float *g_avg, size_t n, float eta)
{
    if (n && (!theta || !g_avg))
        return LOCO_REF_BAD_ARG;
    for (size_t i = 0; i < n; ++i) {
        float step = eta * g_avg[i];
        theta[i] = theta[i] - step;
    }
    return LOCO_REF_OK;
}

int loco_ref_adam_update(float *theta, float *m, float *v, const float *g_avg, size_t n, float eta,
                         float beta1, float beta2, float delta)
{
    if (n && (!theta || !m || !v || !g_avg))
        return LOCO_REF_BAD_ARG;
    if (!(beta1 >= 0.0f && beta1 <= 1.0f) || !(beta2 >= 0.0f && beta2 <= 1.0f) || !(delta >= 0.0f))
        return LOCO_REF_BAD_ARG;
    const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
    for (size_t i = 0; i < n; ++i) {
        float g = g_avg[i];
        float b1g = beta1 * g;
        float m_new = fmaf(omb1, m[i], b1g);
        float g2 = g * g;
        float b2g2 = beta2 * g2;
        float v_new = fmaf(omb2, v[i], b2g2);
        float root = sqrtf(v_new + delta);
        float eta_k = eta / root;
        float step = eta_k * m_new;
        m[i] = m_new;
        v[i] = v_new;
        theta[i] = theta[i] - step;
    }
    return LOCO_REF_OK;
}

/* ------------------------------------------------------------------------------------
 * Averaged gradient handed on in bf16 (the paper trains in bf16, App. B.2): the fp32
 * result of Eq. 8 rounded to the nearest bf16, ties to even.  bf16 is the upper half of
 * a binary32, so rounding adds half an ulp of the kept part (0x7FFF plus the lowest kept
 * bit) and truncates; NaN stays NaN.
 * ---------------------------------------------------------------------------------- */
static uint16_t bf16_nearest_even(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) /* NaN: keep it one */
        return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

int loco_ref_round_to_bf16(const float *in, size_t n, uint16_t *out)
{
    if (n && (!in || !out))
        return LOCO_REF_BAD_ARG;
    for (size_t i = 0; i < n; ++i)
        out[i] = bf16_nearest_even(in[i]);
    return LOCO_REF_OK;
}
