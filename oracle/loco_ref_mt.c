/*
 * loco_ref_mt.c -- runs the CPU oracle of loco_ref.c on several host threads.
 *
 * TEST INFRASTRUCTURE ONLY (same rule as loco_ref.c).  Nothing is recomputed
 * here: each thread calls the oracle's own range function on a disjoint range.
 * Blocks (Alg. 1 steps 1-2) and elements (Eq. 8) are independent, so the bytes
 * written are the same as those of a single-threaded call.
 */
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>

int loco_ref_compensate_quantize_blocks(const void *, int, float *, size_t, int, int, float, int,
                                        uint8_t *, float *, size_t, size_t);
int loco_ref_dequant_reduce_range(const uint8_t *, size_t, const float *, size_t, int, size_t, int,
                                  int, float *, size_t, size_t);
int loco_ref_compensate_quantize_bf16_scales_blocks(const void *, int, float *, size_t, int, int, float,
                                                    int, uint8_t *, uint16_t *, size_t, size_t);
int loco_ref_dequant_reduce_bf16_scales_range(const uint8_t *, size_t, const uint16_t *, size_t, int,
                                              size_t, int, int, float *, size_t, size_t);
int loco_ref_fixed_compensate_quantize_range(const void *, int, int8_t *, size_t, int, int, int, float,
                                             int, uint8_t *, size_t, size_t);
int loco_ref_fixed_dequant_reduce_range(const uint8_t *, size_t, int, size_t, int, int, float *, size_t,
                                        size_t);

#define LOCO_REF_MAX_THREADS 256

typedef struct {
    int kind; /* 0 = compensate_quantize, 1 = dequant_reduce, 2 and 3 = their fixed-scale forms,
                 4 and 5 = their forms with bf16 block steps */
    uint16_t *scales16_out;
    const uint16_t *scales16;
    int8_t *err_state8;
    int log2_s, se_mult;
    const void *grad;
    int grad_dtype;
    float *err_state;
    size_t n;
    int bits, block_size;
    float beta;
    int reset;
    uint8_t *codes_out;
    float *scales_out;
    const uint8_t *codes;
    size_t code_stride;
    const float *scales;
    size_t scale_stride;
    int num_workers;
    float *grad_out;
    size_t lo, hi;
    int status;
} job_t;

static void *run_job(void *p)
{
    job_t *j = (job_t *)p;
    if (j->kind == 0)
        j->status = loco_ref_compensate_quantize_blocks(j->grad, j->grad_dtype, j->err_state, j->n,
                                                        j->bits, j->block_size, j->beta, j->reset,
                                                        j->codes_out, j->scales_out, j->lo, j->hi);
    else if (j->kind == 1)
        j->status = loco_ref_dequant_reduce_range(j->codes, j->code_stride, j->scales,
                                                  j->scale_stride, j->num_workers, j->n, j->bits,
                                                  j->block_size, j->grad_out, j->lo, j->hi);
    else if (j->kind == 2)
        j->status = loco_ref_fixed_compensate_quantize_range(j->grad, j->grad_dtype, j->err_state8, j->n,
                                                             j->bits, j->log2_s, j->se_mult, j->beta,
                                                             j->reset, j->codes_out, j->lo, j->hi);
    else if (j->kind == 4)
        j->status = loco_ref_compensate_quantize_bf16_scales_blocks(j->grad, j->grad_dtype, j->err_state,
                                                                    j->n, j->bits, j->block_size, j->beta,
                                                                    j->reset, j->codes_out,
                                                                    j->scales16_out, j->lo, j->hi);
    else if (j->kind == 5)
        j->status = loco_ref_dequant_reduce_bf16_scales_range(j->codes, j->code_stride, j->scales16,
                                                              j->scale_stride, j->num_workers, j->n,
                                                              j->bits, j->block_size, j->grad_out, j->lo,
                                                              j->hi);
    else
        j->status = loco_ref_fixed_dequant_reduce_range(j->codes, j->code_stride, j->num_workers, j->n,
                                                        j->bits, j->log2_s, j->grad_out, j->lo, j->hi);
    return 0;
}

static int run_split(job_t *proto, size_t units, size_t granule, int threads)
{
    if (threads < 1)
        threads = 1;
    if (threads > LOCO_REF_MAX_THREADS)
        threads = LOCO_REF_MAX_THREADS;
    pthread_t tid[LOCO_REF_MAX_THREADS];
    job_t jobs[LOCO_REF_MAX_THREADS];
    size_t per = (units + (size_t)threads - 1) / (size_t)threads;
    per = (per + granule - 1) / granule * granule; /* keep range starts on a granule */
    int used = 0;
    for (int t = 0; t < threads; ++t) {
        size_t lo = (size_t)t * per;
        if (lo >= units && t > 0)
            break;
        size_t hi = lo + per < units ? lo + per : units;
        jobs[t] = *proto;
        jobs[t].lo = lo;
        jobs[t].hi = hi;
        jobs[t].status = 0;
        if (pthread_create(&tid[t], 0, run_job, &jobs[t]) != 0) {
            run_job(&jobs[t]); /* no thread to be had: do the range here */
            tid[t] = pthread_self();
        }
        used = t + 1;
    }
    int status = 0;
    for (int t = 0; t < used; ++t) {
        if (!pthread_equal(tid[t], pthread_self()))
            pthread_join(tid[t], 0);
        if (jobs[t].status)
            status = jobs[t].status;
    }
    return status;
}

int loco_ref_compensate_quantize_mt(const void *grad, int grad_dtype, float *err_state, size_t n,
                                    int bits, int block_size, float beta, int reset,
                                    uint8_t *codes_out, float *scales_out, int threads)
{
    if (block_size < 1)
        return 1;
    job_t j = {0};
    j.kind = 0;
    j.grad = grad;
    j.grad_dtype = grad_dtype;
    j.err_state = err_state;
    j.n = n;
    j.bits = bits;
    j.block_size = block_size;
    j.beta = beta;
    j.reset = reset;
    j.codes_out = codes_out;
    j.scales_out = scales_out;
    size_t nb = (n + (size_t)block_size - 1) / (size_t)block_size;
    /* two blocks per granule: a range then starts at an even element index,
       which 4-bit packing needs when block_size is odd */
    return run_split(&j, nb, 2, threads);
}

int loco_ref_dequant_reduce_mt(const uint8_t *codes, size_t code_stride_bytes, const float *scales,
                               size_t scale_stride_elems, int num_workers, size_t n, int bits,
                               int block_size, float *grad_out, int threads)
{
    job_t j = {0};
    j.kind = 1;
    j.codes = codes;
    j.code_stride = code_stride_bytes;
    j.scales = scales;
    j.scale_stride = scale_stride_elems;
    j.num_workers = num_workers;
    j.n = n;
    j.bits = bits;
    j.block_size = block_size;
    j.grad_out = grad_out;
    return run_split(&j, n, 64, threads);
}

int loco_ref_fixed_compensate_quantize_mt(const void *grad, int grad_dtype, int8_t *err_state8, size_t n,
                                          int bits, int log2_s, int se_mult, float beta, int reset,
                                          uint8_t *codes_out, int threads)
{
    job_t j = {0};
    j.kind = 2;
    j.grad = grad;
    j.grad_dtype = grad_dtype;
    j.err_state8 = err_state8;
    j.n = n;
    j.bits = bits;
    j.log2_s = log2_s;
    j.se_mult = se_mult;
    j.beta = beta;
    j.reset = reset;
    j.codes_out = codes_out;
    return run_split(&j, n, 64, threads);
}

int loco_ref_fixed_dequant_reduce_mt(const uint8_t *codes, size_t code_stride_bytes, int num_workers,
                                     size_t n, int bits, int log2_s, float *grad_out, int threads)
{
    job_t j = {0};
    j.kind = 3;
    j.codes = codes;
    j.code_stride = code_stride_bytes;
    j.num_workers = num_workers;
    j.n = n;
    j.bits = bits;
    j.log2_s = log2_s;
    j.grad_out = grad_out;
    return run_split(&j, n, 64, threads);
}

int loco_ref_compensate_quantize_bf16_scales_mt(const void *grad, int grad_dtype, float *err_state,
                                                size_t n, int bits, int block_size, float beta,
                                                int reset, uint8_t *codes_out, uint16_t *scales16_out,
                                                int threads)
{
    if (block_size < 1)
        return 1;
    job_t j = {0};
    j.kind = 4;
    j.grad = grad;
    j.grad_dtype = grad_dtype;
    j.err_state = err_state;
    j.n = n;
    j.bits = bits;
    j.block_size = block_size;
    j.beta = beta;
    j.reset = reset;
    j.codes_out = codes_out;
    j.scales16_out = scales16_out;
    size_t nb = (n + (size_t)block_size - 1) / (size_t)block_size;
    return run_split(&j, nb, 2, threads);
}

int loco_ref_dequant_reduce_bf16_scales_mt(const uint8_t *codes, size_t code_stride_bytes,
                                           const uint16_t *scales16, size_t scale_stride_elems,
                                           int num_workers, size_t n, int bits, int block_size,
                                           float *grad_out, int threads)
{
    job_t j = {0};
    j.kind = 5;
    j.codes = codes;
    j.code_stride = code_stride_bytes;
    j.scales16 = scales16;
    j.scale_stride = scale_stride_elems;
    j.num_workers = num_workers;
    j.n = n;
    j.bits = bits;
    j.block_size = block_size;
    j.grad_out = grad_out;
    return run_split(&j, n, 64, threads);
}
