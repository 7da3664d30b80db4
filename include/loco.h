/*
 * loco.h -- C ABI of the MI355X (gfx950) library for LoCo's per-step local path.
 *
 * LoCo (arXiv 2407.04480), Algorithm 1: every step each worker adds its error
 * state to the fresh gradient, compresses the sum to p-bit integers, keeps a
 * moving average of the compression error, and, after the low-bit payloads have
 * been exchanged, decodes and averages the N payloads it received.  This
 * library holds the two element-wise passes of that step and the state's
 * initialisation; the exchange itself, the optimizer and everything else are
 * the caller's.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers on the current HIP device (memory of another
 *     device is refused with LOCO_ERR_BAD_POINTER while pointer checks are on); the caller
 *     owns every buffer.  The library allocates nothing, frees nothing and never
 *     synchronises: work is enqueued on `stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and is ordered by it.
 *   - Sizes are in elements unless a name says bytes; n may exceed 2^31.
 *   - Buffers must not overlap, except that err_state is updated in place.
 *   - Inputs must be finite; NaN and infinities are not checked and give
 *     unspecified codes.
 *   - Errors are returned, never thrown; on an error nothing has been enqueued.
 *     n == 0 is LOCO_OK and enqueues nothing.
 *   - By default each call checks that every device buffer lies inside one
 *     allocation known to the HIP runtime (loco_set_pointer_checks).
 *
 * Payload format (the paper leaves scale granularity and packing open; Eq. 1 is
 * applied per block of block_size consecutive elements):
 *   scales[b] = D_b = max|h| / qmax over block b, fp32, qmax = 2^(bits-1) - 1;
 *               +0 for a block whose D_b would be zero or subnormal
 *   code q_i  = clamp(rint(h_i * (1/D_b)), -2^(bits-1), qmax), ties to even
 *   bits = 8:   codes[i] = (int8) q_i
 *   bits = 4:   codes[i/2] holds q_i as a two's complement nibble, even i in the low
 *               nibble, odd i in the high nibble; an unused last nibble is 0
 *   decode:     d_i = (float) q_i * D_b
 */
#ifndef LOCO_H
#define LOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LOCO_OK = 0,
    LOCO_ERR_INVALID_ARG = 1, /* NULL pointer, beta outside [0,1] or NaN, W < 1, stride too small, or so
                                 large that W payloads would not fit the address space */
    LOCO_ERR_UNSUPPORTED = 2, /* bits, block_size, dtype, worker count or decomposition outside the supported
                                 sets; more than 2^48 elements, or more workgroups than one launch holds */
    LOCO_ERR_ALIGNMENT = 3,   /* a pointer or stride breaks the alignment rule of the call */
    LOCO_ERR_LAUNCH = 4,      /* the HIP runtime refused the launch */
    LOCO_ERR_BAD_POINTER = 5  /* a buffer is not device memory, or too small for the call */
} loco_status_t;

typedef enum { LOCO_F32 = 0, LOCO_BF16 = 1 } loco_dtype_t;

/* Short text for a status code; static storage. */
const char *loco_status_string(loco_status_t status);

/* Bytes of packed codes for n elements: ceil(n * bits / 8).  0 if bits is not 4 or 8. */
size_t loco_code_bytes(size_t n, int bits);

/* Number of blocks (= number of fp32 scales) for n elements: ceil(n / block_size). */
size_t loco_num_blocks(size_t n, int block_size);

/* 1 (default): validate device buffers against the runtime's allocation table on
 * every call (a few microseconds of host time).  0: trust the caller.  Returns the
 * previous setting.  Process-wide. */
int loco_set_pointer_checks(int enabled);

/*
 * e~_0 = 0 (stated below Eq. 5); also the hard form of the periodic reset of Eq. 7.
 *   err_state  [n] fp32, device, 16-byte aligned; overwritten with +0.
 * Uses a fill kernel, so the call may be captured into a HIP graph.
 */
loco_status_t loco_error_state_init(float *err_state, size_t n, void *stream);

/*
 * Algorithm 1, steps 1 and 2, fused into one pass over the shard:
 *   h   = g + e~                      (Eq. 2; the state is fp32, so no decompression)
 *   q   = compressor(h; s_b, bits)    (Eq. 1, Eq. 3; per-block scale, see above)
 *   d   = decompressor(q; s_b)        (Eq. 1)
 *   e~' = (1-beta) e~ + beta (h - d)  (Eq. 4, Eq. 5), or 0 when reset != 0 (Eq. 7)
 *
 *   grad        [n] device, LOCO_F32 or LOCO_BF16, read only, 16-byte aligned
 *   err_state   [n] fp32 device, read and overwritten in place, 16-byte aligned
 *   bits        4 or 8
 *   block_size  32, 64, 128, 256 or 512
 *   beta        moving-average coefficient of Eq. 5, 0 <= beta <= 1
 *   reset       non-zero on a step where Eq. 7 zeroes the state: codes and scales are
 *               still those of the old state, the state written is +0
 *   codes_out   [loco_code_bytes(n, bits)] device, 16-byte aligned
 *   scales_out  [loco_num_blocks(n, block_size)] fp32 device, 4-byte aligned
 * The arithmetic is IEEE binary32 with one rounding per operation (Eq. 5 is
 * fmaf(1-beta, e~, beta*(h-d))), so codes, scales and state are reproducible bit
 * for bit.
 * Performance note.  Any 16-byte aligned placement of the buffers runs at the full rate: the
 * order in which the tiles are handed to the chip follows the address of err_state, not its
 * element index, so a state that is a slice of a larger buffer costs nothing.
 */
loco_status_t loco_compensate_quantize(const void *grad, loco_dtype_t grad_dtype,
                                       float *err_state, size_t n, int bits, int block_size,
                                       float beta, int reset, uint8_t *codes_out,
                                       float *scales_out, void *stream);

/*
 * Algorithm 1, step 3 / Eq. 8: decode the payloads of W workers and average them in
 * fp32:  out_i = (sum_{w=0}^{W-1} (float) q^w_i * D^w_b) * (1/W), summed in worker order.
 *
 * Payload w is at codes + w*code_stride_bytes and scales + w*scale_stride_elems, the
 * layout of an all-to-all receive buffer (Sec. 3.3).
 *   codes               device, 16-byte aligned; code_stride_bytes a multiple of 16 and
 *                       >= loco_code_bytes(n, bits) (ignored when W == 1)
 *   scales              fp32 device; scale_stride_elems >= loco_num_blocks(n, block_size)
 *   num_workers         W >= 1 (N of Eq. 8)
 *   bits, block_size    as for loco_compensate_quantize
 *   grad_out            [n] fp32 device, overwritten, 16-byte aligned
 * Performance notes.  Strides that are multiples of 256 bytes (code_stride_bytes, and
 * 4 * scale_stride_elems) keep every wavefront load inside its cache lines; a code stride that is only
 * 16-byte aligned costs about a tenth of the rate.  A wavefront reads the same position of all W
 * payloads at once: when the strides are multiples of a large power of two (a shard of exactly 2^k
 * elements laid out back to back), those W reads meet in one memory channel and the call can lose up
 * to a quarter of its rate for W >= 32; padding each payload by a few hundred bytes avoids it.  A shard
 * length that is not a multiple of the tile costs nothing measurable, and neither does a grad_out that
 * is a slice of a larger buffer (the tile order follows its address).
 */
loco_status_t loco_dequant_reduce(const uint8_t *codes, size_t code_stride_bytes,
                                  const float *scales, size_t scale_stride_elems,
                                  int num_workers, size_t n, int bits, int block_size,
                                  float *grad_out, void *stream);

/*
 * Algorithm 1, steps 1 and 2, with the reset schedule of Eq. 7 evaluated on the device:
 * the kernel reads the step index k from device memory and zeroes the state when
 * reset_period > 0 and k % reset_period == 0 (Algorithm 1: "e_{k+1} = 0 if k % T_c = 0";
 * T_c = 512 or 1024 in Sec. 3.2).  Nothing about the step is baked into the launch, so one
 * captured HIP graph of a training step can be replayed across reset steps while another
 * node advances the counter (loco_step_index_advance).
 *   step_index_dev  one int64 in device memory, 8-byte aligned, read only; k >= 0
 *   reset_period    T_c >= 0; 0 means the state is never reset
 * Everything else as loco_compensate_quantize; the step index must not change while the
 * call's kernel runs (stream order with the call that advances it is enough).
 */
loco_status_t loco_compensate_quantize_scheduled(const void *grad, loco_dtype_t grad_dtype,
                                                 float *err_state, size_t n, int bits, int block_size,
                                                 float beta, const int64_t *step_index_dev,
                                                 int64_t reset_period, uint8_t *codes_out,
                                                 float *scales_out, void *stream);

/*
 * The step counter k of Algorithm 1 kept in device memory for the _scheduled calls.
 *   loco_step_index_set      k = value
 *   loco_step_index_advance  k = k + 1
 * One small kernel each (no memset, no host write), so both may be captured into a HIP
 * graph.  step_index_dev: one int64, device, 8-byte aligned.
 */
loco_status_t loco_step_index_set(int64_t *step_index_dev, int64_t value, void *stream);
loco_status_t loco_step_index_advance(int64_t *step_index_dev, void *stream);

/* ------------------------------------------------------------------------------------
 * Algorithm 1 exactly as printed: one global scale s for the gradient codes and the error
 * state itself kept as 8-bit codes (Eq. 1-3, 5, 7; s = 2^19 or 2^17, s_e = 4s or 6s in
 * Sec. 3.1-3.2).  No scales array; 4.5 bytes per element with a bf16 gradient and p = 4.
 *   s   = 2^log2_s, -64 <= log2_s <= 64 (the paper's values are powers of two)
 *   s_e = se_mult * s, 1 <= se_mult <= 64
 * Same conventions as above (device pointers, caller-owned buffers, stream order, status).
 * ---------------------------------------------------------------------------------- */

/* 1 when step k is a reset step of Eq. 7 (k % reset_period == 0, reset_period > 0), else 0. */
int loco_reset_due(long long step_index, long long reset_period);

/* e_0 = 0 for the 8-bit error state.  err_state8: [n] int8 device, 16-byte aligned. */
loco_status_t loco_error_state8_init(int8_t *err_state8, size_t n, void *stream);

/*
 * Algorithm 1, steps 1 and 2 with the global scale:
 *   e^  = decompressor(e; s_e) = float(e) / s_e
 *   h   = g + e^                                        (Eq. 2)
 *   q   = round_p-bit(h * s), clamped to the p-bit range (Eq. 1, 3), packed as above
 *   d   = float(q) / s
 *   e~' = (1-beta) e^ + beta (h - d)                     (Eq. 5 on the decoded state)
 *   e'  = round_8-bit(e~' * s_e), or 0 when reset != 0   (Eq. 7)
 *
 *   grad         [n] device, LOCO_F32 or LOCO_BF16, read only, 16-byte aligned
 *   err_state8   [n] int8 device, read and overwritten in place, 16-byte aligned
 *   bits         4 or 8
 *   codes_out    [loco_code_bytes(n, bits)] device, 16-byte aligned
 */
loco_status_t loco_compensate_quantize_fixed(const void *grad, loco_dtype_t grad_dtype,
                                             int8_t *err_state8, size_t n, int bits, int log2_s,
                                             int se_mult, float beta, int reset, uint8_t *codes_out,
                                             void *stream);

/*
 * The same compressor with the compensation error kept in high precision: Algorithm 1 without
 * decompressor(e; s_e) and compressor(.; s_e, 8), which is the paper's ablation row without error
 * compression (Table 9, Sec. 5.4):
 *   h = g + e~;  q, d as above;  e~' = (1-beta) e~ + beta (h - d), or 0 when reset != 0.
 *   err_state    [n] fp32 device, read and overwritten in place, 16-byte aligned
 * Other arguments as for loco_compensate_quantize_fixed; the payload is the same, so the receive
 * side is loco_dequant_reduce_fixed.  State of the same type as loco_error_state_init writes.
 */
loco_status_t loco_compensate_quantize_fixed_f32state(const void *grad, loco_dtype_t grad_dtype,
                                                      float *err_state, size_t n, int bits, int log2_s,
                                                      float beta, int reset, uint8_t *codes_out,
                                                      void *stream);

/*
 * The two calls above with Eq. 7's schedule read from device memory, as
 * loco_compensate_quantize_scheduled: reset when reset_period > 0 and k % reset_period == 0.
 */
loco_status_t loco_compensate_quantize_fixed_scheduled(const void *grad, loco_dtype_t grad_dtype,
                                                       int8_t *err_state8, size_t n, int bits, int log2_s,
                                                       int se_mult, float beta, const int64_t *step_index_dev,
                                                       int64_t reset_period, uint8_t *codes_out, void *stream);
loco_status_t loco_compensate_quantize_fixed_f32state_scheduled(const void *grad, loco_dtype_t grad_dtype,
                                                                float *err_state, size_t n, int bits,
                                                                int log2_s, float beta,
                                                                const int64_t *step_index_dev,
                                                                int64_t reset_period, uint8_t *codes_out,
                                                                void *stream);

/*
 * Algorithm 1, step 3 / Eq. 8 with the global scale:
 *   out_i = (sum_{w=0}^{W-1} float(q^w_i) / s) * (1/W)
 * Payload w is at codes + w*code_stride_bytes (a multiple of 16, >= loco_code_bytes(n, bits);
 * ignored when W == 1).  grad_out: [n] fp32 device, 16-byte aligned.
 * The codes are summed as integers and converted once, which equals the binary32 sum in
 * worker order as long as every partial sum stays below 2^24: num_workers <= 2^21 (4 bits)
 * or 2^17 (8 bits); more is LOCO_ERR_UNSUPPORTED.  The same bound holds for the _bf16, _sgd
 * and _adam forms of this call.
 */
loco_status_t loco_dequant_reduce_fixed(const uint8_t *codes, size_t code_stride_bytes, int num_workers,
                                        size_t n, int bits, int log2_s, float *grad_out, void *stream);

/*
 * Element-wise clipping of the local gradient fused in front of step 1 (the paper's
 * MoE-from-scratch runs clip g "to reduce sensitivity to s", Sec. 5.2; no threshold is given):
 *   g' = min(max(g, -clip_abs), clip_abs), then exactly as the call without _clip.
 * clip_abs > 0; +infinity means no clipping and is what the plain calls pass.
 */
loco_status_t loco_compensate_quantize_clip(const void *grad, loco_dtype_t grad_dtype, float clip_abs,
                                            float *err_state, size_t n, int bits, int block_size,
                                            float beta, int reset, uint8_t *codes_out, float *scales_out,
                                            void *stream);
loco_status_t loco_compensate_quantize_fixed_clip(const void *grad, loco_dtype_t grad_dtype, float clip_abs,
                                                  int8_t *err_state8, size_t n, int bits, int log2_s,
                                                  int se_mult, float beta, int reset, uint8_t *codes_out,
                                                  void *stream);

/*
 * The optimizer step that consumes the averaged gradient g~ of Eq. 8, fused into the reduce
 * so that g~ is never written to memory and read back (saves 8 bytes per element):
 *   _sgd   Eq. 9:   theta' = theta - eta g~
 *   _adam  Eq. 10 with Adam's pre-conditioner, exactly as written in Sec. 4 (no bias
 *          correction, delta inside the root, m_0 = v_0 = 0):
 *            m' = (1-beta1) m + beta1 g~,  v' = (1-beta2) v + beta2 g~^2,
 *            theta' = theta - (eta / sqrt(v' + delta)) m'
 * theta, m, v: [n] fp32 device, 16-byte aligned, updated in place.  eta finite;
 * 0 <= beta1, beta2 <= 1; 0 <= delta < inf.  Payload arguments as for the plain reduce.
 * Binary32, one rounding per operation, correctly rounded square root and division.
 */
loco_status_t loco_dequant_reduce_sgd(const uint8_t *codes, size_t code_stride_bytes, const float *scales,
                                      size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                      int block_size, float eta, float *theta, void *stream);
loco_status_t loco_dequant_reduce_adam(const uint8_t *codes, size_t code_stride_bytes, const float *scales,
                                       size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                       int block_size, float eta, float beta1, float beta2, float delta,
                                       float *m, float *v, float *theta, void *stream);
loco_status_t loco_dequant_reduce_fixed_sgd(const uint8_t *codes, size_t code_stride_bytes, int num_workers,
                                            size_t n, int bits, int log2_s, float eta, float *theta,
                                            void *stream);
loco_status_t loco_dequant_reduce_fixed_adam(const uint8_t *codes, size_t code_stride_bytes, int num_workers,
                                             size_t n, int bits, int log2_s, float eta, float beta1,
                                             float beta2, float delta, float *m, float *v, float *theta,
                                             void *stream);

/*
 * Eq. 8 with the averaged gradient handed on in bf16 (the paper trains in bf16, App. B.2):
 * the fp32 average rounded to the nearest bf16, ties to even; 2 bytes per element written
 * instead of 4.  grad_out_bf16: [n] bf16 bit patterns, device, 16-byte aligned.
 */
loco_status_t loco_dequant_reduce_bf16(const uint8_t *codes, size_t code_stride_bytes, const float *scales,
                                       size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                       int block_size, uint16_t *grad_out_bf16, void *stream);
loco_status_t loco_dequant_reduce_fixed_bf16(const uint8_t *codes, size_t code_stride_bytes, int num_workers,
                                             size_t n, int bits, int log2_s, uint16_t *grad_out_bf16,
                                             void *stream);

/*
 * Algorithm 1 with the block steps kept in bf16 (2 bytes per block instead of 4;
 * the paper's Eq. 1 has one global s and no per-block steps at all, so the step
 * format is this library's choice).  The step D_b = max|h| / qmax is rounded to
 * the nearest bf16 (ties to even) BEFORE use: compressor (Eq. 1, Eq. 3), the
 * sender's own decompressor (Eq. 4) and every receiver (Eq. 8) work with the
 * stored value, so the error feedback of Eq. 5 still sees exactly what the
 * receivers decode.  The zero/subnormal test is made on the rounded step.
 * Arguments as in loco_compensate_quantize / loco_dequant_reduce except that the
 * steps are uint16_t bf16 bit patterns (scales_out_bf16 2-byte aligned, so a
 * payload may be written anywhere into a receive buffer; the reduce wants the
 * base of that buffer 4-byte aligned, stride in elements of any parity).
 * The reduce may read the whole aligned 32-bit word that holds a step, i.e. up to 2 bytes
 * past an array with an odd number of steps; it never writes there, and the word lies in
 * the same allocation granule as the last step.
 */
loco_status_t loco_compensate_quantize_bf16_scales(const void *grad, loco_dtype_t grad_dtype, float *err_state,
                                                   size_t n, int bits, int block_size, float beta, int reset,
                                                   uint8_t *codes_out, uint16_t *scales_out_bf16, void *stream);
loco_status_t loco_dequant_reduce_bf16_scales(const uint8_t *codes, size_t code_stride_bytes,
                                              const uint16_t *scales_bf16, size_t scale_stride_elems,
                                              int num_workers, size_t n, int bits, int block_size,
                                              float *grad_out, void *stream);

/*
 * Measurement aid: loco_compensate_quantize (bits = 4 only) with the codes gathered in LDS and
 * written as 16-byte stores from a few lanes instead of 2-byte stores from every lane; same
 * arithmetic, same bytes.  It exists so that the comparison of the two store shapes can be
 * repeated (the direct stores are 1-2 % faster and are what loco_compensate_quantize uses).
 */
loco_status_t loco_compensate_quantize_staged_codes(const void *grad, loco_dtype_t grad_dtype,
                                                    float *err_state, size_t n, int bits, int block_size,
                                                    float beta, int reset, uint8_t *codes_out,
                                                    float *scales_out, void *stream);

/*
 * Measurement aid: loco_compensate_quantize with the number of wavefronts resident per SIMD
 * chosen by the caller: 4 (what loco_compensate_quantize itself runs with), 6 or 8 (all that the
 * kernel's registers allow); anything else is LOCO_ERR_UNSUPPORTED.  Same arithmetic, same bytes.
 * It exists so that the comparison behind the library's choice can be repeated (4 is 1-3 % faster).
 */
loco_status_t loco_compensate_quantize_resident(const void *grad, loco_dtype_t grad_dtype,
                                                float *err_state, size_t n, int bits, int block_size,
                                                float beta, int reset, uint8_t *codes_out,
                                                float *scales_out, int waves_per_simd, void *stream);

/*
 * Measurement and tuning aid: loco_dequant_reduce with the work decomposition chosen by the
 * caller instead of by the library (same arithmetic, same result bit for bit):
 *   0  what loco_dequant_reduce picks (see loco_dequant_reduce_decomposition)
 *   1  a lane owns 4 consecutive elements; block steps by scalar loads (B >= 128) or one
 *      vector load per payload (B <= 64)
 *   2  as 1, block steps of a group of payloads by one vector load (B >= 128 only)
 *   3, 4, 5  a lane loads 4, 8, 16 bytes of codes per payload (8 .. 32 consecutive elements;
 *      3 is for 4-bit codes only) and the sums are transposed through LDS before the stores
 * A decomposition that does not exist for (bits, block_size) is LOCO_ERR_UNSUPPORTED.
 * loco_dequant_reduce_decomposition returns the library's own choice (1..5) for a worker
 * count, bit width and block size and a shard of 2^22 elements or more (below that, 4-bit codes
 * take 4 or 1 where this says 5), or -1 for arguments outside the supported sets.
 */
loco_status_t loco_dequant_reduce_decomposed(const uint8_t *codes, size_t code_stride_bytes,
                                             const float *scales, size_t scale_stride_elems,
                                             int num_workers, size_t n, int bits, int block_size,
                                             float *grad_out, int decomposition, void *stream);
int loco_dequant_reduce_decomposition(int num_workers, int bits, int block_size);

/*
 * Measurement aids, not part of the method: plain streaming kernels with the same
 * 16-byte-per-lane accesses as the kernels above, each in the launch shape that is
 * fastest for it.  They give the practical HBM ceiling for a pure read stream, a pure
 * write stream, a one-to-one mix and two reads per write (the mix of the compensate-
 * quantize pass), and the scale factor for hardware byte counters.
 * `bytes` is a multiple of 16 and every pointer 16-byte aligned.
 *   loco_stream_copy  dst[i] = src[i]
 *   loco_stream_read  reads all of src; sink16 is 16 bytes of device memory that may be
 *                     written (only if a lane's four words xor to a fixed constant, which
 *                     keeps the loads alive without a store stream)
 *   loco_stream_fill  dst[i] = 0
 *   loco_stream_sum2  dst[i] = src_a[i] + src_b[i] on 32-bit words (wrapping)
 *   loco_stream_update3  a[i] += 1, b[i] += a[i], c[i] += b[i] in place on 32-bit words: the
 *                     traffic of an optimizer step with two moment arrays and nothing else
 * loco_runtime_copy is the HIP runtime's own device-to-device copy (hipMemcpyDtoDAsync) on
 * the same stream, as an independent figure beside loco_stream_copy; any size and alignment.
 */
loco_status_t loco_stream_copy(void *dst, const void *src, size_t bytes, void *stream);
loco_status_t loco_stream_read(const void *src, size_t bytes, void *sink16, void *stream);
loco_status_t loco_stream_fill(void *dst, size_t bytes, void *stream);
loco_status_t loco_stream_sum2(void *dst, const void *src_a, const void *src_b, size_t bytes, void *stream);
loco_status_t loco_stream_update3(void *a, void *b, void *c, size_t bytes, void *stream);
loco_status_t loco_runtime_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * Measurement aid, not part of the method: what the current device reports
 * about itself, for deriving the HBM peak (transfers per memory clock x bus
 * width / 8) beside the published figure.  Each pointer may be NULL; values
 * are written to host memory: memory clock in kHz, memory bus width in bits,
 * number of compute units, engine clock in kHz.  LOCO_ERR_LAUNCH if the
 * runtime cannot answer.
 */
loco_status_t loco_device_info(int *memory_clock_khz, int *memory_bus_bits, int *compute_units,
                               int *engine_clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* LOCO_H */
