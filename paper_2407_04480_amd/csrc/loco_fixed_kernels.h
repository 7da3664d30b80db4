// Device code for LoCo's local step exactly as Algorithm 1 of arXiv 2407.04480 prints it:
// one global scale s = 2^log2_s for the p-bit gradient codes (Eq. 1, 3) and the error state
// itself stored as 8-bit codes with scale s_e = se_mult * s (Eq. 2, 7).
//
//   fixed_cq_kernel  e^ = float(e)/s_e; h = g + e^; q = clamp(rint(h s)); d = float(q)/s;
//                    e~' = (1-beta) e^ + beta (h - d); e' = clamp(rint(e~' s_e)) or 0 on reset
//   fixed_dr_kernel  out = (sum_w float(q^w)/s) * (1/W)                          (Eq. 8)
//   fixed_f32_cq_kernel  the same compressor with the state kept in fp32 (no s_e)
//
// 4.5 bytes move per element (bf16 gradient, 8-bit state in and out, 4-bit codes) against
// about 20 VALU operations, so fixed_cq_kernel sits where the HBM and the VALU limits of
// the chip meet; every operation saved shows.  There is no fp32 stream and no block
// reduction, so a lane owns 8 consecutive elements: 16 B of bf16 gradient, 8 B of state
// and 4 or 8 B of codes, each contiguous across the wavefront.
//
// Floating point: the operations and their order are those of the method, one binary32
// rounding each (compile with -ffp-contract=off).  Two rewrites are exact by construction:
//   float(q)/s        = float(q) * (1/s)       because s is a power of two;
//   float(e)/s_e      = e*r, then one fma-fma correction step with r = fl(1/s_e): for every
//                       integer numerator in [-128, 127] and every se_mult in 1..64 this is
//                       the correctly rounded quotient (checked exhaustively in the tests);
//                       when se_mult is a power of two the first product is already exact.
// In the reduce kernel the sum of Eq. 8 is taken over the integer codes: every partial sum
// of float(q)/s is an integer below 2^24 over s, hence exact in binary32 in any order.
#pragma once

#include "loco_kernels.h"

namespace loco {

constexpr int kOctet = 8;                  // elements per lane per unit
constexpr int kUnit = kWave * kOctet;      // 512 elements per wavefront instruction

template <typename G> struct GradOctet;
template <> struct GradOctet<bf16_t> {
    template <bool NT>
    static __device__ __forceinline__ void load8(const void* base, size_t i, float (&g)[8]) {
        const u32x4 a = vload<NT>(reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + i));
        const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            g[2 * k] = __uint_as_float(w[k] << 16);
            g[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
        }
    }
};
template <> struct GradOctet<float> {
    template <bool NT>
    static __device__ __forceinline__ void load8(const void* base, size_t i, float (&g)[8]) {
        const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + i);
        const f32x4 a = vload<NT>(p), b = vload<NT>(p + 1);
        g[0] = a.x; g[1] = a.y; g[2] = a.z; g[3] = a.w;
        g[4] = b.x; g[5] = b.y; g[6] = b.z; g[7] = b.w;
    }
};

struct FixedScales {
    float s, inv_s;        // 2^log2_s and its exact reciprocal
    float s_e, inv_se;     // se_mult * s and fl(1 / s_e)
    float beta, one_minus_beta;
};

// Algorithm 1 steps 1-2 on one octet.  e8[2]: the 8 state bytes; returns codes and new state.
template <int BITS, bool POW2>
__device__ __forceinline__ void fixed_cq_octet(const float (&g)[8], const uint32_t (&e8)[2],
                                               const FixedScales& k, bool reset,
                                               uint32_t (&codes)[BITS / 4], uint32_t (&e8_new)[2]) {
    constexpr float QMAX = (float)((1 << (BITS - 1)) - 1);
    constexpr float QMIN = -(float)(1 << (BITS - 1));
    codes[0] = 0;
    if constexpr (BITS == 8) codes[1] = 0;
    uint32_t st[2] = {0u, 0u};
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float ef = (float)(int8_t)(e8[j >> 2] >> (8 * (j & 3)));   // sign-extending byte select
        float e_hat = ef * k.inv_se;                                       // float(e) / s_e ...
        if constexpr (!POW2) {                                             // ... correctly rounded
            const float rem = __builtin_fmaf(-e_hat, k.s_e, ef);
            e_hat = __builtin_fmaf(rem, k.inv_se, e_hat);
        }
        const float h = g[j] + e_hat;                                      // Eq. 2
        const float qf = fminf(fmaxf(rintf(h * k.s), QMIN), QMAX);         // Eq. 1, 3
        const float d = qf * k.inv_s;                                      // float(q) / s
        const float delta = h - d;                                         // Eq. 4
        const float bd = k.beta * delta;
        const float e_new = __builtin_fmaf(k.one_minus_beta, e_hat, bd);   // Eq. 5
        // Eq. 7: round, move [-128, 127] to [0, 255] (exact), convert with saturation into byte j
        const float t = rintf(e_new * k.s_e) + 128.0f;
        st[j >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(t, (uint32_t)(j & 3), st[j >> 2]);
        const uint32_t q = (uint32_t)(int)qf;
        if constexpr (BITS == 4) codes[0] |= (q & 15u) << (4 * j);
        else codes[j >> 2] |= (q & 255u) << (8 * (j & 3));
    }
    e8_new[0] = reset ? 0u : st[0] ^ 0x80808080u;   // back to two's complement
    e8_new[1] = reset ? 0u : st[1] ^ 0x80808080u;
}

// Resident wavefronts per SIMD, as for cq_kernel (kCqWavesPerSimd): 5 measured best for a bf16
// gradient with 4-bit codes (82 % of HBM peak against 78-79 % with all 8), 4 for the rest.
template <typename G, int BITS>
constexpr int fixed_cq_waves_per_simd() { return (sizeof(G) == 2 && BITS == 4) ? 5 : 4; }

// One wavefront per UNITS*512 elements, THREADS/64 wavefronts per workgroup;
// grid = ceil(n / (UNITS*512*THREADS/64)).  The last wavefront may take the guarded path.
template <typename G, int BITS, bool POW2, int UNITS, int THREADS, bool NT, bool CLIP, int XCDK = 0>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, fixed_cq_waves_per_simd<G, BITS>())))
fixed_cq_kernel(const void* __restrict__ grad, int8_t* __restrict__ err8, size_t n, FixedScales k,
                int reset, const long long* __restrict__ step_index, long long reset_period, float clip,
                uint8_t* __restrict__ codes) {
    constexpr size_t TILE = (size_t)kUnit * UNITS;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const size_t tile0 = wave_tile_index<THREADS, XCDK>() * TILE;
    if (tile0 >= n) return;
    const bool rst = step_index ? reset_step_due(step_index, reset_period) : reset != 0;   // Eq. 7

    if (tile0 + TILE <= n) {
        float g[UNITS][8];
        uint32_t e8[UNITS][2];
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const size_t i = tile0 + (size_t)u * kUnit + (size_t)lane * kOctet;
            GradOctet<G>::template load8<NT>(grad, i, g[u]);
#pragma unroll
            for (int j = 0; j < 8; ++j) g[u][j] = clip_grad<CLIP>(g[u][j], clip);
            const u32x2 v = vload<NT>(reinterpret_cast<const u32x2*>(err8 + i));
            e8[u][0] = v.x; e8[u][1] = v.y;
        }
#pragma unroll
        for (int u = 0; u < UNITS; ++u) {
            const size_t i = tile0 + (size_t)u * kUnit + (size_t)lane * kOctet;
            uint32_t c[BITS / 4], en[2];
            fixed_cq_octet<BITS, POW2>(g[u], e8[u], k, rst, c, en);
            vstore<NT>(reinterpret_cast<u32x2*>(err8 + i), u32x2{en[0], en[1]});
            if constexpr (BITS == 4) vstore<NT>(reinterpret_cast<uint32_t*>(codes + (i >> 1)), c[0]);
            else vstore<NT>(reinterpret_cast<u32x2*>(codes + i), u32x2{c[0], c[1]});
        }
    } else {
#pragma unroll 1
        for (int u = 0; u < UNITS; ++u) {
            const size_t i = tile0 + (size_t)u * kUnit + (size_t)lane * kOctet;
            if (i >= n) continue;
            float g[8];
            uint32_t e8[2] = {0u, 0u}, c[BITS / 4], en[2];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool in = i + j < n;
                g[j] = in ? clip_grad<CLIP>(Grad<G>::load1(grad, i + j), clip) : 0.0f;
                if (in) e8[j >> 2] |= (uint32_t)(uint8_t)err8[i + j] << (8 * (j & 3));
            }
            fixed_cq_octet<BITS, POW2>(g, e8, k, rst, c, en);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (i + j < n) err8[i + j] = (int8_t)(en[j >> 2] >> (8 * (j & 3)));
            if constexpr (BITS == 4) {
#pragma unroll
                for (int b = 0; b < 4; ++b)   // elements past n carry g = 0, e = 0: their nibble is 0
                    if (i + 2 * b < n) codes[(i >> 1) + b] = (uint8_t)(c[0] >> (8 * b));
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (i + j < n) codes[i + j] = (uint8_t)(c[j >> 2] >> (8 * (j & 3)));
            }
        }
    }
}

// ---- global scale, compensation error kept in fp32 ----
// Algorithm 1 without the 8-bit round trip of the state (the paper's ablation row without error
// compression, Table 9): h = g + e~; q = clamp(rint(h s)); d = float(q)/s;
// e~' = (1-beta) e~ + beta (h - d), or 0 on a reset step.  The fp32 state makes the traffic mix
// that of cq_kernel without the block steps, so the decomposition is cq_kernel's: a lane owns
// a quad per slot (16 B of state, 8 B of bf16 gradient, 2 or 4 B of codes).
template <int BITS>
__device__ __forceinline__ uint32_t fixed_f32_quad(const float (&h)[4], float (&e)[4], const FixedScales& k,
                                                   bool reset) {
    constexpr float QMAX = (float)((1 << (BITS - 1)) - 1);
    constexpr float QMIN = -(float)(1 << (BITS - 1));
    uint32_t pk = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float qf = fminf(fmaxf(rintf(h[j] * k.s), QMIN), QMAX);    // Eq. 1, 3
        const float d = qf * k.inv_s;                                     // float(q) / s, exact
        const float delta = h[j] - d;                                     // Eq. 4
        const float bd = k.beta * delta;
        e[j] = reset ? 0.0f : __builtin_fmaf(k.one_minus_beta, e[j], bd); // Eq. 5 / Eq. 7
        pk |= ((uint32_t)(int)qf & (BITS == 4 ? 15u : 255u)) << (BITS * j);
    }
    return pk;
}

template <typename G, int BITS, int SLOTS, int THREADS, bool NT, int XCDK = 0>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, kCqWavesPerSimd)))
fixed_f32_cq_kernel(const void* __restrict__ grad, float* __restrict__ err, size_t n, FixedScales k, int reset,
                    const long long* __restrict__ step_index, long long reset_period,
                    uint8_t* __restrict__ codes, uint32_t lead_tiles) {
    constexpr size_t TILE = (size_t)kSlot * SLOTS;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const size_t wave = wave_tile_index<THREADS, XCDK>();
    if (wave < lead_tiles) return;   // see xcd_run_lead_tiles
    const size_t tile0 = (wave - lead_tiles) * TILE;
    if (tile0 >= n) return;
    const bool rst = step_index ? reset_step_due(step_index, reset_period) : reset != 0;   // Eq. 7

    if (tile0 + TILE <= n) {
        float h[SLOTS][4], e[SLOTS][4];
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            Grad<G>::template load4<NT>(grad, i, h[s]);
            const f32x4 v = vload<NT>(reinterpret_cast<const f32x4*>(err + i));
            e[s][0] = v.x; e[s][1] = v.y; e[s][2] = v.z; e[s][3] = v.w;
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
#pragma unroll
            for (int j = 0; j < 4; ++j) h[s][j] = h[s][j] + e[s][j];   // Eq. 2
            const uint32_t pk = fixed_f32_quad<BITS>(h[s], e[s], k, rst);
            vstore<NT>(reinterpret_cast<f32x4*>(err + i), f32x4{e[s][0], e[s][1], e[s][2], e[s][3]});
            if constexpr (BITS == 4) vstore<NT>(reinterpret_cast<uint16_t*>(codes + (i >> 1)), (uint16_t)pk);
            else vstore<NT>(reinterpret_cast<uint32_t*>(codes + i), pk);
        }
    } else {
#pragma unroll 1
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            if (i >= n) continue;
            float h[4], e[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool in = i + j < n;
                e[j] = in ? err[i + j] : 0.0f;
                h[j] = (in ? Grad<G>::load1(grad, i + j) : 0.0f) + e[j];   // past n: code 0
            }
            const uint32_t pk = fixed_f32_quad<BITS>(h, e, k, rst);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i + j < n) err[i + j] = e[j];
            if constexpr (BITS == 4) {
                codes[i >> 1] = (uint8_t)pk;
                if (i + 2 < n) codes[(i >> 1) + 1] = (uint8_t)(pk >> 8);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (i + j < n) codes[i + j] = (uint8_t)(pk >> (8 * j));
            }
        }
    }
}

// ---- Eq. 8 with the global scale ----
// Integer sum of the workers' codes, several fields per register (SWAR): 4-bit codes are
// biased to 0..15 and summed in bytes (at most 17 workers before a byte could overflow, so
// the byte sums are widened every 16 workers); 8-bit codes are biased to 0..255 and summed
// in 16-bit halves (up to 256 workers per widening).  A lane owns 4 consecutive elements
// per slot, as in dr_kernel, so the fp32 output is written 16 B per lane, gap-free.
// Resident wavefronts per SIMD: with a fused optimizer (arrays updated in place) 4 measured
// 3-6 points of HBM peak faster than the 8 the registers allow, the plain outputs like all 8.
constexpr int fixed_dr_waves_per_simd(Epilogue e) { return (e == Epilogue::kSgd || e == Epilogue::kAdam) ? 4 : 8; }
// The fp32 output of 8-bit payloads, from 4 of them on, also likes 4 (80 % against 76.5 % at W = 8, +1 to
// +3 points at W = 4..32), while with one or two payloads it wants all 8; the host picks by W.
constexpr int kFixedDr8ManyWorkersWaves = 4, kFixedDr8ManyWorkers = 4;

template <int BITS, int SLOTS, int THREADS, int WU, bool NT, Epilogue EPI, int XCDK = 0,
          int WAVES = fixed_dr_waves_per_simd(EPI)>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, WAVES)))
fixed_dr_kernel(const uint8_t* __restrict__ codes, size_t code_stride, int W, size_t n, float inv_s,
                float inv_w, EpilogueArgs epi, uint32_t lead_tiles) {
    constexpr size_t TILE = (size_t)kSlot * SLOTS;
    constexpr uint32_t SLOT_CODE_BYTES = kSlot * BITS / 8;
    constexpr int FLUSH = BITS == 4 ? 16 : 256;   // workers per widening of the packed sums
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const size_t tile0 = wave_tile_index_tail_first<THREADS, XCDK>(n, TILE, lead_tiles) * TILE;
    if (tile0 >= n) return;

    if (tile0 + TILE <= n) {
        const uint8_t* cbase = codes + tile0 * BITS / 8;   // uniform, advanced per worker
        const uint32_t code_off = lane * (kQuad * BITS / 8);
        int total[SLOTS][4];
        EpilogueState<EPI> est[SLOTS];
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            epilogue_prefetch<EPI, NT>(epi, tile0 + (size_t)s * kSlot + (size_t)lane * kQuad, est[s]);
#pragma unroll
            for (int j = 0; j < 4; ++j) total[s][j] = 0;
        }
        for (int w0 = 0; w0 < W; w0 += FLUSH) {
            const int wend = min(W, w0 + FLUSH);
            uint32_t lo[SLOTS], hi[SLOTS];   // packed partial sums of the biased codes
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) lo[s] = hi[s] = 0u;
            // payloads in chunks of WU, a last shorter one included: all loads of a chunk first, then its sums
            auto chunk = [&](int count) {
                uint32_t c[WU][SLOTS];
#pragma unroll
                for (int u = 0; u < WU; ++u)
                    if (u < count) {
#pragma unroll
                        for (int s = 0; s < SLOTS; ++s)
                            c[u][s] = load_quad_codes<BITS, NT>(cbase + (size_t)(s * SLOT_CODE_BYTES + code_off));
                        cbase += code_stride;
                    }
#pragma unroll
                for (int u = 0; u < WU; ++u)
                    if (u < count)
#pragma unroll
                        for (int s = 0; s < SLOTS; ++s) {
                            if constexpr (BITS == 4) {
                                const uint32_t x = c[u][s] ^ 0x8888u;            // q + 8 in every nibble
                                lo[s] += x & 0x0F0Fu;                            // elements 0, 2
                                hi[s] += (x >> 4) & 0x0F0Fu;                     // elements 1, 3
                            } else {
                                const uint32_t x = c[u][s] ^ 0x80808080u;        // q + 128 in every byte
                                lo[s] += x & 0x00FF00FFu;                        // elements 0, 2
                                hi[s] += (x >> 8) & 0x00FF00FFu;                 // elements 1, 3
                            }
                        }
            };
            int w = w0;
            if (wend - w0 < WU) {
                // fewer payloads than one chunk: one at a time (two payloads fetched together measured 9
                // points of HBM peak slower than one after the other; after a full chunk it is the reverse)
                for (; w < wend; ++w) chunk(1);
            } else {
                for (; w + WU <= wend; w += WU) chunk(WU);
                if (w < wend) chunk(wend - w);
            }
            constexpr int FIELD = BITS == 4 ? 8 : 16;      // width of one packed sum
            constexpr uint32_t MASK = (1u << FIELD) - 1u;
            const int bias = (wend - w0) * (1 << (BITS - 1));
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) {
                total[s][0] += (int)(lo[s] & MASK) - bias;
                total[s][1] += (int)(hi[s] & MASK) - bias;
                total[s][2] += (int)((lo[s] >> FIELD) & MASK) - bias;
                total[s][3] += (int)((hi[s] >> FIELD) & MASK) - bias;
            }
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            float g[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) g[j] = ((float)total[s][j] * inv_s) * inv_w;   // (sum float(q)/s) * (1/W)
            epilogue_finish<EPI, NT>(epi, i, g, est[s]);
        }
    } else {
        // last, partial tile (see load_bytes_clamped in loco_kernels.h)
        constexpr int QB = kQuad * BITS / 8;        // code bytes per quad: 2 or 4
        const size_t last_quad = (n - 1) & ~(size_t)(kQuad - 1);
        size_t at[SLOTS];
        uint32_t have[SLOTS];
        int total[SLOTS][4];
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            at[s] = i < n ? i : last_quad;
            have[s] = code_bytes_present<BITS>(at[s], n, kQuad);
#pragma unroll
            for (int j = 0; j < 4; ++j) total[s][j] = 0;
        }
        for (int w0 = 0; w0 < W; w0 += kTailPayloads) {
            uint32_t c[kTailPayloads][SLOTS];
#pragma unroll
            for (int u = 0; u < kTailPayloads; ++u) {
                const size_t w = (size_t)(w0 + u < W ? w0 + u : W - 1);
#pragma unroll
                for (int s = 0; s < SLOTS; ++s) {
                    uint32_t word[1] = {0u};
                    if constexpr (QB == 4) {
                        load_bytes_clamped<4>(codes + w * code_stride + at[s], have[s], word);
                    } else {
                        const uint8_t* p = codes + w * code_stride + (at[s] >> 1);
                        word[0] = (uint32_t)p[0] | ((uint32_t)p[have[s] - 1u] << 8);
                    }
                    c[u][s] = word[0];
                }
            }
#pragma unroll
            for (int u = 0; u < kTailPayloads; ++u)
                if (w0 + u < W)
#pragma unroll
                    for (int s = 0; s < SLOTS; ++s)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            total[s][j] += ((int)(c[u][s] << (32 - BITS * (j + 1)))) >> (32 - BITS);   // signed field j
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i + j < n) epilogue_element<EPI>(epi, i + j, ((float)total[s][j] * inv_s) * inv_w);
        }
    }
}

// Zero fill of a byte array (8-bit state init), 16 bytes per lane and slot.
template <int SLOTS, int THREADS, bool NT>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, kFillWavesPerSimd)))
fill_zero_bytes_kernel(uint8_t* __restrict__ dst, size_t nbytes) {
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const size_t tile0 = wave_tile_index<THREADS, 0>() * ((size_t)kWave * 16 * SLOTS);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const size_t i = tile0 + ((size_t)s * kWave + lane) * 16;
        if (i + 16 <= nbytes) {
            vstore<NT>(reinterpret_cast<u32x4*>(dst + i), u32x4{0u, 0u, 0u, 0u});
        } else {
            for (size_t j = i; j < nbytes; ++j) dst[j] = 0;
        }
    }
}

}  // namespace loco
