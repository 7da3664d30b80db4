// Device code for LoCo's per-step local path on gfx950 (CDNA4, wave64).
//
// Two streaming kernels, both bound by HBM bandwidth (no contraction, so no MFMA):
//   cq_kernel  Algorithm 1 steps 1-2 of arXiv 2407.04480 (Eq. 1-5, 7): compensate, block
//              quantise, self-decode, fold the error into the moving average; one pass.
//   dr_kernel  Algorithm 1 step 3 (Eq. 8): decode W payloads and average in fp32.
//
// Work decomposition shared by both: a lane owns 8 consecutive elements ("octet"), a
// 256-thread workgroup owns TILES_PER_WG consecutive tiles of 2048 elements.  A
// quantisation block of 32..512 elements is therefore 4..64 consecutive lanes of one
// wavefront, and its max-abs is an all-reduce over those lanes with DPP / swizzle
// cross-lane moves; no LDS memory and no barrier is needed.  One lane's 8 codes are one
// dword (4-bit) or two (8-bit), so a wavefront writes 256 or 512 contiguous bytes.
//
// Floating point: every operation below is one IEEE binary32 operation in the order
// the method states; the file must be compiled with -ffp-contract=off and without any
// fast-math flag.  The only fused operation is the fmaf of Eq. 5.
#pragma once

#include <hip/hip_runtime.h>
#include <float.h>
#include <stdint.h>

namespace loco {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct bf16_t { uint16_t bits; };  // storage tag only; widened with integer shifts

constexpr int kThreads = 256;             // 4 wavefronts
constexpr int kOctet = 8;                 // elements per lane per tile
constexpr int kTile = kThreads * kOctet;  // 2048 elements

template <bool NT, typename V>
__device__ __forceinline__ V vload(const V* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename V>
__device__ __forceinline__ void vstore(V* p, V v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// ---- cross-lane all-reduce (max) over aligned groups of LANES consecutive lanes ----
// Operands are bit patterns of non-negative floats, which order like unsigned ints.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
template <int LANES>
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v) {
    static_assert(LANES == 4 || LANES == 8 || LANES == 16 || LANES == 32 || LANES == 64, "group size");
    v = max(v, dpp_move<0xB1>(v));                       // quad_perm [1,0,3,2]: lane ^ 1
    v = max(v, dpp_move<0x4E>(v));                       // quad_perm [2,3,0,1]: lane ^ 2
    if constexpr (LANES >= 8) v = max(v, dpp_move<0x141>(v));   // row_half_mirror: other quad of 8
    if constexpr (LANES >= 16) v = max(v, dpp_move<0x140>(v));  // row_mirror: other half of 16
    if constexpr (LANES >= 32)                                   // ds_swizzle bit mode, lane ^ 16
        v = max(v, (uint32_t)__builtin_amdgcn_ds_swizzle((int)v, 0x401F));
    if constexpr (LANES >= 64) v = max(v, (uint32_t)__shfl_xor((int)v, 32, 64));
    return v;
}

// ---- gradient loads: 8 elements widened to fp32 ----
template <typename G> struct Grad;
template <> struct Grad<float> {
    template <bool NT>
    static __device__ __forceinline__ void load8(const void* base, size_t i, float (&g)[8]) {
        const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + i);
        f32x4 a = vload<NT>(p), b = vload<NT>(p + 1);
        g[0] = a.x; g[1] = a.y; g[2] = a.z; g[3] = a.w;
        g[4] = b.x; g[5] = b.y; g[6] = b.z; g[7] = b.w;
    }
    static __device__ __forceinline__ float load1(const void* base, size_t i) {
        return static_cast<const float*>(base)[i];
    }
};
template <> struct Grad<bf16_t> {
    template <bool NT>
    static __device__ __forceinline__ void load8(const void* base, size_t i, float (&g)[8]) {
        const u32x4* p = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + i);
        u32x4 a = vload<NT>(p);
        uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {  // bf16 is the high half of a binary32: exact
            g[2 * k] = __uint_as_float(w[k] << 16);
            g[2 * k + 1] = __uint_as_float(w[k] & 0xFFFF0000u);
        }
    }
    static __device__ __forceinline__ float load1(const void* base, size_t i) {
        return __uint_as_float((uint32_t)static_cast<const uint16_t*>(base)[i] << 16);
    }
};

// ---- Algorithm 1 steps 1-2 on one octet held in registers ----
// h: compensated gradient (Eq. 2), e: old state.  Writes the new state, the packed codes
// and the block's step D.  All lanes of a quantisation block call this together.
template <int BITS, int BLOCK>
__device__ __forceinline__ void cq_octet(const float (&h)[8], const float (&e)[8], float beta,
                                         float one_minus_beta, bool reset, float (&e_new)[8],
                                         uint32_t (&packed)[BITS / 4], float& step) {
    constexpr int QMAX = (1 << (BITS - 1)) - 1;
    constexpr int QMIN = -(1 << (BITS - 1));
    float a = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) a = fmaxf(a, fabsf(h[j]));
    a = __uint_as_float(group_max_u32<BLOCK / kOctet>(__float_as_uint(a)));

    float D = a / (float)QMAX;           // step of the block: 1/s_b, correctly rounded
    const bool live = !(D < FLT_MIN);    // zero or subnormal step: encode nothing
    const float r = live ? 1.0f / D : 0.0f;
    D = live ? D : 0.0f;
    step = D;

    packed[0] = 0;
    if constexpr (BITS == 8) packed[1] = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int q = (int)rintf(h[j] * r);                 // Eq. 1: nearest integer, ties to even
        q = min(max(q, QMIN), QMAX);                  // ... within the p-bit range
        const float d = (float)q * D;                 // decompressor
        const float delta = h[j] - d;                 // Eq. 4
        const float bd = beta * delta;
        e_new[j] = reset ? 0.0f : __builtin_fmaf(one_minus_beta, e[j], bd);  // Eq. 5 / Eq. 7
        if constexpr (BITS == 4) packed[0] |= ((uint32_t)q & 15u) << (4 * j);
        else packed[j >> 2] |= ((uint32_t)q & 255u) << (8 * (j & 3));
    }
}

// grid: ceil(n / (kTile * TILES)) workgroups of kThreads.  Workgroups whose chunk lies
// wholly inside [0, n) take the vector path; the last one may take the guarded path,
// which touches memory element by element and never beyond n.
template <typename G, int BITS, int BLOCK, int TILES, bool NT>
__global__ void __launch_bounds__(kThreads)
cq_kernel(const void* __restrict__ grad, float* __restrict__ err, size_t n, float beta,
          float one_minus_beta, int reset, uint8_t* __restrict__ codes, float* __restrict__ scales) {
    constexpr int GROUP = BLOCK / kOctet;  // lanes per quantisation block
    const size_t chunk0 = (size_t)blockIdx.x * (size_t)(kTile * TILES);
    const bool rst = reset != 0;

    if (chunk0 + (size_t)(kTile * TILES) <= n) {
        float g[TILES][8], e[TILES][8];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const size_t i = chunk0 + (size_t)t * kTile + (size_t)threadIdx.x * kOctet;
            Grad<G>::template load8<NT>(grad, i, g[t]);
            const f32x4* pe = reinterpret_cast<const f32x4*>(err + i);
            f32x4 a = vload<NT>(pe), b = vload<NT>(pe + 1);
            e[t][0] = a.x; e[t][1] = a.y; e[t][2] = a.z; e[t][3] = a.w;
            e[t][4] = b.x; e[t][5] = b.y; e[t][6] = b.z; e[t][7] = b.w;
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const size_t i = chunk0 + (size_t)t * kTile + (size_t)threadIdx.x * kOctet;
            float h[8], en[8], step;
            uint32_t pk[BITS / 4];
#pragma unroll
            for (int j = 0; j < 8; ++j) h[j] = g[t][j] + e[t][j];  // Eq. 2
            cq_octet<BITS, BLOCK>(h, e[t], beta, one_minus_beta, rst, en, pk, step);
            f32x4* pe = reinterpret_cast<f32x4*>(err + i);
            vstore<NT>(pe, f32x4{en[0], en[1], en[2], en[3]});
            vstore<NT>(pe + 1, f32x4{en[4], en[5], en[6], en[7]});
            if constexpr (BITS == 4) {
                vstore<NT>(reinterpret_cast<uint32_t*>(codes + (i >> 1)), pk[0]);
            } else {
                vstore<NT>(reinterpret_cast<u32x2*>(codes + i), u32x2{pk[0], pk[1]});
            }
            if ((threadIdx.x & (GROUP - 1)) == 0) scales[i / BLOCK] = step;
        }
    } else {
#pragma unroll 1
        for (int t = 0; t < TILES; ++t) {
            const size_t i = chunk0 + (size_t)t * kTile + (size_t)threadIdx.x * kOctet;
            if (chunk0 + (size_t)t * kTile >= n) break;  // uniform over the workgroup
            float h[8], e[8], en[8], step;
            uint32_t pk[BITS / 4];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const bool in = i + j < n;
                e[j] = in ? err[i + j] : 0.0f;
                const float gj = in ? Grad<G>::load1(grad, i + j) : 0.0f;
                h[j] = gj + e[j];  // elements past n read as h = 0: neutral for the max, code 0
            }
            cq_octet<BITS, BLOCK>(h, e, beta, one_minus_beta, rst, en, pk, step);
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (i + j < n) err[i + j] = en[j];
            if constexpr (BITS == 4) {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (i + 2 * k < n) codes[(i >> 1) + k] = (uint8_t)(pk[0] >> (8 * k));
            } else {
#pragma unroll
                for (int j = 0; j < 8; ++j)
                    if (i + j < n) codes[i + j] = (uint8_t)(pk[j >> 2] >> (8 * (j & 3)));
            }
            if ((threadIdx.x & (GROUP - 1)) == 0 && i < n) scales[i / BLOCK] = step;
        }
    }
}

// ---- Algorithm 1 step 3 / Eq. 8 ----
template <int BITS>
__device__ __forceinline__ void dr_accumulate(const uint32_t (&c)[BITS / 4], float D, float (&acc)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int q;
        if constexpr (BITS == 4) q = ((int)(c[0] << (28 - 4 * j))) >> 28;          // signed nibble j
        else q = ((int)(c[j >> 2] << (24 - 8 * (j & 3)))) >> 24;                   // signed byte j
        const float d = (float)q * D;   // decompressor of Eq. 1
        acc[j] = acc[j] + d;            // sum of Eq. 8, in worker order
    }
}

// grid: ceil(n / (kTile * TILES)) workgroups of kThreads; WU payloads are in flight per lane.
template <int BITS, int BLOCK, int TILES, int WU, bool NT>
__global__ void __launch_bounds__(kThreads)
dr_kernel(const uint8_t* __restrict__ codes, size_t code_stride, const float* __restrict__ scales,
          size_t scale_stride, int W, size_t n, float inv_w, float* __restrict__ out) {
    constexpr int CW = BITS / 4;  // dwords of codes per octet
    const size_t chunk0 = (size_t)blockIdx.x * (size_t)(kTile * TILES);

    if (chunk0 + (size_t)(kTile * TILES) <= n) {
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            const size_t i = chunk0 + (size_t)t * kTile + (size_t)threadIdx.x * kOctet;
            const uint8_t* pc = codes + (i * BITS) / 8;
            const float* ps = scales + i / BLOCK;
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            int w = 0;
            for (; w + WU <= W; w += WU) {
                uint32_t c[WU][CW];
                float D[WU];
#pragma unroll
                for (int u = 0; u < WU; ++u) {
                    if constexpr (BITS == 4) {
                        c[u][0] = vload<NT>(reinterpret_cast<const uint32_t*>(pc));
                    } else {
                        u32x2 v = vload<NT>(reinterpret_cast<const u32x2*>(pc));
                        c[u][0] = v.x; c[u][1] = v.y;
                    }
                    D[u] = *ps;
                    pc += code_stride;
                    ps += scale_stride;
                }
#pragma unroll
                for (int u = 0; u < WU; ++u) dr_accumulate<BITS>(c[u], D[u], acc);
            }
            for (; w < W; ++w) {
                uint32_t c[CW];
                if constexpr (BITS == 4) {
                    c[0] = vload<NT>(reinterpret_cast<const uint32_t*>(pc));
                } else {
                    u32x2 v = vload<NT>(reinterpret_cast<const u32x2*>(pc));
                    c[0] = v.x; c[1] = v.y;
                }
                const float D = *ps;
                pc += code_stride;
                ps += scale_stride;
                dr_accumulate<BITS>(c, D, acc);
            }
            f32x4* po = reinterpret_cast<f32x4*>(out + i);
            vstore<NT>(po, f32x4{acc[0] * inv_w, acc[1] * inv_w, acc[2] * inv_w, acc[3] * inv_w});
            vstore<NT>(po + 1, f32x4{acc[4] * inv_w, acc[5] * inv_w, acc[6] * inv_w, acc[7] * inv_w});
        }
    } else {
#pragma unroll 1
        for (int t = 0; t < TILES; ++t) {
            const size_t i = chunk0 + (size_t)t * kTile + (size_t)threadIdx.x * kOctet;
            if (i >= n) continue;
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int w = 0; w < W; ++w) {
                const uint8_t* pc = codes + (size_t)w * code_stride;
                uint32_t c[CW] = {};
                if constexpr (BITS == 4) {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (i + 2 * k < n) c[0] |= (uint32_t)pc[(i >> 1) + k] << (8 * k);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (i + j < n) c[j >> 2] |= (uint32_t)pc[i + j] << (8 * (j & 3));
                }
                const float D = scales[(size_t)w * scale_stride + i / BLOCK];
                dr_accumulate<BITS>(c, D, acc);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (i + j < n) out[i + j] = acc[j] * inv_w;
        }
    }
}

// ---- helpers: zero fill and plain copy, same launch shape ----
// grid: ceil(n16 / (kThreads * TILES)) workgroups; n16 = number of 16-byte units.
template <int TILES, bool NT>
__global__ void __launch_bounds__(kThreads)
fill_zero_kernel(float* __restrict__ dst, size_t n) {
    const size_t chunk0 = (size_t)blockIdx.x * (size_t)(kThreads * 4 * TILES);
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const size_t i = chunk0 + (size_t)t * (kThreads * 4) + (size_t)threadIdx.x * 4;
        if (i + 4 <= n) {
            vstore<NT>(reinterpret_cast<f32x4*>(dst + i), f32x4{0.f, 0.f, 0.f, 0.f});
        } else {
            for (size_t j = i; j < n; ++j) dst[j] = 0.0f;
        }
    }
}

template <int TILES, bool NT>
__global__ void __launch_bounds__(kThreads)
copy_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n16) {
    const size_t chunk0 = (size_t)blockIdx.x * (size_t)(kThreads * TILES);
    u32x4 v[TILES];
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const size_t i = chunk0 + (size_t)t * kThreads + threadIdx.x;
        if (i < n16) v[t] = vload<NT>(src + i);
    }
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
        const size_t i = chunk0 + (size_t)t * kThreads + threadIdx.x;
        if (i < n16) vstore<NT>(dst + i, v[t]);
    }
}

}  // namespace loco
