// Device code for LoCo's per-step local path on gfx950 (CDNA4, wave64).
//
// Two streaming kernels, both bound by HBM bandwidth (no contraction, so no MFMA):
//   cq_kernel  Algorithm 1 steps 1-2 of arXiv 2407.04480 (Eq. 1-5, 7): compensate, block
//              quantise, self-decode, fold the error into the moving average; one pass.
//   dr_kernel  Algorithm 1 step 3 (Eq. 8): decode W payloads and average in fp32.
//
// Work decomposition shared by both: a lane owns 4 consecutive elements (a "quad"), so
// one wavefront instruction moves 256 consecutive elements (a "slot": 1 KB of fp32 state,
// 512 B of bf16 gradient) with every lane's 16 bytes adjacent to its neighbour's.  A
// wavefront owns SLOTS consecutive slots, a tile of its own whatever the workgroup size
// (one to four wavefronts per workgroup, chosen per kernel by measurement on MI355X, as is
// the non-temporal hint on every streaming access).  A quantisation block of 32..512
// elements lies inside one wavefront's tile, so its max-abs is an all-reduce over 8..64
// lanes (and at most two slots) with DPP moves and lane reads; no LDS, no barrier.
//
// Floating point: every operation below is one IEEE binary32 operation in the order the
// method states; the file must be compiled with -ffp-contract=off and without any
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

constexpr int kWave = 64;
constexpr int kQuad = 4;               // elements per lane per slot
constexpr int kSlot = kWave * kQuad;   // 256 elements per wavefront instruction

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

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Element-wise clipping of the local gradient to [-c, c] before compensation (used by the
// paper's MoE-from-scratch runs, Sec. 5.2, to reduce sensitivity to s); one v_med3_f32.
template <bool CLIP>
__device__ __forceinline__ float clip_grad(float g, float c) {
    if constexpr (CLIP) return fminf(fmaxf(g, -c), c);
    else return g;
}

// Eq. 7 evaluated on the device: step k is a reset step when k % T_c == 0.  k comes from
// device memory (a plain, wavefront-uniform load), so a step captured into a HIP graph
// follows the schedule on every replay while another node advances the counter.  The
// paper's periods (512, 1024; 128 in the ablation) are powers of two and take the mask;
// any other period takes the 64-bit remainder, once per wavefront.
__device__ __forceinline__ bool reset_step_due(const long long* step_index, long long period) {
    if (period <= 0) return false;
    const long long k = *step_index;
    if ((period & (period - 1)) == 0) return (k & (period - 1)) == 0;
    return k % period == 0;
}

// ---- cross-lane all-reduce (max) over aligned groups of LANES consecutive lanes ----
// Operands are bit patterns of non-negative floats, which order like unsigned ints.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}
template <int LANES>
__device__ __forceinline__ uint32_t group_max_u32(uint32_t v, int lane) {
    static_assert(LANES == 8 || LANES == 16 || LANES == 32 || LANES == 64, "group size");
    v = umax(v, dpp_move<0xB1>(v));                          // quad_perm [1,0,3,2]: lane ^ 1
    v = umax(v, dpp_move<0x4E>(v));                          // quad_perm [2,3,0,1]: lane ^ 2
    v = umax(v, dpp_move<0x141>(v));                         // row_half_mirror: other quad of 8
    if constexpr (LANES >= 16) v = umax(v, dpp_move<0x140>(v));  // row_mirror: other half of 16
    if constexpr (LANES >= 32) {
        // every lane of a 16-lane row now holds the row's maximum: combine rows through SGPRs
        const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 0);
        const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
        const uint32_t r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 32);
        const uint32_t r3 = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
        const uint32_t lo = umax(r0, r1), hi = umax(r2, r3);
        if constexpr (LANES == 32) v = lane < 32 ? lo : hi;
        else v = umax(lo, hi);
    }
    return v;
}

// Which tile does this wavefront own?  Workgroups are handed to the 8 XCDs (each with
// its own L2) in turn: workgroup b runs on XCD b % 8.  With XCDK = K > 0 (a power of two),
// every run of 8K workgroups is dealt out so that each XCD gets K consecutive chunks of
// the array: neighbouring tiles - which share cache lines of block steps - then meet in
// one L2 instead of being fetched by all eight, while the machine as a whole still
// sweeps the array front to back.  The launch rounds the grid up to a multiple of 8K;
// tiles past the end return at once.
template <int THREADS, int XCDK>
__device__ __forceinline__ size_t wave_tile_index() {
    size_t b = blockIdx.x;
    if constexpr (XCDK > 0) {
        static_assert((XCDK & (XCDK - 1)) == 0, "XCDK must be a power of two");
        const uint32_t in_run = blockIdx.x & (8u * XCDK - 1u);
        b = (size_t)(blockIdx.x - in_run) + (in_run & 7u) * XCDK + (in_run >> 3);
    }
    return b * (THREADS / kWave) + (size_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}

// The runs pay most when each covers an aligned piece of the array that dominates the traffic: the
// compressor with runs of 32768 elements (128 KB of fp32 state) measured 85 % of the HBM peak with the
// state at a multiple of 128 KB and 80.5-82 % when it starts 16...48 KB or 80...112 KB behind one (period
// 128 KB; where the gradient, the codes and the steps start makes no difference).  So the tile order is
// laid over the ADDRESSES, not the element indices: the first `lead` tile indices stay empty, as many as
// the state's first byte lies behind a multiple of the run, and every run then starts at such a
// multiple (to within one tile).  Host side; the kernel subtracts.  The reduces do the same with the
// array they write or update in place (the output, or the parameters): Adam fused in measured 80 % at a
// multiple of 128 KB against 75-77 % at 48...80 KB behind one, SGD 84 against 82-83, the plain output 82
// against 80.5-81.5.
inline uint32_t xcd_run_lead_tiles(const void* base, size_t run_bytes, size_t tile_bytes) {
    return run_bytes ? (uint32_t)((reinterpret_cast<uintptr_t>(base) % run_bytes) / tile_bytes) : 0u;
}

// The same for the reduces, with the first and the last workgroup that has elements exchanged: the
// last tile may be a partial one, whose wavefront takes the slow byte-wise path W payloads long; in the
// workgroup that is dispatched first that time hides behind all the others, in the one dispatched
// last it would be added to the kernel's (8 % at 128 payloads and 5e7 elements).
template <int THREADS, int XCDK>
__device__ __forceinline__ size_t wave_tile_index_tail_first(size_t n, size_t tile_elems, uint32_t lead_tiles) {
    size_t b = blockIdx.x;
    if constexpr (XCDK > 0) {
        static_assert((XCDK & (XCDK - 1)) == 0, "XCDK must be a power of two");
        const uint32_t in_run = blockIdx.x & (8u * XCDK - 1u);
        b = (size_t)(blockIdx.x - in_run) + (in_run & 7u) * XCDK + (in_run >> 3);
    }
    // the first lead_tiles tile indices are empty (see xcd_run_lead_tiles)
    const size_t first = lead_tiles / (THREADS / kWave);
    const size_t last = (lead_tiles + (n + tile_elems - 1) / tile_elems - 1) / (THREADS / kWave);   // n > 0
    if (b == first) b = last;
    else if (b == last) b = first;
    const size_t wave = b * (THREADS / kWave) + (size_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    if (wave < lead_tiles) return ~(size_t)0 / tile_elems;   // no tile: times tile_elems it is beyond any n
    return wave - lead_tiles;
}

// ---- gradient loads: one quad widened to fp32 ----
template <typename G> struct Grad;
template <> struct Grad<float> {
    template <bool NT>
    static __device__ __forceinline__ void load4(const void* base, size_t i, float (&g)[4]) {
        f32x4 a = vload<NT>(reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + i));
        g[0] = a.x; g[1] = a.y; g[2] = a.z; g[3] = a.w;
    }
    static __device__ __forceinline__ float load1(const void* base, size_t i) {
        return static_cast<const float*>(base)[i];
    }
};
template <> struct Grad<bf16_t> {
    template <bool NT>
    static __device__ __forceinline__ void load4(const void* base, size_t i, float (&g)[4]) {
        u32x2 a = vload<NT>(reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(base) + i));
        // bf16 is the high half of a binary32: widening is exact
        g[0] = __uint_as_float(a.x << 16); g[1] = __uint_as_float(a.x & 0xFFFF0000u);
        g[2] = __uint_as_float(a.y << 16); g[3] = __uint_as_float(a.y & 0xFFFF0000u);
    }
    static __device__ __forceinline__ float load1(const void* base, size_t i) {
        return __uint_as_float((uint32_t)static_cast<const uint16_t*>(base)[i] << 16);
    }
};

// ---- block steps ----
// A block step as it is stored: binary32, or bf16 bits (uint16_t).  A bf16 step is rounded
// (nearest, ties to even, in integer arithmetic so that subnormal steps round like any
// other) before anything uses it, so compressor, own decompressor and the receivers all
// work with the stored value.  Steps are non-negative and finite.
__device__ __forceinline__ float round_step_to_bf16(float D) {
    uint32_t u = __float_as_uint(D);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return __uint_as_float(u & 0xFFFF0000u);
}
template <typename S> __device__ __forceinline__ S step_to_storage(float D);
template <> __device__ __forceinline__ float step_to_storage<float>(float D) { return D; }
template <> __device__ __forceinline__ uint16_t step_to_storage<uint16_t>(float D) {
    return (uint16_t)(__float_as_uint(D) >> 16);   // already rounded: the low half is zero
}
__device__ __forceinline__ float step_from_storage(float v) { return v; }
__device__ __forceinline__ float step_from_storage(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
// Step k of an array at a wavefront-uniform index.  The scalar unit loads whole dwords only,
// so a bf16 step is taken out of the dword that holds it; the array starts on a dword
// boundary (checked by the host) and device allocations end on one.
__device__ __forceinline__ float load_uniform_step(const float* base, size_t k) { return base[k]; }
__device__ __forceinline__ float load_uniform_step(const uint16_t* base, size_t k) {
    const uint32_t word = reinterpret_cast<const uint32_t*>(base)[k >> 1];
    return __uint_as_float((k & 1) ? (word & 0xFFFF0000u) : (word << 16));
}

// ---- Algorithm 1 steps 1-2 on a wavefront's tile held in registers ----
// h: compensated gradient (Eq. 2), e: old state; on return e holds the new state, packed
// the codes of each quad (16 or 32 bits) and step the quad's block step D.
template <int BITS, int BLOCK, int SLOTS, bool S16>
__device__ __forceinline__ void cq_tile(const float (&h)[SLOTS][4], float (&e)[SLOTS][4], float beta,
                                        float one_minus_beta, bool reset, int lane,
                                        uint32_t (&packed)[SLOTS], float (&step)[SLOTS]) {
    constexpr int QMAX = (1 << (BITS - 1)) - 1;
    constexpr int QMIN = -(1 << (BITS - 1));
    static_assert(BLOCK <= kSlot || SLOTS % (BLOCK / kSlot) == 0, "a block must lie inside the tile");
    float a[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s)
        a[s] = fmaxf(fmaxf(fabsf(h[s][0]), fabsf(h[s][1])), fmaxf(fabsf(h[s][2]), fabsf(h[s][3])));
    if constexpr (BLOCK > kSlot) {  // a block spans BLOCK/256 adjacent slots of this wavefront
        constexpr int SPAN = BLOCK / kSlot;
#pragma unroll
        for (int s = 0; s < SLOTS; s += SPAN) {
            float m = a[s];
#pragma unroll
            for (int k = 1; k < SPAN; ++k) m = fmaxf(m, a[s + k]);
            m = __uint_as_float(group_max_u32<kWave>(__float_as_uint(m), lane));
#pragma unroll
            for (int k = 0; k < SPAN; ++k) a[s + k] = m;
        }
    } else {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s)
            a[s] = __uint_as_float(group_max_u32<BLOCK / kQuad>(__float_as_uint(a[s]), lane));
    }
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        float D = a[s] / (float)QMAX;        // step of the block: 1/s_b, correctly rounded
        if constexpr (S16) D = round_step_to_bf16(D);
        const bool live = !(D < FLT_MIN);    // zero or subnormal step: encode nothing
        const float r = live ? 1.0f / D : 0.0f;
        D = live ? D : 0.0f;
        step[s] = D;
        uint32_t pk = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int q = (int)rintf(h[s][j] * r);              // Eq. 1: nearest integer, ties to even
            q = min(max(q, QMIN), QMAX);                  // ... within the p-bit range
            const float d = (float)q * D;                 // decompressor
            const float delta = h[s][j] - d;              // Eq. 4
            const float bd = beta * delta;
            e[s][j] = reset ? 0.0f : __builtin_fmaf(one_minus_beta, e[s][j], bd);  // Eq. 5 / Eq. 7
            pk |= ((uint32_t)q & (BITS == 4 ? 15u : 255u)) << (BITS * j);
        }
        packed[s] = pk;
    }
}

// Resident wavefronts per SIMD for the compressor.  Its registers would allow 8; with 4 (16 per
// CU, each with two slots of every stream in flight) the kernel measured 1-3 points of HBM peak
// faster on every gradient type, bit width and block size, with 3 it starts to lose.  Fewer
// wavefronts touch fewer DRAM pages at a time for the five streams the kernel reads and writes.
constexpr int kCqWavesPerSimd = 4;
// (WAVES on the kernel: other values exist only behind the measurement call that repeats the comparison.)

// One wavefront per SLOTS*256 elements; THREADS/64 wavefronts per workgroup, each with its
// own contiguous tile.  step_index == nullptr: `reset` is the caller's flag for this step.
// grid = ceil(n / (SLOTS*256*THREADS/64)), rounded up to a multiple of 8*XCDK.  A wavefront
// whose tile lies inside [0, n) takes the vector path; the last one may take the guarded
// path, which touches memory element by element and never at or beyond n.
// STAGE_CODES (a measurement variant, 4-bit codes): the tile's nibbles are gathered in LDS and
// leave as 16-byte stores from a few lanes instead of 2-byte stores from all 64.  Either way a
// wavefront hands the memory pipeline the same 128 contiguous bytes per slot; measured, the
// staged form is 1-2 % slower (an LDS round trip in front of the store), so it is not the default.
template <typename G, int BITS, int BLOCK, int SLOTS, int THREADS, bool NT, int XCDK, bool CLIP, typename S,
          bool STAGE_CODES = false, int WAVES = kCqWavesPerSimd>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, WAVES)))
cq_kernel(const void* __restrict__ grad, float* __restrict__ err, size_t n, float beta,
          float one_minus_beta, int reset, const long long* __restrict__ step_index, long long reset_period,
          float clip, uint8_t* __restrict__ codes, S* __restrict__ scales, uint32_t lead_tiles) {
    constexpr bool S16 = sizeof(S) == 2;
    constexpr int GROUP = BLOCK >= kSlot ? kWave : BLOCK / kQuad;  // lanes per block within a slot
    constexpr size_t TILE = (size_t)kSlot * SLOTS;
    const int lane = threadIdx.x & (kWave - 1);
    // the first lead_tiles tile indices are left empty (see xcd_run_lead_tiles)
    const size_t wave = wave_tile_index<THREADS, XCDK>();
    if (wave < lead_tiles) return;  // whole wavefront
    const size_t tile0 = (wave - lead_tiles) * TILE;
    if (tile0 >= n) return;
    // the caller's flag, or Eq. 7's schedule read from the step counter in device memory
    const bool rst = step_index ? reset_step_due(step_index, reset_period) : reset != 0;

    float h[SLOTS][4], e[SLOTS][4], step[SLOTS];
    uint32_t pk[SLOTS];
    if (tile0 + TILE <= n) {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            Grad<G>::template load4<NT>(grad, i, h[s]);
            const f32x4 v = vload<NT>(reinterpret_cast<const f32x4*>(err + i));
            e[s][0] = v.x; e[s][1] = v.y; e[s][2] = v.z; e[s][3] = v.w;
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j) h[s][j] = clip_grad<CLIP>(h[s][j], clip) + e[s][j];  // Eq. 2
        cq_tile<BITS, BLOCK, SLOTS, S16>(h, e, beta, one_minus_beta, rst, lane, pk, step);
        if constexpr (STAGE_CODES && BITS == 4) {
            // SLOTS * 128 bytes of codes per wavefront: lane L puts its 2 bytes of slot s at
            // s*128 + 2L, lanes 0 .. SLOTS*8-1 then each take 16 bytes out and store them
            __shared__ uint16_t staged[THREADS / kWave][SLOTS * kWave];
            const uint32_t wv = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
#pragma unroll
            for (int s = 0; s < SLOTS; ++s) staged[wv][s * kWave + lane] = (uint16_t)pk[s];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (lane < SLOTS * 8) {
                const u32x4 v = reinterpret_cast<const u32x4*>(staged[wv])[lane];
                vstore<NT>(reinterpret_cast<u32x4*>(codes + (tile0 >> 1)) + lane, v);
            }
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            vstore<NT>(reinterpret_cast<f32x4*>(err + i), f32x4{e[s][0], e[s][1], e[s][2], e[s][3]});
            if constexpr (BITS == 4) {
                if constexpr (!STAGE_CODES) vstore<NT>(reinterpret_cast<uint16_t*>(codes + (i >> 1)), (uint16_t)pk[s]);
            } else {
                vstore<NT>(reinterpret_cast<uint32_t*>(codes + i), pk[s]);
            }
            // Block steps: move the slot's NBLK steps into lanes 0..NBLK-1 so that one
            // store writes them side by side from a wavefront-uniform base address
            // (measured: up to 13 % faster than letting each block's first lane store).
            if constexpr (BLOCK > kSlot) {
                if (lane == 0 && s % (BLOCK / kSlot) == 0)
                    scales[(tile0 + (size_t)s * kSlot) / BLOCK] = step_to_storage<S>(step[s]);
            } else {
                constexpr int NBLK = kWave / GROUP;
                const float v = NBLK > 1 ? __shfl(step[s], (lane * GROUP) & (kWave - 1), kWave) : step[s];
                if (lane < NBLK) scales[(tile0 + (size_t)s * kSlot) / BLOCK + lane] = step_to_storage<S>(v);
            }
        }
    } else {
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool in = i + j < n;
                e[s][j] = in ? err[i + j] : 0.0f;
                const float gj = in ? Grad<G>::load1(grad, i + j) : 0.0f;
                h[s][j] = clip_grad<CLIP>(gj, clip) + e[s][j];  // past n: h = 0, neutral for the max, code 0
            }
        }
        cq_tile<BITS, BLOCK, SLOTS, S16>(h, e, beta, one_minus_beta, rst, lane, pk, step);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i + j < n) err[i + j] = e[s][j];
            if constexpr (BITS == 4) {
                if (i < n) codes[i >> 1] = (uint8_t)pk[s];
                if (i + 2 < n) codes[(i >> 1) + 1] = (uint8_t)(pk[s] >> 8);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (i + j < n) codes[i + j] = (uint8_t)(pk[s] >> (8 * j));
            }
            if constexpr (BLOCK > kSlot) {
                if (lane == 0 && s % (BLOCK / kSlot) == 0 && i < n) scales[i / BLOCK] = step_to_storage<S>(step[s]);
            } else {
                if ((lane & (GROUP - 1)) == 0 && i < n) scales[i / BLOCK] = step_to_storage<S>(step[s]);
            }
        }
    }
}

// ---- what happens to the averaged gradient g~ of Eq. 8 ----
// kStore   write it out in fp32 (Algorithm 1 step 3 as such);
// kStoreBf16  write it out rounded to bf16 (nearest, ties to even), 2 B/element instead of 4;
// kSgd     Eq. 9:   theta' = theta - eta g~
// kAdam    Eq. 10:  m' = (1-b1) m + b1 g~;  v' = (1-b2) v + b2 g~^2;
//                   theta' = theta - (eta / sqrt(v' + delta)) m'
// Fusing the optimizer into the reduce saves writing g~ and reading it back (8 B/element).
// The optimizer state of a quad is fetched before the decode loop so its latency is hidden.
enum class Epilogue { kStore, kStoreBf16, kSgd, kAdam };

struct EpilogueArgs {
    float* out;                  // kStore (fp32), kStoreBf16 (the same pointer, holding bf16)
    float* theta;                // kSgd, kAdam (in place)
    float* m;                    // kAdam (in place)
    float* v;                    // kAdam (in place)
    float eta, beta1, one_minus_beta1, beta2, one_minus_beta2, delta;
};

template <Epilogue E> struct EpilogueState { f32x4 theta, m, v; };

// Resident wavefronts per SIMD for dr_kernel by what follows the sum.  With Adam the kernel
// updates three fp32 arrays in place on top of the payloads, a traffic mix like the
// compressor's, and like it runs 3 points of HBM peak faster with 4 than with the 8 its
// registers allow; the plain outputs and SGD are fastest with all 8.
constexpr int dr_waves_per_simd(Epilogue e) { return e == Epilogue::kAdam ? 4 : 8; }

// fp32 -> bf16, nearest with ties to even (the hardware conversion of gfx950); NaN stays NaN.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
    const __bf16 b = (__bf16)x;
    return __builtin_bit_cast(uint16_t, b);
}

template <Epilogue E, bool NT>
__device__ __forceinline__ void epilogue_prefetch(const EpilogueArgs& a, size_t i, EpilogueState<E>& st) {
    if constexpr (E == Epilogue::kSgd || E == Epilogue::kAdam)
        st.theta = vload<NT>(reinterpret_cast<const f32x4*>(a.theta + i));
    if constexpr (E == Epilogue::kAdam) {
        st.m = vload<NT>(reinterpret_cast<const f32x4*>(a.m + i));
        st.v = vload<NT>(reinterpret_cast<const f32x4*>(a.v + i));
    }
}

// One element of the optimizer step; g is the averaged gradient.
template <Epilogue E>
__device__ __forceinline__ void optimizer_element(const EpilogueArgs& a, float g, float& theta, float& m, float& v) {
    if constexpr (E == Epilogue::kSgd) {
        const float step = a.eta * g;
        theta = theta - step;
    } else if constexpr (E == Epilogue::kAdam) {
        const float b1g = a.beta1 * g;
        m = __builtin_fmaf(a.one_minus_beta1, m, b1g);
        const float g2 = g * g;
        const float b2g2 = a.beta2 * g2;
        v = __builtin_fmaf(a.one_minus_beta2, v, b2g2);
        const float root = sqrtf(v + a.delta);      // correctly rounded (see the build flags)
        const float eta_k = a.eta / root;
        const float step = eta_k * m;
        theta = theta - step;
    }
}

template <Epilogue E, bool NT>
__device__ __forceinline__ void epilogue_finish(const EpilogueArgs& a, size_t i, const float (&g)[4],
                                                EpilogueState<E>& st) {
    if constexpr (E == Epilogue::kStore) {
        vstore<NT>(reinterpret_cast<f32x4*>(a.out + i), f32x4{g[0], g[1], g[2], g[3]});
    } else if constexpr (E == Epilogue::kStoreBf16) {
        const uint32_t lo = (uint32_t)f32_to_bf16_bits(g[0]) | ((uint32_t)f32_to_bf16_bits(g[1]) << 16);
        const uint32_t hi = (uint32_t)f32_to_bf16_bits(g[2]) | ((uint32_t)f32_to_bf16_bits(g[3]) << 16);
        vstore<NT>(reinterpret_cast<u32x2*>(reinterpret_cast<uint16_t*>(a.out) + i), u32x2{lo, hi});
    } else {
        float th[4] = {st.theta.x, st.theta.y, st.theta.z, st.theta.w};
        float m[4] = {0.f, 0.f, 0.f, 0.f}, v[4] = {0.f, 0.f, 0.f, 0.f};
        if constexpr (E == Epilogue::kAdam) {
            m[0] = st.m.x; m[1] = st.m.y; m[2] = st.m.z; m[3] = st.m.w;
            v[0] = st.v.x; v[1] = st.v.y; v[2] = st.v.z; v[3] = st.v.w;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) optimizer_element<E>(a, g[j], th[j], m[j], v[j]);
        vstore<NT>(reinterpret_cast<f32x4*>(a.theta + i), f32x4{th[0], th[1], th[2], th[3]});
        if constexpr (E == Epilogue::kAdam) {
            vstore<NT>(reinterpret_cast<f32x4*>(a.m + i), f32x4{m[0], m[1], m[2], m[3]});
            vstore<NT>(reinterpret_cast<f32x4*>(a.v + i), f32x4{v[0], v[1], v[2], v[3]});
        }
    }
}

// Guarded (element-by-element) form for the last, partial tile.
template <Epilogue E>
__device__ __forceinline__ void epilogue_element(const EpilogueArgs& a, size_t i, float g) {
    if constexpr (E == Epilogue::kStore) {
        a.out[i] = g;
    } else if constexpr (E == Epilogue::kStoreBf16) {
        reinterpret_cast<uint16_t*>(a.out)[i] = f32_to_bf16_bits(g);
    } else {
        float th = a.theta[i], m = 0.f, v = 0.f;
        if constexpr (E == Epilogue::kAdam) { m = a.m[i]; v = a.v[i]; }
        optimizer_element<E>(a, g, th, m, v);
        a.theta[i] = th;
        if constexpr (E == Epilogue::kAdam) { a.m[i] = m; a.v[i] = v; }
    }
}

// ---- Algorithm 1 step 3 / Eq. 8 ----
// One worker's contribution to one quad: acc_j = acc_j + (float) q_j * D, j = 0..3, where c
// holds the quad's codes in its low 16 (4-bit) or 32 (8-bit) bits.
//
// W decodes per output element make the arithmetic a visible share of this kernel's time (at
// W = 8 the vector ALUs are busy two thirds of it), so the decode is kept to three instructions
// per element and worker:
//   8-bit  v_cvt_f32_i32 with a sign-extending byte select, v_mul, v_add;
//   4-bit  v_cvt_off_f32_i4, which maps a two's complement nibble q straight to the float
//          q/16, then v_mul by 16*D, v_add.  (q/16) * (16 D) is q * D with the same single
//          rounding as long as 16 D does not overflow; the kernels take this path first and
//          sum a tile again with the plain one if a step of 2^120 or more was met.
template <int BITS>
__device__ __forceinline__ void dr_accumulate(uint32_t c, float D, float (&acc)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int q = ((int)(c << (32 - BITS * (j + 1)))) >> (32 - BITS);  // signed field j
        const float d = (float)q * D;   // decompressor of Eq. 1
        acc[j] = acc[j] + d;            // sum of Eq. 8, in worker order
    }
}
// v_cvt_off_f32_i4 of the low nibble of byte SEL of x (an SDWA byte select instead of a shift).
template <int SEL>
__device__ __forceinline__ float cvt_off_i4_byte(uint32_t x) {
    static_assert(SEL >= 0 && SEL < 4, "byte select");
    float f;
    if constexpr (SEL == 0) f = __builtin_amdgcn_cvt_off_f32_i4((int)x);
    else if constexpr (SEL == 1)
        asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1" : "=v"(f) : "v"(x));
    else if constexpr (SEL == 2)
        asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2" : "=v"(f) : "v"(x));
    else
        asm("v_cvt_off_f32_i4_sdwa %0, %1 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3" : "=v"(f) : "v"(x));
    return f;
}
__device__ __forceinline__ void dr_accumulate_nibbles_x16(uint32_t c, float D16, float (&acc)[4]) {
    const uint32_t t = c >> 4;
    const float f0 = __builtin_amdgcn_cvt_off_f32_i4((int)c);   // q0 / 16
    const float f1 = __builtin_amdgcn_cvt_off_f32_i4((int)t);   // q1 / 16
    const float f2 = cvt_off_i4_byte<1>(c);                       // q2 / 16
    const float f3 = cvt_off_i4_byte<1>(t);                       // q3 / 16
    acc[0] = acc[0] + f0 * D16;
    acc[1] = acc[1] + f1 * D16;
    acc[2] = acc[2] + f2 * D16;
    acc[3] = acc[3] + f3 * D16;
}

template <int BITS, bool NT>
__device__ __forceinline__ uint32_t load_quad_codes(const uint8_t* p) {
    if constexpr (BITS == 4) return vload<NT>(reinterpret_cast<const uint16_t*>(p));
    else return vload<NT>(reinterpret_cast<const uint32_t*>(p));
}

// ---- the last, partial tile of a reduce ----
// A tile that n cuts short is summed with byte loads that never leave the payloads: a lane whose
// elements do not exist works on the last group of elements that does, and a byte that does not exist
// is replaced by the last one that does; what such duplicates decode to is never stored.  All loads
// are unconditional, so the loads of kTailPayloads payloads are in flight together: a lane waits
// W / kTailPayloads times, not once per payload and element (a ragged shard with 128 payloads spent
// 0.15 - 0.45 ms in this path alone when it did).
constexpr int kTailPayloads = 4;
template <int BYTES>
__device__ __forceinline__ void load_bytes_clamped(const uint8_t* p, uint32_t have, uint32_t (&out)[BYTES / 4]) {
#pragma unroll
    for (int k = 0; k < BYTES / 4; ++k) out[k] = 0u;
#pragma unroll
    for (int k = 0; k < BYTES; ++k) out[k / 4] |= (uint32_t)p[(uint32_t)k < have ? (uint32_t)k : have - 1u] << (8 * (k % 4));
}
// Bytes of codes that exist for a group of `group` elements starting at element i < n.
template <int BITS>
__device__ __forceinline__ uint32_t code_bytes_present(size_t i, size_t n, uint32_t group) {
    const size_t left = n - i;
    const uint32_t elems = left < group ? (uint32_t)left : group;
    return (elems * BITS + 7u) / 8u;
}

constexpr uint32_t kBigStepBits = 0x7B800000u;  // 2^120 as a binary32 bit pattern

// Same decomposition as cq_kernel; WU payloads are in flight per lane and slot.  Addresses
// are a wavefront-uniform base (SGPRs, advanced per worker on the scalar unit) plus a
// 32-bit lane offset; with BLOCK >= 256 a slot lies in one block, so its step is a scalar
// load shared by the wavefront.
template <int BITS, int BLOCK, int SLOTS, int THREADS, int WU, bool NT, int XCDK, Epilogue EPI, typename S,
          bool LANE_STEPS = false, int WAVES = dr_waves_per_simd(EPI)>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, WAVES)))
dr_kernel(const uint8_t* __restrict__ codes, size_t code_stride, const S* __restrict__ scales,
          size_t scale_stride, int W, size_t n, float inv_w, EpilogueArgs epi, uint32_t lead_tiles) {
    constexpr size_t TILE = (size_t)kSlot * SLOTS;
    constexpr bool UNIFORM_STEP = BLOCK >= kSlot;
    constexpr uint32_t SLOT_CODE_BYTES = kSlot * BITS / 8;
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const size_t wave = wave_tile_index_tail_first<THREADS, XCDK>(n, TILE, lead_tiles);
    const size_t tile0 = wave * TILE;
    if (tile0 >= n) return;

    if (tile0 + TILE <= n) {
        const uint8_t* cbase = codes + tile0 * BITS / 8;   // uniform
        size_t sidx = tile0 / BLOCK;                        // uniform
        const uint32_t code_off = lane * (kQuad * BITS / 8);
        const uint32_t step_off = UNIFORM_STEP ? 0u : lane / (uint32_t)(BLOCK / kQuad);
        float acc[SLOTS][4];
        EpilogueState<EPI> est[SLOTS];
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            epilogue_prefetch<EPI, NT>(epi, tile0 + (size_t)s * kSlot + (size_t)lane * kQuad, est[s]);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[s][j] = 0.0f;
        }

        // LANE_STEPS (blocks of 128 elements and more): the steps of a whole chunk of workers
        // come in with ONE vector load, lane (u, s, half) fetching the step of worker u, slot s
        // (and half-slot, when a slot holds two blocks), and are handed to the wavefront with
        // lane reads.  Through the scalar cache instead, the lines of steps were fetched from
        // memory about twice (3.7 % more read traffic at 4 bits, B = 256).
        constexpr int NBPS = BLOCK >= kSlot ? 1 : kSlot / BLOCK;   // blocks per slot
        constexpr int PER_W = SLOTS * NBPS;                        // steps per worker in this tile
        static_assert(!LANE_STEPS || (NBPS <= 2 && WU * PER_W <= kWave), "steps of a chunk fit one wavefront load");
        const uint32_t ls_u = lane / PER_W, ls_r = lane % PER_W;
        const size_t ls_off = (size_t)ls_u * scale_stride + ((ls_r / NBPS) * kSlot) / BLOCK + (NBPS == 2 ? ls_r % NBPS : 0);
        auto load_chunk = [&](int count, uint32_t (&c)[WU][SLOTS], float (&D)[WU][SLOTS]) {
            float lane_step = 0.0f;
            if constexpr (LANE_STEPS) {
                if (lane < (uint32_t)(count * PER_W)) lane_step = step_from_storage(scales[sidx + ls_off]);
            }
#pragma unroll
            for (int u = 0; u < WU; ++u) {
                if (u < count) {
#pragma unroll
                    for (int s = 0; s < SLOTS; ++s) {
                        c[u][s] = load_quad_codes<BITS, NT>(cbase + (size_t)(s * SLOT_CODE_BYTES + code_off));
                        if constexpr (LANE_STEPS) {
                            // filled in below, once the chunk's loads are all issued
                        } else if constexpr (UNIFORM_STEP) {
                            D[u][s] = load_uniform_step(scales, sidx + (s * kSlot) / BLOCK);
                        } else if constexpr (BLOCK * 2 == kSlot) {
                            // two blocks per slot: two scalar loads and a select by half-wavefront measured
                            // 1-4 % faster than a vector load (with 4 or 8 blocks per slot it is slower)
                            const float lo = load_uniform_step(scales, sidx + (size_t)(s * 2));
                            const float hi = load_uniform_step(scales, sidx + (size_t)(s * 2 + 1));
                            D[u][s] = step_off ? hi : lo;
                        } else {
                            D[u][s] = step_from_storage(scales[sidx + (size_t)(s * (kSlot / BLOCK) + step_off)]);
                        }
                    }
                    cbase += code_stride;
                    sidx += scale_stride;
                }
            }
            if constexpr (LANE_STEPS) {
#pragma unroll
                for (int u = 0; u < WU; ++u)
                    if (u < count)
#pragma unroll
                        for (int s = 0; s < SLOTS; ++s) {
                            if constexpr (NBPS == 1) {
                                D[u][s] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lane_step), u * PER_W + s));
                            } else {
                                const float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lane_step), (u * SLOTS + s) * 2));
                                const float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, lane_step), (u * SLOTS + s) * 2 + 1));
                                D[u][s] = lane < 32 ? lo : hi;
                            }
                        }
            }
        };
        // 4-bit codes take the 16*D shortcut of dr_accumulate without asking whether it holds:
        // `top` gathers the largest step seen, as a bit pattern (a negative step compares as larger
        // than any positive one), and if that turns out to be 2^120 or more the tile is summed
        // again from the start with the plain arithmetic.  Steps that large do not come out of the
        // compressor for finite gradients of ordinary size, and a loop without a second path
        // keeps the sums in the same registers from one iteration to the next.
        uint32_t top = 0;
        auto accumulate_chunk = [&](int count, const uint32_t (&c)[WU][SLOTS], const float (&D)[WU][SLOTS]) {
#pragma unroll
            for (int u = 0; u < WU; ++u)
                if (u < count)
#pragma unroll
                    for (int s = 0; s < SLOTS; ++s) {
                        if constexpr (BITS == 4) {
                            top = umax(top, __float_as_uint(D[u][s]));
                            dr_accumulate_nibbles_x16(c[u][s], D[u][s] * 16.0f, acc[s]);
                        } else {
                            dr_accumulate<8>(c[u][s], D[u][s], acc[s]);
                        }
                    }
        };

        const int chunks = W / WU, rest = W % WU;
        // From three chunks on, 4-bit codes run with two register sets: the loads of one chunk are
        // in flight while the other is summed (2-4 points of HBM peak at W = 16..48).  With two
        // chunks that would put all 2*WU payloads in flight at once, which measured slower; 8-bit
        // codes gain nothing from it, and the variants with lane-loaded or bf16 steps would not
        // fit the 64 registers that eight resident wavefronts per SIMD leave each.
        constexpr bool TWO_SETS = BITS == 4 && !LANE_STEPS && sizeof(S) == 4;
        if (TWO_SETS && chunks >= 3) {
            uint32_t ca[WU][SLOTS], cb2[WU][SLOTS];
            float Da[WU][SLOTS], Db[WU][SLOTS];
            load_chunk(WU, ca, Da);
            int i = 1;
            for (; i + 1 < chunks; i += 2) {
                load_chunk(WU, cb2, Db);
                accumulate_chunk(WU, ca, Da);
                load_chunk(WU, ca, Da);
                accumulate_chunk(WU, cb2, Db);
            }
            if (i < chunks) {
                load_chunk(WU, cb2, Db);
                accumulate_chunk(WU, ca, Da);
                accumulate_chunk(WU, cb2, Db);
            } else {
                accumulate_chunk(WU, ca, Da);
            }
        } else {
            for (int i = 0; i < chunks; ++i) {
                uint32_t c[WU][SLOTS];
                float D[WU][SLOTS];
                load_chunk(WU, c, D);
                accumulate_chunk(WU, c, D);
            }
        }
        if (rest) {
            uint32_t c[WU][SLOTS];
            float D[WU][SLOTS];
            load_chunk(rest, c, D);
            accumulate_chunk(rest, c, D);
        }
        if constexpr (BITS == 4) {
            if (__builtin_expect(__any(top >= kBigStepBits), 0)) {
                const uint8_t* p = codes + tile0 * BITS / 8 + code_off;
                const S* ps = scales + tile0 / BLOCK + (lane * kQuad) / (uint32_t)BLOCK;
#pragma unroll
                for (int s = 0; s < SLOTS; ++s)
#pragma unroll
                    for (int j = 0; j < 4; ++j) acc[s][j] = 0.0f;
#pragma unroll 1
                for (int w = 0; w < W; ++w, p += code_stride, ps += scale_stride)
#pragma unroll
                    for (int s = 0; s < SLOTS; ++s)
                        dr_accumulate<4>(load_quad_codes<BITS, NT>(p + s * SLOT_CODE_BYTES),
                                         step_from_storage(ps[(s * kSlot) / BLOCK]), acc[s]);
            }
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            const float g[4] = {acc[s][0] * inv_w, acc[s][1] * inv_w, acc[s][2] * inv_w, acc[s][3] * inv_w};
            epilogue_finish<EPI, NT>(epi, i, g, est[s]);
        }
    } else {
        // last, partial tile (see load_bytes_clamped)
        constexpr int QB = kQuad * BITS / 8;        // code bytes per quad: 2 or 4
        const size_t last_quad = (n - 1) & ~(size_t)(kQuad - 1);
        size_t at[SLOTS];
        uint32_t have[SLOTS];
        float acc[SLOTS][4];
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
            at[s] = i < n ? i : last_quad;
            have[s] = code_bytes_present<BITS>(at[s], n, kQuad);
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[s][j] = 0.0f;
        }
        for (int w0 = 0; w0 < W; w0 += kTailPayloads) {
            uint32_t c[kTailPayloads][SLOTS];
            float D[kTailPayloads][SLOTS];
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
                    D[u][s] = step_from_storage(scales[w * scale_stride + at[s] / BLOCK]);
                }
            }
#pragma unroll
            for (int u = 0; u < kTailPayloads; ++u)
                if (w0 + u < W)
#pragma unroll
                    for (int s = 0; s < SLOTS; ++s) dr_accumulate<BITS>(c[u][s], D[u][s], acc[s]);
        }
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i + j < n) epilogue_element<EPI>(epi, i + j, acc[s][j] * inv_w);
        }
    }
}

// Eight nibbles of one dword: acc_j = acc_j + (q_j / 16) * (16 D), j = 0..7.
__device__ __forceinline__ void dr_accumulate_octet_x16(uint32_t c, float D16, float* acc) {
    const uint32_t t = c >> 4;
    acc[0] = acc[0] + cvt_off_i4_byte<0>(c) * D16;
    acc[1] = acc[1] + cvt_off_i4_byte<0>(t) * D16;
    acc[2] = acc[2] + cvt_off_i4_byte<1>(c) * D16;
    acc[3] = acc[3] + cvt_off_i4_byte<1>(t) * D16;
    acc[4] = acc[4] + cvt_off_i4_byte<2>(c) * D16;
    acc[5] = acc[5] + cvt_off_i4_byte<2>(t) * D16;
    acc[6] = acc[6] + cvt_off_i4_byte<3>(c) * D16;
    acc[7] = acc[7] + cvt_off_i4_byte<3>(t) * D16;
}
// One dword of codes in the plain form (any step): 8 nibbles or 4 bytes.
template <int BITS>
__device__ __forceinline__ void dr_accumulate_dword(uint32_t c, float D, float* acc) {
#pragma unroll
    for (int j = 0; j < 32 / BITS; ++j) {
        const int q = ((int)(c << (32 - BITS * (j + 1)))) >> (32 - BITS);
        const float d = (float)q * D;
        acc[j] = acc[j] + d;
    }
}

// ---- Algorithm 1 step 3 / Eq. 8 with wide code loads ----
// The same arithmetic as dr_kernel in another decomposition: a lane loads CB = 4, 8 or 16
// bytes of codes per worker, i.e. EL = 8*CB/BITS consecutive elements, so a wavefront
// instruction fetches 256 B .. 1 KB of one payload instead of 128 B (4-bit quads) and a
// wavefront owns one unit of 64*EL elements.  A lane's EL sums are consecutive in memory;
// before they are written they are transposed through a wavefront-private piece of LDS
// into the quad layout, so that every store instruction (and every optimizer-state access
// of the fused epilogues) covers 1 KB without gaps.  No barrier: a wavefront only reads
// what it wrote itself, and its LDS instructions execute in order.
//
// Block steps: a lane's EL <= 32 elements lie inside one block.  A unit inside one block
// takes a scalar load, two blocks per unit take two scalar loads and a select, more blocks
// per unit a vector load in which the lanes of a block share the address.
template <int CB> struct CodeWord;
template <> struct CodeWord<4> { typedef uint32_t type; };
template <> struct CodeWord<8> { typedef u32x2 type; };
template <> struct CodeWord<16> { typedef u32x4 type; };
template <int CB>
__device__ __forceinline__ uint32_t code_dword(const typename CodeWord<CB>::type& v, int k) {
    if constexpr (CB == 4) return v;
    else return v[k];
}

// Index of 16-byte piece p of a wavefront's LDS region: the low three bits are mixed with
// the next three, so that the eight lanes served together hit different banks both when
// lanes write their own consecutive pieces and when they read the transposed ones.
__device__ __forceinline__ uint32_t lds_piece(uint32_t p) { return p ^ ((p >> 3) & 7u); }

template <int BITS, int BLOCK, int CB, int THREADS, int WU, bool NT, int XCDK, Epilogue EPI, typename S>
__global__ void __launch_bounds__(THREADS)
dr_wide_kernel(const uint8_t* __restrict__ codes, size_t code_stride, const S* __restrict__ scales,
               size_t scale_stride, int W, size_t n, float inv_w, EpilogueArgs epi, uint32_t lead_tiles) {
    constexpr int EL = CB * 8 / BITS;             // elements per lane
    constexpr int NQ = EL / kQuad;                // quads (16-byte pieces of fp32) per lane
    constexpr int DW = CB / 4;                    // code dwords per lane and worker
    constexpr int PER_DW = 32 / BITS;             // elements per code dword
    constexpr size_t UNIT = (size_t)kWave * EL;
    constexpr bool UNIFORM_STEP = BLOCK >= (int)UNIT;
    constexpr int NBLK = UNIFORM_STEP ? 1 : (int)UNIT / BLOCK;   // blocks per unit
    static_assert(EL >= 8 && EL <= 32 && EL <= BLOCK, "a lane's elements lie inside one block");
    typedef typename CodeWord<CB>::type code_t;
    __shared__ f32x4 stage[THREADS / kWave][kWave * NQ];
    const uint32_t lane = threadIdx.x & (kWave - 1);
    const uint32_t wv = (uint32_t)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const size_t tile0 = wave_tile_index_tail_first<THREADS, XCDK>(n, UNIT, lead_tiles) * UNIT;
    if (tile0 >= n) return;

    if (tile0 + UNIT <= n) {
        const uint8_t* cbase = codes + tile0 * BITS / 8;   // uniform, advanced per worker
        size_t sidx = tile0 / BLOCK;                        // uniform, advanced per worker
        const uint32_t code_off = lane * CB;
        const uint32_t step_off = UNIFORM_STEP ? 0u : (lane * EL) / (uint32_t)BLOCK;
        float acc[EL];
#pragma unroll
        for (int j = 0; j < EL; ++j) acc[j] = 0.0f;

        // One chunk of `count` workers: all loads first, then the sums.  4-bit codes take the 16*D
        // shortcut (see dr_accumulate) without asking whether it holds: `top` gathers the largest
        // step seen, as a bit pattern (a negative step compares as larger than any positive one),
        // and if that turns out to be 2^120 or more the unit is summed again from the start with
        // the plain arithmetic.  Steps that large do not come out of the compressor for finite
        // gradients of ordinary size, and a loop without a second path keeps the EL sums in the
        // same registers from one iteration to the next.
        uint32_t top = 0;
        auto load_chunk = [&](int count, code_t (&c)[WU], float (&D)[WU]) {
#pragma unroll
            for (int u = 0; u < WU; ++u) {
                if (u < count) {
                    c[u] = vload<NT>(reinterpret_cast<const code_t*>(cbase + code_off));
                    if constexpr (UNIFORM_STEP) {
                        D[u] = load_uniform_step(scales, sidx);
                    } else if constexpr (NBLK == 2) {
                        const float lo = load_uniform_step(scales, sidx);
                        const float hi = load_uniform_step(scales, sidx + 1);
                        D[u] = step_off ? hi : lo;
                    } else {
                        D[u] = step_from_storage(scales[sidx + step_off]);
                    }
                    cbase += code_stride;
                    sidx += scale_stride;
                }
            }
        };
        auto accumulate_chunk = [&](int count, const code_t (&c)[WU], const float (&D)[WU]) {
#pragma unroll
            for (int u = 0; u < WU; ++u)
                if (u < count) {
                    if constexpr (BITS == 4) {
                        top = umax(top, __float_as_uint(D[u]));
                        const float D16 = D[u] * 16.0f;
#pragma unroll
                        for (int k = 0; k < DW; ++k) dr_accumulate_octet_x16(code_dword<CB>(c[u], k), D16, acc + k * PER_DW);
                    } else {
#pragma unroll
                        for (int k = 0; k < DW; ++k) dr_accumulate_dword<8>(code_dword<CB>(c[u], k), D[u], acc + k * PER_DW);
                    }
                }
        };
        const int chunks = W / WU, rest = W % WU;
        // two register sets: the loads of one chunk are in flight while the other is summed
        code_t ca[WU], cb2[WU];
        float Da[WU], Db[WU];
        if (chunks > 0) {
            load_chunk(WU, ca, Da);
            int i = 1;
            for (; i + 1 < chunks; i += 2) {
                load_chunk(WU, cb2, Db);
                accumulate_chunk(WU, ca, Da);
                load_chunk(WU, ca, Da);
                accumulate_chunk(WU, cb2, Db);
            }
            if (i < chunks) {
                load_chunk(WU, cb2, Db);
                accumulate_chunk(WU, ca, Da);
                accumulate_chunk(WU, cb2, Db);
            } else {
                accumulate_chunk(WU, ca, Da);
            }
        }
        if (rest) {
            code_t c[WU];
            float D[WU];
            load_chunk(rest, c, D);
            accumulate_chunk(rest, c, D);
        }
        if constexpr (BITS == 4) {
            if (__builtin_expect(__any(top >= kBigStepBits), 0)) {
                const uint8_t* p = codes + tile0 * BITS / 8 + code_off;
                const S* ps = scales + tile0 / BLOCK + (lane * EL) / (uint32_t)BLOCK;
#pragma unroll
                for (int j = 0; j < EL; ++j) acc[j] = 0.0f;
#pragma unroll 1
                for (int w = 0; w < W; ++w, p += code_stride, ps += scale_stride) {
                    const code_t c = vload<NT>(reinterpret_cast<const code_t*>(p));
                    const float D = step_from_storage(*ps);
#pragma unroll
                    for (int k = 0; k < DW; ++k) dr_accumulate_dword<4>(code_dword<CB>(c, k), D, acc + k * PER_DW);
                }
            }
        }

        // the optimizer state of the fused epilogues is fetched only now (its latency hides behind the
        // transposition): held across the decode loop it would cost up to 96 registers per lane
        EpilogueState<EPI> est[NQ];
#pragma unroll
        for (int k = 0; k < NQ; ++k)
            epilogue_prefetch<EPI, NT>(epi, tile0 + (size_t)k * kSlot + (size_t)lane * kQuad, est[k]);
        // transpose: lane L holds elements [L*EL, L*EL + EL) of the unit; store k wants lane L
        // to hold elements [k*256 + 4L, +4)
        f32x4* mine = stage[wv];
#pragma unroll
        for (int k = 0; k < NQ; ++k)
            mine[lds_piece(lane * NQ + k)] = f32x4{acc[4 * k] * inv_w, acc[4 * k + 1] * inv_w,
                                                   acc[4 * k + 2] * inv_w, acc[4 * k + 3] * inv_w};
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int k = 0; k < NQ; ++k) {
            const f32x4 v = mine[lds_piece((uint32_t)k * kWave + lane)];
            const float g[4] = {v.x, v.y, v.z, v.w};
            epilogue_finish<EPI, NT>(epi, tile0 + (size_t)k * kSlot + (size_t)lane * kQuad, g, est[k]);
        }
    } else {
        // last, partial unit (see load_bytes_clamped); a lane's EL elements lie inside one block
        const size_t mine = tile0 + (size_t)lane * EL;
        const size_t first = mine < n ? mine : (n - 1) / EL * EL;
        const uint32_t have = code_bytes_present<BITS>(first, n, EL);
        float acc[EL];
#pragma unroll
        for (int j = 0; j < EL; ++j) acc[j] = 0.0f;
        for (int w0 = 0; w0 < W; w0 += kTailPayloads) {
            uint32_t c[kTailPayloads][DW];
            float D[kTailPayloads];
#pragma unroll
            for (int u = 0; u < kTailPayloads; ++u) {
                const size_t w = (size_t)(w0 + u < W ? w0 + u : W - 1);
                load_bytes_clamped<CB>(codes + w * code_stride + first * BITS / 8, have, c[u]);
                D[u] = step_from_storage(scales[w * scale_stride + first / BLOCK]);
            }
#pragma unroll
            for (int u = 0; u < kTailPayloads; ++u)
                if (w0 + u < W)
#pragma unroll
                    for (int k = 0; k < DW; ++k) dr_accumulate_dword<BITS>(c[u][k], D[u], acc + k * PER_DW);
        }
#pragma unroll
        for (int j = 0; j < EL; ++j)
            if (mine + j < n) epilogue_element<EPI>(epi, mine + j, acc[j] * inv_w);
    }
}

// The step counter k of Eq. 7 in device memory: set it (add == 0) or add to it (add != 0).
// One lane writes, with an ordinary vector store.
__global__ void step_index_kernel(long long* step_index, long long value, int add) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *step_index = add ? *step_index + value : value;
}

// ---- helpers: zero fill of the state, plain streaming kernels (16 bytes per lane and slot) ----
constexpr int kFillWavesPerSimd = 3;   // see stream_waves_per_simd
template <int SLOTS, int THREADS, bool NT>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, kFillWavesPerSimd)))
fill_zero_kernel(float* __restrict__ dst, size_t n) {
    const int lane = threadIdx.x & (kWave - 1);
    const size_t wave = (size_t)blockIdx.x * (THREADS / kWave) + (threadIdx.x >> 6);
    const size_t tile0 = wave * ((size_t)kSlot * SLOTS);
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const size_t i = tile0 + (size_t)s * kSlot + (size_t)lane * kQuad;
        if (i + 4 <= n) {
            vstore<NT>(reinterpret_cast<f32x4*>(dst + i), f32x4{0.f, 0.f, 0.f, 0.f});
        } else {
            for (size_t j = i; j < n; ++j) dst[j] = 0.0f;
        }
    }
}

// Plain streaming kernels for measuring what the memory system sustains for a given mix of
// reads and writes: kCopy dst = src; kRead loads src and stores (to sink) only if the words of
// a lane's 16 bytes xor to `never`, so that the loads cannot be dropped; kFill writes zeros;
// kSum2 dst = src + src2 word by word (two read streams, one write stream).
enum class StreamMode { kCopy, kRead, kFill, kSum2 };
// Resident wavefronts per SIMD at which each stream measured fastest in its launch shape: a pure
// write stream wants few (90 % of HBM peak with 2-3 against 82 % with 8), a pure read stream 6
// (94 % against 89 %), two reads and a write 5, the copy all 8.
constexpr int stream_waves_per_simd(StreamMode m) {
    return m == StreamMode::kFill ? kFillWavesPerSimd : m == StreamMode::kRead ? 6 : m == StreamMode::kSum2 ? 5 : 8;
}
template <StreamMode MODE, int SLOTS, int THREADS, bool NT>
__global__ void __launch_bounds__(THREADS) __attribute__((amdgpu_waves_per_eu(1, stream_waves_per_simd(MODE))))
stream_kernel(u32x4* __restrict__ dst, const u32x4* __restrict__ src, const u32x4* __restrict__ src2,
              size_t n16, uint32_t never) {
    const int lane = threadIdx.x & (kWave - 1);
    const size_t wave = (size_t)blockIdx.x * (THREADS / kWave) + (threadIdx.x >> 6);
    const size_t tile0 = wave * ((size_t)kWave * SLOTS);
    u32x4 v[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const size_t i = tile0 + (size_t)s * kWave + lane;
        v[s] = u32x4{0u, 0u, 0u, 0u};
        if constexpr (MODE != StreamMode::kFill)
            if (i < n16) v[s] = vload<NT>(src + i);
        if constexpr (MODE == StreamMode::kSum2)
            if (i < n16) v[s] += vload<NT>(src2 + i);
    }
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const size_t i = tile0 + (size_t)s * kWave + lane;
        if constexpr (MODE == StreamMode::kRead) {
            if (i < n16 && (v[s].x ^ v[s].y ^ v[s].z ^ v[s].w) == never) dst[0] = v[s];
        } else {
            if (i < n16) vstore<NT>(dst + i, v[s]);
        }
    }
}

// In-place update of three arrays (a += 1; b += a; c += b on 32-bit words): the traffic of an
// optimizer with two moment arrays and nothing else, three read and three write streams.
template <int SLOTS, int THREADS, bool NT>
__global__ void __launch_bounds__(THREADS)
update3_kernel(u32x4* __restrict__ a, u32x4* __restrict__ b, u32x4* __restrict__ c, size_t n16) {
    const int lane = threadIdx.x & (kWave - 1);
    const size_t wave = (size_t)blockIdx.x * (THREADS / kWave) + (threadIdx.x >> 6);
    const size_t tile0 = wave * ((size_t)kWave * SLOTS);
    u32x4 x[SLOTS], y[SLOTS], z[SLOTS];
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const size_t i = tile0 + (size_t)s * kWave + lane;
        if (i < n16) { x[s] = vload<NT>(a + i); y[s] = vload<NT>(b + i); z[s] = vload<NT>(c + i); }
    }
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
        const size_t i = tile0 + (size_t)s * kWave + lane;
        if (i < n16) {
            x[s] += 1u; y[s] += x[s]; z[s] += y[s];
            vstore<NT>(a + i, x[s]); vstore<NT>(b + i, y[s]); vstore<NT>(c + i, z[s]);
        }
    }
}

}  // namespace loco
