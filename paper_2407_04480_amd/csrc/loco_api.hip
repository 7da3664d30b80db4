// Host side of the C ABI declared in include/loco.h: argument checks, dispatch on
// (gradient type, bits, block size), launches on the caller's stream.  No allocation,
// no synchronisation, no CPU fallback: without a GPU every compute call fails.
#include "loco.h"
#include "loco_kernels.h"
#include "loco_fixed_kernels.h"

#include <atomic>
#include <cmath>
#include <cstdint>
#include <tuple>
#include <type_traits>
#include <utility>

namespace {

using namespace loco;

// Launch shapes chosen by measurement on MI355X (sweeps at the 7B-shard size): slots of
// 256 elements per wavefront, threads per workgroup, payloads in flight per lane in the
// reduce kernel, the non-temporal hint on the streaming accesses, XCD-aware tile order.
// Compensate-quantize: two slots per wavefront, at most 4 wavefronts resident per SIMD (see
// kCqWavesPerSimd); with that, one-wavefront workgroups for 8-bit codes and two wavefronts for
// 4-bit codes measured best (up to 2 points over the other choice, and over 4 slots or 256 threads).
// Its tiles go to the XCDs in runs of 32768 consecutive elements (128 KB of state; see
// wave_tile_index): with the residency above that measured 2-3.5 points of HBM peak faster than the
// hardware's own round robin (bf16, 4-bit, B = 256: 83.2 % against 81.1 %; 8-bit, B = 64: 84.7 against
// 81.2; 2.2e9 elements: 84.2 against 80.7), twice that 1 point less, four times nothing, and HALF of it
// 6 points slower than no runs at all; run lengths that are no powers of two (24576...49152 elements) 3-6
// points slower than 32768; the same order for fp32 gradients.  (At full residency the runs had measured
// no gain.)  The runs are counted from a multiple of 128 KB of the state's address, not from its first
// element (xcd_run_lead_tiles).
constexpr int kCqXcdRunElements = 32768;
template <int BITS, int BLOCK = 256> struct CqShape {
    static constexpr int kSlots = 2, kThreads = BITS == 8 ? 64 : 128;
    static constexpr int kXcdRun = kCqXcdRunElements / (kSlot * kSlots * (kThreads / kWave));
};
template <int BITS> struct DrShape;
template <> struct DrShape<4> { static constexpr int kSlots = 2, kThreads = 128, kInFlight = 4; };
template <> struct DrShape<8> { static constexpr int kSlots = 1, kThreads = 256, kInFlight = 4; };
// With few workers the reduce is mostly a write stream, which measured 3-9 % faster with
// 2 KB of output per wavefront and 8 KB per workgroup; with two or three payloads of 4-bit codes
// 4 KB per wavefront (B = 256, W = 2: 80 % of HBM peak against 73 %; W = 3: 79 against 77; B = 64 the
// same either way); up to three payloads of 8-bit codes with 6 resident wavefronts per SIMD instead of
// 8 (W = 1: 82.6 % against 79.2 %; W = 2, 3: 80-83 % against 75-79 % in the many-payload shape).
struct DrFewWorkersShape { static constexpr int kSlots = 2, kThreads = 256, kInFlight = 4; };
struct DrTwoOrThreeWorkersShape { static constexpr int kSlots = 4, kThreads = 256, kInFlight = 4; };
constexpr bool dr_few_workers(int bits, int W) { return bits == 4 ? W <= 4 : W <= 3; }
constexpr int kDrFewPayloads8BitWaves = 6;
constexpr bool kNonTemporal = true;
// Consecutive workgroups' tiles per XCD (see wave_tile_index): dequant-reduce loses nothing with
// runs of 32, which keeps each cache line of block steps in one L2 instead of fetching it into all
// eight (and is, for its two main shapes, again 32768 elements per run).
constexpr int kDrXcdRun = 32;
// The hardware's own round robin of workgroups over the XCDs instead of runs of tiles per XCD: when the
// payloads together hold 2^33 bytes of codes or more (and there are at least 8 of them) it measured 2-6
// points of HBM peak faster for the quad layout, the 8-byte code loads and the fixed-scale reduce (4-bit,
// 2.2e9 elements, W = 16: 82.5 % against 76 %; 8.4e8 elements, W = 32: 76.5 against 74.0; 8-bit, W = 32:
// 74.2 against 72.5; fixed-scale, 2.2e9 elements, W = 16: 77.7 against 75.1), although every L2 then
// fetches the lines of block steps for itself (read traffic 1.24x instead of 1.04x of the algorithmic
// bytes at 4 bits, B = 256).  Below that amount the runs are 1-3 points faster; the 16-byte code loads are
// the same either way.  Not when the payload strides are multiples of a large power of two: the W loads of
// a wavefront then meet in one memory channel, which the round robin suffers from far more (down to
// 40-60 % of the rate).
constexpr int kDrNaturalOrderWorkers = 8;
constexpr size_t kDrNaturalOrderBytes = (size_t)1 << 33;
// Plain streaming kernels, each in the shape that measured fastest for its mix (together with
// the resident wavefronts per SIMD set on the kernels): a pure write stream likes 4 KB per
// workgroup, a copy one wavefront per KB, a pure read 4 KB per wavefront.
struct FillShape { static constexpr int kSlots = 1, kThreads = 256; };
struct CopyShape { static constexpr int kSlots = 1, kThreads = 64; };
struct ReadShape { static constexpr int kSlots = 4, kThreads = 64; };
struct Sum2Shape { static constexpr int kSlots = 1, kThreads = 64; };
struct Update3Shape { static constexpr int kSlots = 4, kThreads = 64; };
static_assert(CqShape<4, 512>::kSlots % 2 == 0 && CqShape<8, 512>::kSlots % 2 == 0,
              "block size 512 spans two slots of one wavefront");

std::atomic<int> g_pointer_checks{1};

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// No device holds this many elements; refusing more keeps every byte count below in range.
constexpr size_t kMaxElements = (size_t)1 << 48;

bool block_size_ok(int b) { return b == 32 || b == 64 || b == 128 || b == 256 || b == 512; }

// Is [p, p+bytes) inside one device allocation known to the runtime?
loco_status_t check_device_range(const void* p, size_t bytes) {
    if (!g_pointer_checks.load(std::memory_order_relaxed) || bytes == 0) return LOCO_OK;
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();
        return LOCO_ERR_BAD_POINTER;
    }
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged) return LOCO_ERR_BAD_POINTER;
    int current = -1;   // the kernels run on the current device: memory of another GPU is refused
    if (hipGetDevice(&current) != hipSuccess) {
        (void)hipGetLastError();
        return LOCO_ERR_BAD_POINTER;
    }
    if (attr.type == hipMemoryTypeDevice && attr.device != current) return LOCO_ERR_BAD_POINTER;
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange(&base, &size, const_cast<void*>(p)) != hipSuccess) {
        (void)hipGetLastError();
        return LOCO_ERR_BAD_POINTER;
    }
    const uintptr_t lo = reinterpret_cast<uintptr_t>(base), q = reinterpret_cast<uintptr_t>(p);
    if (q < lo || bytes > size || q - lo > size - bytes) return LOCO_ERR_BAD_POINTER;
    return LOCO_OK;
}

// Bytes from the start of payload 0 to the end of payload W-1: (W - 1) * stride + last, or false
// when that does not fit a size_t (a stride or worker count that cannot describe real memory).
bool payload_span(size_t W, size_t stride, size_t last, size_t unit, size_t* bytes) {
    if (W > 1 && stride > (SIZE_MAX / unit - last) / (W - 1)) return false;
    *bytes = ((W - 1) * stride + last) * unit;
    return true;
}

// Workgroups needed for `units` at `per_group` each, rounded up to a multiple of `round`
// (8 where the kernel spreads tiles over the XCDs itself).
loco_status_t grid_for(size_t units, size_t per_group, unsigned* grid, size_t round = 1) {
    size_t g = (units + per_group - 1) / per_group;
    g = (g + round - 1) / round * round;
    if (g == 0 || g > 0x7FFFFFFFull) return LOCO_ERR_UNSUPPORTED;
    *grid = (unsigned)g;
    return LOCO_OK;
}

// One kernel launch through the runtime's C entry point, which returns the status of THIS
// launch: an error some earlier call of the caller's left behind is neither reported as ours
// nor cleared.  The arguments are converted to the kernel's exact parameter types first.
template <typename... P, size_t... I>
loco_status_t launch_packed(void (*kernel)(P...), unsigned grid, unsigned threads, hipStream_t s,
                            std::tuple<P...>& vals, std::index_sequence<I...>) {
    void* ptrs[] = {static_cast<void*>(&std::get<I>(vals))...};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kernel), dim3(grid), dim3(threads), ptrs, 0, s);
    return e == hipSuccess ? LOCO_OK : LOCO_ERR_LAUNCH;
}
template <typename... P, typename... A>
loco_status_t launch(void (*kernel)(P...), unsigned grid, unsigned threads, hipStream_t s, A... args) {
    static_assert(sizeof...(P) == sizeof...(A), "one argument per kernel parameter");
    std::tuple<P...> vals(static_cast<P>(args)...);
    return launch_packed(kernel, grid, threads, s, vals, std::index_sequence_for<P...>{});
}

struct CqArgs {
    const void* grad;
    float* err;
    size_t n;
    float beta;
    int reset;
    const long long* step_index;   // device; nullptr: `reset` decides
    long long reset_period;
    float clip;   // +inf: no clipping
    uint8_t* codes;
    void* scales;      // float[nb], or uint16_t[nb] holding bf16 steps
    bool scales_bf16;
    bool stage_codes;  // measurement variant: 4-bit codes leave through LDS as 16-byte stores
    int waves;         // measurement variant: resident wavefronts per SIMD (0: the library's own)
};

template <typename G, int BITS, int BLOCK>
loco_status_t launch_cq(hipStream_t s, const CqArgs& a) {
    const float one_minus_beta = 1.0f - a.beta;
    using Shape = CqShape<BITS, BLOCK>;
    constexpr int kRun = Shape::kXcdRun;
    constexpr size_t kTile = (size_t)kSlot * Shape::kSlots;
    const uint32_t lead = xcd_run_lead_tiles(a.err, kRun ? kCqXcdRunElements * sizeof(float) : 0, kTile * sizeof(float));
    unsigned grid;
    if (loco_status_t st = grid_for(a.n + lead * kTile, kTile * (Shape::kThreads / kWave), &grid, kRun ? 8 * kRun : 1))
        return st;
    if constexpr (BITS == 4) {
        if (a.stage_codes)
            return launch(cq_kernel<G, BITS, BLOCK, Shape::kSlots, Shape::kThreads, kNonTemporal, kRun, false, float, true>,
                          grid, Shape::kThreads, s, a.grad, a.err, a.n, a.beta, one_minus_beta, a.reset, a.step_index,
                          a.reset_period, a.clip, a.codes, static_cast<float*>(a.scales), lead);
    }
    if (a.waves == 6 || a.waves == 8) {
        if (a.waves == 6)
            return launch(cq_kernel<G, BITS, BLOCK, Shape::kSlots, Shape::kThreads, kNonTemporal, kRun, false, float, false, 6>,
                          grid, Shape::kThreads, s, a.grad, a.err, a.n, a.beta, one_minus_beta, a.reset, a.step_index,
                          a.reset_period, a.clip, a.codes, static_cast<float*>(a.scales), lead);
        return launch(cq_kernel<G, BITS, BLOCK, Shape::kSlots, Shape::kThreads, kNonTemporal, kRun, false, float, false, 8>,
                      grid, Shape::kThreads, s, a.grad, a.err, a.n, a.beta, one_minus_beta, a.reset, a.step_index,
                      a.reset_period, a.clip, a.codes, static_cast<float*>(a.scales), lead);
    }
    if (a.scales_bf16)   // offered without clipping only
        return launch(cq_kernel<G, BITS, BLOCK, Shape::kSlots, Shape::kThreads, kNonTemporal, kRun, false, uint16_t>,
                      grid, Shape::kThreads, s, a.grad, a.err, a.n, a.beta, one_minus_beta, a.reset, a.step_index,
                      a.reset_period, a.clip, a.codes, static_cast<uint16_t*>(a.scales), lead);
    if (std::isinf(a.clip))
        return launch(cq_kernel<G, BITS, BLOCK, Shape::kSlots, Shape::kThreads, kNonTemporal, kRun, false, float>,
                      grid, Shape::kThreads, s, a.grad, a.err, a.n, a.beta, one_minus_beta, a.reset, a.step_index,
                      a.reset_period, a.clip, a.codes, static_cast<float*>(a.scales), lead);
    return launch(cq_kernel<G, BITS, BLOCK, Shape::kSlots, Shape::kThreads, kNonTemporal, kRun, true, float>,
                  grid, Shape::kThreads, s, a.grad, a.err, a.n, a.beta, one_minus_beta, a.reset, a.step_index,
                  a.reset_period, a.clip, a.codes, static_cast<float*>(a.scales), lead);
}

template <typename G, int BITS>
loco_status_t dispatch_cq_block(int block, hipStream_t s, const CqArgs& a) {
    switch (block) {
        case 32: return launch_cq<G, BITS, 32>(s, a);
        case 64: return launch_cq<G, BITS, 64>(s, a);
        case 128: return launch_cq<G, BITS, 128>(s, a);
        case 256: return launch_cq<G, BITS, 256>(s, a);
        case 512: return launch_cq<G, BITS, 512>(s, a);
        default: return LOCO_ERR_UNSUPPORTED;
    }
}

struct DrArgs {
    const uint8_t* codes;
    size_t code_stride;
    const void* scales;   // float, or uint16_t holding bf16 steps
    bool scales_bf16;
    size_t scale_stride;
    int W;
    size_t n;
};

bool dr_natural_order(int W, size_t n, int bits, size_t code_stride, size_t step_stride_bytes) {
    const bool aliased = code_stride % 4096 == 0 || (step_stride_bytes != 0 && step_stride_bytes % 4096 == 0);
    return W >= kDrNaturalOrderWorkers && (size_t)W * loco_code_bytes(n, bits) >= kDrNaturalOrderBytes && !aliased;
}

// With fp32 arrays updated in place behind the decode (theta; m and v for Adam) one slot per
// wavefront and 256 threads measured best, whatever the worker count.
constexpr bool dr_updates_in_place(Epilogue e) { return e == Epilogue::kSgd || e == Epilogue::kAdam; }
template <int BITS, Epilogue EPI>
using DrShapeFor = std::conditional_t<dr_updates_in_place(EPI), DrShape<8>, DrShape<BITS>>;

// Decompositions of the reduce.  kQuad is dr_kernel as described in loco_kernels.h;
// kQuadLaneSteps the same with the block steps of a chunk of workers fetched by one vector
// load (blocks of 128 elements and more); kWide4/8/16 is dr_wide_kernel with that many code
// bytes per lane and worker.  Measured on MI355X (2^26 .. 2.2e9 elements):
//   - up to 16 payloads of 4-bit codes with blocks of 256 elements and more, and for 8-bit codes
//     up to 64 payloads, the quad layout is the fastest;
//   - with more payloads its code loads (2 bytes per lane at 4 bits) become the limit: 4-bit codes
//     with blocks of 32..128 elements gain 6-10 points of HBM peak from wide loads from W = 16 on
//     (blocks of 32 and 64 elements already 1-4 points from 4-byte loads at W = 8..15),
//     with larger blocks 1-5 points from W = 64 on, 8-bit codes 2 points at W = 128;
//   - lane-loaded steps remove the doubled fetch of step lines that the scalar cache causes
//     (read traffic 1.037x -> 1.001x of the algorithmic bytes at 4 bits, B = 256) but cost
//     1-6 % of speed at 4 bits; at 8 bits with B >= 256 they are 1-3 points faster.
enum DrDecomposition { kDrAuto = 0, kDrQuad = 1, kDrQuadLaneSteps = 2, kDrWide4 = 3, kDrWide8 = 4, kDrWide16 = 5 };
template <int CB> struct DrWideShape { static constexpr int kThreads = CB == 16 ? 128 : 256, kInFlight = 4; };

int dr_auto_for_large_shards(int bits, int block, int W, Epilogue kind, bool scales_bf16);

// Shards below 2^22 elements do not fill the machine with the 2048-element units of the 16-byte code
// loads of 4-bit codes (2^20 elements, W = 128: 33 us against 20 us for the quad layout; equal from 2^22
// on), so there the choice falls back to what it would be with fewer payloads.
constexpr size_t kDrWide16MinElements = (size_t)1 << 22;
int dr_auto_decomposition(int bits, int block, int W, Epilogue kind, bool scales_bf16, size_t n) {
    const int how = dr_auto_for_large_shards(bits, block, W, kind, scales_bf16);
    if (how == kDrWide16 && bits == 4 && n < kDrWide16MinElements && kind != Epilogue::kStoreBf16)
        return block <= 128 ? kDrWide8 : kDrQuad;
    return how;
}

int dr_auto_for_large_shards(int bits, int block, int W, Epilogue kind, bool scales_bf16) {
    if (scales_bf16) return kDrQuad;
    // bf16 output of 4-bit codes: half the bytes written per element leave the quad layout's 2-byte code
    // loads as the limit at any worker count (W = 8: 80 % of HBM peak against 74 %, W = 1: 77 % against 65 %)
    if (kind == Epilogue::kStoreBf16 && bits == 4) return kDrWide16;
    if (W >= 96) return kDrWide16;                       // every bit width, block size and epilogue
    if (bits == 4) {
        if (block <= 128 && W >= 16) return W >= 64 ? kDrWide16 : kDrWide8;
        if (block <= 64 && W >= 8 && kind == Epilogue::kStore) return kDrWide4;   // 1-4 points over the quad layout
        if (block >= 256 && W >= 64) return kDrWide16;
        return kDrQuad;
    }
    return kind == Epilogue::kStore && block >= 256 && !dr_few_workers(bits, W) ? kDrQuadLaneSteps : kDrQuad;
}

// Empty tiles in front of a reduce's tile order, so that its runs of tiles start at multiples of their
// own size in the ADDRESSES of the array the kernel writes or updates in place (see xcd_run_lead_tiles).
template <Epilogue EPI>
uint32_t dr_lead_tiles(const EpilogueArgs& epi, int xcd_run, size_t tile_elems, int waves_per_group) {
    const void* base = (EPI == Epilogue::kStore || EPI == Epilogue::kStoreBf16) ? epi.out : epi.theta;
    const size_t elem = EPI == Epilogue::kStoreBf16 ? 2 : 4;
    return xcd_run_lead_tiles(base, (size_t)xcd_run * waves_per_group * tile_elems * elem, tile_elems * elem);
}

template <int BITS, int BLOCK, Epilogue EPI, typename Shape, typename S, bool LANE_STEPS, int XCD_RUN = kDrXcdRun>
loco_status_t launch_dr_quad(hipStream_t s, const DrArgs& a, const EpilogueArgs& epi) {
    constexpr size_t kTile = (size_t)kSlot * Shape::kSlots;
    const uint32_t lead = dr_lead_tiles<EPI>(epi, XCD_RUN, kTile, Shape::kThreads / kWave);
    unsigned grid;
    if (loco_status_t st = grid_for(a.n + lead * kTile, kTile * (Shape::kThreads / kWave), &grid, XCD_RUN ? 8 * XCD_RUN : 1))
        return st;
    constexpr int kWaves = (BITS == 8 && std::is_same_v<Shape, DrFewWorkersShape> && !dr_updates_in_place(EPI))
                               ? kDrFewPayloads8BitWaves : dr_waves_per_simd(EPI);
    return launch(dr_kernel<BITS, BLOCK, Shape::kSlots, Shape::kThreads, Shape::kInFlight, kNonTemporal, XCD_RUN, EPI, S,
                            LANE_STEPS, kWaves>,
                  grid, Shape::kThreads, s, a.codes, a.code_stride, static_cast<const S*>(a.scales), a.scale_stride, a.W,
                  a.n, 1.0f / (float)a.W, epi, lead);
}

template <int BITS, int BLOCK, int CB, Epilogue EPI = Epilogue::kStore, int XCD_RUN = kDrXcdRun>
loco_status_t launch_dr_wide(hipStream_t s, const DrArgs& a, const EpilogueArgs& epi) {
    using Shape = DrWideShape<CB>;
    constexpr size_t kUnitElems = (size_t)kWave * (CB * 8 / BITS);
    const uint32_t lead = dr_lead_tiles<EPI>(epi, XCD_RUN, kUnitElems, Shape::kThreads / kWave);
    unsigned grid;
    if (loco_status_t st = grid_for(a.n + lead * kUnitElems, kUnitElems * (Shape::kThreads / kWave), &grid, XCD_RUN ? 8 * XCD_RUN : 1))
        return st;
    return launch(dr_wide_kernel<BITS, BLOCK, CB, Shape::kThreads, Shape::kInFlight, kNonTemporal, XCD_RUN, EPI, float>,
                  grid, Shape::kThreads, s, a.codes, a.code_stride, static_cast<const float*>(a.scales), a.scale_stride,
                  a.W, a.n, 1.0f / (float)a.W, epi, lead);
}

template <int BITS, int BLOCK, Epilogue EPI>
loco_status_t launch_dr(int how, hipStream_t s, const DrArgs& a, const EpilogueArgs& epi) {
    const bool natural = dr_natural_order(a.W, a.n, BITS, a.code_stride, a.scale_stride * sizeof(float));
    if constexpr (EPI == Epilogue::kStore) {   // the other decompositions: plain fp32 output, fp32 steps
        if (how != kDrQuad && a.scales_bf16) return LOCO_ERR_UNSUPPORTED;
        if (how == kDrQuadLaneSteps) {
            if constexpr (BLOCK >= 128) {
                if (dr_few_workers(BITS, a.W)) return launch_dr_quad<BITS, BLOCK, EPI, DrFewWorkersShape, float, true>(s, a, epi);
                if (natural) return launch_dr_quad<BITS, BLOCK, EPI, DrShape<BITS>, float, true, 0>(s, a, epi);
                return launch_dr_quad<BITS, BLOCK, EPI, DrShape<BITS>, float, true>(s, a, epi);
            }
            return LOCO_ERR_UNSUPPORTED;
        }
        if (how == kDrWide4) {
            if constexpr (BITS == 4) return launch_dr_wide<BITS, BLOCK, 4>(s, a, epi);
            return LOCO_ERR_UNSUPPORTED;
        }
        if (how == kDrWide8) {
            if (natural) return launch_dr_wide<BITS, BLOCK, 8, EPI, 0>(s, a, epi);
            return launch_dr_wide<BITS, BLOCK, 8>(s, a, epi);
        }
        if (how == kDrWide16) return launch_dr_wide<BITS, BLOCK, 16>(s, a, epi);
        if (a.scales_bf16) {
            if (dr_few_workers(BITS, a.W)) return launch_dr_quad<BITS, BLOCK, EPI, DrFewWorkersShape, uint16_t, false>(s, a, epi);
            return launch_dr_quad<BITS, BLOCK, EPI, DrShape<BITS>, uint16_t, false>(s, a, epi);
        }
    }
    if constexpr (EPI != Epilogue::kStore) {   // many payloads: the wide loads, whatever follows the sum
        if (how == kDrWide8) return launch_dr_wide<BITS, BLOCK, 8, EPI>(s, a, epi);
        if (how == kDrWide16) return launch_dr_wide<BITS, BLOCK, 16, EPI>(s, a, epi);
    }
    if (how != kDrQuad) return LOCO_ERR_UNSUPPORTED;
    if constexpr (!dr_updates_in_place(EPI)) {
        if constexpr (BITS == 4 && BLOCK <= 256) {   // (blocks of 512 elements lose 7 points with it)
            if (a.W == 2 || a.W == 3) return launch_dr_quad<BITS, BLOCK, EPI, DrTwoOrThreeWorkersShape, float, false>(s, a, epi);
        }
        if (dr_few_workers(BITS, a.W)) return launch_dr_quad<BITS, BLOCK, EPI, DrFewWorkersShape, float, false>(s, a, epi);
    }
    if constexpr (EPI == Epilogue::kStore) {
        if (natural) return launch_dr_quad<BITS, BLOCK, EPI, DrShape<BITS>, float, false, 0>(s, a, epi);
    }
    return launch_dr_quad<BITS, BLOCK, EPI, DrShapeFor<BITS, EPI>, float, false>(s, a, epi);
}

template <int BITS, Epilogue EPI>
loco_status_t dispatch_dr_block(int block, int how, hipStream_t s, const DrArgs& a, const EpilogueArgs& epi) {
    switch (block) {
        case 32: return launch_dr<BITS, 32, EPI>(how, s, a, epi);
        case 64: return launch_dr<BITS, 64, EPI>(how, s, a, epi);
        case 128: return launch_dr<BITS, 128, EPI>(how, s, a, epi);
        case 256: return launch_dr<BITS, 256, EPI>(how, s, a, epi);
        case 512: return launch_dr<BITS, 512, EPI>(how, s, a, epi);
        default: return LOCO_ERR_UNSUPPORTED;
    }
}

template <Epilogue EPI>
loco_status_t dispatch_dr(int bits, int block, int how, hipStream_t s, const DrArgs& a, const EpilogueArgs& epi) {
    return bits == 4 ? dispatch_dr_block<4, EPI>(block, how, s, a, epi) : dispatch_dr_block<8, EPI>(block, how, s, a, epi);
}

// Checks the buffers an epilogue touches (16-byte aligned fp32 arrays of n elements, inside
// one allocation) and its hyper-parameters.
loco_status_t check_epilogue(Epilogue kind, const EpilogueArgs& e, size_t n) {
    const float* arrays[4] = {e.out, e.theta, e.m, e.v};
    const bool stores = kind == Epilogue::kStore || kind == Epilogue::kStoreBf16;
    const bool used[4] = {stores, !stores, kind == Epilogue::kAdam, kind == Epilogue::kAdam};
    for (int k = 0; k < 4; ++k) {
        if (!used[k]) continue;
        if (!arrays[k]) return LOCO_ERR_INVALID_ARG;
        if (!aligned(arrays[k], 16)) return LOCO_ERR_ALIGNMENT;
        const size_t esz = kind == Epilogue::kStoreBf16 ? 2 : sizeof(float);
        if (loco_status_t st = check_device_range(arrays[k], n * esz)) return st;
    }
    if (!stores && !std::isfinite(e.eta)) return LOCO_ERR_INVALID_ARG;
    if (kind == Epilogue::kAdam) {
        if (!(e.beta1 >= 0.0f && e.beta1 <= 1.0f) || !(e.beta2 >= 0.0f && e.beta2 <= 1.0f)) return LOCO_ERR_INVALID_ARG;
        if (!(e.delta >= 0.0f) || std::isinf(e.delta)) return LOCO_ERR_INVALID_ARG;
    }
    return LOCO_OK;
}

EpilogueArgs make_epilogue(float* out, float* theta, float* m, float* v, float eta, float beta1, float beta2,
                           float delta) {
    EpilogueArgs e;
    e.out = out; e.theta = theta; e.m = m; e.v = v;
    e.eta = eta; e.beta1 = beta1; e.one_minus_beta1 = 1.0f - beta1;
    e.beta2 = beta2; e.one_minus_beta2 = 1.0f - beta2; e.delta = delta;
    return e;
}

// Launch shapes of the fixed-scale kernels (units of 512 elements per wavefront).
// (tile runs per XCD: none for the 8-bit state, where every run length tried was 2-6 points slower; for the
// fp32 state 32768 elements like cq_kernel: 83 % of HBM peak against 79-80 %)
struct FixedCqShape { static constexpr int kUnits = 2, kThreads = 128, kXcdRun = 0; };
struct FixedF32CqShape { static constexpr int kSlots = 2, kThreads = 64, kXcdRun = kCqXcdRunElements / (kSlot * 2); };    // 128 threads measured 1.5 points slower
struct FixedDrShape { static constexpr int kSlots = 2, kThreads = 128, kInFlight = 4; };
struct FixedDrWideShape { static constexpr int kSlots = 1, kThreads = 256, kInFlight = 4; };  // Adam, as DrShapeFor
template <Epilogue EPI>
using FixedDrShapeFor = std::conditional_t<EPI == Epilogue::kAdam, FixedDrWideShape, FixedDrShape>;

bool fixed_args_ok(int bits, int log2_s, int se_mult) {
    return (bits == 4 || bits == 8) && log2_s >= -64 && log2_s <= 64 && se_mult >= 1 && se_mult <= 64;
}

struct FixedCqArgs {
    const void* grad;
    int8_t* err8;
    size_t n;
    FixedScales k;
    int reset;
    const long long* step_index;   // device; nullptr: `reset` decides
    long long reset_period;
    float clip;
    uint8_t* codes;
};

template <typename G, int BITS, bool POW2>
loco_status_t launch_fixed_cq(unsigned grid, hipStream_t s, const FixedCqArgs& a) {
    if (std::isinf(a.clip))
        return launch(fixed_cq_kernel<G, BITS, POW2, FixedCqShape::kUnits, FixedCqShape::kThreads, kNonTemporal, false, FixedCqShape::kXcdRun>,
                      grid, FixedCqShape::kThreads, s, a.grad, a.err8, a.n, a.k, a.reset, a.step_index, a.reset_period,
                      a.clip, a.codes);
    return launch(fixed_cq_kernel<G, BITS, POW2, FixedCqShape::kUnits, FixedCqShape::kThreads, kNonTemporal, true, FixedCqShape::kXcdRun>,
                  grid, FixedCqShape::kThreads, s, a.grad, a.err8, a.n, a.k, a.reset, a.step_index, a.reset_period,
                  a.clip, a.codes);
}

template <typename G>
loco_status_t dispatch_fixed_cq(int bits, bool pow2, unsigned grid, hipStream_t s, const FixedCqArgs& a) {
    if (bits == 4) return pow2 ? launch_fixed_cq<G, 4, true>(grid, s, a) : launch_fixed_cq<G, 4, false>(grid, s, a);
    return pow2 ? launch_fixed_cq<G, 8, true>(grid, s, a) : launch_fixed_cq<G, 8, false>(grid, s, a);
}

loco_status_t reduce_block(const uint8_t* codes, size_t code_stride_bytes, const void* scales,
                           size_t scale_stride_elems, int num_workers, size_t n, int bits, int block_size,
                           Epilogue kind, const EpilogueArgs& epi, void* stream, bool scales_bf16 = false,
                           int decomposition = kDrAuto) {
    if (scales_bf16 && kind != Epilogue::kStore) return LOCO_ERR_UNSUPPORTED;
    const size_t step_bytes = scales_bf16 ? sizeof(uint16_t) : sizeof(float);
    if (bits != 4 && bits != 8) return LOCO_ERR_UNSUPPORTED;
    if (!block_size_ok(block_size)) return LOCO_ERR_UNSUPPORTED;
    if (decomposition < kDrAuto || decomposition > kDrWide16) return LOCO_ERR_UNSUPPORTED;
    if (num_workers < 1) return LOCO_ERR_INVALID_ARG;
    if (n == 0) return LOCO_OK;
    if (n > kMaxElements) return LOCO_ERR_UNSUPPORTED;
    if (!codes || !scales) return LOCO_ERR_INVALID_ARG;
    const size_t cb = loco_code_bytes(n, bits), nb = loco_num_blocks(n, block_size);
    const size_t W = (size_t)num_workers;
    if (W == 1) {  // strides are not used
        code_stride_bytes = 0;
        scale_stride_elems = 0;
    } else {
        if (code_stride_bytes < cb || scale_stride_elems < nb) return LOCO_ERR_INVALID_ARG;
        if (code_stride_bytes % 16 != 0) return LOCO_ERR_ALIGNMENT;
    }
    if (!aligned(codes, 16) || !aligned(scales, 4)) return LOCO_ERR_ALIGNMENT;
    size_t code_span, step_span;
    if (!payload_span(W, code_stride_bytes, cb, 1, &code_span) ||
        !payload_span(W, scale_stride_elems, nb, step_bytes, &step_span))
        return LOCO_ERR_INVALID_ARG;
    if (loco_status_t st = check_device_range(codes, code_span)) return st;
    if (loco_status_t st = check_device_range(scales, step_span)) return st;
    if (loco_status_t st = check_epilogue(kind, epi, n)) return st;
    const int how = decomposition == kDrAuto ? dr_auto_decomposition(bits, block_size, num_workers, kind, scales_bf16, n)
                                             : decomposition;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const DrArgs a{codes, code_stride_bytes, scales, scales_bf16, scale_stride_elems, num_workers, n};
    switch (kind) {
        case Epilogue::kStore: return dispatch_dr<Epilogue::kStore>(bits, block_size, how, s, a, epi);
        case Epilogue::kStoreBf16: return dispatch_dr<Epilogue::kStoreBf16>(bits, block_size, how, s, a, epi);
        case Epilogue::kSgd: return dispatch_dr<Epilogue::kSgd>(bits, block_size, how, s, a, epi);
        case Epilogue::kAdam: return dispatch_dr<Epilogue::kAdam>(bits, block_size, how, s, a, epi);
    }
    return LOCO_ERR_UNSUPPORTED;
}

// Runs of 32 tiles per XCD measured about one point of HBM peak faster for the fp32 output and the
// fused optimizers of the fixed-scale reduce, and slower for the bf16 output.
template <Epilogue EPI> constexpr int fixed_dr_xcd_run() { return EPI == Epilogue::kStoreBf16 ? 0 : 32; }

// One launch of the fixed-scale reduce in a given shape, tile order and residency.
template <int BITS, typename Shape, Epilogue EPI, int RUN, int WAVES = fixed_dr_waves_per_simd(EPI)>
loco_status_t launch_fixed_dr_shape(hipStream_t s, const uint8_t* codes, size_t cs, int W, size_t n, float inv_s,
                                    float inv_w, const EpilogueArgs& epi) {
    constexpr size_t kTile = (size_t)kSlot * Shape::kSlots;
    const uint32_t lead = dr_lead_tiles<EPI>(epi, RUN, kTile, Shape::kThreads / kWave);
    unsigned grid;
    if (loco_status_t st = grid_for(n + lead * kTile, kTile * (Shape::kThreads / kWave), &grid, RUN ? 8 * RUN : 1)) return st;
    return launch(fixed_dr_kernel<BITS, Shape::kSlots, Shape::kThreads, Shape::kInFlight, kNonTemporal, EPI, RUN, WAVES>, grid,
                  Shape::kThreads, s, codes, cs, W, n, inv_s, inv_w, epi, lead);
}

template <Epilogue EPI>
loco_status_t launch_fixed_dr(int bits, hipStream_t s, const uint8_t* codes, size_t cs, int W,
                              size_t n, float inv_s, float inv_w, const EpilogueArgs& epi) {
    using Shape = FixedDrShapeFor<EPI>;
    constexpr int kRun = fixed_dr_xcd_run<EPI>();
    if constexpr (EPI == Epilogue::kStore) {
        // few payloads, as for the block form: 4 KB of output per wavefront for two or three payloads of
        // 4-bit codes (78 % of HBM peak against 69 %), 6 resident wavefronts for one payload of 8-bit codes
        // (82 % against 71 %)
        if (bits == 4 && (W == 2 || W == 3))
            return launch_fixed_dr_shape<4, DrTwoOrThreeWorkersShape, EPI, kRun>(s, codes, cs, W, n, inv_s, inv_w, epi);
        if (bits == 8 && W == 1)
            return launch_fixed_dr_shape<8, DrFewWorkersShape, EPI, kRun, kDrFewPayloads8BitWaves>(s, codes, cs, W, n, inv_s, inv_w, epi);
        if (bits == 4 && dr_natural_order(W, n, 4, cs, 0))   // see kDrNaturalOrderBytes
            return launch_fixed_dr_shape<4, Shape, EPI, 0>(s, codes, cs, W, n, inv_s, inv_w, epi);
    }
    if (bits == 4) return launch_fixed_dr_shape<4, Shape, EPI, kRun>(s, codes, cs, W, n, inv_s, inv_w, epi);
    if constexpr (EPI == Epilogue::kStore) {
        if (W >= kFixedDr8ManyWorkers)
            return launch_fixed_dr_shape<8, Shape, EPI, kRun, kFixedDr8ManyWorkersWaves>(s, codes, cs, W, n, inv_s, inv_w, epi);
    }
    return launch_fixed_dr_shape<8, Shape, EPI, kRun>(s, codes, cs, W, n, inv_s, inv_w, epi);
}

// The reduce kernel sums the integer codes and converts once; every partial sum must stay
// below 2^24 in magnitude for that to equal the sequential binary32 sum of Eq. 8.
constexpr int kFixedMaxWorkers4 = (1 << 24) / 8, kFixedMaxWorkers8 = (1 << 24) / 128;

loco_status_t reduce_fixed(const uint8_t* codes, size_t code_stride_bytes, int num_workers, size_t n,
                           int bits, int log2_s, Epilogue kind, const EpilogueArgs& epi, void* stream) {
    if (!fixed_args_ok(bits, log2_s, 1)) return LOCO_ERR_UNSUPPORTED;
    if (num_workers < 1) return LOCO_ERR_INVALID_ARG;
    if (num_workers > (bits == 4 ? kFixedMaxWorkers4 : kFixedMaxWorkers8)) return LOCO_ERR_UNSUPPORTED;
    if (n == 0) return LOCO_OK;
    if (n > kMaxElements) return LOCO_ERR_UNSUPPORTED;
    if (!codes) return LOCO_ERR_INVALID_ARG;
    const size_t cb = loco_code_bytes(n, bits);
    const size_t W = (size_t)num_workers;
    if (W == 1) {
        code_stride_bytes = 0;
    } else {
        if (code_stride_bytes < cb) return LOCO_ERR_INVALID_ARG;
        if (code_stride_bytes % 16 != 0) return LOCO_ERR_ALIGNMENT;
    }
    if (!aligned(codes, 16)) return LOCO_ERR_ALIGNMENT;
    size_t code_span;
    if (!payload_span(W, code_stride_bytes, cb, 1, &code_span)) return LOCO_ERR_INVALID_ARG;
    if (loco_status_t st = check_device_range(codes, code_span)) return st;
    if (loco_status_t st = check_epilogue(kind, epi, n)) return st;
    const float inv_s = std::ldexp(1.0f, -log2_s), inv_w = 1.0f / (float)num_workers;
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (kind) {
        case Epilogue::kStore: return launch_fixed_dr<Epilogue::kStore>(bits, s, codes, code_stride_bytes, num_workers, n, inv_s, inv_w, epi);
        case Epilogue::kStoreBf16: return launch_fixed_dr<Epilogue::kStoreBf16>(bits, s, codes, code_stride_bytes, num_workers, n, inv_s, inv_w, epi);
        case Epilogue::kSgd: return launch_fixed_dr<Epilogue::kSgd>(bits, s, codes, code_stride_bytes, num_workers, n, inv_s, inv_w, epi);
        case Epilogue::kAdam: return launch_fixed_dr<Epilogue::kAdam>(bits, s, codes, code_stride_bytes, num_workers, n, inv_s, inv_w, epi);
    }
    return LOCO_ERR_UNSUPPORTED;
}

// The step counter of the scheduled calls: 8-byte aligned device memory holding one int64.
loco_status_t check_step_index(const int64_t* step_index_dev, int64_t reset_period) {
    if (!step_index_dev) return LOCO_ERR_INVALID_ARG;
    if (reset_period < 0) return LOCO_ERR_INVALID_ARG;
    if (!aligned(step_index_dev, 8)) return LOCO_ERR_ALIGNMENT;
    return check_device_range(step_index_dev, sizeof(int64_t));
}

loco_status_t compress_block(const void* grad, loco_dtype_t grad_dtype, float clip_abs, float* err_state,
                             size_t n, int bits, int block_size, float beta, int reset,
                             const int64_t* step_index_dev, int64_t reset_period, uint8_t* codes_out,
                             void* scales_out, bool scales_bf16, void* stream, bool stage_codes = false,
                             int waves = 0) {
    const size_t step_bytes = scales_bf16 ? sizeof(uint16_t) : sizeof(float);
    if (bits != 4 && bits != 8) return LOCO_ERR_UNSUPPORTED;
    if (!block_size_ok(block_size)) return LOCO_ERR_UNSUPPORTED;
    if (grad_dtype != LOCO_F32 && grad_dtype != LOCO_BF16) return LOCO_ERR_UNSUPPORTED;
    if (!(beta >= 0.0f && beta <= 1.0f)) return LOCO_ERR_INVALID_ARG;  // also rejects NaN
    if (!(clip_abs > 0.0f)) return LOCO_ERR_INVALID_ARG;               // NaN, zero, negative
    if (n == 0) return LOCO_OK;
    if (n > kMaxElements) return LOCO_ERR_UNSUPPORTED;
    if (!grad || !err_state || !codes_out || !scales_out) return LOCO_ERR_INVALID_ARG;
    if (!aligned(grad, 16) || !aligned(err_state, 16) || !aligned(codes_out, 16) || !aligned(scales_out, step_bytes))
        return LOCO_ERR_ALIGNMENT;
    const size_t gsz = grad_dtype == LOCO_BF16 ? 2 : 4;
    if (loco_status_t st = check_device_range(grad, n * gsz)) return st;
    if (loco_status_t st = check_device_range(err_state, n * sizeof(float))) return st;
    if (loco_status_t st = check_device_range(codes_out, loco_code_bytes(n, bits))) return st;
    if (loco_status_t st = check_device_range(scales_out, loco_num_blocks(n, block_size) * step_bytes))
        return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const CqArgs a{grad, err_state, n, beta, reset, reinterpret_cast<const long long*>(step_index_dev),
                   (long long)reset_period, clip_abs, codes_out, scales_out, scales_bf16, stage_codes, waves};
    if (grad_dtype == LOCO_BF16)
        return bits == 4 ? dispatch_cq_block<bf16_t, 4>(block_size, s, a) : dispatch_cq_block<bf16_t, 8>(block_size, s, a);
    return bits == 4 ? dispatch_cq_block<float, 4>(block_size, s, a) : dispatch_cq_block<float, 8>(block_size, s, a);
}

loco_status_t compress_fixed(const void* grad, loco_dtype_t grad_dtype, float clip_abs, int8_t* err_state8, size_t n,
                             int bits, int log2_s, int se_mult, float beta, int reset,
                             const int64_t* step_index_dev, int64_t reset_period, uint8_t* codes_out, void* stream) {
    if (!fixed_args_ok(bits, log2_s, se_mult)) return LOCO_ERR_UNSUPPORTED;
    if (!(clip_abs > 0.0f)) return LOCO_ERR_INVALID_ARG;
    if (grad_dtype != LOCO_F32 && grad_dtype != LOCO_BF16) return LOCO_ERR_UNSUPPORTED;
    if (!(beta >= 0.0f && beta <= 1.0f)) return LOCO_ERR_INVALID_ARG;
    if (n == 0) return LOCO_OK;
    if (n > kMaxElements) return LOCO_ERR_UNSUPPORTED;
    if (!grad || !err_state8 || !codes_out) return LOCO_ERR_INVALID_ARG;
    if (!aligned(grad, 16) || !aligned(err_state8, 16) || !aligned(codes_out, 16)) return LOCO_ERR_ALIGNMENT;
    const size_t gsz = grad_dtype == LOCO_BF16 ? 2 : 4;
    if (loco_status_t st = check_device_range(grad, n * gsz)) return st;
    if (loco_status_t st = check_device_range(err_state8, n)) return st;
    if (loco_status_t st = check_device_range(codes_out, loco_code_bytes(n, bits))) return st;
    unsigned grid;
    if (loco_status_t st = grid_for(n, (size_t)kUnit * FixedCqShape::kUnits * (FixedCqShape::kThreads / kWave), &grid,
                                    FixedCqShape::kXcdRun ? 8 * FixedCqShape::kXcdRun : 1))
        return st;
    FixedScales k;
    k.s = std::ldexp(1.0f, log2_s);
    k.inv_s = std::ldexp(1.0f, -log2_s);
    k.s_e = (float)se_mult * k.s;
    k.inv_se = 1.0f / k.s_e;
    k.beta = beta;
    k.one_minus_beta = 1.0f - beta;
    const bool pow2 = (se_mult & (se_mult - 1)) == 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const FixedCqArgs a{grad, err_state8, n, k, reset, reinterpret_cast<const long long*>(step_index_dev),
                        (long long)reset_period, clip_abs, codes_out};
    return grad_dtype == LOCO_BF16 ? dispatch_fixed_cq<bf16_t>(bits, pow2, grid, s, a)
                                   : dispatch_fixed_cq<float>(bits, pow2, grid, s, a);
}

loco_status_t compress_fixed_f32state(const void* grad, loco_dtype_t grad_dtype, float* err_state, size_t n, int bits,
                                      int log2_s, float beta, int reset, const int64_t* step_index_dev,
                                      int64_t reset_period, uint8_t* codes_out, void* stream) {
    if (!fixed_args_ok(bits, log2_s, 1)) return LOCO_ERR_UNSUPPORTED;
    if (grad_dtype != LOCO_F32 && grad_dtype != LOCO_BF16) return LOCO_ERR_UNSUPPORTED;
    if (!(beta >= 0.0f && beta <= 1.0f)) return LOCO_ERR_INVALID_ARG;
    if (n == 0) return LOCO_OK;
    if (n > kMaxElements) return LOCO_ERR_UNSUPPORTED;
    if (!grad || !err_state || !codes_out) return LOCO_ERR_INVALID_ARG;
    if (!aligned(grad, 16) || !aligned(err_state, 16) || !aligned(codes_out, 16)) return LOCO_ERR_ALIGNMENT;
    const size_t gsz = grad_dtype == LOCO_BF16 ? 2 : 4;
    if (loco_status_t st = check_device_range(grad, n * gsz)) return st;
    if (loco_status_t st = check_device_range(err_state, n * sizeof(float))) return st;
    if (loco_status_t st = check_device_range(codes_out, loco_code_bytes(n, bits))) return st;
    using Shape = FixedF32CqShape;
    constexpr size_t kTile = (size_t)kSlot * Shape::kSlots;
    const uint32_t lead = xcd_run_lead_tiles(err_state, Shape::kXcdRun ? kCqXcdRunElements * sizeof(float) : 0, kTile * sizeof(float));
    unsigned grid;
    if (loco_status_t st = grid_for(n + lead * kTile, kTile * (Shape::kThreads / kWave), &grid,
                                    Shape::kXcdRun ? 8 * Shape::kXcdRun : 1))
        return st;
    FixedScales k{};
    k.s = std::ldexp(1.0f, log2_s);
    k.inv_s = std::ldexp(1.0f, -log2_s);
    k.beta = beta;
    k.one_minus_beta = 1.0f - beta;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const long long* si = reinterpret_cast<const long long*>(step_index_dev);
    const long long period = (long long)reset_period;
    if (grad_dtype == LOCO_BF16) {
        if (bits == 4) return launch(fixed_f32_cq_kernel<bf16_t, 4, Shape::kSlots, Shape::kThreads, kNonTemporal, Shape::kXcdRun>, grid, Shape::kThreads, s, grad, err_state, n, k, reset, si, period, codes_out, lead);
        return launch(fixed_f32_cq_kernel<bf16_t, 8, Shape::kSlots, Shape::kThreads, kNonTemporal, Shape::kXcdRun>, grid, Shape::kThreads, s, grad, err_state, n, k, reset, si, period, codes_out, lead);
    }
    if (bits == 4) return launch(fixed_f32_cq_kernel<float, 4, Shape::kSlots, Shape::kThreads, kNonTemporal, Shape::kXcdRun>, grid, Shape::kThreads, s, grad, err_state, n, k, reset, si, period, codes_out, lead);
    return launch(fixed_f32_cq_kernel<float, 8, Shape::kSlots, Shape::kThreads, kNonTemporal, Shape::kXcdRun>, grid, Shape::kThreads, s, grad, err_state, n, k, reset, si, period, codes_out, lead);
}

template <StreamMode MODE, typename Shape>
loco_status_t launch_stream(void* dst, const void* src, const void* src2, size_t bytes, void* stream) {
    const size_t n16 = bytes / 16;
    unsigned grid;
    if (loco_status_t st = grid_for(n16, (size_t)Shape::kThreads * Shape::kSlots, &grid)) return st;
    return launch(stream_kernel<MODE, Shape::kSlots, Shape::kThreads, kNonTemporal>, grid, Shape::kThreads,
                  static_cast<hipStream_t>(stream), static_cast<u32x4*>(dst), static_cast<const u32x4*>(src),
                  static_cast<const u32x4*>(src2), n16, 0x9E3779B9u);
}

}  // namespace

extern "C" {

const char* loco_status_string(loco_status_t status) {
    switch (status) {
        case LOCO_OK: return "ok";
        case LOCO_ERR_INVALID_ARG: return "invalid argument";
        case LOCO_ERR_UNSUPPORTED: return "unsupported bits, block size, dtype, size, worker count or decomposition";
        case LOCO_ERR_ALIGNMENT: return "pointer or stride not aligned as required";
        case LOCO_ERR_LAUNCH: return "kernel launch failed";
        case LOCO_ERR_BAD_POINTER: return "buffer is not device memory or is too small";
        default: return "unknown status";
    }
}

size_t loco_code_bytes(size_t n, int bits) {
    if (bits == 8) return n;
    if (bits == 4) return n / 2 + (n & 1);
    return 0;
}

size_t loco_num_blocks(size_t n, int block_size) {
    if (block_size < 1) return 0;
    return n / (size_t)block_size + (n % (size_t)block_size != 0);
}

int loco_set_pointer_checks(int enabled) { return g_pointer_checks.exchange(enabled ? 1 : 0); }

loco_status_t loco_error_state_init(float* err_state, size_t n, void* stream) {
    if (n == 0) return LOCO_OK;
    if (n > kMaxElements) return LOCO_ERR_UNSUPPORTED;
    if (!err_state) return LOCO_ERR_INVALID_ARG;
    if (!aligned(err_state, 16)) return LOCO_ERR_ALIGNMENT;
    if (loco_status_t st = check_device_range(err_state, n * sizeof(float))) return st;
    unsigned grid;
    if (loco_status_t st = grid_for(n, (size_t)FillShape::kThreads * 4 * FillShape::kSlots, &grid)) return st;
    return launch(fill_zero_kernel<FillShape::kSlots, FillShape::kThreads, kNonTemporal>, grid, FillShape::kThreads,
                  static_cast<hipStream_t>(stream), err_state, n);
}

loco_status_t loco_compensate_quantize_clip(const void* grad, loco_dtype_t grad_dtype, float clip_abs,
                                            float* err_state, size_t n, int bits, int block_size, float beta,
                                            int reset, uint8_t* codes_out, float* scales_out, void* stream) {
    return compress_block(grad, grad_dtype, clip_abs, err_state, n, bits, block_size, beta, reset, nullptr, 0,
                          codes_out, scales_out, false, stream);
}

loco_status_t loco_compensate_quantize(const void* grad, loco_dtype_t grad_dtype, float* err_state,
                                       size_t n, int bits, int block_size, float beta, int reset,
                                       uint8_t* codes_out, float* scales_out, void* stream) {
    return compress_block(grad, grad_dtype, INFINITY, err_state, n, bits, block_size, beta, reset, nullptr, 0,
                          codes_out, scales_out, false, stream);
}

loco_status_t loco_compensate_quantize_staged_codes(const void* grad, loco_dtype_t grad_dtype, float* err_state,
                                                    size_t n, int bits, int block_size, float beta, int reset,
                                                    uint8_t* codes_out, float* scales_out, void* stream) {
    if (bits != 4) return LOCO_ERR_UNSUPPORTED;
    return compress_block(grad, grad_dtype, INFINITY, err_state, n, bits, block_size, beta, reset, nullptr, 0,
                          codes_out, scales_out, false, stream, true);
}

loco_status_t loco_compensate_quantize_resident(const void* grad, loco_dtype_t grad_dtype, float* err_state,
                                                size_t n, int bits, int block_size, float beta, int reset,
                                                uint8_t* codes_out, float* scales_out, int waves_per_simd,
                                                void* stream) {
    if (waves_per_simd != kCqWavesPerSimd && waves_per_simd != 6 && waves_per_simd != 8) return LOCO_ERR_UNSUPPORTED;
    return compress_block(grad, grad_dtype, INFINITY, err_state, n, bits, block_size, beta, reset, nullptr, 0,
                          codes_out, scales_out, false, stream, false,
                          waves_per_simd == kCqWavesPerSimd ? 0 : waves_per_simd);
}

loco_status_t loco_compensate_quantize_scheduled(const void* grad, loco_dtype_t grad_dtype, float* err_state,
                                                 size_t n, int bits, int block_size, float beta,
                                                 const int64_t* step_index_dev, int64_t reset_period,
                                                 uint8_t* codes_out, float* scales_out, void* stream) {
    if (n != 0)
        if (loco_status_t st = check_step_index(step_index_dev, reset_period)) return st;
    return compress_block(grad, grad_dtype, INFINITY, err_state, n, bits, block_size, beta, 0, step_index_dev,
                          reset_period, codes_out, scales_out, false, stream);
}

loco_status_t loco_compensate_quantize_bf16_scales(const void* grad, loco_dtype_t grad_dtype, float* err_state,
                                                   size_t n, int bits, int block_size, float beta, int reset,
                                                   uint8_t* codes_out, uint16_t* scales_out_bf16, void* stream) {
    return compress_block(grad, grad_dtype, INFINITY, err_state, n, bits, block_size, beta, reset, nullptr, 0,
                          codes_out, scales_out_bf16, true, stream);
}

loco_status_t loco_dequant_reduce_bf16_scales(const uint8_t* codes, size_t code_stride_bytes,
                                              const uint16_t* scales_bf16, size_t scale_stride_elems,
                                              int num_workers, size_t n, int bits, int block_size,
                                              float* grad_out, void* stream) {
    return reduce_block(codes, code_stride_bytes, scales_bf16, scale_stride_elems, num_workers, n, bits, block_size,
                        Epilogue::kStore, make_epilogue(grad_out, nullptr, nullptr, nullptr, 0, 0, 0, 0), stream,
                        true);
}

loco_status_t loco_dequant_reduce(const uint8_t* codes, size_t code_stride_bytes, const float* scales,
                                  size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                  int block_size, float* grad_out, void* stream) {
    return reduce_block(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                        Epilogue::kStore, make_epilogue(grad_out, nullptr, nullptr, nullptr, 0, 0, 0, 0), stream);
}

loco_status_t loco_dequant_reduce_decomposed(const uint8_t* codes, size_t code_stride_bytes, const float* scales,
                                             size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                             int block_size, float* grad_out, int decomposition, void* stream) {
    return reduce_block(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                        Epilogue::kStore, make_epilogue(grad_out, nullptr, nullptr, nullptr, 0, 0, 0, 0), stream,
                        false, decomposition);
}

int loco_dequant_reduce_decomposition(int num_workers, int bits, int block_size) {
    if ((bits != 4 && bits != 8) || !block_size_ok(block_size) || num_workers < 1) return -1;
    return dr_auto_for_large_shards(bits, block_size, num_workers, Epilogue::kStore, false);
}

loco_status_t loco_dequant_reduce_bf16(const uint8_t* codes, size_t code_stride_bytes, const float* scales,
                                       size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                       int block_size, uint16_t* grad_out_bf16, void* stream) {
    return reduce_block(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                        Epilogue::kStoreBf16,
                        make_epilogue(reinterpret_cast<float*>(grad_out_bf16), nullptr, nullptr, nullptr, 0, 0, 0, 0),
                        stream);
}

loco_status_t loco_dequant_reduce_sgd(const uint8_t* codes, size_t code_stride_bytes, const float* scales,
                                      size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                      int block_size, float eta, float* theta, void* stream) {
    return reduce_block(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                        Epilogue::kSgd, make_epilogue(nullptr, theta, nullptr, nullptr, eta, 0, 0, 0), stream);
}

loco_status_t loco_dequant_reduce_adam(const uint8_t* codes, size_t code_stride_bytes, const float* scales,
                                       size_t scale_stride_elems, int num_workers, size_t n, int bits,
                                       int block_size, float eta, float beta1, float beta2, float delta,
                                       float* m, float* v, float* theta, void* stream) {
    return reduce_block(codes, code_stride_bytes, scales, scale_stride_elems, num_workers, n, bits, block_size,
                        Epilogue::kAdam, make_epilogue(nullptr, theta, m, v, eta, beta1, beta2, delta), stream);
}

loco_status_t loco_stream_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (bytes == 0) return LOCO_OK;
    if (!dst || !src) return LOCO_ERR_INVALID_ARG;
    if (bytes % 16 != 0 || !aligned(dst, 16) || !aligned(src, 16)) return LOCO_ERR_ALIGNMENT;
    if (loco_status_t st = check_device_range(dst, bytes)) return st;
    if (loco_status_t st = check_device_range(src, bytes)) return st;
    return launch_stream<StreamMode::kCopy, CopyShape>(dst, src, nullptr, bytes, stream);
}

loco_status_t loco_runtime_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (bytes == 0) return LOCO_OK;
    if (!dst || !src) return LOCO_ERR_INVALID_ARG;
    if (loco_status_t st = check_device_range(dst, bytes)) return st;
    if (loco_status_t st = check_device_range(src, bytes)) return st;
    const hipError_t e = hipMemcpyDtoDAsync(reinterpret_cast<hipDeviceptr_t>(dst),
                                            reinterpret_cast<hipDeviceptr_t>(const_cast<void*>(src)), bytes,
                                            static_cast<hipStream_t>(stream));
    return e == hipSuccess ? LOCO_OK : LOCO_ERR_LAUNCH;
}

loco_status_t loco_stream_read(const void* src, size_t bytes, void* sink16, void* stream) {
    if (bytes == 0) return LOCO_OK;
    if (!src || !sink16) return LOCO_ERR_INVALID_ARG;
    if (bytes % 16 != 0 || !aligned(src, 16) || !aligned(sink16, 16)) return LOCO_ERR_ALIGNMENT;
    if (loco_status_t st = check_device_range(src, bytes)) return st;
    if (loco_status_t st = check_device_range(sink16, 16)) return st;
    return launch_stream<StreamMode::kRead, ReadShape>(sink16, src, nullptr, bytes, stream);
}

loco_status_t loco_stream_sum2(void* dst, const void* src_a, const void* src_b, size_t bytes, void* stream) {
    if (bytes == 0) return LOCO_OK;
    if (!dst || !src_a || !src_b) return LOCO_ERR_INVALID_ARG;
    if (bytes % 16 != 0 || !aligned(dst, 16) || !aligned(src_a, 16) || !aligned(src_b, 16)) return LOCO_ERR_ALIGNMENT;
    if (loco_status_t st = check_device_range(dst, bytes)) return st;
    if (loco_status_t st = check_device_range(src_a, bytes)) return st;
    if (loco_status_t st = check_device_range(src_b, bytes)) return st;
    return launch_stream<StreamMode::kSum2, Sum2Shape>(dst, src_a, src_b, bytes, stream);
}

loco_status_t loco_stream_update3(void* a, void* b, void* c, size_t bytes, void* stream) {
    if (bytes == 0) return LOCO_OK;
    if (!a || !b || !c) return LOCO_ERR_INVALID_ARG;
    if (bytes % 16 != 0 || !aligned(a, 16) || !aligned(b, 16) || !aligned(c, 16)) return LOCO_ERR_ALIGNMENT;
    if (loco_status_t st = check_device_range(a, bytes)) return st;
    if (loco_status_t st = check_device_range(b, bytes)) return st;
    if (loco_status_t st = check_device_range(c, bytes)) return st;
    const size_t n16 = bytes / 16;
    unsigned grid;
    if (loco_status_t st = grid_for(n16, (size_t)Update3Shape::kThreads * Update3Shape::kSlots, &grid)) return st;
    return launch(update3_kernel<Update3Shape::kSlots, Update3Shape::kThreads, kNonTemporal>, grid, Update3Shape::kThreads,
                  static_cast<hipStream_t>(stream), static_cast<u32x4*>(a), static_cast<u32x4*>(b),
                  static_cast<u32x4*>(c), n16);
}

loco_status_t loco_stream_fill(void* dst, size_t bytes, void* stream) {
    if (bytes == 0) return LOCO_OK;
    if (!dst) return LOCO_ERR_INVALID_ARG;
    if (bytes % 16 != 0 || !aligned(dst, 16)) return LOCO_ERR_ALIGNMENT;
    if (loco_status_t st = check_device_range(dst, bytes)) return st;
    return launch_stream<StreamMode::kFill, FillShape>(dst, nullptr, nullptr, bytes, stream);
}

loco_status_t loco_device_info(int* memory_clock_khz, int* memory_bus_bits, int* compute_units,
                               int* engine_clock_khz) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return LOCO_ERR_LAUNCH;
    const struct { int* out; hipDeviceAttribute_t attr; } wanted[] = {
        {memory_clock_khz, hipDeviceAttributeMemoryClockRate},
        {memory_bus_bits, hipDeviceAttributeMemoryBusWidth},
        {compute_units, hipDeviceAttributeMultiprocessorCount},
        {engine_clock_khz, hipDeviceAttributeClockRate},
    };
    for (const auto& w : wanted) {
        if (!w.out) continue;
        if (hipDeviceGetAttribute(w.out, w.attr, dev) != hipSuccess) return LOCO_ERR_LAUNCH;
    }
    return LOCO_OK;
}

int loco_reset_due(long long step_index, long long reset_period) {
    return reset_period > 0 && step_index % reset_period == 0;
}

loco_status_t loco_step_index_set(int64_t* step_index_dev, int64_t value, void* stream) {
    if (loco_status_t st = check_step_index(step_index_dev, 0)) return st;
    return launch(step_index_kernel, 1, kWave, static_cast<hipStream_t>(stream),
                  reinterpret_cast<long long*>(step_index_dev), (long long)value, 0);
}

loco_status_t loco_step_index_advance(int64_t* step_index_dev, void* stream) {
    if (loco_status_t st = check_step_index(step_index_dev, 0)) return st;
    return launch(step_index_kernel, 1, kWave, static_cast<hipStream_t>(stream),
                  reinterpret_cast<long long*>(step_index_dev), 1LL, 1);
}

loco_status_t loco_error_state8_init(int8_t* err_state8, size_t n, void* stream) {
    if (n == 0) return LOCO_OK;
    if (n > kMaxElements) return LOCO_ERR_UNSUPPORTED;
    if (!err_state8) return LOCO_ERR_INVALID_ARG;
    if (!aligned(err_state8, 16)) return LOCO_ERR_ALIGNMENT;
    if (loco_status_t st = check_device_range(err_state8, n)) return st;
    unsigned grid;
    if (loco_status_t st = grid_for(n, (size_t)FillShape::kThreads * 16 * FillShape::kSlots, &grid)) return st;
    return launch(fill_zero_bytes_kernel<FillShape::kSlots, FillShape::kThreads, kNonTemporal>, grid, FillShape::kThreads,
                  static_cast<hipStream_t>(stream), reinterpret_cast<uint8_t*>(err_state8), n);
}

loco_status_t loco_compensate_quantize_fixed(const void* grad, loco_dtype_t grad_dtype, int8_t* err_state8,
                                             size_t n, int bits, int log2_s, int se_mult, float beta,
                                             int reset, uint8_t* codes_out, void* stream) {
    return compress_fixed(grad, grad_dtype, INFINITY, err_state8, n, bits, log2_s, se_mult, beta, reset, nullptr, 0,
                          codes_out, stream);
}

loco_status_t loco_compensate_quantize_fixed_clip(const void* grad, loco_dtype_t grad_dtype, float clip_abs,
                                                  int8_t* err_state8, size_t n, int bits, int log2_s,
                                                  int se_mult, float beta, int reset, uint8_t* codes_out,
                                                  void* stream) {
    return compress_fixed(grad, grad_dtype, clip_abs, err_state8, n, bits, log2_s, se_mult, beta, reset, nullptr, 0,
                          codes_out, stream);
}

loco_status_t loco_compensate_quantize_fixed_scheduled(const void* grad, loco_dtype_t grad_dtype, int8_t* err_state8,
                                                       size_t n, int bits, int log2_s, int se_mult, float beta,
                                                       const int64_t* step_index_dev, int64_t reset_period,
                                                       uint8_t* codes_out, void* stream) {
    if (n != 0)
        if (loco_status_t st = check_step_index(step_index_dev, reset_period)) return st;
    return compress_fixed(grad, grad_dtype, INFINITY, err_state8, n, bits, log2_s, se_mult, beta, 0, step_index_dev,
                          reset_period, codes_out, stream);
}

loco_status_t loco_compensate_quantize_fixed_f32state(const void* grad, loco_dtype_t grad_dtype, float* err_state,
                                                      size_t n, int bits, int log2_s, float beta, int reset,
                                                      uint8_t* codes_out, void* stream) {
    return compress_fixed_f32state(grad, grad_dtype, err_state, n, bits, log2_s, beta, reset, nullptr, 0, codes_out,
                                   stream);
}

loco_status_t loco_compensate_quantize_fixed_f32state_scheduled(const void* grad, loco_dtype_t grad_dtype,
                                                                float* err_state, size_t n, int bits, int log2_s,
                                                                float beta, const int64_t* step_index_dev,
                                                                int64_t reset_period, uint8_t* codes_out,
                                                                void* stream) {
    if (n != 0)
        if (loco_status_t st = check_step_index(step_index_dev, reset_period)) return st;
    return compress_fixed_f32state(grad, grad_dtype, err_state, n, bits, log2_s, beta, 0, step_index_dev, reset_period,
                                   codes_out, stream);
}

loco_status_t loco_dequant_reduce_fixed(const uint8_t* codes, size_t code_stride_bytes, int num_workers,
                                        size_t n, int bits, int log2_s, float* grad_out, void* stream) {
    return reduce_fixed(codes, code_stride_bytes, num_workers, n, bits, log2_s, Epilogue::kStore,
                        make_epilogue(grad_out, nullptr, nullptr, nullptr, 0, 0, 0, 0), stream);
}

loco_status_t loco_dequant_reduce_fixed_bf16(const uint8_t* codes, size_t code_stride_bytes, int num_workers,
                                             size_t n, int bits, int log2_s, uint16_t* grad_out_bf16,
                                             void* stream) {
    return reduce_fixed(codes, code_stride_bytes, num_workers, n, bits, log2_s, Epilogue::kStoreBf16,
                        make_epilogue(reinterpret_cast<float*>(grad_out_bf16), nullptr, nullptr, nullptr, 0, 0, 0, 0),
                        stream);
}

loco_status_t loco_dequant_reduce_fixed_sgd(const uint8_t* codes, size_t code_stride_bytes, int num_workers,
                                            size_t n, int bits, int log2_s, float eta, float* theta, void* stream) {
    return reduce_fixed(codes, code_stride_bytes, num_workers, n, bits, log2_s, Epilogue::kSgd,
                        make_epilogue(nullptr, theta, nullptr, nullptr, eta, 0, 0, 0), stream);
}

loco_status_t loco_dequant_reduce_fixed_adam(const uint8_t* codes, size_t code_stride_bytes, int num_workers,
                                             size_t n, int bits, int log2_s, float eta, float beta1, float beta2,
                                             float delta, float* m, float* v, float* theta, void* stream) {
    return reduce_fixed(codes, code_stride_bytes, num_workers, n, bits, log2_s, Epilogue::kAdam,
                        make_epilogue(nullptr, theta, m, v, eta, beta1, beta2, delta), stream);
}

}  // extern "C"
