// C ABI of the Distributed Lion sweep: argument validation and kernel launches.
// The entry points and their contracts are documented in include/dlion.h.
#include "dlion_kernels.hpp"

#include <hip/hip_runtime.h>

#include <mutex>
#include <type_traits>

namespace {

using namespace dlion;

constexpr int64_t kMaxTiles = (int64_t)0x7FFFFFFF;   // one-wave workgroups: one tile per workgroup

inline bool aligned_to(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline int64_t tiles_for(int64_t numel) { return (numel + kTile - 1) / kTile; }
inline int64_t words_for(int64_t numel) { return (numel + 63) / 64; }

inline bool power_of_two(int32_t n) { return n > 0 && (n & (n - 1)) == 0; }

#define DLION_TRY(expr)                 \
    do {                                \
        const dlion_status st_ = (expr); \
        if (st_ != DLION_OK)            \
            return st_;                 \
    } while (0)

// Launch-shape overrides (dlion_set_tuning); every field -1 = the library decides.
dlion_tuning g_tuning = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1};
inline const dlion_tuning &tuning() { return g_tuning; }

// Scratch of dlion_step_noalloc: device memory inside the library's code object, so that the entry
// point needs no allocation by anybody.  Every GPU the library runs on holds its own copy at its
// own address; in host code the array's name is only a handle for hipGetSymbolAddress, never a
// pointer to pass on.
static __device__ __align__(256) unsigned char dlion_static_scratch[DLION_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

// Device address of the scratch on the current device, looked up once per device.
dlion_status static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return DLION_ELAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(dlion_static_scratch)) != hipSuccess || !p)
            return DLION_ELAUNCH;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return DLION_OK;
}

Hyper make_hyper(int32_t N, int mode, float beta1, float beta2, float lr, float lambda)
{
    Hyper h;
    h.beta1 = beta1;
    h.omb1 = 1.0f - beta1;
    h.beta2 = beta2;
    h.omb2 = 1.0f - beta2;
    h.lr = lr;
    h.lambda = lambda;
    h.inv_n = power_of_two(N) ? 1.0f / static_cast<float>(N) : 0.0f;
    h.N = N;
    h.mode = mode;
    h.stream_counts = 0;
    h.worker_begin = 0;
    h.worker_end = N;
    h.carry = kCarryNone;
    h.carry_in = 0;
    h.carry_out = 0;
    h.xcd_quads = 0;
    h.beta1_pw = nullptr;
    h.beta2_pw = nullptr;
    return h;
}

// The memory-side cache holds 256 MB; a counts array (2 B per coordinate) well below that is
// still there when the next call reads it.
inline int32_t counts_exceed_cache(int64_t coords) { return coords * 2 > (int64_t)192 << 20; }

// Rows that do not start on a 128-byte line: a wave's piece of such a row shares its first and
// last line with the neighbouring tiles.  The worker/fused kernels then put 4 consecutive tiles
// on one XCD, so that most shared lines meet in one L2 instead of being fetched, and written
// back in part, by two (d = 50 M, N = 8, row stride d + 1: 61.8 -> 69.6 % of peak; stride d + 16:
// 71.9 -> 75.2 %).  Aligned rows lose 0-0.7 % with that numbering and keep the plain one.
inline bool rows_split_lines(const void *base, int64_t stride, size_t elem, int32_t N)
{
    return !aligned_to(base, 128) || (N > 1 && (static_cast<uint64_t>(stride) * elem) % 128 != 0);
}
inline int32_t step_quads(bool split)
{
    const int forced = tuning().step_quads;
    return forced >= 0 ? (forced > 0) : (split ? 1 : 0);
}

inline dim3 grid_for(int64_t tiles) { return dim3(static_cast<uint32_t>(tiles)); }

// Enqueues one kernel and reports what the launch call itself returned: an error that an earlier
// call of this thread left behind is neither reported as ours nor cleared.
template <typename T> struct same { using type = T; };
template <typename... P>
dlion_status launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t s, typename same<P>::type... args)
{
    void *argv[] = {static_cast<void *>(&args)...};
    const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, argv, lds, s);
    return e == hipSuccess ? DLION_OK : DLION_ELAUNCH;
}

// ------------------------------------------------------------------ launch shape
// HBM delivers the most when the chip keeps only a modest, compact window of addresses in
// flight.  A wave of the worker/fused kernels has one worker's loads outstanding at a time
// (1 KB of m and 0.5 or 1 KB of g), and the number of resident waves per compute unit is capped:
// bf16 gradients, 11 / 12 / 14 / 16 waves give 78.5 / 80.1 / 78.5 / 77.3 % of peak at N = 8,
// d = 124 M, and 79.3 / 80.3 / 79.9 / 79.4 % at d = 1.3 G; the launches of a split step that only
// hand their votes on want 14 (N = 32, d = 350 M: 12 / 14 / 16 waves 80.0 / 80.9 / 80.3 %), its
// last launches 16-18; fp32 gradients 11-12 (tensor list, N = 16: 11 / 12 / 14 waves 79.1 / 79.1 /
// 77.2 %).  Issuing two workers' loads back to back with fewer waves is 0.5-4 % slower; uncapped
// the kernel reaches 68 %.  A tensor list takes one wave more for a whole step: its waves start
// with a table lookup during which they have nothing in flight.  The cap is applied by reserving
// (unused) dynamic LDS per workgroup (lds_reservation).
//
// What was tried and dropped for many workers in one launch: 16-wave workgroups walking over
// the workers in lockstep cut the per-CU translation-cache misses 15x at N = 32 (5.5 M against
// 84 M per launch) but were 1-3 % slower on the same allocation; the large run-to-run spread
// of one launch at N = 32 (65-76 % of peak) follows the row stride, not the launch shape.  What
// works is fewer workers per launch (launch_step below).
struct LaunchShape {
    int unroll;          // workers whose loads are issued back to back (8, 4, 2 or 1)
    int blocks_per_cu;   // resident workgroups per compute unit (0: no cap)
};

constexpr size_t kLdsPerCu = 160 * 1024;
constexpr size_t kMaxDynamicLds = 160 * 1024;
constexpr int64_t kResidentWaves = 256 * 32;   // one-wave workgroups the 256 compute units hold at once

// LDS reservation that admits at most `blocks_per_cu` workgroups per compute unit.  The 160 KB are
// handed out in units of 1280 bytes (128 per compute unit), so the caps that can be reached are
// floor(128 / n): 32, 25, 21, 18, 16, 14, 12, 11, 10, 9, 8 ...; 13 and 15 do not exist (measured:
// reservations asking for 14 and 15, or for 16 and 17, run at the same speed).
constexpr size_t kLdsGranule = 1280;

// the next reachable cap above k
inline int next_cap(int k)
{
    const int granules = static_cast<int>(kLdsPerCu / kLdsGranule);
    int n = granules / (k + 1) + 1;                       // granules reserved for cap k
    while (n > 1 && granules / n <= k)
        --n;
    return granules / n;
}

inline size_t lds_reservation(int blocks_per_cu)
{
    if (blocks_per_cu <= 0)
        return 0;
    const size_t granules = kLdsPerCu / kLdsGranule;                              // 128
    const size_t n = granules / (static_cast<size_t>(blocks_per_cu) + 1) + 1;     // smallest n with granules / n <= cap
    const size_t bytes = n * kLdsGranule;
    return bytes > kMaxDynamicLds ? kMaxDynamicLds : bytes;
}

// What a launch of the worker/fused kernels is within its step.
enum StepRole {
    kWholeStep,   // all workers of the step in this launch
    kHandOn,      // some of the workers; the votes are handed on to a later launch (no x)
    kLastPass,    // the last workers: adds up what was handed on, then aggregates and updates x
};

// wide_g: fp32 gradients (a wave then has 2 KB per worker in flight, 1.5 KB with bf16 ones).
LaunchShape step_shape(int32_t N, bool wide_g, StepRole role)
{
    const dlion_tuning &tn = tuning();
    LaunchShape s;
    s.unroll = tn.unroll > 0 ? tn.unroll : 1;
    while (s.unroll > N)
        s.unroll >>= 1;
    if (s.unroll < 1)
        s.unroll = 1;
    const int forced = (role == kHandOn && tn.blocks_per_cu_pass >= 0) ? tn.blocks_per_cu_pass : tn.blocks_per_cu;
    if (forced >= 0) {
        s.blocks_per_cu = forced;
    } else {
        const int waves = wide_g ? (role == kLastPass ? 12 : 11) : (role == kWholeStep ? 12 : (role == kHandOn ? 14 : 16));
        s.blocks_per_cu = s.unroll == 1 ? waves : (waves * 3 / 2 / s.unroll < 3 ? 3 : waves * 3 / 2 / s.unroll);
    }
    return s;
}

// ------------------------------------------------------------------ dispatch
template <typename GT, int kUnroll, bool kApply, class Addr>
dlion_status launch_step_flags(const Addr &addr, const Hyper &h, bool packed, bool counts, size_t lds,
                               hipStream_t s)
{
    const dim3 grid = grid_for(addr.total_tiles - addr.first_tile), block(kLanes);
    const size_t stage = kLanes * sizeof(uint64_t);
    if (packed && lds < stage)
        lds = stage;                                      // packed words are staged in LDS, 512 B per wave
    if (packed && counts)
        return launch(step_kernel<GT, kUnroll, kApply, true, true, Addr>, grid, block, lds, s, addr, h);
    if (packed)
        return launch(step_kernel<GT, kUnroll, kApply, true, false, Addr>, grid, block, lds, s, addr, h);
    if (counts)
        return launch(step_kernel<GT, kUnroll, kApply, false, true, Addr>, grid, block, lds, s, addr, h);
    return launch(step_kernel<GT, kUnroll, kApply, false, false, Addr>, grid, block, lds, s, addr, h);
}

template <typename GT, bool kApply, class Addr>
dlion_status launch_step_unroll(const Addr &addr, const Hyper &h, bool packed, bool counts, int64_t problem_tiles,
                                hipStream_t s)
{
    const StepRole role = h.carry_out != 0 ? kHandOn : ((h.carry != kCarryNone && h.carry_in) ? kLastPass : kWholeStep);
    LaunchShape shape = step_shape(h.worker_end - h.worker_begin, Grad<GT>::kVecBytes == 16, role);
    // A problem whose waves all fit on the chip at once never reaches the steady state the cap
    // is tuned for; it is latency-bound and wants every wave resident (d = 1,000,003, N = 4:
    // 12.7 -> 10.4 us).
    if (tuning().blocks_per_cu < 0) {
        if (problem_tiles <= kResidentWaves)
            shape.blocks_per_cu = 0;
        else if (role == kWholeStep && shape.blocks_per_cu > 0 && (std::is_same<Addr, SegAddr>::value || h.beta1_pw))
            // a tensor list's waves start with a table lookup, those of a step with per-worker
            // coefficients by fetching them, and have nothing else in flight meanwhile; the next cap
            // up makes up for it (per-worker coefficients, bf16, N = 8: 12 -> 14 waves, d = 124 M
            // 78.9 -> 81.3 % of peak, d = 1.3 G 77.9 -> 80.9 %; the ViT list with bf16 gradients and
            // N = 8: 79.3 -> 81.1 %, with fp32 gradients 11 -> 12 waves)
            shape.blocks_per_cu = next_cap(shape.blocks_per_cu);
    }
    const size_t lds = lds_reservation(shape.blocks_per_cu);
    switch (shape.unroll) {
    case 8: return launch_step_flags<GT, 8, kApply, Addr>(addr, h, packed, counts, lds, s);
    case 4: return launch_step_flags<GT, 4, kApply, Addr>(addr, h, packed, counts, lds, s);
    case 2: return launch_step_flags<GT, 2, kApply, Addr>(addr, h, packed, counts, lds, s);
    default: return launch_step_flags<GT, 1, kApply, Addr>(addr, h, packed, counts, lds, s);
    }
}

template <bool kApply, class Addr>
dlion_status launch_step_once(const Addr &addr, const Hyper &h, dlion_dtype g_dtype, bool packed, bool counts,
                              int64_t problem_tiles, hipStream_t s)
{
    if (g_dtype == DLION_BF16)
        return launch_step_unroll<uint16_t, kApply, Addr>(addr, h, packed, counts, problem_tiles, s);
    return launch_step_unroll<float, kApply, Addr>(addr, h, packed, counts, problem_tiles, s);
}

// How a step is cut into launches.
//
// By tiles.  Workgroups are handed to the 8 XCDs round-robin and every XCD works through its own
// share at its own pace, so over a long launch the XCDs drift apart and the window of addresses in
// flight widens; launches of kBlockTiles tiles bring them back together (N = 8, bf16: d = 1.3 G
// 77.6 -> 80.2 % of peak with 67 M coordinates per launch, 81.2 % with 134 M; d = 350 M 76.9 ->
// 79.1 %; d = 124 M unchanged).  A launch boundary costs about 4.5 us when launches are short
// (16384 tiles) and nothing measurable from 131072 tiles on.
//
// By workers.  One launch over all N rows keeps 2N + 1 streams (and as many pages) open across
// the chip at once, and from N = 16 on that costs more bandwidth than handing the votes from one
// launch over kPassWorkers workers to the next (fused step, bf16 gradients, d = 350 M, N = 32:
// one launch 20.6 ms, launches over 8 workers 18.0 ms; 6 / 7 / 9 / 10 / 11 workers per launch are
// all 0.1-1.5 % slower than 8, 16 lose 5 %; N = 12 gains nothing, and below ~16 M coordinates the
// extra launches cost what they save).  The worker step needs no hand-over.  The fused step hands
// the votes on in the caller's workspace or, without one, in the caller's counts array, and stays
// one launch per block when it has neither: the library owns no memory.  All launches of one
// block of tiles run before the next block starts, so the hand-over is still in the memory-side
// cache when it is read back (a running uint16 count handed on over the whole of d = 350 M
// instead: 19.2 against 18.5 ms).
//
// Hand-over formats (Carry): in a workspace and with at most kNibblePasses launches, every
// launch but the last writes its own plane of 4-bit partial counts (0.5 B per coordinate written,
// and read once by the last launch: 3 B per coordinate at N = 32, 0.9 % on top of the step's
// algorithmic bytes, which is most of what separates it from the single-launch rate at N = 8);
// with more launches a running uint16 count per coordinate (2 B read + 2 B written per launch);
// in the counts array the running count, indexed by coordinate.  Block sizes between 131072 and
// 524288 tiles are within 0.15 % of each other at N = 32.
constexpr int kPassWorkers = 8;
constexpr int kPassMinN = 16;
constexpr int kNibblePasses = 8;            // at most 7 planes of partial counts
constexpr int kNibbleMaxWorkers = 15;       // a partial count must fit 4 bits
constexpr int64_t kPassMinTiles = 8 * kResidentWaves;
constexpr int64_t kBlockTiles = 64 * kResidentWaves;         // 134 M coordinates per launch
constexpr int64_t kPassBlockTiles = 32 * kResidentWaves;     // 67 M when the block is cut into launches over few workers
constexpr int64_t kPassMinBlockTiles = 4 * kResidentWaves;   // a workspace that holds less is not used

struct Workspace {
    void *base = nullptr;
    int64_t bytes = 0;
};

struct StepPlan {
    int passes = 1;          // launches per block of tiles
    int carry = kCarryNone;
    int64_t block = 0;       // tiles per block
    int64_t ws_tile = 0;     // workspace bytes per tile
};

inline int64_t ws_bytes_per_tile(int carry, int passes)
{
    if (carry == kCarryNibbles)
        return (int64_t)(passes - 1) * kNibbleCarryPerTile * 2;
    return carry == kCarryRunning ? kRunningCarryPerTile * 2 : 0;
}

// passes of the default split for N workers over `tiles` tiles (1: no split)
inline int default_passes(int32_t N, int64_t tiles)
{
    int per = tuning().pass_workers;                      // 0 = always one launch
    if (per < 0)
        per = (N >= kPassMinN && tiles >= kPassMinTiles) ? kPassWorkers : 0;
    return (per <= 0 || per >= N) ? 1 : (N + per - 1) / per;
}

inline int workspace_carry(int32_t N, int passes)
{
    const int most = (N + passes - 1) / passes;           // workers of the largest launch
    return (passes <= kNibblePasses && most <= kNibbleMaxWorkers) ? kCarryNibbles : kCarryRunning;
}

inline int64_t default_block_tiles(int passes)
{
    const int64_t forced = tuning().block_tiles;           // 0 = all tiles in one block
    return forced >= 0 ? forced : (passes > 1 ? kPassBlockTiles : kBlockTiles);
}

StepPlan plan_step(int32_t N, int64_t tiles, bool apply, bool counts, const Workspace &ws)
{
    StepPlan pl;
    pl.passes = default_passes(N, tiles);
    pl.block = default_block_tiles(pl.passes);
    if (pl.block <= 0 || pl.block > tiles)
        pl.block = tiles;
    if (pl.passes > 1 && apply) {
        // the fused step needs somewhere to hand the votes on: the workspace, else the counts output
        const int carry = workspace_carry(N, pl.passes);
        const int64_t per_tile = ws_bytes_per_tile(carry, pl.passes);
        const int64_t fit = ws.base ? ws.bytes / per_tile : 0;
        if (fit >= pl.block || fit >= kPassMinBlockTiles) {
            pl.carry = carry;
            pl.ws_tile = per_tile;
            if (fit < pl.block)
                pl.block = fit;
        } else if (counts) {
            pl.carry = kCarryCounts;
        } else {
            pl.passes = 1;
        }
    }
    return pl;
}

template <class Addr> inline void set_workspace(Addr &a, const StepPlan &pl, const Workspace &ws)
{
    a.ws = (pl.carry == kCarryNibbles || pl.carry == kCarryRunning) ? static_cast<uint16_t *>(ws.base) : nullptr;
    a.ws_plane = pl.block * kNibbleCarryPerTile;
}

template <bool kApply, class Addr>
dlion_status launch_step(const Addr &addr, const Hyper &h0, dlion_dtype g_dtype, bool packed, bool counts,
                         hipStream_t s, const Workspace &ws = Workspace())
{
    const int N = h0.N;
    const int64_t tiles = addr.total_tiles;
    const StepPlan pl = plan_step(N, tiles, kApply, counts, ws);
    Hyper h = h0;
    Addr a = addr;
    set_workspace(a, pl, ws);
    for (int64_t first = 0; first < tiles; first += pl.block) {
        a.first_tile = first;
        a.total_tiles = first + pl.block < tiles ? first + pl.block : tiles;
        for (int pass = 0; pass < pl.passes; ++pass) {
            // spread evenly: N = 30 runs as 8, 8, 7, 7
            h.worker_begin = static_cast<int32_t>((int64_t)N * pass / pl.passes);
            h.worker_end = static_cast<int32_t>((int64_t)N * (pass + 1) / pl.passes);
            const bool last = pass == pl.passes - 1;
            h.carry = pl.carry;
            h.carry_in = h.carry_out = 0;
            h.stream_counts = h0.stream_counts;
            bool counts_out = counts;
            if (pl.carry == kCarryCounts) {
                h.carry_in = pass > 0;
                // the running count is read again right away: keep it cached; the result follows the caller's hint
                if (!last && pl.block < tiles)
                    h.stream_counts = 0;
            } else if (pl.carry == kCarryRunning) {
                h.carry_in = pass > 0;
                h.carry_out = !last;
                counts_out = counts && last;
            } else if (pl.carry == kCarryNibbles) {
                h.carry_in = last ? pl.passes - 1 : 0;
                h.carry_out = last ? 0 : pass + 1;
                counts_out = counts && last;
            }
            dlion_status st;
            if (kApply && last)
                st = launch_step_once<true, Addr>(a, h, g_dtype, packed, counts_out, tiles, s);
            else
                st = launch_step_once<false, Addr>(a, h, g_dtype, packed, counts_out, tiles, s);
            if (st != DLION_OK)
                return st;
        }
    }
    return DLION_OK;
}

// Launches of the server-side and update kernels are cut like the step's (XCDs drift apart over a
// long launch: d = 1.3 G, dlion_apply in one launch 78.7 % of peak against 91.9 % at d = 124 M), by
// bytes moved rather than by tiles, since their bytes per coordinate span 3 to 40: about 6 GB per
// launch, which is what a launch of the step over 8 workers moves.  A grid unit of the kernel covers
// tiles_per_unit tiles and moves about bytes_per_coord bytes per coordinate.
constexpr int64_t kBlockBytes = (int64_t)6 << 30;
// The bit-sliced kernels, whose workgroups read for a long time and then write in one burst, want
// much shorter launches: with one round of workgroups per launch (131072 tiles: 256 workgroups of
// 16 waves) the whole chip reads together and then writes together (N = 256, d = 1 G, fused
// update: one launch 6.88 ms, 131072 / 262144 / 524288 / 1048576 tiles per launch 6.04 / 6.02 /
// 6.12 / 6.30 ms; counts only 5.09 against 5.05 ms), as long as a launch still moves about 1 GB.
constexpr int64_t kSlicedBlockTiles = 16 * kResidentWaves;
constexpr int64_t kSlicedBlockBytes = (int64_t)1 << 30;

template <class Addr, class Launch>
dlion_status launch_in_blocks(const Addr &addr, int64_t units, int64_t tiles_per_unit, int64_t bytes_per_coord,
                              bool sliced, Launch launch_one)
{
    const int64_t forced = tuning().block_tiles;           // 0 = all in one launch
    int64_t tiles = (sliced ? kSlicedBlockBytes : kBlockBytes) / (kTile * bytes_per_coord);
    if (sliced) {
        // whole rounds only: a launch of 1.2 rounds runs as long as one of 2
        tiles = (tiles + kSlicedBlockTiles / 2) / kSlicedBlockTiles * kSlicedBlockTiles;
        if (tiles < kSlicedBlockTiles)
            tiles = kSlicedBlockTiles;
    }
    int64_t block = forced > 0 ? forced / tiles_per_unit : (forced == 0 ? units : tiles / tiles_per_unit);
    if (block < 1)
        block = 1;
    Addr a = addr;
    for (int64_t first = 0; first < units; first += block) {
        a.first_tile = first;
        DLION_TRY(launch_one(a, first + block < units ? block : units - first));
    }
    return DLION_OK;
}

template <class Addr>
dlion_status launch_aggregate(const Addr &addr, const Hyper &h, bool apply, bool counts, hipStream_t s)
{
    const int64_t bytes = h.N / 8 + 1 + (apply ? 8 : 0) + (counts ? 2 : 0);
    return launch_in_blocks(addr, addr.total_tiles, 1, bytes, false, [&](const Addr &a, int64_t n) {
        const dim3 grid = grid_for(n), block(kLanes);
        if (apply && counts)
            return launch(aggregate_kernel<true, true, Addr>, grid, block, 0, s, a, h);
        if (apply)
            return launch(aggregate_kernel<true, false, Addr>, grid, block, 0, s, a, h);
        return launch(aggregate_kernel<false, true, Addr>, grid, block, 0, s, a, h);
    });
}

// Bit-sliced counting (flat buffers): planes = bits needed for a count 0..N; waves per
// workgroup is 1, or as many (up to 16) as fit the 160 KB of LDS with one region per wave.
constexpr int kSlicedOneWaveBlocks = 16;
template <int kPlanes, int kWaves>
dlion_status launch_sliced_shape(const FlatAddr &addr, const Hyper &h, bool apply, bool counts, hipStream_t s)
{
    const int64_t W = words_for(addr.p.numel);
    const int64_t groups = (W + kSlicedWords - 1) / kSlicedWords;
    size_t lds = static_cast<size_t>(kWaves) * kPlanes * kSlicedLdsPerPlane * sizeof(uint32_t);
    if (kWaves == 1 && lds_reservation(kSlicedOneWaveBlocks) > lds)
        lds = lds_reservation(kSlicedOneWaveBlocks);          // at most 16 one-wave workgroups per compute unit
    // a word group of kSlicedWords words is kSlicedWords / kWordsPerTile tiles; a workgroup takes kWaves groups
    const int64_t bytes = h.N / 8 + 1 + (apply ? 8 : 0) + (counts ? 2 : 0);
    return launch_in_blocks(addr, (groups + kWaves - 1) / kWaves, kWaves * (kSlicedWords / kWordsPerTile), bytes,
                            kWaves > 1, [&](FlatAddr a, int64_t n) {
        a.first_tile *= kWaves;                          // the kernel counts in word groups
        const dim3 grid = grid_for(n), block(kLanes * kWaves);
        if (apply && counts)
            return launch(aggregate_sliced_kernel<kPlanes, kWaves, true, true>, grid, block, lds, s, a, h);
        if (apply)
            return launch(aggregate_sliced_kernel<kPlanes, kWaves, true, false>, grid, block, lds, s, a, h);
        return launch(aggregate_sliced_kernel<kPlanes, kWaves, false, true>, grid, block, lds, s, a, h);
    });
}

// Waves per workgroup of the bit-sliced kernels.  Workgroups of 8 or 16 waves walk the streams in
// lockstep and write together; with launches of whole rounds they run at 74-86 % of peak for every
// N from 65 to 1000 (d = 124 M to 1 G; a launch of 1.2 rounds, which the byte rule alone gave at
// N = 192 or 512, ran at 60-67 %).  One-wave workgroups (16 to a compute unit, two rows in flight)
// are level with them for the counts and 2-6 % behind for the fused update and the message at large
// d, and well behind when d is small and N large (N = 2000, d = 16 M: 71 against 85 %; N = 65535,
// d = 1 M: 3 against 8 %); they are kept for problems of a few dozen groups of 128 words.  16 waves
// need a workgroup for every compute unit (N = 130, d = 16 M: 8 waves 72-79 %, 16 waves 50-57 %).
constexpr int kSlicedWaves = 8;
constexpr int kSliced16MinWorkers = 128;
constexpr int64_t kSlicedMinGroups = 4096;     // groups of 128 words for 16-wave workgroups: 33.5 M coordinates
constexpr int64_t kSlicedMinGroups8 = 64;      // ... and for 8-wave workgroups

inline int64_t sliced_groups(int64_t numel) { return (words_for(numel) + kSlicedWords - 1) / kSlicedWords; }

// waves per workgroup when `wanted` (8 or 16) lockstep waves suit N
inline int sliced_waves_for(int64_t numel, int wanted)
{
    const int forced = tuning().sliced_waves;              // 1, 8 or 16
    if (forced > 0)
        return forced;
    const int64_t groups = sliced_groups(numel);
    if (wanted >= 16 && groups >= kSlicedMinGroups)
        return 16;
    return groups >= kSlicedMinGroups8 ? 8 : 1;
}

// Flat buffers with more workers than the few-worker kernel takes (aggregate_group_kernel, below) go
// to the bit-sliced kernel at every N and d (the per-nibble kernel, which reads 32 bytes of a row per
// wave, runs the fused update at N = 4096, d = 33 M at 18 % of peak); the per-nibble kernel serves the
// tensor lists' fused aggregate + update beyond the few-worker kernel's N.
inline bool use_sliced(int32_t N)
{
    const int forced = tuning().sliced_min_workers;       // per-nibble kernel below this N
    return forced < 0 || N >= forced;
}

template <int kPlanes, bool kAllow16>
dlion_status launch_sliced_planes(const FlatAddr &addr, const Hyper &h, bool apply, bool counts, hipStream_t s)
{
    const int waves = sliced_waves_for(addr.p.numel, h.N >= kSliced16MinWorkers ? 16 : kSlicedWaves);
    if (waves >= 16 && kAllow16)
        return launch_sliced_shape<kPlanes, kAllow16 ? 16 : 8>(addr, h, apply, counts, s);
    if (waves >= 8)
        return launch_sliced_shape<kPlanes, 8>(addr, h, apply, counts, s);
    return launch_sliced_shape<kPlanes, 1>(addr, h, apply, counts, s);
}

dlion_status launch_sliced(const FlatAddr &addr, const Hyper &h, bool apply, bool counts, hipStream_t s)
{
    if (h.N < 32)
        return launch_sliced_planes<5, true>(addr, h, apply, counts, s);
    if (h.N < 128)
        return launch_sliced_planes<7, true>(addr, h, apply, counts, s);
    if (h.N < 512)
        return launch_sliced_planes<9, true>(addr, h, apply, counts, s);
    if (h.N < 4096)
        return launch_sliced_planes<12, false>(addr, h, apply, counts, s);
    return launch_sliced_planes<16, false>(addr, h, apply, counts, s);
}

template <class Addr> dlion_status launch_apply(const Addr &addr, const Hyper &h, hipStream_t s)
{
    // no occupancy cap here: it only loses (d = 124 M: 88.7 % uncapped, 81 % with 16-24 waves per compute unit)
    return launch_in_blocks(addr, addr.total_tiles, 1, 10, false, [&](const Addr &a, int64_t n) {
        return launch(apply_kernel<Addr>, grid_for(n), dim3(kLanes), 0, s, a, h);
    });
}

// Down-link message: planes needed for Delta.
inline int32_t delta_planes(int32_t N, int mode)
{
    if (mode == DLION_AVG) {
        int32_t bits = 0;
        while ((static_cast<int64_t>(1) << bits) <= static_cast<int64_t>(N))
            ++bits;
        return bits;
    }
    return (N % 2 == 0) ? 2 : 1;
}

constexpr int kGroupEncodeMinWorkers = 12;     // below: the bit-sliced encoder (see the few-worker kernel's launch)

template <int kPlanes, int kWaves>
dlion_status launch_encode_shape(const FlatAddr &addr, const Hyper &h, const DeltaOut &out, hipStream_t s)
{
    const int64_t W = words_for(addr.p.numel);
    const int64_t groups = (W + kSlicedWords - 1) / kSlicedWords;
    return launch_in_blocks(addr, (groups + kWaves - 1) / kWaves, kWaves * (kSlicedWords / kWordsPerTile),
                            h.N / 8 + 1 + out.n_planes / 8, kWaves > 1, [&](FlatAddr a, int64_t n) {
        a.first_tile *= kWaves;
        // one-wave workgroups: at most 16 resident per compute unit (the kernel itself uses no LDS)
        const size_t lds = kWaves == 1 ? lds_reservation(kSlicedOneWaveBlocks) : 0;
        return launch(aggregate_encode_kernel<kPlanes, kWaves>, grid_for(n), dim3(kLanes * kWaves), lds, s, a, h, out);
    });
}

template <int kPlanes>
dlion_status launch_encode_planes(const FlatAddr &addr, const Hyper &h, const DeltaOut &out, hipStream_t s)
{
    // 16 waves from N = 64 on (N = 256, d = 1 G: vote 5.15 -> 5.03 ms, average 6.00 -> 5.49 ms; N = 64:
    // 1.48 -> 1.44 and 1.69 -> 1.60 ms).  The very few workers that the few-worker kernel leaves to this
    // one (N < 12: a message of 30-300 us) run as one-wave workgroups, 16 to a compute unit: packed rows on
    // 1 KB boundaries, N = 8, d = 124 M 62-66 -> 72-73 % of peak, d = 1.3 G 74-77 -> 79-81 %.
    const int waves = h.N < kGroupEncodeMinWorkers && tuning().sliced_waves <= 0
                          ? 1 : sliced_waves_for(addr.p.numel, h.N >= 64 ? 16 : kSlicedWaves);
    if (waves >= 16 && kPlanes <= 9)
        return launch_encode_shape<kPlanes, kPlanes <= 9 ? 16 : 8>(addr, h, out, s);
    if (waves >= 8)
        return launch_encode_shape<kPlanes, 8>(addr, h, out, s);
    return launch_encode_shape<kPlanes, 1>(addr, h, out, s);
}

dlion_status launch_encode(const FlatAddr &addr, const Hyper &h, const DeltaOut &out, hipStream_t s)
{
    if (h.N < 32)
        return launch_encode_planes<5>(addr, h, out, s);
    if (h.N < 128)
        return launch_encode_planes<7>(addr, h, out, s);
    if (h.N < 512)
        return launch_encode_planes<9>(addr, h, out, s);
    if (h.N < 4096)
        return launch_encode_planes<12>(addr, h, out, s);
    return launch_encode_planes<16>(addr, h, out, s);
}

// Few workers on flat buffers (aggregate_group_kernel): eight waves share 8192 coordinates.  enc = the
// down-link planes to write instead of counts / x, or null.
//
// Measured with packed rows that start on 1 KB boundaries, d = 350 M, % of the HBM peak, bit-sliced
// kernel -> this one:
//   counts only      N = 4 / 16 / 32 / 64 / 100: 67.1 / 70.7 / 70.7 / 73.0 / 72.8 -> 74.5 / 81.5 / 81.4 / 77.8 / 75.6
//   fused update     N = 4 / 16 / 32 / 64 / 120: 69.4 / 72.2 / 69.8 / 72.4 / 73.6 -> 80.6 / 78.8 / 79.9 / 79.6 / 78.2
//   message, vote    N = 12 / 16 / 32 / 64:      71.8 / 72.6 / 70.5 / 71.1        -> 72.9 / 79.6 / 77.1 / 73.9
//   message, average N = 12 / 16 / 32 / 64:      74.5 / 71.7 / 70.4 / 72.1        -> 82.9 / 82.5 / 77.0 / 71.5
// The shape that wins depends on what is written.  The fused update (4 KB of x read and written per
// wave) wants one row in flight per wave and three workgroups per compute unit (two: 72-74 %, four:
// 73-75 %); counts and messages want two rows in flight and, as N grows, fewer workgroups.  Below
// N = 12 the message is so short (30-50 us) that the bit-sliced kernel, which has no exchange through
// LDS on its way out, is faster (N = 4: 71 against 44 %).  Rows that do not start on a 128-byte line
// cost either kernel 3-8 % (a wave's 1 KB piece of a row then shares lines with its neighbours').
constexpr int kGroupMaxWorkers = 120;          // counts up to 127 fit the kernel's byte lanes
constexpr int kGroupApplyMaxWorkers = 120;     // fused update: ahead of the bit-sliced kernel up to the limit
constexpr int kGroupCountsMaxWorkers = 64;     // counts only: behind it from N = 65 on (69 against 76 %)
constexpr int kGroupEncodeMaxWorkers = 64;

// resident workgroups (of 8 waves) per compute unit; 0 = as many as fit (4)
inline int group_blocks(const Hyper &h, bool apply, bool encode)
{
    const int forced = tuning().group_blocks;
    if (forced >= 0)
        return forced;
    if (apply)
        return 3;
    if (encode)
        return h.N < 32 || (h.N == 32 && h.mode == DLION_VOTE) ? 0 : 3;
    return h.N < 32 ? 4 : (h.N < 64 ? 3 : 2);
}

template <int kAcc>
dlion_status launch_group_planes(const FlatAddr &addr, const Hyper &h, bool apply, bool counts, const DeltaOut *enc,
                                 const SegTab &tab, hipStream_t s)
{
    const int64_t spans = (words_for(addr.p.numel) + kGroupWords - 1) / kGroupWords;
    const DeltaOut out = enc ? *enc : DeltaOut{nullptr, 0, 0};
    const int64_t bytes = h.N / 8 + 1 + (apply ? 8 : 0) + (counts ? 2 : 0) + out.n_planes / 8;
    // the waves' partial planes, and (down-link message) the planes on their way out
    const size_t need = (static_cast<size_t>(kGroupWaves) * kAcc + (enc ? kAcc + 3 : 0)) * 256 * sizeof(uint32_t);
    const size_t cap = lds_reservation(group_blocks(h, apply, enc != nullptr));
    const size_t lds = cap > need ? cap : need;
    return launch_in_blocks(addr, spans, kGroupCoords / kTile, bytes, false, [&](const FlatAddr &a, int64_t n) {
        const dim3 grid = grid_for(n), block(kLanes * kGroupWaves);
        if (enc)
            return launch(aggregate_group_kernel<kAcc, 2, false, false, true, false>, grid, block, lds, s, a, h, out, tab);
        if (apply && tab.segs && counts)
            return launch(aggregate_group_kernel<kAcc, 1, true, true, false, true>, grid, block, lds, s, a, h, out, tab);
        if (apply && tab.segs)
            return launch(aggregate_group_kernel<kAcc, 1, true, false, false, true>, grid, block, lds, s, a, h, out, tab);
        if (apply && counts)
            return launch(aggregate_group_kernel<kAcc, 1, true, true, false, false>, grid, block, lds, s, a, h, out, tab);
        if (apply)
            return launch(aggregate_group_kernel<kAcc, 1, true, false, false, false>, grid, block, lds, s, a, h, out, tab);
        return launch(aggregate_group_kernel<kAcc, 2, false, true, false, false>, grid, block, lds, s, a, h, out, tab);
    });
}

// tab: the tensor table behind a flat view of a tensor list (x is found through it), or {null, 0}
dlion_status launch_group(const FlatAddr &addr, const Hyper &h, bool apply, bool counts, const DeltaOut *enc, hipStream_t s,
                          const SegTab &tab = SegTab{nullptr, 0})
{
    // planes a wave needs for its own rows: ceil(N / 8) < 2^kAcc
    if (h.N <= 8)
        return launch_group_planes<1>(addr, h, apply, counts, enc, tab, s);
    if (h.N <= 24)
        return launch_group_planes<2>(addr, h, apply, counts, enc, tab, s);
    if (h.N <= 56)
        return launch_group_planes<3>(addr, h, apply, counts, enc, tab, s);
    return launch_group_planes<4>(addr, h, apply, counts, enc, tab, s);
}

// The kernel serves N up to group_max_workers (never beyond kGroupMaxWorkers); a forced value also
// sends the short messages of very few workers through it.
enum GroupUse { kGroupCounts, kGroupApply, kGroupEncode };

inline bool use_group(int32_t N, GroupUse use)
{
    const int forced = tuning().group_max_workers;
    if (forced >= 0)
        return N <= forced;
    if (use == kGroupApply)
        return N <= kGroupApplyMaxWorkers;
    if (use == kGroupEncode)
        return N >= kGroupEncodeMinWorkers && N <= kGroupEncodeMaxWorkers;
    return N <= kGroupCountsMaxWorkers;
}

template <typename GT>
dlion_status launch_global_lion_unroll(const FlatAddr &addr, const Hyper &h, uint64_t *sign_bits, hipStream_t s)
{
    const LaunchShape shape = step_shape(h.N, Grad<GT>::kVecBytes == 16, kWholeStep);
    const size_t lds = lds_reservation(shape.blocks_per_cu);
    const dim3 grid(static_cast<uint32_t>(addr.total_tiles)), block(kLanes);
    if (shape.unroll >= 2 && h.N >= 2)
        return launch(global_lion_kernel<GT, 2>, grid, block, lds, s, addr, h, sign_bits);
    else
        return launch(global_lion_kernel<GT, 1>, grid, block, lds, s, addr, h, sign_bits);
}

// ------------------------------------------------------------------ validation
dlion_status check_common(int64_t d, int32_t N)
{
    if (d <= 0 || N < 1 || N > DLION_MAX_WORKERS)
        return DLION_EINVAL;
    if (tiles_for(d) > kMaxTiles)
        return DLION_EUNSUPPORTED;
    return DLION_OK;
}

dlion_status check_rows(const void *p, int64_t stride, int64_t extent, int32_t N, uintptr_t elem)
{
    if (!p)
        return DLION_EINVAL;
    if (!aligned_to(p, elem))
        return DLION_EALIGN;
    if (N > 1 && stride < extent)
        return DLION_EINVAL;
    return DLION_OK;
}

inline uintptr_t grad_size(dlion_dtype t) { return t == DLION_BF16 ? 2 : 4; }
inline bool dtype_ok(dlion_dtype t) { return t == DLION_F32 || t == DLION_BF16; }
inline bool mode_ok(dlion_mode m) { return m == DLION_VOTE || m == DLION_AVG; }

FlatAddr flat_addr(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride, int64_t d,
                   uint64_t *packed, int64_t packed_stride, uint16_t *counts)
{
    FlatAddr a;
    a.p.x = x;
    a.p.m = m;
    a.p.g = g;
    a.p.m_stride = m_stride;
    a.p.g_stride = g_stride;
    a.p.numel = d;
    a.p.packed = packed;
    a.p.packed_stride = packed_stride;
    a.p.counts = counts;
    a.p.counts_end = d;
    a.total_tiles = tiles_for(d);
    a.first_tile = 0;
    a.ws = nullptr;
    a.ws_plane = 0;
    return a;
}

// What a tensor-list call needs from each segment.
enum SegNeeds { kNeedX = 1, kNeedM = 2, kNeedG = 4 };

dlion_status check_segs(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K, int32_t N,
                        int needs, dlion_dtype g_dtype, int64_t *total_words, int64_t *total_tiles,
                        bool *rows_split = nullptr)
{
    if (!segs_host || !segs_dev || K < 1 || N < 1 || N > DLION_MAX_WORKERS)
        return DLION_EINVAL;
    bool split = false;
    if (!aligned_to(segs_dev, 8))
        return DLION_EALIGN;
    int64_t words = 0, tiles = 0;
    for (int32_t k = 0; k < K; ++k) {
        const dlion_seg &s = segs_host[k];
        if (s.numel <= 0)
            return DLION_EINVAL;
        if (s.word_begin != words || s.tile_begin != tiles)
            return DLION_EINVAL;   // table was not laid out by dlion_mt_layout
        if (needs & kNeedX) {
            if (!s.x)
                return DLION_EINVAL;
            if (!aligned_to(s.x, 4))
                return DLION_EALIGN;
        }
        if (needs & kNeedM) {
            DLION_TRY(check_rows(s.m, s.m_stride, s.numel, N, 4));
            split = split || rows_split_lines(s.m, s.m_stride, 4, N);
        }
        if (needs & kNeedG) {
            DLION_TRY(check_rows(s.g, s.g_stride, s.numel, N, grad_size(g_dtype)));
            split = split || rows_split_lines(s.g, s.g_stride, grad_size(g_dtype), N);
        }
        words += words_for(s.numel);
        tiles += tiles_for(s.numel);
        if (tiles > kMaxTiles)
            return DLION_EUNSUPPORTED;
    }
    *total_words = words;
    *total_tiles = tiles;
    if (rows_split)
        *rows_split = split;
    return DLION_OK;
}

SegAddr seg_addr(const dlion_seg *segs_dev, int32_t K, int64_t total_tiles, uint64_t *packed,
                 int64_t packed_stride, uint16_t *counts)
{
    SegAddr a;
    a.segs = segs_dev;
    a.K = K;
    a.total_tiles = total_tiles;
    a.first_tile = 0;
    a.ws = nullptr;
    a.ws_plane = 0;
    a.packed = packed;
    a.packed_stride = packed_stride;
    a.counts = counts;
    return a;
}

template <int kBatch>
dlion_status launch_membench(const u32x4 *src, int64_t row_stride, int32_t rows, u32x4 *dst, int64_t pieces,
                             bool write, size_t lds, hipStream_t s)
{
    const int64_t block = default_block_tiles(1) > 0 ? default_block_tiles(1) : pieces;
    for (int64_t first = 0; first < pieces; first += block) {
        const dim3 grid = grid_for(first + block < pieces ? block : pieces - first), threads(kLanes);
        DLION_TRY(write ? launch(membench_kernel<true, kBatch>, grid, threads, lds, s, src, row_stride, rows, dst, first)
                        : launch(membench_kernel<false, kBatch>, grid, threads, lds, s, src, row_stride, rows, dst, first));
    }
    return DLION_OK;
}

// Arguments that every form of the flat fused step shares.
dlion_status check_step(const float *x, const float *m, int64_t m_stride, const void *g, int64_t g_stride,
                        dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, const uint64_t *packed_or_null,
                        int64_t packed_stride, const uint16_t *counts_or_null)
{
    DLION_TRY(check_common(d, N));
    if (!dtype_ok(g_dtype) || !mode_ok(mode) || !x)
        return DLION_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(counts_or_null, 2))
        return DLION_EALIGN;
    DLION_TRY(check_rows(m, m_stride, d, N, 4));
    DLION_TRY(check_rows(g, g_stride, d, N, grad_size(g_dtype)));
    if (packed_or_null)
        DLION_TRY(check_rows(packed_or_null, packed_stride, words_for(d), N, 8));
    return DLION_OK;
}

}  // namespace

extern "C" {

dlion_status dlion_worker_step(float *m, int64_t m_stride, const void *g, int64_t g_stride,
                               dlion_dtype g_dtype, uint64_t *packed, int64_t packed_stride, int64_t d,
                               int32_t N, float beta1, float beta2, void *stream)
{
    DLION_TRY(check_common(d, N));
    if (!dtype_ok(g_dtype))
        return DLION_EINVAL;
    DLION_TRY(check_rows(m, m_stride, d, N, 4));
    DLION_TRY(check_rows(g, g_stride, d, N, grad_size(g_dtype)));
    DLION_TRY(check_rows(packed, packed_stride, words_for(d), N, 8));
    Hyper h = make_hyper(N, DLION_VOTE, beta1, beta2, 0.0f, 0.0f);
    // a tile writes 32 bytes of every packed row, a quarter of a line: with 4 consecutive tiles on one XCD
    // the quarters meet in one L2 and leave it as one line (d = 350 M, N = 32: 76.5 -> 78.5 % of peak; N = 8,
    // d = 124 M: 79.0 -> 79.7 %); the fused step with packed output gains nothing from it
    h.xcd_quads = step_quads(true);
    const FlatAddr a = flat_addr(nullptr, m, m_stride, g, g_stride, d, packed, packed_stride, nullptr);
    return launch_step<false>(a, h, g_dtype, true, false, static_cast<hipStream_t>(stream));
}

dlion_status dlion_aggregate(const uint64_t *packed, int64_t packed_stride, int64_t d, int32_t N,
                             uint16_t *counts, void *stream)
{
    DLION_TRY(check_common(d, N));
    DLION_TRY(check_rows(packed, packed_stride, words_for(d), N, 8));
    if (!counts)
        return DLION_EINVAL;
    if (!aligned_to(counts, 2))
        return DLION_EALIGN;
    Hyper h = make_hyper(N, DLION_VOTE, 0.0f, 0.0f, 0.0f, 0.0f);
    h.stream_counts = counts_exceed_cache(d);
    const FlatAddr a = flat_addr(nullptr, nullptr, 0, nullptr, 0, d, const_cast<uint64_t *>(packed),
                                 packed_stride, counts);
    if (use_group(N, kGroupCounts))
        return launch_group(a, h, false, true, nullptr, static_cast<hipStream_t>(stream));
    if (use_sliced(N))
        return launch_sliced(a, h, false, true, static_cast<hipStream_t>(stream));
    return launch_aggregate(a, h, false, true, static_cast<hipStream_t>(stream));
}

dlion_status dlion_apply(float *x, const uint16_t *counts, int64_t d, int32_t N, dlion_mode mode, float lr,
                         float lambda, void *stream)
{
    DLION_TRY(check_common(d, N));
    if (!mode_ok(mode) || !x || !counts)
        return DLION_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(counts, 2))
        return DLION_EALIGN;
    const Hyper h = make_hyper(N, mode, 0.0f, 0.0f, lr, lambda);
    const FlatAddr a = flat_addr(x, nullptr, 0, nullptr, 0, d, nullptr, 0, const_cast<uint16_t *>(counts));
    return launch_apply(a, h, static_cast<hipStream_t>(stream));
}

dlion_status dlion_aggregate_apply(float *x, const uint64_t *packed, int64_t packed_stride, int64_t d,
                                   int32_t N, dlion_mode mode, float lr, float lambda,
                                   uint16_t *counts_or_null, void *stream)
{
    DLION_TRY(check_common(d, N));
    if (!mode_ok(mode) || !x)
        return DLION_EINVAL;
    DLION_TRY(check_rows(packed, packed_stride, words_for(d), N, 8));
    if (!aligned_to(x, 4) || !aligned_to(counts_or_null, 2))
        return DLION_EALIGN;
    Hyper h = make_hyper(N, mode, 0.0f, 0.0f, lr, lambda);
    h.stream_counts = counts_or_null ? counts_exceed_cache(d) : 0;
    const FlatAddr a = flat_addr(x, nullptr, 0, nullptr, 0, d, const_cast<uint64_t *>(packed), packed_stride,
                                 counts_or_null);
    if (use_group(N, kGroupApply))
        return launch_group(a, h, true, counts_or_null != nullptr, nullptr, static_cast<hipStream_t>(stream));
    if (use_sliced(N))
        return launch_sliced(a, h, true, counts_or_null != nullptr, static_cast<hipStream_t>(stream));
    return launch_aggregate(a, h, true, counts_or_null != nullptr, static_cast<hipStream_t>(stream));
}

int64_t dlion_step_mt_workspace_bytes(int64_t total_tiles, int32_t N)
{
    if (total_tiles <= 0 || total_tiles > kMaxTiles || N < 1 || N > DLION_MAX_WORKERS)
        return 0;
    const int passes = default_passes(N, total_tiles);
    if (passes <= 1)
        return 0;
    int64_t block = default_block_tiles(passes);
    if (block <= 0 || block > total_tiles)
        block = total_tiles;
    return block * ws_bytes_per_tile(workspace_carry(N, passes), passes);
}

int64_t dlion_step_workspace_bytes(int64_t d, int32_t N)
{
    return d > 0 ? dlion_step_mt_workspace_bytes(tiles_for(d), N) : 0;
}

dlion_status dlion_step(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                        dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, float beta1, float beta2,
                        float lr, float lambda, uint64_t *packed_or_null, int64_t packed_stride,
                        uint16_t *counts_or_null, void *stream)
{
    return dlion_step_ws(x, m, m_stride, g, g_stride, g_dtype, d, N, mode, beta1, beta2, lr, lambda, packed_or_null,
                         packed_stride, counts_or_null, nullptr, 0, stream);
}

dlion_status dlion_step_ws(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                           dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, float beta1, float beta2,
                           float lr, float lambda, uint64_t *packed_or_null, int64_t packed_stride,
                           uint16_t *counts_or_null, void *workspace_or_null, int64_t workspace_bytes,
                           void *stream)
{
    DLION_TRY(check_step(x, m, m_stride, g, g_stride, g_dtype, d, N, mode, packed_or_null, packed_stride,
                         counts_or_null));
    if (workspace_bytes < 0 || (workspace_or_null == nullptr && workspace_bytes != 0))
        return DLION_EINVAL;
    if (!aligned_to(workspace_or_null, 16))
        return DLION_EALIGN;
    Hyper h = make_hyper(N, mode, beta1, beta2, lr, lambda);
    h.stream_counts = counts_or_null ? counts_exceed_cache(d) : 0;
    h.xcd_quads = step_quads(rows_split_lines(m, m_stride, 4, N) || rows_split_lines(g, g_stride, grad_size(g_dtype), N));
    const FlatAddr a = flat_addr(x, m, m_stride, g, g_stride, d, packed_or_null, packed_stride, counts_or_null);
    Workspace ws;
    ws.base = workspace_or_null;
    ws.bytes = workspace_bytes;
    return launch_step<true>(a, h, g_dtype, packed_or_null != nullptr, counts_or_null != nullptr,
                             static_cast<hipStream_t>(stream), ws);
}

dlion_status dlion_noalloc_init(void)
{
    void *p;
    return static_scratch(&p);
}

dlion_status dlion_step_noalloc(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                                dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, float beta1,
                                float beta2, float lr, float lambda, uint64_t *packed_or_null,
                                int64_t packed_stride, uint16_t *counts_or_null, void *stream)
{
    DLION_TRY(check_step(x, m, m_stride, g, g_stride, g_dtype, d, N, mode, packed_or_null, packed_stride,
                         counts_or_null));
    // what the hand-over of this step needs for its smallest block must fit the static scratch
    const int passes = default_passes(N, tiles_for(d));
    if (passes > 1) {
        const int64_t per_tile = ws_bytes_per_tile(workspace_carry(N, passes), passes);
        int64_t least = default_block_tiles(passes);
        if (least <= 0 || least > tiles_for(d))
            least = tiles_for(d);
        if (least > kPassMinBlockTiles)
            least = kPassMinBlockTiles;
        if (least * per_tile > (int64_t)DLION_NOALLOC_SCRATCH_BYTES)
            return DLION_EUNSUPPORTED;
    }
    void *scratch = nullptr;
    DLION_TRY(static_scratch(&scratch));
    return dlion_step_ws(x, m, m_stride, g, g_stride, g_dtype, d, N, mode, beta1, beta2, lr, lambda, packed_or_null,
                         packed_stride, counts_or_null, scratch, (int64_t)DLION_NOALLOC_SCRATCH_BYTES, stream);
}

// ----------------------------------------------------------------------- tensor lists
dlion_status dlion_mt_layout(dlion_seg *segs_host, int32_t K, int64_t *total_words, int64_t *total_tiles)
{
    if (!segs_host || K < 1)
        return DLION_EINVAL;
    int64_t words = 0, tiles = 0;
    for (int32_t k = 0; k < K; ++k) {
        if (segs_host[k].numel <= 0)
            return DLION_EINVAL;
        segs_host[k].word_begin = words;
        segs_host[k].tile_begin = tiles;
        words += words_for(segs_host[k].numel);
        tiles += tiles_for(segs_host[k].numel);
    }
    if (tiles > kMaxTiles)
        return DLION_EUNSUPPORTED;
    if (total_words)
        *total_words = words;
    if (total_tiles)
        *total_tiles = tiles;
    return DLION_OK;
}

dlion_status dlion_worker_step_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                                  dlion_dtype g_dtype, uint64_t *packed, int64_t packed_stride, int32_t N,
                                  float beta1, float beta2, void *stream)
{
    if (!dtype_ok(g_dtype))
        return DLION_EINVAL;
    int64_t words, tiles;
    bool split;
    DLION_TRY(check_segs(segs_host, segs_dev, K, N, kNeedM | kNeedG, g_dtype, &words, &tiles, &split));
    DLION_TRY(check_rows(packed, packed_stride, words, N, 8));
    Hyper h = make_hyper(N, DLION_VOTE, beta1, beta2, 0.0f, 0.0f);
    h.xcd_quads = step_quads(split);
    const SegAddr a = seg_addr(segs_dev, K, tiles, packed, packed_stride, nullptr);
    return launch_step<false>(a, h, g_dtype, true, false, static_cast<hipStream_t>(stream));
}

dlion_status dlion_aggregate_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                                const uint64_t *packed, int64_t packed_stride, int32_t N, uint16_t *counts,
                                void *stream)
{
    int64_t words, tiles;
    DLION_TRY(check_segs(segs_host, segs_dev, K, N, 0, DLION_F32, &words, &tiles));
    DLION_TRY(check_rows(packed, packed_stride, words, N, 8));
    if (!counts)
        return DLION_EINVAL;
    if (!aligned_to(counts, 2))
        return DLION_EALIGN;
    Hyper h = make_hyper(N, DLION_VOTE, 0.0f, 0.0f, 0.0f, 0.0f);
    h.stream_counts = counts_exceed_cache(64 * words);
    if (use_group(N, kGroupCounts) || use_sliced(N)) {
        // packed words and counts of a tensor list are laid out by word, the padding bits of every
        // tensor's last word are zero: counting is the flat problem over 64 * words coordinates
        const FlatAddr f = flat_addr(nullptr, nullptr, 0, nullptr, 0, 64 * words, const_cast<uint64_t *>(packed),
                                     packed_stride, counts);
        if (use_group(N, kGroupCounts))
            return launch_group(f, h, false, true, nullptr, static_cast<hipStream_t>(stream));
        return launch_sliced(f, h, false, true, static_cast<hipStream_t>(stream));
    }
    const SegAddr a = seg_addr(segs_dev, K, tiles, const_cast<uint64_t *>(packed), packed_stride, counts);
    return launch_aggregate(a, h, false, true, static_cast<hipStream_t>(stream));
}

dlion_status dlion_apply_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                            const uint16_t *counts, int32_t N, dlion_mode mode, float lr, float lambda,
                            void *stream)
{
    if (!mode_ok(mode) || !counts)
        return DLION_EINVAL;
    if (!aligned_to(counts, 2))
        return DLION_EALIGN;
    int64_t words, tiles;
    DLION_TRY(check_segs(segs_host, segs_dev, K, N, kNeedX, DLION_F32, &words, &tiles));
    const Hyper h = make_hyper(N, mode, 0.0f, 0.0f, lr, lambda);
    const SegAddr a = seg_addr(segs_dev, K, tiles, nullptr, 0, const_cast<uint16_t *>(counts));
    return launch_apply(a, h, static_cast<hipStream_t>(stream));
}

dlion_status dlion_aggregate_apply_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                                      const uint64_t *packed, int64_t packed_stride, int32_t N,
                                      dlion_mode mode, float lr, float lambda, uint16_t *counts_or_null,
                                      void *stream)
{
    if (!mode_ok(mode))
        return DLION_EINVAL;
    if (!aligned_to(counts_or_null, 2))
        return DLION_EALIGN;
    int64_t words, tiles;
    DLION_TRY(check_segs(segs_host, segs_dev, K, N, kNeedX, DLION_F32, &words, &tiles));
    DLION_TRY(check_rows(packed, packed_stride, words, N, 8));
    Hyper h = make_hyper(N, mode, 0.0f, 0.0f, lr, lambda);
    h.stream_counts = counts_or_null ? counts_exceed_cache(64 * words) : 0;
    if (use_group(N, kGroupApply)) {
        // words and counts of the list are one flat layout; only x is found through the table
        const FlatAddr f = flat_addr(nullptr, nullptr, 0, nullptr, 0, 64 * words, const_cast<uint64_t *>(packed),
                                     packed_stride, counts_or_null);
        return launch_group(f, h, true, counts_or_null != nullptr, nullptr, static_cast<hipStream_t>(stream),
                            SegTab{segs_dev, K});
    }
    const SegAddr a = seg_addr(segs_dev, K, tiles, const_cast<uint64_t *>(packed), packed_stride, counts_or_null);
    return launch_aggregate(a, h, true, counts_or_null != nullptr, static_cast<hipStream_t>(stream));
}

dlion_status dlion_step_mt(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                           dlion_dtype g_dtype, int32_t N, dlion_mode mode, float beta1, float beta2, float lr,
                           float lambda, uint64_t *packed_or_null, int64_t packed_stride,
                           uint16_t *counts_or_null, void *stream)
{
    return dlion_step_mt_ws(segs_host, segs_dev, K, g_dtype, N, mode, beta1, beta2, lr, lambda, packed_or_null,
                            packed_stride, counts_or_null, nullptr, 0, stream);
}

dlion_status dlion_step_mt_ws(const dlion_seg *segs_host, const dlion_seg *segs_dev, int32_t K,
                              dlion_dtype g_dtype, int32_t N, dlion_mode mode, float beta1, float beta2,
                              float lr, float lambda, uint64_t *packed_or_null, int64_t packed_stride,
                              uint16_t *counts_or_null, void *workspace_or_null, int64_t workspace_bytes,
                              void *stream)
{
    if (!dtype_ok(g_dtype) || !mode_ok(mode))
        return DLION_EINVAL;
    if (workspace_bytes < 0 || (workspace_or_null == nullptr && workspace_bytes != 0))
        return DLION_EINVAL;
    if (!aligned_to(counts_or_null, 2) || !aligned_to(workspace_or_null, 16))
        return DLION_EALIGN;
    int64_t words, tiles;
    bool split;
    DLION_TRY(check_segs(segs_host, segs_dev, K, N, kNeedX | kNeedM | kNeedG, g_dtype, &words, &tiles, &split));
    if (packed_or_null)
        DLION_TRY(check_rows(packed_or_null, packed_stride, words, N, 8));
    Hyper h = make_hyper(N, mode, beta1, beta2, lr, lambda);
    h.stream_counts = counts_or_null ? counts_exceed_cache(64 * words) : 0;
    h.xcd_quads = step_quads(split);
    const SegAddr a = seg_addr(segs_dev, K, tiles, packed_or_null, packed_stride, counts_or_null);
    Workspace ws;
    ws.base = workspace_or_null;
    ws.bytes = workspace_bytes;
    return launch_step<true>(a, h, g_dtype, packed_or_null != nullptr, counts_or_null != nullptr,
                             static_cast<hipStream_t>(stream), ws);
}

// ----------------------------------------------------------------------- wider rows
int32_t dlion_delta_planes(int32_t N, dlion_mode mode)
{
    if (N < 1 || N > DLION_MAX_WORKERS || !mode_ok(mode))
        return 0;
    return delta_planes(N, mode);
}

dlion_status dlion_aggregate_encode(const uint64_t *packed, int64_t packed_stride, int64_t d, int32_t N,
                                    dlion_mode mode, uint64_t *delta, int64_t delta_stride, void *stream)
{
    DLION_TRY(check_common(d, N));
    if (!mode_ok(mode))
        return DLION_EINVAL;
    DLION_TRY(check_rows(packed, packed_stride, words_for(d), N, 8));
    const int32_t planes = delta_planes(N, mode);
    DLION_TRY(check_rows(delta, delta_stride, words_for(d), planes, 8));
    Hyper h = make_hyper(N, mode, 0.0f, 0.0f, 0.0f, 0.0f);
    // planes too large to stay cached until they are applied: streaming stores (same field as for counts)
    h.stream_counts = (int64_t)delta_planes(N, mode) * words_for(d) * 8 > ((int64_t)192 << 20);
    const FlatAddr a = flat_addr(nullptr, nullptr, 0, nullptr, 0, d, const_cast<uint64_t *>(packed),
                                 packed_stride, nullptr);
    const DeltaOut out = {delta, delta_stride, planes};
    if (use_group(N, kGroupEncode))
        return launch_group(a, h, false, false, &out, static_cast<hipStream_t>(stream));
    return launch_encode(a, h, out, static_cast<hipStream_t>(stream));
}

dlion_status dlion_apply_encoded(float *x, const uint64_t *delta, int64_t delta_stride, int64_t d, int32_t N,
                                 dlion_mode mode, float lr, float lambda, void *stream)
{
    DLION_TRY(check_common(d, N));
    if (!mode_ok(mode) || !x)
        return DLION_EINVAL;
    if (!aligned_to(x, 4))
        return DLION_EALIGN;
    const int32_t planes = delta_planes(N, mode);
    DLION_TRY(check_rows(delta, delta_stride, words_for(d), planes, 8));
    const Hyper h = make_hyper(N, mode, 0.0f, 0.0f, lr, lambda);
    const FlatAddr a = flat_addr(x, nullptr, 0, nullptr, 0, d, nullptr, 0, nullptr);
    const DeltaOut in = {const_cast<uint64_t *>(delta), delta_stride, planes};
    hipStream_t s = static_cast<hipStream_t>(stream);
    // resident waves per compute unit, capped like the fused step's (a wave has 4 KB of x and a
    // line of every plane in flight): d = 1.3 G, vote (2 planes) 11 / 12 / 14 / 16 waves 84.8 / 84.5 /
    // 82.5 / 81.4 % of peak, average at N = 8 (4 planes) 82.6 / 84.5 / 83.2 / 80.3 %; d = 350 M,
    // average at N = 32 (6 planes) 79.2 / 83.3 / 86.2 / 86.6 %
    const int env_k = tuning().apply_blocks;
    const size_t lds = lds_reservation(env_k >= 0 ? env_k : (planes <= 5 ? 12 : 16));
    return launch_in_blocks(a, (d + kLineCoords - 1) / kLineCoords, kLineSubs, 8 + planes / 8 + 1, false,
                            [&](const FlatAddr &b, int64_t n) {
        const dim3 grid = grid_for(n), block(kLanes);
        if (planes <= 2)
            return launch(apply_encoded_kernel<2>, grid, block, lds, s, b, h, in);
        if (planes <= 5)
            return launch(apply_encoded_kernel<5>, grid, block, lds, s, b, h, in);
        if (planes <= 9)
            return launch(apply_encoded_kernel<9>, grid, block, lds, s, b, h, in);
        return launch(apply_encoded_kernel<16>, grid, block, lds, s, b, h, in);
    });
}

dlion_status dlion_worker_step_pw(float *m, int64_t m_stride, const void *g, int64_t g_stride,
                                  dlion_dtype g_dtype, uint64_t *packed, int64_t packed_stride, int64_t d,
                                  int32_t N, const float *beta1, const float *beta2, void *stream)
{
    DLION_TRY(check_common(d, N));
    if (!dtype_ok(g_dtype) || !beta1 || !beta2)
        return DLION_EINVAL;
    if (!aligned_to(beta1, 4) || !aligned_to(beta2, 4))
        return DLION_EALIGN;
    DLION_TRY(check_rows(m, m_stride, d, N, 4));
    DLION_TRY(check_rows(g, g_stride, d, N, grad_size(g_dtype)));
    DLION_TRY(check_rows(packed, packed_stride, words_for(d), N, 8));
    Hyper h = make_hyper(N, DLION_VOTE, 0.0f, 0.0f, 0.0f, 0.0f);
    h.beta1_pw = beta1;
    h.beta2_pw = beta2;
    // a tile writes 32 bytes of every packed row, a quarter of a line: with 4 consecutive tiles on one XCD
    // the quarters meet in one L2 and leave it as one line (d = 350 M, N = 32: 76.5 -> 78.5 % of peak; N = 8,
    // d = 124 M: 79.0 -> 79.7 %); the fused step with packed output gains nothing from it
    h.xcd_quads = step_quads(true);
    const FlatAddr a = flat_addr(nullptr, m, m_stride, g, g_stride, d, packed, packed_stride, nullptr);
    return launch_step<false>(a, h, g_dtype, true, false, static_cast<hipStream_t>(stream));
}

dlion_status dlion_step_pw_ws(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                              dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, const float *beta1,
                              const float *beta2, float lr, float lambda, uint64_t *packed_or_null,
                              int64_t packed_stride, uint16_t *counts_or_null, void *workspace_or_null,
                              int64_t workspace_bytes, void *stream)
{
    DLION_TRY(check_step(x, m, m_stride, g, g_stride, g_dtype, d, N, mode, packed_or_null, packed_stride,
                         counts_or_null));
    if (!beta1 || !beta2 || workspace_bytes < 0 || (workspace_or_null == nullptr && workspace_bytes != 0))
        return DLION_EINVAL;
    if (!aligned_to(beta1, 4) || !aligned_to(beta2, 4) || !aligned_to(workspace_or_null, 16))
        return DLION_EALIGN;
    Hyper h = make_hyper(N, mode, 0.0f, 0.0f, lr, lambda);
    h.beta1_pw = beta1;
    h.beta2_pw = beta2;
    h.stream_counts = counts_or_null ? counts_exceed_cache(d) : 0;
    h.xcd_quads = step_quads(rows_split_lines(m, m_stride, 4, N) || rows_split_lines(g, g_stride, grad_size(g_dtype), N));
    const FlatAddr a = flat_addr(x, m, m_stride, g, g_stride, d, packed_or_null, packed_stride, counts_or_null);
    Workspace ws;
    ws.base = workspace_or_null;
    ws.bytes = workspace_bytes;
    return launch_step<true>(a, h, g_dtype, packed_or_null != nullptr, counts_or_null != nullptr,
                             static_cast<hipStream_t>(stream), ws);
}

dlion_status dlion_step_pw(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                           dlion_dtype g_dtype, int64_t d, int32_t N, dlion_mode mode, const float *beta1,
                           const float *beta2, float lr, float lambda, uint64_t *packed_or_null,
                           int64_t packed_stride, uint16_t *counts_or_null, void *stream)
{
    return dlion_step_pw_ws(x, m, m_stride, g, g_stride, g_dtype, d, N, mode, beta1, beta2, lr, lambda,
                            packed_or_null, packed_stride, counts_or_null, nullptr, 0, stream);
}

dlion_status dlion_global_lion_step(float *x, float *m, int64_t m_stride, const void *g, int64_t g_stride,
                                    dlion_dtype g_dtype, int64_t d, int32_t N, float beta1, float beta2,
                                    float lr, float lambda, uint64_t *sign_bits_or_null, void *stream)
{
    DLION_TRY(check_common(d, N));
    if (!dtype_ok(g_dtype) || !x)
        return DLION_EINVAL;
    if (!aligned_to(x, 4) || !aligned_to(sign_bits_or_null, 8))
        return DLION_EALIGN;
    DLION_TRY(check_rows(m, m_stride, d, N, 4));
    DLION_TRY(check_rows(g, g_stride, d, N, grad_size(g_dtype)));
    const Hyper h = make_hyper(N, DLION_VOTE, beta1, beta2, lr, lambda);
    const FlatAddr a = flat_addr(x, m, m_stride, g, g_stride, d, nullptr, 0, nullptr);
    if (g_dtype == DLION_BF16)
        return launch_global_lion_unroll<uint16_t>(a, h, sign_bits_or_null, static_cast<hipStream_t>(stream));
    return launch_global_lion_unroll<float>(a, h, sign_bits_or_null, static_cast<hipStream_t>(stream));
}

dlion_status dlion_membench(const void *src, int64_t src_row_stride_bytes, int32_t rows, void *dst,
                            int64_t bytes_per_row, int32_t write, int32_t loads_in_flight, int32_t waves_per_cu,
                            void *stream)
{
    if (!src || !dst || rows < 1 || bytes_per_row <= 0 || bytes_per_row % 1024 != 0 || waves_per_cu < 0 ||
        waves_per_cu > 64 || (rows > 1 && src_row_stride_bytes < bytes_per_row))
        return DLION_EINVAL;
    if (loads_in_flight != 1 && loads_in_flight != 2 && loads_in_flight != 4 && loads_in_flight != 8 &&
        loads_in_flight != 16)
        return DLION_EINVAL;
    if (!aligned_to(src, 16) || !aligned_to(dst, 16) || src_row_stride_bytes % 16 != 0)
        return DLION_EALIGN;
    const int64_t pieces = bytes_per_row / 1024;
    if (pieces > kMaxTiles)
        return DLION_EUNSUPPORTED;
    const size_t lds = lds_reservation(waves_per_cu);
    const u32x4 *s4 = static_cast<const u32x4 *>(src);
    u32x4 *d4 = static_cast<u32x4 *>(dst);
    const int64_t stride = src_row_stride_bytes / 16;
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (loads_in_flight) {
    case 1: return launch_membench<1>(s4, stride, rows, d4, pieces, write != 0, lds, s);
    case 2: return launch_membench<2>(s4, stride, rows, d4, pieces, write != 0, lds, s);
    case 4: return launch_membench<4>(s4, stride, rows, d4, pieces, write != 0, lds, s);
    case 8: return launch_membench<8>(s4, stride, rows, d4, pieces, write != 0, lds, s);
    default: return launch_membench<16>(s4, stride, rows, d4, pieces, write != 0, lds, s);
    }
}

const char *dlion_status_str(dlion_status s)
{
    switch (s) {
    case DLION_OK: return "ok";
    case DLION_EINVAL: return "invalid argument (size, stride, count, enum or null pointer)";
    case DLION_EALIGN: return "pointer not aligned to its element type";
    case DLION_ELAUNCH: return "HIP runtime refused the kernel launch";
    case DLION_EUNSUPPORTED: return "request outside what this build supports";
    }
    return "unknown status";
}

int dlion_version(void) { return 210; }

void dlion_tuning_defaults(dlion_tuning *t)
{
    if (t) {
        const dlion_tuning d = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1};
        *t = d;
    }
}

dlion_status dlion_set_tuning(const dlion_tuning *t)
{
    dlion_tuning v;
    dlion_tuning_defaults(&v);
    if (t)
        v = *t;
    const bool unroll_ok = v.unroll == -1 || v.unroll == 1 || v.unroll == 2 || v.unroll == 4 || v.unroll == 8;
    const bool waves_ok = v.sliced_waves == -1 || v.sliced_waves == 1 || v.sliced_waves == 8 || v.sliced_waves == 16;
    if (!unroll_ok || !waves_ok || v.blocks_per_cu < -1 || v.blocks_per_cu > 64 || v.blocks_per_cu_pass < -1 || v.blocks_per_cu_pass > 64 || v.pass_workers < -1 ||
        v.step_quads < -1 || v.step_quads > 1 || v.sliced_min_workers < -1 || v.apply_blocks < -1 ||
        v.apply_blocks > 64 || v.block_tiles < -1 || v.block_tiles > kMaxTiles || v.group_blocks < -1 ||
        v.group_blocks > 64 || v.group_max_workers < -1 || v.group_max_workers > kGroupMaxWorkers)
        return DLION_EINVAL;
    g_tuning = v;
    return DLION_OK;
}

void dlion_get_tuning(dlion_tuning *t)
{
    if (t)
        *t = g_tuning;
}

}  // extern "C"
