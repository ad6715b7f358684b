// Device code of the Distributed Lion sweep for gfx950 (CDNA4, 64-wide wavefronts).
//
// Work decomposition: the coordinate range of a tensor is cut into TILES of 256
// coordinates (= 4 packed uint64 words).  One wavefront owns one tile and walks
// over all N workers for it, so the vote count of a coordinate never leaves
// the lane that owns the coordinate and no inter-wave communication, atomics
// or barriers are needed anywhere on the worker/fused path.
//
// Two code paths per tile:
//   * vector path (full tile): lane l owns coordinates 4l..4l+3 and moves them
//     with one 128-bit access per stream, whatever the alignment of the rows.
//     Its four sign bits form a nibble; the nibbles of the 16 lanes of a DPP
//     row are OR-combined into one canonical packed word per row.
//   * guarded path (ragged last tile of a tensor): lane l owns coordinates
//     64k+l, k=0..3, moved with dword accesses; a 64-lane ballot of the sign
//     predicate is already a canonical packed word.
//
// All fp32 arithmetic goes through __fmul_rn/__fadd_rn/__fsub_rn so that no
// multiply-add is ever fused (Section 3.2's expressions, each operation rounded
// on its own); the sign is taken as !(c < 0), i.e. 0 votes +1.
//
// Kernels, in file order: step_kernel (worker step / fused step, also the launches of a step that
// is cut by workers), aggregate_kernel (server side, per-nibble), aggregate_sliced_kernel and
// aggregate_encode_kernel (server side and down-link message, bit-sliced, many workers),
// apply_encoded_kernel (worker side of the down-link), aggregate_group_kernel (server side and
// message, few workers), global_lion_kernel, apply_kernel, membench_kernel (memory-rate probe).
// Loads of m, g, x and the packed rows are streaming (non-temporal) loads throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "../../include/dlion.h"

namespace dlion {

constexpr int kLanes = 64;                    // one-wave workgroups everywhere on the worker/fused path
constexpr int kVec = 4;                       // coordinates per lane on the vector path
constexpr int kTile = kLanes * kVec;          // 256 coordinates = 4 packed words: what one wave owns
constexpr int kWordsPerTile = kTile / 64;


typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

// How the votes of the workers that earlier launches handled reach the current one, when a step
// over many workers runs as several launches over a few workers each (Hyper::carry).
enum Carry : int32_t {
    kCarryNone = 0,
    kCarryCounts = 1,    // running count in the caller's counts array (uint16, indexed by coordinate)
    kCarryRunning = 2,   // running count in the workspace, private to the lane: 4 x uint16 per lane and tile
    kCarryNibbles = 3,   // one plane per launch in the workspace: the lane's 4 partial counts (each <= 15)
                         // are the nibbles of one uint16; the last launch adds the planes up
};

struct Hyper {
    float beta1, omb1, beta2, omb2;  // omb = 1.0f - beta, formed on the host in fp32
    float lr, lambda;
    float inv_n;      // 1/N when N is a power of two (then S*inv_n == S/N exactly), else 0
    int32_t N;
    int32_t mode;     // dlion_mode
    int32_t stream_counts;   // counts array too large to stay cached: write it with streaming stores
    // The worker/fused kernels walk workers [worker_begin, worker_end) of the N: a step over many
    // workers may be run as several launches over a few workers each.
    int32_t worker_begin, worker_end;
    int32_t carry;       // Carry
    int32_t carry_in;    // counts / running: 1 = start from the stored count; nibbles: planes to add up
    int32_t carry_out;   // running: 1 = store the count; nibbles: 1 + plane to write; else 0
    int32_t xcd_quads;   // worker/fused kernels: 4 consecutive tiles per XCD (quad_tile_index)
    const float *beta1_pw;   // per-worker coefficients (device arrays of N floats), or null:
    const float *beta2_pw;   // then beta1/beta2 above are shared by all workers
};

// Coefficients of one worker (footnote of Algorithm 1: each worker may set its own).
struct Coef {
    float beta1, omb1, beta2, omb2;
};

// One flat problem as a tile sees it.
struct Problem {
    float *x;
    float *m;
    const void *g;
    int64_t m_stride, g_stride;
    int64_t numel;
    uint64_t *packed;       // worker 0, first word of this tensor (may be null)
    int64_t packed_stride;
    uint16_t *counts;       // first count of this tensor (may be null)
    int64_t counts_end;     // counts[0..counts_end) may be written: numel (flat buffer) or
                            // numel rounded up to a whole word (tensor list)
};

// Where a tile's votes wait between the launches of one step (kCarryRunning, kCarryNibbles): the
// launches of one block of tiles [first_tile, total_tiles) share ws, laid out by tile within the
// block and by lane within the tile, so that every lane reads back exactly what it wrote.
struct CarrySlot {
    uint16_t *tile;     // this tile's first element (null when the step has no workspace carry)
    int64_t plane;      // kCarryNibbles: uint16 elements from one plane to the next
};

// ---------------------------------------------------------------- addressing
// Flat buffer: the problem travels in the kernel arguments.
struct FlatAddr {
    Problem p;
    int64_t total_tiles;
    int64_t first_tile;    // worker/fused kernels: the launch covers tiles [first_tile, total_tiles)
    uint16_t *ws;          // workspace carry of this block of tiles, or null
    int64_t ws_plane;
    __device__ int64_t resolve(int64_t tile, Problem &out) const
    {
        out = p;
        return tile;
    }
};

// Tensor list: a device table of segments ordered by tile_begin; the owner of a
// tile is found by bisection (all operands are wave-uniform, so these are
// scalar loads).
struct SegAddr {
    const dlion_seg *segs;
    int32_t K;
    int64_t total_tiles;
    int64_t first_tile;
    uint16_t *ws;
    int64_t ws_plane;
    uint64_t *packed;
    int64_t packed_stride;
    uint16_t *counts;
    __device__ int64_t resolve(int64_t tile, Problem &out) const
    {
        int32_t lo = 0, hi = K - 1;
        while (lo < hi) {
            int32_t mid = (lo + hi + 1) >> 1;
            if (segs[mid].tile_begin <= tile)
                lo = mid;
            else
                hi = mid - 1;
        }
        const dlion_seg s = segs[lo];
        out.x = s.x;
        out.m = s.m;
        out.g = s.g;
        out.m_stride = s.m_stride;
        out.g_stride = s.g_stride;
        out.numel = s.numel;
        out.packed = packed ? packed + s.word_begin : nullptr;
        out.packed_stride = packed_stride;
        out.counts = counts ? counts + 64 * s.word_begin : nullptr;
        out.counts_end = ((s.numel + 63) >> 6) << 6;
        return tile - s.tile_begin;
    }
};

// uint16 elements of workspace one tile takes per plane (kCarryNibbles) / in all (kCarryRunning)
constexpr int kNibbleCarryPerTile = kLanes;
constexpr int kRunningCarryPerTile = kLanes * kVec;

template <class Addr> __device__ __forceinline__ CarrySlot carry_slot(const Addr &addr, int64_t tile, const Hyper &h)
{
    CarrySlot c = {nullptr, addr.ws_plane};
    if (addr.ws)
        c.tile = addr.ws + (tile - addr.first_tile) * (h.carry == kCarryRunning ? kRunningCarryPerTile : kNibbleCarryPerTile);
    return c;
}

// Tile numbering for kernels that READ bit-packed rows.  A tile needs only 32 bytes of each
// packed row, a quarter of a 128-byte line, and every XCD has its own L2: with the plain
// numbering the four quarters of a line are fetched by four different L2s, i.e. up to four
// times from memory.  Within every group of 32 workgroups, XCD x (workgroups b with b % 8 == x)
// takes tiles 4x..4x+3 instead, so the line is fetched once.  Groups stay in order, so the
// window of addresses in flight remains compact.
__device__ __forceinline__ int64_t quad_tile_index()
{
    uint32_t block = blockIdx.x;
    const uint32_t group = block & ~31u;
    if (group + 32 <= gridDim.x)                           // whole group of 32 exists
        block = group + ((block & 7u) << 2) + ((block >> 3) & 3u);
    return block;
}

// Plain numbering: workgroup b owns tile b.  Workgroups are handed to the 8 XCDs round-robin
// (workgroup b runs on XCD b % 8), so all XCDs work inside the same narrow window of addresses.
// That is what DRAM page locality wants: renumbering so that every XCD walks its own contiguous
// eighth of the tiles costs 15 % of the bandwidth.  Grouping 4 consecutive tiles per XCD
// (quad_tile_index) costs the fused step 1-5 %; the worker step, whose tiles each write a quarter
// line of every packed row, gains 1-2 % from it and is launched that way.
__device__ __forceinline__ int64_t wave_tile_index()
{
    return blockIdx.x;     // uniform across the wavefront: everything derived from it stays scalar
}

// Cache policy of the small per-coordinate arrays.  x is touched once per step: streaming
// (non-temporal) accesses, +14 % on the apply kernel.  counts written by one call are read by
// the next (aggregate -> apply) and up to ~250 MB of them stay in the memory-side cache, so
// they use ordinary accesses unless the array is too large for that (h.stream_counts).
// Streaming stores carry the device-scope bit next to the streaming hint: with one L2 per XCD a
// device-scope store is written through to memory at once instead of waiting in the L2 for its
// eviction, and the steadier stream of writes is worth 1 % of the HBM peak to the fused step
// (N = 32, d = 350 M: 79.7 -> 80.6 %; the hint alone 79.7 %, the bit alone 79.4 %), 2-3 % to
// dlion_apply_encoded.  The compiler has no way to ask for the bit on a wide store, hence the
// instructions are written out; the memory clobber keeps them in program order.  A store of more
// than 64 bits must not be followed at once by a vector-ALU write to the registers that hold its
// data (the hardware reads them a cycle late); the compiler pads its own stores for that but
// cannot see into this one, hence the two idle cycles after it.
#define DLION_STREAM_STORE_POLICY "sc1 nt"
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void stream_store_b128(u32x4 v, void *p)
{
    asm volatile("global_store_dwordx4 %0, %1, off " DLION_STREAM_STORE_POLICY "\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store_b64(u32x2 v, void *p)
{
    asm volatile("global_store_dwordx2 %0, %1, off " DLION_STREAM_STORE_POLICY : : "v"(p), "v"(v) : "memory");
}

template <typename T> __device__ __forceinline__ T stream_load(const T *p)
{
    return __builtin_nontemporal_load(p);
}
// Four consecutive elements of a row, of x or of the counts, in one access.  The callers'
// arrays are only promised the alignment of their element type (rows of a contiguous [N, d]
// array with d not a multiple of 4 start anywhere), so the vector types used for the access
// carry the element's alignment: the compiler still selects one 128-bit (or 64-bit)
// instruction, which global memory on this target accepts at any alignment, and assumes
// nothing about the low address bits.  These are plain functions, not templates, because a
// deduced template argument would drop the alignment of the typedef.
typedef f32x4 f32x4_e __attribute__((aligned(4)));
typedef u32x2 bf16x4_e __attribute__((aligned(2)));
typedef u16x4 u16x4_e __attribute__((aligned(2)));

__device__ __forceinline__ f32x4 row_load4(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4_e *>(p));
}
__device__ __forceinline__ u32x2 row_load4(const uint16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const bf16x4_e *>(p));
}
__device__ __forceinline__ void row_store4(f32x4 v, float *p)
{
    stream_store_b128(__builtin_bit_cast(u32x4, v), p);
}
__device__ __forceinline__ f32x4 x_load4(const float *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const f32x4_e *>(p));
}
__device__ __forceinline__ void x_store4(f32x4 v, float *p)
{
    stream_store_b128(__builtin_bit_cast(u32x4, v), p);
}
__device__ __forceinline__ u16x4 counts_load4(const uint16_t *p)
{
    return *reinterpret_cast<const u16x4_e *>(p);
}
// Streaming or ordinary store, chosen at run time.
__device__ __forceinline__ void counts_store4(u16x4 v, uint16_t *p, bool stream)
{
    if (stream)
        stream_store_b64(__builtin_bit_cast(u32x2, v), p);
    else
        *reinterpret_cast<u16x4_e *>(p) = v;
}
#define COUNTS_STORE4(v, p) counts_store4(v, p, h.stream_counts)

// eight counts in one 128-bit store
typedef u32x4 u16x8_e __attribute__((aligned(2)));
__device__ __forceinline__ void counts_store8(u32x4 v, uint16_t *p, bool stream)
{
    if (stream)
        stream_store_b128(v, p);
    else
        *reinterpret_cast<u16x8_e *>(p) = v;
}

// ---------------------------------------------------------------- gradients
template <typename GT> struct Grad;
template <> struct Grad<float> {
    static constexpr int kVecBytes = 16;
    static __device__ __forceinline__ f32x4 load4(const void *g, int64_t idx)
    {
        return row_load4(static_cast<const float *>(g) + idx);
    }
    static __device__ __forceinline__ float load1(const void *g, int64_t idx)
    {
        return stream_load(static_cast<const float *>(g) + idx);
    }
};
template <> struct Grad<uint16_t> {   // bf16 bit patterns; widening to fp32 is exact
    static constexpr int kVecBytes = 8;
    static __device__ __forceinline__ f32x4 load4(const void *g, int64_t idx)
    {
        const u32x2 raw = row_load4(static_cast<const uint16_t *>(g) + idx);
        f32x4 r;
        r.x = __uint_as_float(raw.x << 16);
        r.y = __uint_as_float(raw.x & 0xFFFF0000u);
        r.z = __uint_as_float(raw.y << 16);
        r.w = __uint_as_float(raw.y & 0xFFFF0000u);
        return r;
    }
    static __device__ __forceinline__ float load1(const void *g, int64_t idx)
    {
        const uint16_t raw = stream_load(static_cast<const uint16_t *>(g) + idx);
        return __uint_as_float(static_cast<uint32_t>(raw) << 16);
    }
};

// ---------------------------------------------------------------- arithmetic
// Worker update for one coordinate (Section 3.2, first display).  Returns the
// vote (true = +1) and replaces m by the new momentum.
__device__ __forceinline__ float lion_blend(float &m, float g, const Coef &k)
{
    const float c = __fadd_rn(__fmul_rn(k.beta1, m), __fmul_rn(k.omb1, g));
    m = __fadd_rn(__fmul_rn(k.beta2, m), __fmul_rn(k.omb2, g));
    return c;
}
__device__ __forceinline__ bool lion_worker(float &m, float g, const Coef &k)
{
    return !(lion_blend(m, g, k) < 0.0f);
}

// i is uniform across the wave: scalar loads
__device__ __forceinline__ Coef worker_coef(const Hyper &h, int i)
{
    Coef k = {h.beta1, h.omb1, h.beta2, h.omb2};
    if (h.beta1_pw) {
        k.beta1 = h.beta1_pw[i];
        k.omb1 = __fsub_rn(1.0f, k.beta1);
        k.beta2 = h.beta2_pw[i];
        k.omb2 = __fsub_rn(1.0f, k.beta2);
    }
    return k;
}

// Aggregation of p votes for +1 out of N (Section 3.2, second display).
__device__ __forceinline__ float aggregate_votes(uint32_t p, const Hyper &h)
{
    const int32_t S = 2 * static_cast<int32_t>(p) - h.N;
    if (h.mode == DLION_AVG) {
        if (h.inv_n != 0.0f)
            return __fmul_rn(static_cast<float>(S), h.inv_n);   // exact: N is a power of two
        return static_cast<float>(S) / static_cast<float>(h.N);
    }
    return static_cast<float>((S > 0) - (S < 0));
}

// Weight update (Section 3.2, third display).
__device__ __forceinline__ float lion_apply(float x, float Delta, const Hyper &h)
{
    return __fsub_rn(x, __fmul_rn(h.lr, __fadd_rn(Delta, __fmul_rn(h.lambda, x))));
}

// ---------------------------------------------------------------- bit packing
// DPP lane exchange within a row of 16 lanes.
template <int kCtrl> __device__ __forceinline__ uint32_t dpp(uint32_t v)
{
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kCtrl, 0xF, 0xF, true));
}

// Each lane holds the 4 sign bits of coordinates 4l..4l+3 of a tile.  Lanes
// 16w..16w+15 together hold word w of the tile; OR them together so that the
// first lane of each row ends up with the canonical 64-bit word.
__device__ __forceinline__ uint64_t row_gather_nibbles(uint32_t nibble, int lane)
{
    uint32_t v = nibble << ((lane & 7) * 4);          // position inside this half's dword
    v |= dpp<0xB1>(v);                                // quad_perm [1,0,3,2]: lane ^ 1
    v |= dpp<0x4E>(v);                                // quad_perm [2,3,0,1]: lane ^ 2
    v |= dpp<0x141>(v);                               // row_half_mirror: other quad of the half
    const uint32_t other = dpp<0x128>(v);             // row_ror 8: the other half of the row
    // lanes 0..7 of a row hold the low dword, lanes 8..15 the high dword
    return (lane & 8) ? ((static_cast<uint64_t>(v) << 32) | other)
                      : ((static_cast<uint64_t>(other) << 32) | v);
}

// ---------------------------------------------------------------- fused / worker tile
// kApply : read x, aggregate, write x (fused step); else worker step only.
// kPacked: write packed words.   kCounts: write counts.
// Vector path over one full tile: the loads of kUnroll workers are issued back to back before
// any arithmetic.
template <typename GT, int kUnroll, bool kApply, bool kPacked, bool kCounts>
__device__ __forceinline__ void step_tile_vector(const Problem &p, int64_t t, int lane, const Hyper &h,
                                                 const CarrySlot &carry, uint64_t *stage)
{
    const int64_t j0 = t * kTile + lane * kVec;
    // packed words wait in `stage` (LDS, private to the wave) until kPackWorkers workers are done
    constexpr int kPackWorkers = kLanes / kWordsPerTile;
    int staged = 0;                                        // uniform
    auto flush_packed = [&](int i_next) {                  // workers [i_next - staged, i_next)
        if (!kPacked)
            return;
        // the wave's own LDS writes, then its reads: program order is enough inside one wave,
        // the fences only keep the compiler from moving the accesses
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int worker = lane / kWordsPerTile;           // lane -> (worker, word of the tile)
        const int word = lane % kWordsPerTile;
        if (worker < staged) {
            const uint64_t v = stage[lane];
            p.packed[(int64_t)(i_next - staged + worker) * p.packed_stride + t * kWordsPerTile + word] = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        staged = 0;
    };
    f32x4 xv;
    if (kApply)
        xv = x_load4(p.x + j0);
    // votes of the workers that earlier launches of this step handled (all branches uniform)
    uint32_t cnt0 = 0, cnt1 = 0, cnt2 = 0, cnt3 = 0;
    if (h.carry == kCarryCounts) {
        if (h.carry_in) {
            const u16x4 c = counts_load4(p.counts + j0);
            cnt0 = c.x, cnt1 = c.y, cnt2 = c.z, cnt3 = c.w;
        }
    } else if (h.carry == kCarryRunning) {
        if (h.carry_in) {
            const u16x4 c = *reinterpret_cast<const u16x4 *>(carry.tile + lane * kVec);
            cnt0 = c.x, cnt1 = c.y, cnt2 = c.z, cnt3 = c.w;
        }
    } else if (h.carry == kCarryNibbles) {
        for (int pl = 0; pl < h.carry_in; ++pl) {
            const uint32_t v = carry.tile[pl * carry.plane + lane];
            cnt0 += v & 15u;
            cnt1 += (v >> 4) & 15u;
            cnt2 += (v >> 8) & 15u;
            cnt3 += v >> 12;
        }
    }
    const int N = h.N, i_begin = h.worker_begin, i_end = h.worker_end;

    // Per-worker coefficients: lane l keeps those of worker (i & ~63) + l, fetched once per block
    // of 64 workers (outer loop below); each worker's pair is then broadcast from its lane, so
    // that no memory access sits between a worker's loads and its arithmetic.
    uint32_t pw_beta1 = 0, pw_beta2 = 0;
    auto coef_of = [&](int i) {
        Coef k = {h.beta1, h.omb1, h.beta2, h.omb2};
        if (h.beta1_pw) {                               // uniform
            k.beta1 = __uint_as_float(__builtin_amdgcn_readlane(pw_beta1, i & 63));
            k.omb1 = __fsub_rn(1.0f, k.beta1);
            k.beta2 = __uint_as_float(__builtin_amdgcn_readlane(pw_beta2, i & 63));
            k.omb2 = __fsub_rn(1.0f, k.beta2);
        }
        return k;
    };

    auto one_worker = [&](int i, f32x4 mv, f32x4 gv) {
        const Coef k = coef_of(i);
        float m0 = mv.x, m1 = mv.y, m2 = mv.z, m3 = mv.w;
        const bool b0 = lion_worker(m0, gv.x, k);
        const bool b1 = lion_worker(m1, gv.y, k);
        const bool b2 = lion_worker(m2, gv.z, k);
        const bool b3 = lion_worker(m3, gv.w, k);
        mv.x = m0;
        mv.y = m1;
        mv.z = m2;
        mv.w = m3;
        row_store4(mv, p.m + (int64_t)i * p.m_stride + j0);
        cnt0 += b0;
        cnt1 += b1;
        cnt2 += b2;
        cnt3 += b3;
        if (kPacked) {
            const uint32_t nib = (b0 ? 1u : 0u) | (b1 ? 2u : 0u) | (b2 ? 4u : 0u) | (b3 ? 8u : 0u);
            const uint64_t word = row_gather_nibbles(nib, lane);
            // staged in LDS: one store instruction then writes the words of up to kPackWorkers
            // workers (a store by 4 scattered lanes per worker costs the kernel 10 % of its time)
            if ((lane & 15) == 0)
                stage[staged * kWordsPerTile + (lane >> 4)] = word;
            if (++staged == kPackWorkers)
                flush_packed(i + 1);
        }
    };

    for (int c0 = i_begin; c0 < i_end;) {
        // workers [c0, c1): the rest of c0's block of 64
        const int c1 = min(i_end, (c0 | 63) + 1);
        if (h.beta1_pw) {                                   // uniform
            const int w = (c0 & ~63) + lane;
            pw_beta1 = w < N ? __float_as_uint(h.beta1_pw[w]) : 0u;
            pw_beta2 = w < N ? __float_as_uint(h.beta2_pw[w]) : 0u;
        }
        int i = c0;
        for (; i + kUnroll <= c1; i += kUnroll) {
            f32x4 mv[kUnroll], gv[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                mv[u] = row_load4(p.m + (int64_t)(i + u) * p.m_stride + j0);
                gv[u] = Grad<GT>::load4(p.g, (int64_t)(i + u) * p.g_stride + j0);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                one_worker(i + u, mv[u], gv[u]);
        }
        for (; i < c1; ++i) {
            const f32x4 mv = row_load4(p.m + (int64_t)i * p.m_stride + j0);
            const f32x4 gv = Grad<GT>::load4(p.g, (int64_t)i * p.g_stride + j0);
            one_worker(i, mv, gv);
        }
        c0 = c1;
    }
    if (kPacked && staged > 0)
        flush_packed(i_end);

    if (kApply) {
        xv.x = lion_apply(xv.x, aggregate_votes(cnt0, h), h);
        xv.y = lion_apply(xv.y, aggregate_votes(cnt1, h), h);
        xv.z = lion_apply(xv.z, aggregate_votes(cnt2, h), h);
        xv.w = lion_apply(xv.w, aggregate_votes(cnt3, h), h);
        x_store4(xv, p.x + j0);
    }
    if (kCounts) {
        u16x4 c;
        c.x = static_cast<uint16_t>(cnt0);
        c.y = static_cast<uint16_t>(cnt1);
        c.z = static_cast<uint16_t>(cnt2);
        c.w = static_cast<uint16_t>(cnt3);
        COUNTS_STORE4(c, p.counts + j0);
    }
    // hand the votes on to the next launch of this step: read back soon, so ordinary stores
    if (h.carry_out) {                                      // uniform
        if (h.carry == kCarryRunning) {
            u16x4 c;
            c.x = static_cast<uint16_t>(cnt0);
            c.y = static_cast<uint16_t>(cnt1);
            c.z = static_cast<uint16_t>(cnt2);
            c.w = static_cast<uint16_t>(cnt3);
            *reinterpret_cast<u16x4 *>(carry.tile + lane * kVec) = c;
        } else if (h.carry == kCarryNibbles) {
            carry.tile[(h.carry_out - 1) * carry.plane + lane] =
                static_cast<uint16_t>(cnt0 | (cnt1 << 4) | (cnt2 << 8) | (cnt3 << 12));
        }
    }
}

// Guarded path (ragged last tile of a tensor): lane l owns coordinates 64k+l, k = 0..3, of the
// tile; every access checks j < numel; a 64-lane ballot is already a canonical packed word.  The
// lane's four counts travel in the 16-bit fields of one 64-bit register.
template <typename GT, bool kApply, bool kPacked, bool kCounts>
__device__ __forceinline__ void step_tile_guarded(const Problem &p, int64_t t, int lane, const Hyper &h,
                                                  const CarrySlot &carry)
{
    const int64_t W = (p.numel + 63) >> 6;
    uint64_t cnt = 0;                                       // field k = votes for coordinate 64k + lane
    if (h.carry == kCarryRunning) {
        if (h.carry_in) {
            const u16x4 c = *reinterpret_cast<const u16x4 *>(carry.tile + lane * kVec);
            cnt = static_cast<uint64_t>(c.x) | (static_cast<uint64_t>(c.y) << 16) |
                  (static_cast<uint64_t>(c.z) << 32) | (static_cast<uint64_t>(c.w) << 48);
        }
    } else if (h.carry == kCarryNibbles) {
        for (int pl = 0; pl < h.carry_in; ++pl) {
            const uint64_t v = carry.tile[pl * carry.plane + lane];
            cnt += (v & 15u) | (((v >> 4) & 15u) << 16) | (((v >> 8) & 15u) << 32) | ((v >> 12) << 48);
        }
    }
#pragma unroll 1
    for (int k = 0; k < kWordsPerTile; ++k) {
        const int64_t w = t * kWordsPerTile + k;
        if (w >= W)
            break;                                   // uniform: whole wave leaves together
        const int64_t j = w * 64 + lane;
        const bool valid = j < p.numel;
        uint32_t c = static_cast<uint32_t>(cnt >> (16 * k)) & 0xFFFFu;
        if (h.carry == kCarryCounts && h.carry_in && valid)
            c = p.counts[j];
        for (int i = h.worker_begin; i < h.worker_end; ++i) {
            bool plus = false;
            if (valid) {
                float *mp = p.m + (int64_t)i * p.m_stride + j;
                float mv = *mp;
                const float gv = Grad<GT>::load1(p.g, (int64_t)i * p.g_stride + j);
                plus = lion_worker(mv, gv, worker_coef(h, i));
                *mp = mv;
            }
            c += plus;
            if (kPacked) {
                const uint64_t word = __ballot(plus);   // invalid lanes contribute 0: tail bits zero
                if (lane == 0)
                    p.packed[(int64_t)i * p.packed_stride + w] = word;
            }
        }
        if (kApply && valid)
            p.x[j] = lion_apply(p.x[j], aggregate_votes(c, h), h);
        if (kCounts && j < p.counts_end)
            p.counts[j] = static_cast<uint16_t>(c);     // 0 past numel (tensor-list padding)
        cnt = (cnt & ~(static_cast<uint64_t>(0xFFFFu) << (16 * k))) | (static_cast<uint64_t>(c) << (16 * k));
    }
    if (h.carry_out) {
        if (h.carry == kCarryRunning) {
            u16x4 c;
            c.x = static_cast<uint16_t>(cnt);
            c.y = static_cast<uint16_t>(cnt >> 16);
            c.z = static_cast<uint16_t>(cnt >> 32);
            c.w = static_cast<uint16_t>(cnt >> 48);
            *reinterpret_cast<u16x4 *>(carry.tile + lane * kVec) = c;
        } else if (h.carry == kCarryNibbles) {
            carry.tile[(h.carry_out - 1) * carry.plane + lane] = static_cast<uint16_t>(
                (cnt & 15u) | (((cnt >> 16) & 15u) << 4) | (((cnt >> 32) & 15u) << 8) | (((cnt >> 48) & 15u) << 12));
        }
    }
}

template <typename GT, int kUnroll, bool kApply, bool kPacked, bool kCounts, class Addr>
__global__ __launch_bounds__(kLanes) void step_kernel(Addr addr, Hyper h)
{
    const int64_t tile = addr.first_tile + (h.xcd_quads ? quad_tile_index() : wave_tile_index());
    if (tile >= addr.total_tiles)
        return;
    const int lane = threadIdx.x;
    // dynamic LDS: reserved to cap the resident waves; its first 512 bytes stage packed words
    extern __shared__ uint64_t step_lds[];
    Problem p;
    const int64_t t = addr.resolve(tile, p);              // tile within its tensor
    const CarrySlot carry = carry_slot(addr, tile, h);
    if ((t + 1) * kTile <= p.numel)
        step_tile_vector<GT, kUnroll, kApply, kPacked, kCounts>(p, t, lane, h, carry, step_lds);
    else if (t * kTile < p.numel)                         // ragged end of a tensor
        step_tile_guarded<GT, kApply, kPacked, kCounts>(p, t, lane, h, carry);
}

// A nibble's four bits, one per byte (bit 0 of each byte): 24-bit multiply, full rate.
__device__ __forceinline__ uint32_t nibble_to_bytes(uint32_t nib)
{
    return __umul24(nib, 0x00204081u) & 0x01010101u;
}

// ---------------------------------------------------------------- server side from packed words
// Vector path: lane l owns coordinates 4l..4l+3 = nibble (l & 15) of word (l >> 4) of the
// tile.  Votes are accumulated four at a time in the bytes of one register (a nibble is
// spread to one bit per byte by a multiply), flushed to 32-bit counters every 255 workers.
template <bool kApply, bool kCounts>
__device__ __forceinline__ void agg_subtile_vector(const Problem &p, int64_t t, int lane, const Hyper &h)
{
    const uint32_t *half = reinterpret_cast<const uint32_t *>(p.packed + t * kWordsPerTile + (lane >> 4)) +
                           ((lane >> 3) & 1);
    const int shift = (lane & 7) * 4;
    const int64_t stride32 = p.packed_stride * 2;
    uint32_t cnt0 = 0, cnt1 = 0, cnt2 = 0, cnt3 = 0;
    const int N = h.N;
    for (int base = 0; base < N; base += 255) {
        const int end = (N - base < 255) ? N : base + 255;
        uint32_t acc = 0;
        int i = base;
        for (; i + 8 <= end; i += 8) {
            uint32_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                v[u] = stream_load(half + (int64_t)(i + u) * stride32);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                acc += nibble_to_bytes((v[u] >> shift) & 0xFu);
        }
        for (; i < end; ++i)
            acc += nibble_to_bytes((stream_load(half + (int64_t)i * stride32) >> shift) & 0xFu);
        cnt0 += acc & 0xFFu;
        cnt1 += (acc >> 8) & 0xFFu;
        cnt2 += (acc >> 16) & 0xFFu;
        cnt3 += acc >> 24;
    }
    const int64_t j0 = t * kTile + lane * kVec;
    if (kApply) {
        f32x4 xv = x_load4(p.x + j0);
        xv.x = lion_apply(xv.x, aggregate_votes(cnt0, h), h);
        xv.y = lion_apply(xv.y, aggregate_votes(cnt1, h), h);
        xv.z = lion_apply(xv.z, aggregate_votes(cnt2, h), h);
        xv.w = lion_apply(xv.w, aggregate_votes(cnt3, h), h);
        x_store4(xv, p.x + j0);
    }
    if (kCounts) {
        u16x4 c;
        c.x = static_cast<uint16_t>(cnt0);
        c.y = static_cast<uint16_t>(cnt1);
        c.z = static_cast<uint16_t>(cnt2);
        c.w = static_cast<uint16_t>(cnt3);
        COUNTS_STORE4(c, p.counts + j0);
    }
}

// Guarded path: lane l owns bit l of word 4t+k.
template <bool kApply, bool kCounts>
__device__ __forceinline__ void agg_subtile_guarded(const Problem &p, int64_t t, int lane, const Hyper &h)
{
    const int64_t W = (p.numel + 63) >> 6;
#pragma unroll 1
    for (int k = 0; k < kWordsPerTile; ++k) {
        const int64_t w = t * kWordsPerTile + k;
        if (w >= W)
            break;
        const int64_t j = w * 64 + lane;
        const bool valid = j < p.numel;
        uint32_t cnt = 0;
        for (int i = 0; i < h.N; ++i) {
            const uint64_t word = p.packed[(int64_t)i * p.packed_stride + w];
            cnt += static_cast<uint32_t>((word >> lane) & 1u);
        }
        if (!valid)
            cnt = 0;                      // tail bits are zero by contract; do not rely on it
        if (kApply && valid)
            p.x[j] = lion_apply(p.x[j], aggregate_votes(cnt, h), h);
        if (kCounts && j < p.counts_end)
            p.counts[j] = static_cast<uint16_t>(cnt);
    }
}

template <bool kApply, bool kCounts, class Addr>
__global__ __launch_bounds__(kLanes) void aggregate_kernel(Addr addr, Hyper h)
{
    const int64_t tile = addr.first_tile + quad_tile_index();
    if (tile >= addr.total_tiles)
        return;
    const int lane = threadIdx.x;
    Problem p;
    const int64_t t = addr.resolve(tile, p);
    if ((t + 1) * kTile <= p.numel)
        agg_subtile_vector<kApply, kCounts>(p, t, lane, h);
    else if (t * kTile < p.numel)
        agg_subtile_guarded<kApply, kCounts>(p, t, lane, h);
}

// ---------------------------------------------------------------- server side, bit-sliced
// Bit-sliced ("vertical") counting.  One wave owns kSlicedWords consecutive packed words;
// lane l reads kWpl consecutive words of every stream (1 KB contiguous per load instruction)
// and adds the N words into kPlanes bit-planes with carry-save adders: after the loop, bit c
// of plane b of a word is bit b of the vote count of that word's coordinate c.  About one
// bitwise operation per 32 coordinates and input word replaces 32 extract-and-add steps.  The planes
// are then staged through LDS so that the lanes can switch from "kWpl words each" to "eight
// consecutive coordinates each" (counts) or "four consecutive coordinates each" (x) and write
// with 128-bit accesses.
constexpr int kWpl = 2;                                // consecutive words of each stream a lane reads
constexpr int kSlices = 2 * kWpl;                      // 32-bit slices a lane carries
constexpr int kSlicedWords = kLanes * kWpl;            // words per wave
constexpr int kSlicedCoords = kSlicedWords * 64;

typedef u32x4 words2_e __attribute__((aligned(8)));

// two consecutive packed words (only promised the alignment of one) in one 128-bit access
__device__ __forceinline__ u32x4 packed_load2(const uint64_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const words2_e *>(p));
}

// carry-save adder on 32 independent bit positions: a + b + c = 2*carry + sum.  gfx950 has a
// three-input boolean instruction, so each output is one operation (truth tables: majority
// 0xE8, parity 0x96; both symmetric in their operands).
__device__ __forceinline__ void csa(uint32_t &carry, uint32_t &sum, uint32_t a, uint32_t b, uint32_t c)
{
    carry = __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);
    sum = __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

// Planes of one lane: v[b][q] = bits b of the counts of the 32 coordinates of slice q.
template <int kPlanes> struct Planes {
    uint32_t v[kPlanes][kSlices];
};

// Counting loop shared by the kernels below: adds the N words of every stream into `out`.
// w0 = first word of the wave; kWaves > 1: a barrier per batch of 16 streams (lockstep).
template <int kPlanes, int kWaves>
__device__ __forceinline__ void sliced_count(const Problem &p, int N, int64_t w0, int64_t W, int lane,
                                             Planes<kPlanes> &out)
{
    static_assert(kPlanes >= 5 && kPlanes <= 16, "planes");
    static_assert(kWpl == 2, "a lane reads its two words of a row as one 128-bit load");
    // rows whose loads a wave has outstanding at once: one-wave workgroups, 16 or so to a compute unit,
    // want two (32 KB per compute unit) unless the rows are few (N < 32: four, for fewer round trips); the
    // 8 or 16 waves of a lockstep workgroup four
    constexpr int kSlicedInFlight = (kWaves == 1 && kPlanes > 5) ? 2 : 4;
    const int64_t wl0 = w0 + (int64_t)lane * kWpl;              // first word of the lane
    // whole group inside the word range: full-width loads, no per-lane guards
    const bool fast = w0 + kSlicedWords <= W;

    uint32_t ones[kSlices], twos[kSlices], fours[kSlices], eights[kSlices];
    uint32_t hi[kPlanes - 4][kSlices];                          // planes 4.. (sixteens and up)
#pragma unroll
    for (int q = 0; q < kSlices; ++q) {
        ones[q] = twos[q] = fours[q] = eights[q] = 0;
#pragma unroll
        for (int b = 0; b < kPlanes - 4; ++b)
            hi[b][q] = 0;
    }

    // Tree over the weight-2 carries of 8 pairs of words, then a ripple into the upper planes.
    auto add_pairs = [&](uint32_t (&t)[8][kSlices]) {
#pragma unroll
        for (int q = 0; q < kSlices; ++q) {
            uint32_t f0, f1, f2, f3, e0, e1, s16;
            csa(f0, twos[q], twos[q], t[0][q], t[1][q]);
            csa(f1, twos[q], twos[q], t[2][q], t[3][q]);
            csa(f2, twos[q], twos[q], t[4][q], t[5][q]);
            csa(f3, twos[q], twos[q], t[6][q], t[7][q]);
            csa(e0, fours[q], fours[q], f0, f1);
            csa(e1, fours[q], fours[q], f2, f3);
            csa(s16, eights[q], eights[q], e0, e1);
            // ripple the weight-16 carry into the upper planes
#pragma unroll
            for (int b = 0; b < kPlanes - 4; ++b) {
                const uint32_t c = hi[b][q] & s16;
                hi[b][q] ^= s16;
                s16 = c;
            }
        }
    };
    // adds one batch of 16 words per slice
    auto add_batch = [&](const uint32_t (&v)[16][kSlices]) {
        uint32_t t[8][kSlices];
#pragma unroll
        for (int k = 0; k < 8; ++k)
#pragma unroll
            for (int q = 0; q < kSlices; ++q)
                csa(t[k][q], ones[q], ones[q], v[2 * k][q], v[2 * k + 1][q]);
        add_pairs(t);
    };
    // One batch of 16 rows starting at row i, full-width loads, kSlicedInFlight rows at a time:
    // the memory system gives the most with 24-32 KB of loads outstanding per compute unit, which
    // 16 waves reach with two 1 KB loads each (all 16 rows of a batch at once: 256 KB, and 6 % less
    // bandwidth).  The running sums pass through an empty asm statement after every group, so
    // that the compiler can neither issue the next group's loads early nor postpone the adds.
    // guard_rows: rows past N count as zeros.
    auto count_rows = [&](int i, auto guard_rows) {
        // the row base is uniform; each lane adds a small unsigned byte offset
        const uint32_t lane_bytes = static_cast<uint32_t>(lane) * (8u * kWpl);
        uint32_t t[8][kSlices];
#pragma unroll
        for (int k0 = 0; k0 < 16; k0 += kSlicedInFlight) {
            uint32_t v[kSlicedInFlight][kSlices];
#pragma unroll
            for (int k = 0; k < kSlicedInFlight; ++k) {
#pragma unroll
                for (int q = 0; q < kSlices; ++q)
                    v[k][q] = 0;
                if (!decltype(guard_rows)::value || i + k0 + k < N) {        // uniform
                    const char *row = reinterpret_cast<const char *>(p.packed + (int64_t)(i + k0 + k) * p.packed_stride + w0);
                    const u32x4 r = packed_load2(reinterpret_cast<const uint64_t *>(row + lane_bytes));
                    v[k][0] = r.x;
                    v[k][1] = r.y;
                    v[k][2] = r.z;
                    v[k][3] = r.w;
                }
            }
#pragma unroll
            for (int k = 0; k < kSlicedInFlight; k += 2)
#pragma unroll
                for (int q = 0; q < kSlices; ++q)
                    csa(t[(k0 + k) / 2][q], ones[q], ones[q], v[k][q], v[k + 1][q]);
#pragma unroll
            for (int q = 0; q < kSlices; ++q)
                asm volatile("" : "+v"(ones[q]) : : "memory");
        }
        add_pairs(t);
    };
    if (fast) {
        int i = 0;
        for (; i + 16 <= N; i += 16) {
            count_rows(i, std::false_type());
            if (kWaves > 1)
                __builtin_amdgcn_s_barrier();
        }
        if (i < N) {
            count_rows(i, std::true_type());
            if (kWaves > 1)
                __builtin_amdgcn_s_barrier();
        }
    } else {
        // ragged end of the word range: per-lane guards (same number of batches, hence of barriers)
        for (int i = 0; i < N; i += 16) {
            uint32_t v[16][kSlices];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
#pragma unroll
                for (int q = 0; q < kWpl; ++q) {
                    uint64_t word = 0;
                    if (i + k < N && wl0 + q < W)
                        word = stream_load(p.packed + (int64_t)(i + k) * p.packed_stride + wl0 + q);
                    v[k][2 * q] = static_cast<uint32_t>(word);
                    v[k][2 * q + 1] = static_cast<uint32_t>(word >> 32);
                }
            }
            add_batch(v);
            if (kWaves > 1)
                __builtin_amdgcn_s_barrier();
        }
    }
#pragma unroll
    for (int q = 0; q < kSlices; ++q) {
        out.v[0][q] = ones[q];
        out.v[1][q] = twos[q];
        out.v[2][q] = fours[q];
        out.v[3][q] = eights[q];
#pragma unroll
        for (int b = 0; b < kPlanes - 4; ++b)
            out.v[4 + b][q] = hi[b][q];
    }
}

// Majority vote in the bit-sliced domain: compares the count of every coordinate with
// K = floor(N/2) on all bit positions at once, from the top plane down.  plus = count > K, i.e.
// S > 0; tie = count == K for even N, i.e. S == 0.
template <int kPlanes>
__device__ __forceinline__ void sliced_vote(const Planes<kPlanes> &pl, int N, uint32_t (&plus)[kSlices],
                                            uint32_t (&tie)[kSlices])
{
    const uint32_t K = static_cast<uint32_t>(N) >> 1;
    const uint32_t even = (N & 1) ? 0u : 0xFFFFFFFFu;
#pragma unroll
    for (int q = 0; q < kSlices; ++q) {
        uint32_t gt = 0, eq = 0xFFFFFFFFu;
#pragma unroll
        for (int b = kPlanes - 1; b >= 0; --b) {
            if ((K >> b) & 1u) {
                eq &= pl.v[b][q];
            } else {
                gt |= eq & pl.v[b][q];
                eq &= ~pl.v[b][q];
            }
        }
        plus[q] = gt;
        tie[q] = eq & even;
    }
}

__device__ __forceinline__ float decode_vote(uint32_t plus, uint32_t tie)
{
    return plus ? 1.0f : (tie ? 0.0f : -1.0f);
}

// kWaves waves per workgroup, each with its own word group and its own LDS region.  With more
// than one, the waves walk over the streams in lockstep (a barrier per batch of 16 streams,
// so that the compute unit works inside 16 pages at a time instead of up to N), and they start
// writing their results together: the memory system handles a few large bursts of writes much
// better than a trickle of small ones between reads.  A wave without words terminates at once;
// barriers only wait for waves that are alive, and all of those run the same number of batches.
constexpr int kSlicedLdsPerPlane = kLanes * kSlices;   // dwords per wave and plane

template <int kPlanes, int kWaves, bool kApply, bool kCounts>
__global__ __launch_bounds__(kLanes * kWaves) void aggregate_sliced_kernel(FlatAddr addr, Hyper h)
{
    extern __shared__ uint32_t sliced_lds[];                    // [kWaves][kPlanes][kSlicedLdsPerPlane]
    const Problem &p = addr.p;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t(*lds)[kSlicedLdsPerPlane] =
        reinterpret_cast<uint32_t(*)[kSlicedLdsPerPlane]>(sliced_lds + wave * kPlanes * kSlicedLdsPerPlane);
    const int64_t W = (p.numel + 63) >> 6;
    // first word of the wave (addr.first_tile: the first word group of this launch)
    const int64_t w0 = (addr.first_tile + (int64_t)blockIdx.x * kWaves + wave) * kSlicedWords;
    if (w0 >= W)
        return;
    Planes<kPlanes> pl;
    sliced_count<kPlanes, kWaves>(p, h.N, w0, W, lane, pl);
    // stage: lds[b][2*wl + half] = low / high dword of plane b of word wl of the group
#pragma unroll
    for (int q = 0; q < kSlices; ++q) {
#pragma unroll
        for (int b = 0; b < kPlanes; ++b)
            lds[b][lane * kSlices + q] = pl.v[b][q];
    }
    __syncthreads();

    // counts of the 4 coordinates whose bits sit at [shift, shift+4) of dword `dword` of every plane
    auto unpack4 = [&](int dword, int shift, uint32_t (&cnt)[4]) {
        // byte k of lo / up collects bits 0..7 / 8..15 of the count of coordinate k
        uint32_t lo = 0, up = 0;
#pragma unroll
        for (int b = 0; b < kPlanes; ++b) {
            const uint32_t bytes = nibble_to_bytes((lds[b][dword] >> shift) & 0xFu);
            if (b < 8)
                lo += bytes << b;
            else
                up += bytes << (b - 8);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            cnt[k] = ((lo >> (8 * k)) & 0xFFu) | (kPlanes > 8 ? ((up >> (8 * k)) & 0xFFu) << 8 : 0u);
    };

    if (kCounts) {
        // lane l owns the 8 coordinates of byte l&7 of word 8*s + (l>>3): 16 bytes of counts per
        // lane, 1 KB per store instruction.  Stores of 8 bytes per lane (4 coordinates) reach
        // memory as 32-byte pieces and cost 13 % of the whole pass at N = 256 (6.45 -> 5.71 ms).
        constexpr int kSteps = kSlicedWords / 8;
        auto counts8 = [&](int s, u32x4 &c, uint32_t (&c0)[4], uint32_t (&c1)[4]) {
            const int wl = s * 8 + (lane >> 3);                     // word within the group
            const int dword = 2 * wl + ((lane >> 2) & 1);
            const int shift = (lane & 3) * 8;
            unpack4(dword, shift, c0);
            unpack4(dword, shift + 4, c1);
            c.x = c0[0] | (c0[1] << 16);
            c.y = c0[2] | (c0[3] << 16);
            c.z = c1[0] | (c1[1] << 16);
            c.w = c1[2] | (c1[3] << 16);
        };
        if ((w0 + kSlicedWords) * 64 <= p.numel) {                  // uniform: the whole group is inside
            // all results first, then the stores back to back (and, with several waves, together)
            u32x4 c[kSteps];
#pragma unroll
            for (int s = 0; s < kSteps; ++s) {
                uint32_t c0[4], c1[4];
                counts8(s, c[s], c0, c1);
            }
            if (kWaves > 1)
                __builtin_amdgcn_s_barrier();
            uint16_t *dst = p.counts + w0 * 64 + lane * 8;         // + 512 coordinates per step
            if (h.stream_counts) {
#pragma unroll
                for (int s = 0; s < kSteps; ++s)
                    stream_store_b128(c[s], dst + s * 512);
            } else {
#pragma unroll
                for (int s = 0; s < kSteps; ++s)
                    *reinterpret_cast<u16x8_e *>(dst + s * 512) = c[s];
            }
        } else {
            if (kWaves > 1)
                __builtin_amdgcn_s_barrier();                        // same number of barriers on every path
#pragma unroll 1
            for (int s = 0; s < kSteps; ++s) {
                const int64_t j0 = (w0 + s * 8 + (lane >> 3)) * 64 + (lane & 7) * 8;
                if (j0 >= p.numel)
                    continue;
                u32x4 c;
                uint32_t c0[4], c1[4];
                counts8(s, c, c0, c1);
                if (j0 + 8 <= p.numel) {
                    counts_store8(c, p.counts + j0, h.stream_counts);
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        if (j0 + k < p.numel)
                            p.counts[j0 + k] = static_cast<uint16_t>(c0[k]);
                        if (j0 + 4 + k < p.numel)
                            p.counts[j0 + 4 + k] = static_cast<uint16_t>(c1[k]);
                    }
                }
            }
        }
    }
    if (kApply) {
        // lane l owns coordinates 4*(l&15).. of word 4*s + (l>>4): 16 bytes of x per lane
        constexpr int kSteps = kSlicedWords / kWordsPerTile;        // 32 steps of 256 coordinates
        auto step_coord = [&](int s) { return (w0 + s * kWordsPerTile + (lane >> 4)) * 64 + (lane & 15) * kVec; };
        auto step_delta = [&](int s, float (&Delta)[4]) {
            uint32_t cnt[4];
            unpack4(2 * (s * kWordsPerTile + (lane >> 4)) + ((lane >> 3) & 1), (lane & 7) * 4, cnt);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                Delta[k] = aggregate_votes(cnt[k], h);
        };
        if ((w0 + kSlicedWords) * 64 <= p.numel) {                  // uniform: the whole group is inside
            // kXBatch loads of x in flight per wave.  What this phase costs is its stores: at N = 256,
            // d = 1 G the pass takes 4.60 ms without the x phase, 5.24 ms with its loads only, 5.90 ms
            // with its stores only and 6.89 ms with both (batches of 2 to 16 loads, ordinary instead of
            // streaming accesses or a cheaper decoding of the vote change nothing or lose)
            constexpr int kXBatch = 4;
#pragma unroll 1
            for (int s0 = 0; s0 < kSteps; s0 += kXBatch) {
                f32x4 xv[kXBatch];
#pragma unroll
                for (int u = 0; u < kXBatch; ++u)
                    xv[u] = x_load4(p.x + step_coord(s0 + u));
#pragma unroll
                for (int u = 0; u < kXBatch; ++u) {
                    float Delta[4];
                    step_delta(s0 + u, Delta);
                    xv[u].x = lion_apply(xv[u].x, Delta[0], h);
                    xv[u].y = lion_apply(xv[u].y, Delta[1], h);
                    xv[u].z = lion_apply(xv[u].z, Delta[2], h);
                    xv[u].w = lion_apply(xv[u].w, Delta[3], h);
                    x_store4(xv[u], p.x + step_coord(s0 + u));
                }
            }
        } else {
#pragma unroll 1
            for (int s = 0; s < kSteps; ++s) {
                const int64_t j0 = step_coord(s);
                if (j0 >= p.numel)
                    continue;
                float Delta[4];
                step_delta(s, Delta);
                if (j0 + kVec <= p.numel) {
                    f32x4 xv = x_load4(p.x + j0);
                    xv.x = lion_apply(xv.x, Delta[0], h);
                    xv.y = lion_apply(xv.y, Delta[1], h);
                    xv.z = lion_apply(xv.z, Delta[2], h);
                    xv.w = lion_apply(xv.w, Delta[3], h);
                    x_store4(xv, p.x + j0);
                } else {
#pragma unroll
                    for (int k = 0; k < kVec; ++k)
                        if (j0 + k < p.numel)
                            p.x[j0 + k] = lion_apply(p.x[j0 + k], Delta[k], h);
                }
            }
        }
    }
}

// ---------------------------------------------------------------- server -> worker message
// The aggregated update as bit-planes over the same 64-coordinate words as the workers'
// messages ("Communication Cost" paragraph; Table 1):
//   majority vote: plane 0 "plus" (S > 0) and, for even N only, plane 1 "tie" (S == 0);
//   averaging    : plane b = bit b of the count p, b < bits(N) = ceil(log2(N+1)).
// The counting loop leaves exactly such planes in registers, so the averaged message is
// written straight from them, and the vote needs one bit-sliced comparison against N/2:
// no transposition, no LDS, and 1/8 .. bits(N)/8 bytes written per coordinate instead of 2.
struct DeltaOut {
    uint64_t *planes;      // plane b at planes + b*stride
    int64_t stride;
    int32_t n_planes;      // planes to write: 1 or 2 (vote), bits(N) (average)
};

template <int kPlanes, int kWaves>
__global__ __launch_bounds__(kLanes * kWaves) void aggregate_encode_kernel(FlatAddr addr, Hyper h, DeltaOut out)
{
    const Problem &p = addr.p;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t W = (p.numel + 63) >> 6;
    const int64_t w0 = (addr.first_tile + (int64_t)blockIdx.x * kWaves + wave) * kSlicedWords;
    if (w0 >= W)
        return;
    Planes<kPlanes> pl;
    sliced_count<kPlanes, kWaves>(p, h.N, w0, W, lane, pl);
    if (kWaves > 1)
        __builtin_amdgcn_s_barrier();        // start the write burst together

    uint32_t res[2][kSlices];                // vote: plus (S > 0), tie (S == 0; written only when N is even)
    if (h.mode == DLION_VOTE)
        sliced_vote<kPlanes>(pl, h.N, res[0], res[1]);
    const int64_t wl0 = w0 + (int64_t)lane * kWpl;
    const bool whole = w0 + kSlicedWords <= W;              // uniform: every lane's words exist
#pragma unroll 1
    for (int b = 0; b < out.n_planes; ++b) {
        uint64_t word[kWpl];
#pragma unroll
        for (int q = 0; q < kWpl; ++q) {
            uint32_t lo, up;
            if (h.mode == DLION_VOTE) {
                lo = b == 0 ? res[0][2 * q] : res[1][2 * q];
                up = b == 0 ? res[0][2 * q + 1] : res[1][2 * q + 1];
            } else {
                lo = up = 0;
#pragma unroll
                for (int bb = 0; bb < kPlanes; ++bb) {      // select plane b without indexing registers
                    if (bb == b) {
                        lo = pl.v[bb][2 * q];
                        up = pl.v[bb][2 * q + 1];
                    }
                }
            }
            word[q] = (static_cast<uint64_t>(up) << 32) | lo;
            const int64_t left = p.numel - (wl0 + q) * 64;    // coordinates in this word
            if (left < 64)
                word[q] &= left > 0 ? (static_cast<uint64_t>(1) << left) - 1 : 0;   // bits past d are zero
        }
        uint64_t *dst = out.planes + (int64_t)b * out.stride + wl0;
        if (whole) {
            // both words of the lane in one 128-bit store: 1 KB per instruction
            u32x4 v;
            v.x = static_cast<uint32_t>(word[0]);
            v.y = static_cast<uint32_t>(word[0] >> 32);
            v.z = static_cast<uint32_t>(word[1]);
            v.w = static_cast<uint32_t>(word[1] >> 32);
            if (h.stream_counts) {
                stream_store_b128(v, dst);
            } else {
                *reinterpret_cast<words2_e *>(dst) = v;
            }
        } else {
#pragma unroll
            for (int q = 0; q < kWpl; ++q)
                if (wl0 + q < W)
                    dst[q] = word[q];
        }
    }
}

// Worker side of the down-link: decode the planes and take the step.  Same tiling as the
// per-nibble server kernel: lane l owns coordinates 4l..4l+3 of a 256-coordinate tile, i.e.
// nibble (l & 15) of word (l >> 4); the guarded path gives lane l bit l of one word.
// One wave owns kLineSubs = 4 consecutive sub-tiles = 16 words = one 128-byte line of every
// plane, so that each line is read by exactly one wave (and one L2): lane l loads dword
// (l & 31) of the line, and for sub-tile s takes the dword that holds its nibble from lane
// 8s + (l >> 3) with a lane permute.
constexpr int kLineSubs = 4;
constexpr int kLineCoords = kLineSubs * kTile;   // 1024

template <int kMaxPlanes>
__global__ __launch_bounds__(kLanes) void apply_encoded_kernel(FlatAddr addr, Hyper h, DeltaOut in)
{
    const Problem &p = addr.p;
    const int64_t t = addr.first_tile + blockIdx.x;             // line index (first_tile: first line of this launch)
    const int lane = threadIdx.x;
    const bool full = (t + 1) * kLineCoords <= p.numel;
    if (full) {
        // all planes' loads first (n_planes <= kMaxPlanes; the test is uniform)
        uint32_t raw[kMaxPlanes];
#pragma unroll
        for (int b = 0; b < kMaxPlanes; ++b) {
            const uint32_t *line = reinterpret_cast<const uint32_t *>(in.planes + (int64_t)b * in.stride +
                                                                      t * (kLineSubs * kWordsPerTile));
            raw[b] = b < in.n_planes ? line[lane & 31] : 0u;
        }
        f32x4 xv[kLineSubs];
#pragma unroll
        for (int s = 0; s < kLineSubs; ++s)
            xv[s] = x_load4(p.x + t * kLineCoords + s * kTile + lane * kVec);
        const int shift = (lane & 7) * 4;
#pragma unroll
        for (int s = 0; s < kLineSubs; ++s) {
            const int from = (8 * s + (lane >> 3)) << 2;       // byte address of the source lane
            float Delta[4];
            if (h.mode == DLION_VOTE) {
                const uint32_t plus = (static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from, raw[0])) >> shift) & 0xFu;
                const uint32_t tie = (static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from, raw[kMaxPlanes > 1 ? 1 : 0])) >> shift) & 0xFu;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    Delta[k] = decode_vote((plus >> k) & 1u, in.n_planes > 1 ? (tie >> k) & 1u : 0u);
            } else {
                uint32_t lo = 0, up = 0;
#pragma unroll
                for (int b = 0; b < kMaxPlanes; ++b) {
                    const uint32_t dw = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from, raw[b]));
                    const uint32_t bytes = nibble_to_bytes((dw >> shift) & 0xFu);
                    if (b < 8)
                        lo += bytes << b;
                    else
                        up += bytes << (b - 8);
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    Delta[k] = aggregate_votes(((lo >> (8 * k)) & 0xFFu) | (((up >> (8 * k)) & 0xFFu) << 8), h);
            }
            xv[s].x = lion_apply(xv[s].x, Delta[0], h);
            xv[s].y = lion_apply(xv[s].y, Delta[1], h);
            xv[s].z = lion_apply(xv[s].z, Delta[2], h);
            xv[s].w = lion_apply(xv[s].w, Delta[3], h);
            x_store4(xv[s], p.x + t * kLineCoords + s * kTile + lane * kVec);
        }
        return;
    }
    // ragged end: lane l owns bit l of one word at a time
    const int64_t W = (p.numel + 63) >> 6;
#pragma unroll 1
    for (int k = 0; k < kLineSubs * kWordsPerTile; ++k) {
        const int64_t w = t * (kLineSubs * kWordsPerTile) + k;
        if (w >= W)
            break;
        const int64_t j = w * 64 + lane;
        float Delta;
        if (h.mode == DLION_VOTE) {
            const uint32_t plus = static_cast<uint32_t>((in.planes[w] >> lane) & 1u);
            const uint32_t tie = in.n_planes > 1 ? static_cast<uint32_t>((in.planes[in.stride + w] >> lane) & 1u) : 0u;
            Delta = decode_vote(plus, tie);
        } else {
            uint32_t cnt = 0;
            for (int b = 0; b < in.n_planes; ++b)
                cnt |= static_cast<uint32_t>((in.planes[(int64_t)b * in.stride + w] >> lane) & 1u) << b;
            Delta = aggregate_votes(cnt, h);
        }
        if (j < p.numel)
            p.x[j] = lion_apply(p.x[j], Delta, h);
    }
}

// ---------------------------------------------------------------- server side, few workers
// Server side for few workers (N <= 120), flat buffers.  With few rows a coordinate's x (8 bytes)
// or counts (2 bytes) weigh as much as its votes (N/8 bytes), and a wave of the bit-sliced kernel
// above, which owns 8192 coordinates alone, walks through some 16 dependent round trips to memory
// (N/4 for the rows, 8 for x).  Here the eight waves of a workgroup share those 8192 coordinates
// (128 words): wave w reads rows w, w + 8, ... over the whole span (1 KB per row and load: shorter
// pieces of a row, e.g. one 128-byte line per wave, reach half the bandwidth however they are
// loaded) and adds them up bit-sliced; the partial planes meet in LDS; then wave w owns
// coordinates 1024w .. 1024w + 1023 of the span, one 128-byte line of every plane, as in
// apply_encoded_kernel: lanes 0..31 add the partial planes of waves 0..3 for one dword of the line
// each, lanes 32..63 those of waves 4..7, and one exchange across the halves completes the
// count.  Every wave then has three or four round trips, and a workgroup's loads are in flight
// together.  Ragged ends are handled by guards (words past the end read as zero, outputs past the
// end are not written), so that every wave of a workgroup reaches the one barrier.
constexpr int kGroupWaves = 8;
constexpr int kGroupWords = 128;                        // words per workgroup
constexpr int kGroupCoords = kGroupWords * 64;          // 8192
constexpr int kLineWords = kLineSubs * kWordsPerTile;   // 16 words = 1024 coordinates per wave

// bit-sliced a + b on kIn planes -> kIn + 1 planes
template <int kIn>
__device__ __forceinline__ void add_planes(const uint32_t (&a)[kIn], const uint32_t (&b)[kIn], uint32_t (&sum)[kIn + 1])
{
    uint32_t carry = 0;
#pragma unroll
    for (int k = 0; k < kIn; ++k)
        csa(carry, sum[k], a[k], b[k], carry);
    sum[kIn] = carry;
}

// counts of four coordinates, one per byte: nibble `shift / 4` of the dword that lane `from / 4` holds
template <int kPlanes> __device__ __forceinline__ uint32_t line_counts4(const uint32_t (&pl)[kPlanes], int from, int shift)
{
    uint32_t bytes = 0;
#pragma unroll
    for (int b = 0; b < kPlanes; ++b) {
        const uint32_t dw = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from, pl[b]));
        bytes += nibble_to_bytes((dw >> shift) & 0xFu) << b;
    }
    return bytes;
}

// Tensor list behind a flat view: packed words and counts of a list are one flat layout by word, only x
// lives in the tensors.  The kernel then runs on the flat problem of 64 * total_words coordinates (x
// null) and finds x through the table: a line of 1024 coordinates that lies in the whole words of one
// tensor (a scalar search, the common case) is updated as in the flat case, any other line coordinate
// by coordinate, every lane searching the owner of its word.
struct SegTab {
    const dlion_seg *segs;     // device table ordered by word_begin, or null (flat buffer)
    int32_t K;
};

__device__ __forceinline__ int32_t seg_of_word(const SegTab &tab, int64_t word)
{
    int32_t lo = 0, hi = tab.K - 1;
    while (lo < hi) {
        const int32_t mid = (lo + hi + 1) >> 1;
        if (tab.segs[mid].word_begin <= word)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo;
}

// kAcc = planes a wave needs for its own rows, ceil(N / 8) < 2^kAcc; the count has kAcc + 3 planes.
// kInFlight = rows whose loads a wave has outstanding at once (1 KB each).  kSeg: x through `tab`.
template <int kAcc, int kInFlight, bool kApply, bool kCounts, bool kEncode, bool kSeg>
__global__ __launch_bounds__(kLanes * kGroupWaves) void aggregate_group_kernel(FlatAddr addr, Hyper h, DeltaOut out,
                                                                               SegTab tab)
{
    static_assert(!kSeg || (kApply && !kEncode), "the table is only needed to find x");
    static_assert(kAcc >= 1 && kAcc <= 4, "planes");           // counts up to 127 fit a byte
    constexpr int kPlanes = kAcc + 3;
    extern __shared__ uint32_t group_lds[];                     // [kGroupWaves][kAcc][256 dwords of the span]
    const Problem &p = addr.p;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = h.N;
    const int64_t W = (p.numel + 63) >> 6;
    const int64_t span = addr.first_tile + blockIdx.x;
    const int64_t w0 = span * kGroupWords;

    // ---- this wave's rows over the whole span: lane l holds words 2l, 2l + 1 as four 32-bit slices
    uint32_t acc[kAcc][4];
#pragma unroll
    for (int b = 0; b < kAcc; ++b)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            acc[b][q] = 0;
    {
        const bool whole = w0 + kGroupWords <= W;              // uniform
        const int64_t wl = w0 + lane * 2;
#pragma unroll 1
        for (int r0 = wave; r0 < N; r0 += kGroupWaves * kInFlight) {
            u32x4 v[kInFlight];
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                v[u] = u32x4{0u, 0u, 0u, 0u};
                const int r = r0 + u * kGroupWaves;
                if (r < N) {                                    // uniform
                    const uint64_t *src = p.packed + (int64_t)r * p.packed_stride + wl;
                    if (whole || wl + 1 < W) {
                        v[u] = packed_load2(src);
                    } else if (wl < W) {
                        const uint64_t word = stream_load(src);
                        v[u].x = static_cast<uint32_t>(word);
                        v[u].y = static_cast<uint32_t>(word >> 32);
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kInFlight; ++u) {
                const uint32_t w4[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    uint32_t c = w4[q];
#pragma unroll
                    for (int b = 0; b < kAcc; ++b) {
                        const uint32_t carry = acc[b][q] & c;
                        acc[b][q] ^= c;
                        c = carry;
                    }
                }
            }
        }
    }
    // ---- this wave's line of the span
    const int64_t t = span * kGroupWaves + wave;                // line index: words 16t .. 16t + 15
    const int64_t c0 = t * kLineCoords;
    const bool line_full = c0 + kLineCoords <= p.numel;         // uniform
    {
        uint32_t *mine = group_lds + wave * kAcc * 256 + lane * 4;
#pragma unroll
        for (int b = 0; b < kAcc; ++b)
            *reinterpret_cast<u32x4 *>(mine + b * 256) = u32x4{acc[b][0], acc[b][1], acc[b][2], acc[b][3]};
    }
    __syncthreads();
    // x of the line's first coordinate if the line can be updated with full-width accesses
    float *xline = nullptr;
    if (kApply && line_full) {
        if (kSeg) {
            const dlion_seg sg = tab.segs[seg_of_word(tab, t * kLineWords)];       // uniform
            const int64_t local = (t * kLineWords - sg.word_begin) * 64;
            if (local + kLineCoords <= sg.numel)
                xline = sg.x + local;
        } else {
            xline = p.x + c0;
        }
    }
    f32x4 xv[kLineSubs];
    if (kApply && xline) {
#pragma unroll
        for (int s = 0; s < kLineSubs; ++s)
            xv[s] = x_load4(xline + s * kTile + lane * kVec);
    }
    const bool line_exists = c0 < p.numel;                      // uniform
    if (!kEncode && !line_exists)
        return;
    const int half = lane >> 5, dw = lane & 31;
    uint32_t pl[kPlanes];
    {
        const uint32_t *src = group_lds + (4 * half * kAcc) * 256 + wave * 32 + dw;
        uint32_t a[4][kAcc];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int b = 0; b < kAcc; ++b)
                a[k][b] = src[(k * kAcc + b) * 256];
        uint32_t s01[kAcc + 1], s23[kAcc + 1], s4[kAcc + 2];
        add_planes<kAcc>(a[0], a[1], s01);
        add_planes<kAcc>(a[2], a[3], s23);
        add_planes<kAcc + 1>(s01, s23, s4);
        uint32_t carry = 0;                                     // waves 0..3 + waves 4..7
#pragma unroll
        for (int b = 0; b < kAcc + 2; ++b) {
            const uint32_t other = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, s4[b]));
            csa(carry, pl[b], s4[b], other, carry);
        }
        pl[kAcc + 2] = carry;
    }
    // from here on lane l holds, for dword l & 31 of the line, plane b = bit b of its 32 counts
    uint32_t plus = 0, tie = 0;
    if (h.mode == DLION_VOTE) {                                 // count > N/2; count == N/2 for even N
        const uint32_t K = static_cast<uint32_t>(N) >> 1;
        uint32_t eq = 0xFFFFFFFFu;
#pragma unroll
        for (int b = kPlanes - 1; b >= 0; --b) {
            if ((K >> b) & 1u) {
                eq &= pl[b];
            } else {
                plus |= eq & pl[b];
                eq &= ~pl[b];
            }
        }
        tie = (N & 1) ? 0u : eq;
    }
    if (kEncode) {
        // The planes of the message go back through LDS, so that wave b can write plane b of the whole
        // span with full-width stores (1 KB per instruction; a line per wave and plane reaches half the
        // bandwidth).  Bits past d are zero; words past W do not exist.
        uint32_t *stage = group_lds + kGroupWaves * kAcc * 256;    // [kPlanes][256 dwords of the span]
        if (line_exists && half == 0) {
            const int64_t left = p.numel - (c0 + 32 * dw);         // coordinates from this dword on
            const uint32_t mask = left >= 32 ? 0xFFFFFFFFu : (left > 0 ? (1u << left) - 1u : 0u);
            if (h.mode == DLION_VOTE) {
                stage[wave * 32 + dw] = plus & mask;
                stage[256 + wave * 32 + dw] = tie & mask;
            } else {
#pragma unroll
                for (int b = 0; b < kPlanes; ++b)
                    stage[b * 256 + wave * 32 + dw] = pl[b] & mask;
            }
        }
        __syncthreads();
        if (wave < out.n_planes) {
            const u32x4 val = *reinterpret_cast<const u32x4 *>(stage + wave * 256 + lane * 4);
            const int64_t wl = w0 + lane * 2;
            uint64_t *dst = out.planes + (int64_t)wave * out.stride + wl;
            if (wl + 1 < W) {
                if (h.stream_counts)
                    stream_store_b128(val, dst);
                else
                    *reinterpret_cast<words2_e *>(dst) = val;
            } else if (wl < W) {
                *dst = (static_cast<uint64_t>(val.y) << 32) | val.x;
            }
        }
        return;
    }
    if (kApply) {
        // lane l owns coordinates 4l..4l+3 of sub-tile s: nibble l & 7 of dword 8s + (l >> 3)
        const int shift = (lane & 7) * 4;
#pragma unroll
        for (int s = 0; s < kLineSubs; ++s) {
            const int from = (8 * s + (lane >> 3)) << 2;
            const int64_t j = c0 + s * kTile + lane * kVec;
            float Delta[4];
            uint32_t bytes = 0;
            if (h.mode == DLION_VOTE && !kCounts) {
                const uint32_t pn = (static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from, plus)) >> shift) & 0xFu;
                const uint32_t tn = (static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(from, tie)) >> shift) & 0xFu;
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    Delta[k] = decode_vote((pn >> k) & 1u, (tn >> k) & 1u);
            } else {
                bytes = line_counts4<kPlanes>(pl, from, shift);
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    Delta[k] = aggregate_votes((bytes >> (8 * k)) & 0xFFu, h);
            }
            if (xline) {
                if (kCounts) {
                    u16x4 c;
                    c.x = static_cast<uint16_t>(bytes & 0xFFu);
                    c.y = static_cast<uint16_t>((bytes >> 8) & 0xFFu);
                    c.z = static_cast<uint16_t>((bytes >> 16) & 0xFFu);
                    c.w = static_cast<uint16_t>(bytes >> 24);
                    COUNTS_STORE4(c, p.counts + j);
                }
                xv[s].x = lion_apply(xv[s].x, Delta[0], h);
                xv[s].y = lion_apply(xv[s].y, Delta[1], h);
                xv[s].z = lion_apply(xv[s].z, Delta[2], h);
                xv[s].w = lion_apply(xv[s].w, Delta[3], h);
                x_store4(xv[s], xline + s * kTile + lane * kVec);
            } else {
                // coordinate by coordinate; the lane's four coordinates share a word, hence an owner
                float *xs = p.x;                                // flat: coordinate j is x[j]
                int64_t local = j, numel = p.numel;
                if (kSeg) {
                    numel = 0;
                    if (j < p.numel) {
                        const dlion_seg sg = tab.segs[seg_of_word(tab, j >> 6)];
                        xs = sg.x;
                        local = j - sg.word_begin * 64;
                        numel = sg.numel;
                    }
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    if (local + k < numel)
                        xs[local + k] = lion_apply(xs[local + k], Delta[k], h);
                    if (kCounts && j + k < p.counts_end)
                        p.counts[j + k] = static_cast<uint16_t>(local + k < numel ? (bytes >> (8 * k)) & 0xFFu : 0u);
                }
            }
        }
    } else if (kCounts) {
        // counts only: lane l owns coordinates 8l..8l+7 of one half of the line, i.e. byte l & 3 of
        // dword 16h + (l >> 2), and stores its eight counts with one 128-bit access
        const int shift = (lane & 3) * 8;
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
            const int from = (16 * hh + (lane >> 2)) << 2;
            const uint32_t lo = line_counts4<kPlanes>(pl, from, shift);
            const uint32_t up = line_counts4<kPlanes>(pl, from, shift + 4);
            const int64_t j = c0 + hh * (kLineCoords / 2) + lane * 8;
            if (line_full) {
                u32x4 c;
                c.x = (lo & 0xFFu) | ((lo & 0xFF00u) << 8);
                c.y = ((lo >> 16) & 0xFFu) | ((lo >> 24) << 16);
                c.z = (up & 0xFFu) | ((up & 0xFF00u) << 8);
                c.w = ((up >> 16) & 0xFFu) | ((up >> 24) << 16);
                counts_store8(c, p.counts + j, h.stream_counts);
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k)
                    if (j + k < p.counts_end)
                        p.counts[j + k] = static_cast<uint16_t>(j + k < p.numel ? ((k < 4 ? lo : up) >> (8 * (k & 3))) & 0xFFu : 0u);
            }
        }
    }
}

// ---------------------------------------------------------------- Global Lion (comparison scheme)
// Appendix, "Global Lion Convergence": the workers' full-precision blends c_i are averaged and
// x <- x - lr*(sign(mean_i c_i) + lambda*x); each worker's momentum moves as in Distributed
// Lion.  The mean is the fp32 sum over i = 0..N-1 in that order divided by (float)N, and the
// sign maps 0 to +1 (so that N = 1 is the same single-worker Lion).  Same tiling as the fused
// step; sign_bits (optional) receives sign(mean c) packed like a worker's message.
__device__ __forceinline__ bool global_sign(float sum, const Hyper &h)
{
    const float mean = (h.inv_n != 0.0f) ? __fmul_rn(sum, h.inv_n) : sum / static_cast<float>(h.N);
    return !(mean < 0.0f);
}

template <typename GT, int kUnroll>
__global__ __launch_bounds__(kLanes) void global_lion_kernel(FlatAddr addr, Hyper h, uint64_t *sign_bits)
{
    const Problem &p = addr.p;
    const int64_t t = blockIdx.x;
    const int lane = threadIdx.x;
    const int N = h.N;
    const Coef k = {h.beta1, h.omb1, h.beta2, h.omb2};
    const bool vec = (t + 1) * kTile <= p.numel;
    if (vec) {
        const int64_t j0 = t * kTile + lane * kVec;
        f32x4 xv = x_load4(p.x + j0);
        float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
        auto one_worker = [&](int i, f32x4 mv, f32x4 gv) {
            float m0 = mv.x, m1 = mv.y, m2 = mv.z, m3 = mv.w;
            s0 = __fadd_rn(s0, lion_blend(m0, gv.x, k));
            s1 = __fadd_rn(s1, lion_blend(m1, gv.y, k));
            s2 = __fadd_rn(s2, lion_blend(m2, gv.z, k));
            s3 = __fadd_rn(s3, lion_blend(m3, gv.w, k));
            mv.x = m0;
            mv.y = m1;
            mv.z = m2;
            mv.w = m3;
            row_store4(mv, p.m + (int64_t)i * p.m_stride + j0);
        };
        int i = 0;
        for (; i + kUnroll <= N; i += kUnroll) {
            f32x4 mv[kUnroll], gv[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                mv[u] = row_load4(p.m + (int64_t)(i + u) * p.m_stride + j0);
                gv[u] = Grad<GT>::load4(p.g, (int64_t)(i + u) * p.g_stride + j0);
            }
#pragma unroll
            for (int u = 0; u < kUnroll; ++u)
                one_worker(i + u, mv[u], gv[u]);
        }
        for (; i < N; ++i) {
            const f32x4 mv = row_load4(p.m + (int64_t)i * p.m_stride + j0);
            const f32x4 gv = Grad<GT>::load4(p.g, (int64_t)i * p.g_stride + j0);
            one_worker(i, mv, gv);
        }
        const bool b0 = global_sign(s0, h), b1 = global_sign(s1, h), b2 = global_sign(s2, h), b3 = global_sign(s3, h);
        xv.x = lion_apply(xv.x, b0 ? 1.0f : -1.0f, h);
        xv.y = lion_apply(xv.y, b1 ? 1.0f : -1.0f, h);
        xv.z = lion_apply(xv.z, b2 ? 1.0f : -1.0f, h);
        xv.w = lion_apply(xv.w, b3 ? 1.0f : -1.0f, h);
        x_store4(xv, p.x + j0);
        if (sign_bits) {
            const uint32_t nib = (b0 ? 1u : 0u) | (b1 ? 2u : 0u) | (b2 ? 4u : 0u) | (b3 ? 8u : 0u);
            const uint64_t word = row_gather_nibbles(nib, lane);
            if ((lane & 15) == 0)
                sign_bits[t * kWordsPerTile + (lane >> 4)] = word;
        }
        return;
    }
    const int64_t W = (p.numel + 63) >> 6;
#pragma unroll 1
    for (int kk = 0; kk < kWordsPerTile; ++kk) {
        const int64_t w = t * kWordsPerTile + kk;
        if (w >= W)
            break;
        const int64_t j = w * 64 + lane;
        const bool valid = j < p.numel;
        float sum = 0.0f;
        if (valid) {
            for (int i = 0; i < N; ++i) {
                float *mp = p.m + (int64_t)i * p.m_stride + j;
                float mv = *mp;
                sum = __fadd_rn(sum, lion_blend(mv, Grad<GT>::load1(p.g, (int64_t)i * p.g_stride + j), k));
                *mp = mv;
            }
        }
        const bool plus = valid && global_sign(sum, h);
        if (valid)
            p.x[j] = lion_apply(p.x[j], plus ? 1.0f : -1.0f, h);
        if (sign_bits) {
            const uint64_t word = __ballot(plus);
            if (lane == 0)
                sign_bits[w] = word;
        }
    }
}

// ---------------------------------------------------------------- apply from counts
template <class Addr>
__global__ __launch_bounds__(kLanes) void apply_kernel(Addr addr, Hyper h)
{
    const int64_t tile = addr.first_tile + wave_tile_index();
    if (tile >= addr.total_tiles)
        return;
    const int lane = threadIdx.x;
    Problem p;
    const int64_t t = addr.resolve(tile, p);
    if ((t + 1) * kTile <= p.numel) {
        const int64_t j0 = t * kTile + lane * kVec;
        const u16x4 c = counts_load4(p.counts + j0);
        f32x4 xv = x_load4(p.x + j0);
        xv.x = lion_apply(xv.x, aggregate_votes(c.x, h), h);
        xv.y = lion_apply(xv.y, aggregate_votes(c.y, h), h);
        xv.z = lion_apply(xv.z, aggregate_votes(c.z, h), h);
        xv.w = lion_apply(xv.w, aggregate_votes(c.w, h), h);
        x_store4(xv, p.x + j0);
    } else {
#pragma unroll 1
        for (int k = 0; k < kWordsPerTile; ++k) {
            const int64_t j = (t * kWordsPerTile + k) * 64 + lane;
            if (j < p.numel)
                p.x[j] = lion_apply(p.x[j], aggregate_votes(p.counts[j], h), h);
        }
    }
}

// ---------------------------------------------------------------- memory-rate probe
// None of the method's arithmetic: wave t reads the t-th 1 KB piece of each of `rows` rows (128
// bits per lane, kBatch rows in flight), folds them with XOR so that no load can be dropped, and
// writes one 1 KB piece (kWrite) or nothing.  rows = 1 with kWrite is a plain copy; rows = 16 has
// the 16 : 1 read : write byte mix of counting 256 packed streams into uint16 counts.  Same launch
// style as the real kernels: one-wave workgroups, streaming accesses, plain tile numbering.
template <bool kWrite, int kBatch>
__global__ __launch_bounds__(kLanes) void membench_kernel(const u32x4 *src, int64_t row_stride, int32_t rows,
                                                          u32x4 *dst, int64_t first_piece)
{
    const int64_t at = (first_piece + blockIdx.x) * kLanes + threadIdx.x;      // in 16-byte units
    u32x4 acc = {0u, 0u, 0u, 0u};
    int r = 0;
    for (; r + kBatch <= rows; r += kBatch) {
        u32x4 v[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k)
            v[k] = __builtin_nontemporal_load(src + (int64_t)(r + k) * row_stride + at);
#pragma unroll
        for (int k = 0; k < kBatch; ++k)
            acc ^= v[k];
    }
    for (; r < rows; ++r)
        acc ^= __builtin_nontemporal_load(src + (int64_t)r * row_stride + at);
    if (kWrite)
        stream_store_b128(acc, dst + at);
    else if (acc.x == 0x9E3779B9u && acc.y == 0x7F4A7C15u && acc.z == acc.x && acc.w == acc.y)
        dst[0] = acc;                                        // practically never: keeps the loads alive
}

}  // namespace dlion
