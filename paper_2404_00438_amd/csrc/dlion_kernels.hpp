// Device code of the Distributed Lion sweep for gfx950 (CDNA4, 64-wide wavefronts).
//
// Work decomposition: the coordinate range of a tensor is cut into TILES of 256
// coordinates (= 4 packed uint64 words).  One wavefront owns one tile and walks
// over all N workers for it, so the vote count of a coordinate never leaves
// the lane that owns the coordinate and no inter-wave communication, atomics
// or barriers are needed anywhere on the worker/fused path.
//
// Two code paths per tile:
//   * vector path (full tile, 16-byte aligned rows): lane l owns coordinates
//     4l..4l+3 and moves them with one 128-bit access per stream.  Its four
//     sign bits form a nibble; the nibbles of the 16 lanes of a DPP row are
//     OR-combined into one canonical packed word per row.
//   * guarded path (ragged last tile, or rows that are not 16-byte aligned):
//     lane l owns coordinates 64k+l, k=0..3, moved with dword accesses; a
//     64-lane ballot of the sign predicate is already a canonical packed word.
//
// All fp32 arithmetic goes through __fmul_rn/__fadd_rn/__fsub_rn so that no
// multiply-add is ever fused (Section 3.2's expressions, each operation rounded
// on its own); the sign is taken as !(c < 0), i.e. 0 votes +1.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dlion.h"

namespace dlion {

// Launch-shape knobs (compile-time; the defaults are the measured best on MI355X).
#ifndef DLION_SUBTILES
#define DLION_SUBTILES 1        // 256-coordinate sub-tiles a wave handles together
#endif
#ifndef DLION_WAVES_PER_BLOCK
#define DLION_WAVES_PER_BLOCK 1
#endif
#ifndef DLION_NT_LOAD
#define DLION_NT_LOAD 1         // streaming (non-temporal) loads of m and g
#endif
#ifndef DLION_NT_STORE
#define DLION_NT_STORE 1        // streaming stores of m
#endif
#ifndef DLION_MAX_WAVES_PER_EU
#define DLION_MAX_WAVES_PER_EU 0   // cap on resident waves per SIMD for the streaming kernels (0: no cap)
#endif
#ifndef DLION_XCD_REMAP
#define DLION_XCD_REMAP 0       // give each of the 8 XCDs one contiguous range of tiles
#endif

constexpr int kLanes = 64;
constexpr int kVec = 4;                       // coordinates per lane per sub-tile on the vector path
constexpr int kSubTile = kLanes * kVec;       // 256 coordinates = 4 packed words
constexpr int kWordsPerSub = kSubTile / 64;
constexpr int kSubs = DLION_SUBTILES;
constexpr int kTile = kSubTile * kSubs;       // coordinates one wave owns
constexpr int kWavesPerBlock = DLION_WAVES_PER_BLOCK;
constexpr int kBlock = kLanes * kWavesPerBlock;
constexpr int kXcds = 8;

#if DLION_MAX_WAVES_PER_EU > 0
#define DLION_OCCUPANCY __attribute__((amdgpu_waves_per_eu(1, DLION_MAX_WAVES_PER_EU)))
#else
#define DLION_OCCUPANCY
#endif

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

struct Hyper {
    float beta1, omb1, beta2, omb2;  // omb = 1.0f - beta, formed on the host in fp32
    float lr, lambda;
    float inv_n;      // 1/N when N is a power of two (then S*inv_n == S/N exactly), else 0
    int32_t N;
    int32_t mode;     // dlion_mode
    int32_t stream_counts;   // counts array too large to stay cached: write it with streaming stores
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

// ---------------------------------------------------------------- addressing
// Flat buffer: the problem travels in the kernel arguments.
struct FlatAddr {
    Problem p;
    int64_t total_tiles;
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

template <int kWaves = kWavesPerBlock> __device__ __forceinline__ int64_t wave_tile_index()
{
    // blockIdx and the wave number are uniform across the wavefront; say so, so
    // that everything derived from the tile index stays in scalar registers.
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t block = blockIdx.x;
#if DLION_XCD_REMAP
    // Workgroups are handed to the 8 XCDs round-robin (block b runs on XCD b % 8).
    // Renumber them so that XCD x walks one contiguous range of tiles.
    const uint32_t G = gridDim.x, q = G / kXcds, r = G % kXcds, xcd = block % kXcds;
    block = xcd * q + (xcd < r ? xcd : r) + block / kXcds;
#endif
    return (int64_t)block * kWaves + wave;
}

// Cache policy of the small per-coordinate arrays.  x is touched once per step: streaming
// (non-temporal) accesses, +14 % on the apply kernel.  counts written by one call are read by
// the next (aggregate -> apply) and up to ~250 MB of them stay in the memory-side cache, so
// they use ordinary accesses unless the array is too large for that (h.stream_counts).
#ifndef DLION_NT_X
#define DLION_NT_X 1
#endif
#define C_STORE(v, p)                              \
    do {                                           \
        if (h.stream_counts)                       \
            __builtin_nontemporal_store(v, p);     \
        else                                       \
            *(p) = (v);                            \
    } while (0)
#define C_LOAD(p) (*(p))
#if DLION_NT_X
#define X_STORE(v, p) __builtin_nontemporal_store(v, p)
#define X_LOAD(p) __builtin_nontemporal_load(p)
#else
#define X_STORE(v, p) (*(p) = (v))
#define X_LOAD(p) (*(p))
#endif

template <typename T> __device__ __forceinline__ T stream_load(const T *p)
{
#if DLION_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename T> __device__ __forceinline__ void stream_store(T v, T *p)
{
#if DLION_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

__device__ __forceinline__ bool is_aligned(const void *p, uint64_t a)
{
    return (reinterpret_cast<uint64_t>(p) & (a - 1)) == 0;
}

// ---------------------------------------------------------------- gradients
template <typename GT> struct Grad;
template <> struct Grad<float> {
    static constexpr int kVecBytes = 16;
    static __device__ __forceinline__ f32x4 load4(const void *g, int64_t idx)
    {
        return stream_load(reinterpret_cast<const f32x4 *>(static_cast<const float *>(g) + idx));
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
        const u32x2 raw = stream_load(reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(g) + idx));
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
__device__ __forceinline__ bool lion_worker(float &m, float g, const Hyper &h)
{
    const float c = __fadd_rn(__fmul_rn(h.beta1, m), __fmul_rn(h.omb1, g));
    m = __fadd_rn(__fmul_rn(h.beta2, m), __fmul_rn(h.omb2, g));
    return !(c < 0.0f);
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
// Vector path over kR full sub-tiles starting at sub-tile `t`: the loads of kUnroll workers
// x kR sub-tiles are issued back to back before any arithmetic.
template <typename GT, int kUnroll, int kR, bool kApply, bool kPacked, bool kCounts, bool kLockstep = false>
__device__ __forceinline__ void step_subtiles_vector(const Problem &p, int64_t t, int lane, const Hyper &h)
{
    const int64_t j0 = t * kSubTile + lane * kVec;
    f32x4 xv[kR];
    if (kApply) {
#pragma unroll
        for (int r = 0; r < kR; ++r)
            xv[r] = X_LOAD(reinterpret_cast<const f32x4 *>(p.x + j0 + r * kSubTile));
    }
    uint32_t cnt[kR][4];
#pragma unroll
    for (int r = 0; r < kR; ++r)
        cnt[r][0] = cnt[r][1] = cnt[r][2] = cnt[r][3] = 0;
    const int N = h.N;

    auto one_worker = [&](int i, int r, f32x4 mv, f32x4 gv) {
        float m0 = mv.x, m1 = mv.y, m2 = mv.z, m3 = mv.w;
        const bool b0 = lion_worker(m0, gv.x, h);
        const bool b1 = lion_worker(m1, gv.y, h);
        const bool b2 = lion_worker(m2, gv.z, h);
        const bool b3 = lion_worker(m3, gv.w, h);
        mv.x = m0;
        mv.y = m1;
        mv.z = m2;
        mv.w = m3;
        stream_store(mv, reinterpret_cast<f32x4 *>(p.m + (int64_t)i * p.m_stride + j0 + r * kSubTile));
        cnt[r][0] += b0;
        cnt[r][1] += b1;
        cnt[r][2] += b2;
        cnt[r][3] += b3;
        if (kPacked) {
            const uint32_t nib = (b0 ? 1u : 0u) | (b1 ? 2u : 0u) | (b2 ? 4u : 0u) | (b3 ? 8u : 0u);
            const uint64_t word = row_gather_nibbles(nib, lane);
            if ((lane & 15) == 0)
                p.packed[(int64_t)i * p.packed_stride + (t + r) * kWordsPerSub + (lane >> 4)] = word;
        }
    };

    int i = 0;
    for (; i + kUnroll <= N; i += kUnroll) {
        f32x4 mv[kUnroll][kR], gv[kUnroll][kR];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
            for (int r = 0; r < kR; ++r) {
                mv[u][r] = stream_load(
                    reinterpret_cast<const f32x4 *>(p.m + (int64_t)(i + u) * p.m_stride + j0 + r * kSubTile));
                gv[u][r] = Grad<GT>::load4(p.g, (int64_t)(i + u) * p.g_stride + j0 + r * kSubTile);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
#pragma unroll
            for (int r = 0; r < kR; ++r)
                one_worker(i + u, r, mv[u][r], gv[u][r]);
        }
        if (kLockstep)
            __builtin_amdgcn_s_barrier();     // keep the waves of the workgroup on the same workers
    }
    for (; i < N; ++i) {
        f32x4 mv[kR], gv[kR];
#pragma unroll
        for (int r = 0; r < kR; ++r) {
            mv[r] = stream_load(reinterpret_cast<const f32x4 *>(p.m + (int64_t)i * p.m_stride + j0 + r * kSubTile));
            gv[r] = Grad<GT>::load4(p.g, (int64_t)i * p.g_stride + j0 + r * kSubTile);
        }
#pragma unroll
        for (int r = 0; r < kR; ++r)
            one_worker(i, r, mv[r], gv[r]);
    }

#pragma unroll
    for (int r = 0; r < kR; ++r) {
        if (kApply) {
            xv[r].x = lion_apply(xv[r].x, aggregate_votes(cnt[r][0], h), h);
            xv[r].y = lion_apply(xv[r].y, aggregate_votes(cnt[r][1], h), h);
            xv[r].z = lion_apply(xv[r].z, aggregate_votes(cnt[r][2], h), h);
            xv[r].w = lion_apply(xv[r].w, aggregate_votes(cnt[r][3], h), h);
            X_STORE(xv[r], reinterpret_cast<f32x4 *>(p.x + j0 + r * kSubTile));
        }
        if (kCounts) {
            u16x4 c;
            c.x = static_cast<uint16_t>(cnt[r][0]);
            c.y = static_cast<uint16_t>(cnt[r][1]);
            c.z = static_cast<uint16_t>(cnt[r][2]);
            c.w = static_cast<uint16_t>(cnt[r][3]);
            C_STORE(c, reinterpret_cast<u16x4 *>(p.counts + j0 + r * kSubTile));
        }
    }
}

// Guarded path: lane l owns coordinates 64k+l of the tile; every access checks
// j < numel; a 64-lane ballot is already a canonical packed word.
template <typename GT, bool kApply, bool kPacked, bool kCounts>
__device__ __forceinline__ void step_subtile_guarded(const Problem &p, int64_t t, int lane, const Hyper &h)
{
    const int64_t W = (p.numel + 63) >> 6;
#pragma unroll 1
    for (int k = 0; k < kWordsPerSub; ++k) {
        const int64_t w = t * kWordsPerSub + k;
        if (w >= W)
            break;                                   // uniform: whole wave leaves together
        const int64_t j = w * 64 + lane;
        const bool valid = j < p.numel;
        uint32_t cnt = 0;
        for (int i = 0; i < h.N; ++i) {
            bool plus = false;
            if (valid) {
                float *mp = p.m + (int64_t)i * p.m_stride + j;
                float mv = *mp;
                const float gv = Grad<GT>::load1(p.g, (int64_t)i * p.g_stride + j);
                plus = lion_worker(mv, gv, h);
                *mp = mv;
            }
            cnt += plus;
            if (kPacked) {
                const uint64_t word = __ballot(plus);   // invalid lanes contribute 0: tail bits zero
                if (lane == 0)
                    p.packed[(int64_t)i * p.packed_stride + w] = word;
            }
        }
        if (kApply && valid)
            p.x[j] = lion_apply(p.x[j], aggregate_votes(cnt, h), h);
        if (kCounts && j < p.counts_end)
            p.counts[j] = static_cast<uint16_t>(cnt);   // 0 past numel (tensor-list padding)
    }
}

// kWaves waves per workgroup.  With more than one, the waves of a workgroup walk over the
// workers in lockstep (a barrier per batch of workers): with many workers, waves that drift
// apart touch 3 pages per worker each and thrash the per-CU address-translation cache; kept
// together, the compute unit works inside a handful of pages at any time.  A wave that takes
// the guarded path, or has no tile, simply terminates; the barrier only waits for waves that
// are still alive, and every surviving wave executes the same number of barriers (N is the
// same for every tile).
template <typename GT, int kUnroll, int kWaves, bool kApply, bool kPacked, bool kCounts, class Addr>
__global__ __launch_bounds__(kLanes * kWaves) DLION_OCCUPANCY void step_kernel(Addr addr, Hyper h)
{
    const int64_t tile = wave_tile_index<kWaves>();
    if (tile >= addr.total_tiles)
        return;
    const int lane = threadIdx.x & 63;
    Problem p;
    const int64_t t = addr.resolve(tile, p) * kSubs;      // first sub-tile of this wave
    bool aligned = is_aligned(p.m, 16) && (p.m_stride & 3) == 0 && is_aligned(p.g, Grad<GT>::kVecBytes) &&
                   (p.g_stride & 3) == 0;
    if (kApply)
        aligned = aligned && is_aligned(p.x, 16);
    if (kCounts)
        aligned = aligned && is_aligned(p.counts, 8);
    if (aligned && (t + kSubs) * kSubTile <= p.numel) {
        step_subtiles_vector<GT, kUnroll, kSubs, kApply, kPacked, kCounts, (kWaves > 1)>(p, t, lane, h);
        return;
    }
    // ragged end of a tensor, or rows that cannot take 128-bit accesses
#pragma unroll 1
    for (int r = 0; r < kSubs; ++r) {
        const int64_t sub = t + r;
        if (sub * kSubTile >= p.numel)
            break;
        if (kSubs > 1 && aligned && (sub + 1) * kSubTile <= p.numel)
            step_subtiles_vector<GT, kUnroll, 1, kApply, kPacked, kCounts>(p, sub, lane, h);
        else
            step_subtile_guarded<GT, kApply, kPacked, kCounts>(p, sub, lane, h);
    }
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
    const uint32_t *half = reinterpret_cast<const uint32_t *>(p.packed + t * kWordsPerSub + (lane >> 4)) +
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
    const int64_t j0 = t * kSubTile + lane * kVec;
    if (kApply) {
        f32x4 xv = X_LOAD(reinterpret_cast<const f32x4 *>(p.x + j0));
        xv.x = lion_apply(xv.x, aggregate_votes(cnt0, h), h);
        xv.y = lion_apply(xv.y, aggregate_votes(cnt1, h), h);
        xv.z = lion_apply(xv.z, aggregate_votes(cnt2, h), h);
        xv.w = lion_apply(xv.w, aggregate_votes(cnt3, h), h);
        X_STORE(xv, reinterpret_cast<f32x4 *>(p.x + j0));
    }
    if (kCounts) {
        u16x4 c;
        c.x = static_cast<uint16_t>(cnt0);
        c.y = static_cast<uint16_t>(cnt1);
        c.z = static_cast<uint16_t>(cnt2);
        c.w = static_cast<uint16_t>(cnt3);
        C_STORE(c, reinterpret_cast<u16x4 *>(p.counts + j0));
    }
}

// Guarded path: lane l owns bit l of word 4t+k.
template <bool kApply, bool kCounts>
__device__ __forceinline__ void agg_subtile_guarded(const Problem &p, int64_t t, int lane, const Hyper &h)
{
    const int64_t W = (p.numel + 63) >> 6;
#pragma unroll 1
    for (int k = 0; k < kWordsPerSub; ++k) {
        const int64_t w = t * kWordsPerSub + k;
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
__global__ __launch_bounds__(kBlock) void aggregate_kernel(Addr addr, Hyper h)
{
    const int64_t tile = wave_tile_index();
    if (tile >= addr.total_tiles)
        return;
    const int lane = threadIdx.x & 63;
    Problem p;
    const int64_t t = addr.resolve(tile, p) * kSubs;
    bool aligned = true;
    if (kApply)
        aligned = aligned && is_aligned(p.x, 16);
    if (kCounts)
        aligned = aligned && is_aligned(p.counts, 8);
#pragma unroll 1
    for (int r = 0; r < kSubs; ++r) {
        const int64_t sub = t + r;
        if (sub * kSubTile >= p.numel)
            break;
        if (aligned && (sub + 1) * kSubTile <= p.numel)
            agg_subtile_vector<kApply, kCounts>(p, sub, lane, h);
        else
            agg_subtile_guarded<kApply, kCounts>(p, sub, lane, h);
    }
}

// ---------------------------------------------------------------- server side, many workers
// Bit-sliced ("vertical") counting.  One wave owns kSlicedWords consecutive packed words;
// lane l reads kWpl consecutive words of every stream (1 KB contiguous per load instruction)
// and adds the N words into kPlanes bit-planes with carry-save adders: after the loop, bit c
// of plane b of a word is bit b of the vote count of that word's coordinate c.  About one
// bitwise operation per 32 coordinates and input word replaces 32 extract-and-add steps.  The planes
// are then staged through LDS so that the lanes can switch from "kWpl words each" to "four
// consecutive coordinates each" and write counts / update x with full-width accesses.
#ifndef DLION_SLICED_WORDS_PER_LANE
#define DLION_SLICED_WORDS_PER_LANE 2      // consecutive words of each stream a lane reads (1 or 2)
#endif
constexpr int kWpl = DLION_SLICED_WORDS_PER_LANE;
constexpr int kSlices = 2 * kWpl;                      // 32-bit slices a lane carries
constexpr int kSlicedWords = kLanes * kWpl;            // words per wave
constexpr int kSlicedCoords = kSlicedWords * 64;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// carry-save adder on 32 independent bit positions: a + b + c = 2*carry + sum.  gfx950 has a
// three-input boolean instruction, so each output is one operation (truth tables: majority
// 0xE8, parity 0x96; both symmetric in their operands).
__device__ __forceinline__ void csa(uint32_t &carry, uint32_t &sum, uint32_t a, uint32_t b, uint32_t c)
{
    carry = __builtin_amdgcn_bitop3_b32(a, b, c, 0xE8);
    sum = __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

//
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
    static_assert(kPlanes >= 5 && kPlanes <= 16, "planes");
    static_assert(kWpl == 1 || kWpl == 2, "words per lane");
    extern __shared__ uint32_t sliced_lds[];                    // [kWaves][kPlanes][kSlicedLdsPerPlane]
    const Problem &p = addr.p;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    uint32_t(*lds)[kSlicedLdsPerPlane] =
        reinterpret_cast<uint32_t(*)[kSlicedLdsPerPlane]>(sliced_lds + wave * kPlanes * kSlicedLdsPerPlane);
    const int64_t W = (p.numel + 63) >> 6;
    const int64_t w0 = ((int64_t)blockIdx.x * kWaves + wave) * kSlicedWords;   // first word of the wave
    if (w0 >= W)
        return;
    const int64_t wl0 = w0 + (int64_t)lane * kWpl;              // first word of the lane
    const bool vec = (p.packed_stride % kWpl) == 0 && is_aligned(p.packed, 8 * kWpl);
    // whole group inside the word range and rows that allow full-width loads: no per-lane guards
    const bool fast = vec && w0 + kSlicedWords <= W;
    const int N = h.N;

    uint32_t ones[kSlices], twos[kSlices], fours[kSlices], eights[kSlices];
    uint32_t hi[kPlanes - 4][kSlices];                          // planes 4.. (sixteens and up)
#pragma unroll
    for (int q = 0; q < kSlices; ++q) {
        ones[q] = twos[q] = fours[q] = eights[q] = 0;
#pragma unroll
        for (int b = 0; b < kPlanes - 4; ++b)
            hi[b][q] = 0;
    }

    for (int i = 0; i < N; i += 16) {
        uint32_t v[16][kSlices];
        if (fast && i + 16 <= N) {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                // uniform row base + small per-lane offset
                const uint64_t *row = p.packed + (int64_t)(i + k) * p.packed_stride + w0;
                if (kWpl == 2) {
                    const u32x4 r = stream_load(reinterpret_cast<const u32x4 *>(row) + lane);
                    v[k][0] = r.x;
                    v[k][1] = r.y;
                    v[k][kSlices - 2] = r.z;
                    v[k][kSlices - 1] = r.w;
                } else {
                    const u32x2 r = stream_load(reinterpret_cast<const u32x2 *>(row) + lane);
                    v[k][0] = r.x;
                    v[k][1] = r.y;
                }
            }
        } else {
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
        }
#pragma unroll
        for (int q = 0; q < kSlices; ++q) {
            uint32_t t0, t1, t2, t3, t4, t5, t6, t7, f0, f1, f2, f3, e0, e1, s16;
            csa(t0, ones[q], ones[q], v[0][q], v[1][q]);
            csa(t1, ones[q], ones[q], v[2][q], v[3][q]);
            csa(t2, ones[q], ones[q], v[4][q], v[5][q]);
            csa(t3, ones[q], ones[q], v[6][q], v[7][q]);
            csa(t4, ones[q], ones[q], v[8][q], v[9][q]);
            csa(t5, ones[q], ones[q], v[10][q], v[11][q]);
            csa(t6, ones[q], ones[q], v[12][q], v[13][q]);
            csa(t7, ones[q], ones[q], v[14][q], v[15][q]);
            csa(f0, twos[q], twos[q], t0, t1);
            csa(f1, twos[q], twos[q], t2, t3);
            csa(f2, twos[q], twos[q], t4, t5);
            csa(f3, twos[q], twos[q], t6, t7);
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
        if (kWaves > 1)
            __builtin_amdgcn_s_barrier();
    }

    // stage: lds[b][2*wl + half] = low / high dword of plane b of word wl of the group
#pragma unroll
    for (int q = 0; q < kSlices; ++q) {
        const int at = lane * kSlices + q;
        lds[0][at] = ones[q];
        lds[1][at] = twos[q];
        lds[2][at] = fours[q];
        lds[3][at] = eights[q];
#pragma unroll
        for (int b = 0; b < kPlanes - 4; ++b)
            lds[4 + b][at] = hi[b][q];
    }
    __syncthreads();

    const bool vec_x = !kApply || is_aligned(p.x, 16);
    const bool vec_c = !kCounts || is_aligned(p.counts, 8);
    // now lane l owns coordinates 4*(l&15).. of word 4*s + (l>>4), s = 0..kSlicedWords/4-1
#pragma unroll 2
    for (int s = 0; s < kSlicedWords / kWordsPerSub; ++s) {
        const int wl = s * kWordsPerSub + (lane >> 4);          // word within the group
        const int64_t j0 = (w0 + wl) * 64 + (lane & 15) * kVec;
        if (j0 >= p.numel)
            continue;
        const int dword = 2 * wl + ((lane >> 3) & 1);
        const int shift = (lane & 7) * 4;
        // byte k of lo / hi collects bits 0..7 / 8..15 of the count of coordinate j0 + k
        uint32_t lo = 0, up = 0;
#pragma unroll
        for (int b = 0; b < kPlanes; ++b) {
            const uint32_t bytes = nibble_to_bytes((lds[b][dword] >> shift) & 0xFu);
            if (b < 8)
                lo += bytes << b;
            else
                up += bytes << (b - 8);
        }
        uint32_t cnt[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            cnt[k] = ((lo >> (8 * k)) & 0xFFu) | (kPlanes > 8 ? ((up >> (8 * k)) & 0xFFu) << 8 : 0u);
        const bool full = j0 + kVec <= p.numel;
        if (kApply) {
            if (full && vec_x) {
                f32x4 xv = X_LOAD(reinterpret_cast<const f32x4 *>(p.x + j0));
                xv.x = lion_apply(xv.x, aggregate_votes(cnt[0], h), h);
                xv.y = lion_apply(xv.y, aggregate_votes(cnt[1], h), h);
                xv.z = lion_apply(xv.z, aggregate_votes(cnt[2], h), h);
                xv.w = lion_apply(xv.w, aggregate_votes(cnt[3], h), h);
                X_STORE(xv, reinterpret_cast<f32x4 *>(p.x + j0));
            } else {
#pragma unroll
                for (int k = 0; k < kVec; ++k)
                    if (j0 + k < p.numel)
                        p.x[j0 + k] = lion_apply(p.x[j0 + k], aggregate_votes(cnt[k], h), h);
            }
        }
        if (kCounts) {
            if (full && vec_c) {
                u16x4 c;
                c.x = static_cast<uint16_t>(cnt[0]);
                c.y = static_cast<uint16_t>(cnt[1]);
                c.z = static_cast<uint16_t>(cnt[2]);
                c.w = static_cast<uint16_t>(cnt[3]);
                C_STORE(c, reinterpret_cast<u16x4 *>(p.counts + j0));
            } else {
#pragma unroll
                for (int k = 0; k < kVec; ++k)
                    if (j0 + k < p.numel)
                        p.counts[j0 + k] = static_cast<uint16_t>(cnt[k]);
            }
        }
    }
}

// ---------------------------------------------------------------- apply from counts
template <class Addr>
__global__ __launch_bounds__(kBlock) void apply_kernel(Addr addr, Hyper h)
{
    const int64_t tile = wave_tile_index();
    if (tile >= addr.total_tiles)
        return;
    const int lane = threadIdx.x & 63;
    Problem p;
    const int64_t t = addr.resolve(tile, p) * kSubs;
    const bool aligned = is_aligned(p.x, 16) && is_aligned(p.counts, 8);
#pragma unroll 1
    for (int r = 0; r < kSubs; ++r) {
        const int64_t sub = t + r;
        if (sub * kSubTile >= p.numel)
            break;
        if (aligned && (sub + 1) * kSubTile <= p.numel) {
            const int64_t j0 = sub * kSubTile + lane * kVec;
            const u16x4 c = C_LOAD(reinterpret_cast<const u16x4 *>(p.counts + j0));
            f32x4 xv = X_LOAD(reinterpret_cast<const f32x4 *>(p.x + j0));
            xv.x = lion_apply(xv.x, aggregate_votes(c.x, h), h);
            xv.y = lion_apply(xv.y, aggregate_votes(c.y, h), h);
            xv.z = lion_apply(xv.z, aggregate_votes(c.z, h), h);
            xv.w = lion_apply(xv.w, aggregate_votes(c.w, h), h);
            X_STORE(xv, reinterpret_cast<f32x4 *>(p.x + j0));
        } else {
#pragma unroll 1
            for (int k = 0; k < kWordsPerSub; ++k) {
                const int64_t j = (sub * kWordsPerSub + k) * 64 + lane;
                if (j < p.numel)
                    p.x[j] = lion_apply(p.x[j], aggregate_votes(p.counts[j], h), h);
            }
        }
    }
}

}  // namespace dlion
