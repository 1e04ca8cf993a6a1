// Group-sync kernels for gfx950: the local SGD update of every worker fused
// with the parameter average inside each group and the write-back of the mean
// to every member (Listing 1: optimizer.step() then Average(model, group);
// Sec. III-A step 4; Sec. IV-B2: X_{k+1} = W_k X_k, w_ij = 1/|group|).
//
// The step is a streaming reduction over the worker axis: 8 (or 6) bytes are
// read and 4 written per (worker, column) and about one FMA is spent on them,
// so the kernel is bound by HBM bandwidth and uses no matrix cores.  Mapping:
//   - a workgroup is ONE wavefront and owns a tile of 256 consecutive columns
//     of ONE group; blockIdx.y is the group, blockIdx.x the tile, so
//     consecutive workgroups walk each member row sequentially and the tiles
//     in flight form one contiguous window of every row;
//   - a lane owns one vector of 4 consecutive columns, so every load/store
//     instruction covers 1 KiB of one row (128-bit per lane, fully coalesced).
//     Wider tiles (2, 4 or 8 vectors per lane) measured 2-20 % slower at every
//     group size once the occupancy cap follows the bytes in flight;
//   - member rows are uniform across the wavefront: their indices come from
//     the kernel-argument block through scalar loads (which have their own
//     wait counter, so fetching an index never waits for data loads), and the
//     row base addresses live in scalar registers;
//   - members are accumulated 8 at a time, i.e. a round issues up to 16 loads
//     of 1 KiB per wavefront; interior tiles run a predicate-free body (a load
//     guarded by a lane predicate gets its own basic block and is waited on
//     before the next one is issued).  As compiled, the loads of a round do
//     not all leave at once: each member's row index is a scalar load that is
//     waited for before its two vector loads, and the first sums are taken
//     while the last loads are still being issued, so about ten loads per
//     wavefront are in flight at a time and the stores trail one another by a
//     scalar lookup each.  That pacing was checked against explicit schedules
//     (all 16 loads back to back, sliding windows of 2..8 member pairs,
//     stores spaced by 0..16 sleep units): the best of them (window of 5
//     pairs, stores 2 units apart) is within 0.5 % of this code, back-to-back
//     issue is 3-4 % slower;
//   - the reduction over members is sequential inside a lane (no cross-lane
//     traffic is needed: a column never leaves its lane), one mean is formed
//     per column and stored |group| times, so members end bit-identical;
//   - loads and stores carry the non-temporal hint: every byte is touched
//     exactly once per step;
//   - the launch asks for dynamic LDS that the kernel never touches.  Its
//     only purpose is to cap the number of wavefronts per CU (occupancy_pad
//     below): measured on MI355X, the memory system sustains most when about
//     80 KiB of loads are in flight per CU - five wavefronts per CU for groups
//     of 8 (6.3-6.6 TB/s on this 2:1 read/write mix; full occupancy gives
//     5.4-5.7, two wavefronts per CU 4.4), ten for groups of 4, twenty for
//     pairs;
//   - rows that start on 1-KiB boundaries (ds_padded_ld) make every 1-KiB
//     access one aligned KiB of its row: 2-5 % faster than other 256-byte
//     alignments.
// Also measured and not adopted, all on the 32 x 25.6 M fp32 stacks: persistent
// wavefronts that prefetch the next tile while the current one is reduced and
// stored (5.0-5.5 TB/s: on this target one counter orders loads and stores, so
// waiting for a tile's loads also waits for the previous tile's stores),
// XCD-aware tile orders in runs of 2..64 tiles per XCD (2-12 % slower than the
// plain order, in which the tiles in flight form one contiguous window of every
// row), and the other cache-policy bits on loads and stores (sc0, sc1 with or
// without nt: at best equal to the plain non-temporal hint, without it 10-15 %
// slower).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <utility>
#include <vector>

#include "ds_internal.h"
#include "launch.h"

namespace {

using ds::kPlanTileCols;
using ds::kSyncLoadsPerLane;
using ds::kSyncTileCols;
using ds::kSyncThreads;
using ds::PartitionArg;
using ds::PlanHeader;
using ds::Tile;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Occupancy cap.  The launch requests dynamic LDS that the kernel never touches, so
// that only floor(LDS per CU / request) one-wavefront workgroups fit a CU (160 KiB
// on MI355X; the figure is read from the device).  The
// number aimed for keeps about 80 KiB of first-round loads in flight per CU
// (with bf16 gradients 60 KiB for pairs rising to 72 KiB for groups of 8):
// measured on MI355X over group sizes 1..8, fp32 and bf16 gradients, with and
// without the momentum and SWA buffers, the best cap was within 3.5 % of this
// rule everywhere (e.g. 16 KiB per wavefront -> 5 per CU, 8 KiB -> 10,
// 4 KiB -> 20, 24 KiB -> 3).
constexpr unsigned kLdsGranule = 2048;
constexpr int kInFlightHalfKiB = 160;        // fp32 gradients
constexpr int kInFlightHalfKiBBf16 = 112;    // bf16 gradients: this plus 4 per member of a round ...
constexpr int kInFlightHalfKiBBf16V = 144;   // ... or this with the momentum buffer
constexpr int kMinWavesPerCu = 3;
constexpr int kUncappedWavesPerCu = 26;      // from here on the register file is the limit anyway
constexpr int kUncappedWorkgroupsPerCu = 32;   // a launch of up to this many per CU fits the chip in one go

template <typename V>
__device__ __forceinline__ V stream_load(const V* p) { return __builtin_nontemporal_load(p); }
template <typename V>
__device__ __forceinline__ void stream_store(V v, V* p) { __builtin_nontemporal_store(v, p); }

// Entry i of a packed byte table in the kernel-argument block; i is
// wavefront-uniform, so this is a scalar load plus scalar bit arithmetic.
__device__ __forceinline__ int packed_byte(const uint32_t* words, int i) {
    return static_cast<int>((words[i >> 2] >> ((i & 3) * 8)) & 0xffu);
}

__device__ __forceinline__ float bits_to_f32(uint32_t u) { return __builtin_bit_cast(float, u); }

// four consecutive gradient elements, widened to fp32
__device__ __forceinline__ f32x4 load_grad4(const float* p) {
    return stream_load(reinterpret_cast<const f32x4*>(p));
}
__device__ __forceinline__ f32x4 load_grad4(const uint16_t* p) {
    const u32x2 raw = stream_load(reinterpret_cast<const u32x2*>(p));
    f32x4 v;
    v.x = bits_to_f32(raw.x << 16);          // bf16 is the upper half of an fp32
    v.y = bits_to_f32(raw.x & 0xffff0000u);
    v.z = bits_to_f32(raw.y << 16);
    v.w = bits_to_f32(raw.y & 0xffff0000u);
    return v;
}
__device__ __forceinline__ float load_grad1(const float* p) { return *p; }
__device__ __forceinline__ float load_grad1(const uint16_t* p) {
    return bits_to_f32(static_cast<uint32_t>(*p) << 16);
}

// Optional per-worker state of the fuller local step (Listing 1; Sec. V-A3):
// momentum buffers V (never averaged: only the model is handed to Average) and
// SWA models S.  tile-relative pointers, NULL-free when the matching flag is set.
struct Extras {
    float* v;
    float* s;
    int64_t ldv, lds;       // row strides
    int64_t tsv, tss;       // tile strides (tiled stacks only; see TileWalk)
    float momentum, weight_decay, factor;
};

// Tiled stacks (kTiled instances of the kernels): the W pieces of a 256-column
// tile are one contiguous block, so tile t of a stack is at base + t * tile
// stride (>= W*256) and the row stride handed on to sync_tile is 256.  The grid
// is 1-D, tiles * groups with the group running fastest (tile_major = number of
// groups), so that consecutive workgroups walk the blocks front to back.  The
// row-major instances never read this argument: their tile t is at column
// 256 * t of every row and their grid is (tiles, groups), whose consecutive
// workgroups walk the rows of one group.
struct TileWalk {
    int64_t tsx, tsg;
    int32_t tile_major;
};

// Adds the locally updated parameters of kCount members (perm positions
// q .. q+kCount-1) to the lane's column sums.  Plain step: y = x - lr*g.
// With kOpt: d = g + weight_decay*x; kHasV: v' = momentum*v + d is stored back
// and y = x - lr*v', else y = x - lr*d.  The loads of the first kAhead members
// come first in program order (with kFull nothing is predicated, so they sit in
// one basic block); the loads of member j + kAhead follow the arithmetic of
// member j.  kAhead = kCount (everything first, order of use left to the
// compiler) except for rounds of 4 members with fp32 gradients, where a window
// of 2 members in flight measured 1-2 % faster (groups of 4 run 10 wavefronts
// per CU, and the staggered issue suits that better than bursts of 8 loads).
// With bf16 gradients the same window measured 5 % slower, and for rounds of 8
// every window from 2 to 8 members measured equal or slower than the compiler's
// own order (7 loads, a wait for the first two, 9 loads).
template <typename GT, int kCount, bool kFull, bool kOpt, bool kHasV>
__device__ __forceinline__ void add_members(f32x4& sum, const float* xt, const GT* gt, int64_t ldx, int64_t ldg,
                                            const Extras& ex, const PartitionArg& part, int q, int col, bool live,
                                            float lr) {
    constexpr int kAhead = (kCount == 4 && kFull && sizeof(GT) == 4 && !kHasV) ? 2 : kCount;
    f32x4 x[kCount], g[kCount], mv[kHasV ? kCount : 1];
#pragma unroll
    for (int j = 0; j < kAhead; ++j) {
        const int64_t row = packed_byte(part.perm, q + j);
        if (kFull || live) {
            x[j] = stream_load(reinterpret_cast<const f32x4*>(xt + row * ldx + col));
            g[j] = load_grad4(gt + row * ldg + col);
            if (kHasV) mv[j] = stream_load(reinterpret_cast<const f32x4*>(ex.v + row * ex.ldv + col));
        }
    }
    if (kAhead < kCount) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < kCount; ++j) {
        const int64_t row = kHasV ? packed_byte(part.perm, q + j) : 0;
        if (kFull || live) {
            if (!kOpt) {
                sum += x[j] - lr * g[j];
            } else {
                f32x4 d = g[j] + ex.weight_decay * x[j];
                if (kHasV) {
                    d = ex.momentum * mv[j] + d;
                    stream_store(d, reinterpret_cast<f32x4*>(ex.v + row * ex.ldv + col));
                }
                sum += x[j] - lr * d;
            }
        }
        if (j + kAhead < kCount) {
            // kAhead < kCount implies kFull: nothing is predicated here
            const int64_t next = packed_byte(part.perm, q + j + kAhead);
            x[j + kAhead] = stream_load(reinterpret_cast<const f32x4*>(xt + next * ldx + col));
            g[j + kAhead] = load_grad4(gt + next * ldg + col);
            if (kHasV) mv[j + kAhead] = stream_load(reinterpret_cast<const f32x4*>(ex.v + next * ex.ldv + col));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Writes the mean to kCount members; with kHasS also moves their SWA models:
// s' = factor*s + (1-factor)*mean (the S loads are issued together first).
template <int kCount, bool kFull, bool kHasS>
__device__ __forceinline__ void store_members(const f32x4& mean, float* xt, int64_t ldx, const Extras& ex,
                                              const PartitionArg& part, int q, int col, bool live) {
    f32x4 s[kHasS ? kCount : 1];
    if (kHasS) {
#pragma unroll
        for (int j = 0; j < kCount; ++j) {
            const int64_t row = packed_byte(part.perm, q + j);
            if (kFull || live) s[j] = stream_load(reinterpret_cast<const f32x4*>(ex.s + row * ex.lds + col));
        }
    }
#pragma unroll
    for (int j = 0; j < kCount; ++j) {
        const int64_t row = packed_byte(part.perm, q + j);
        if (kFull || live) {
            stream_store(mean, reinterpret_cast<f32x4*>(xt + row * ldx + col));
            if (kHasS) {
                const f32x4 moved = ex.factor * s[j] + (1.0f - ex.factor) * mean;
                stream_store(moved, reinterpret_cast<f32x4*>(ex.s + row * ex.lds + col));
            }
        }
    }
}

// One tile of one group.  kFull: the tile has all kSyncTileCols columns.
// mean_out receives the lane's four column means (zeros for a lane beyond the
// tile), tail_out the mean of the single column a lane handles at a ragged end
// (zero for every other lane): what the fused consensus needs.
template <typename GT, bool kFull, bool kOpt, bool kHasV, bool kHasS>
__device__ __forceinline__ void sync_tile(float* xt, const GT* gt, int len, int64_t ldx, int64_t ldg,
                                          const Extras& ex, const PartitionArg& part, int first, int n, float lr,
                                          f32x4& mean_out, float& tail_out) {
    constexpr int kChunk = kSyncLoadsPerLane / 2;   // members per round of loads
    const int lane = static_cast<int>(threadIdx.x) & (kSyncThreads - 1);
    const int col = lane * 4;
    const bool live = kFull || col + 4 <= len;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    int q = first;
    const int end = first + n;
    for (; q + kChunk <= end; q += kChunk)
        add_members<GT, kChunk, kFull, kOpt, kHasV>(sum, xt, gt, ldx, ldg, ex, part, q, col, live, lr);
    // remaining members (fewer than kChunk): one specialised, branch-free body each
    switch (end - q) {
#define DS_REST(k) \
    case k: add_members<GT, k, kFull, kOpt, kHasV>(sum, xt, gt, ldx, ldg, ex, part, q, col, live, lr); break;
        DS_REST(1) DS_REST(2) DS_REST(3) DS_REST(4) DS_REST(5) DS_REST(6) DS_REST(7)
#undef DS_REST
        default: break;
    }
    static_assert(kChunk == 8, "the remainder switch lists 1..7 members");
    const float nf = static_cast<float>(n);
    sum = sum / nf;
    mean_out = sum;
    tail_out = 0.f;
    if (!kHasS) {
        for (int m = first; m < end; ++m) store_members<1, kFull, false>(sum, xt, ldx, ex, part, m, col, live);
    } else {
        int m = first;
        for (; m + kChunk <= end; m += kChunk) store_members<kChunk, kFull, true>(sum, xt, ldx, ex, part, m, col, live);
        for (; m < end; ++m) store_members<1, kFull, true>(sum, xt, ldx, ex, part, m, col, live);
    }
    if (!kFull) {
        // ragged end of the tile: fewer than 4 columns, one lane each
        const int c = (len & ~3) + lane;
        if (lane < 3 && c < len) {
            float acc = 0.f;
            for (int m = first; m < end; ++m) {
                const int64_t row = packed_byte(part.perm, m);
                const float x = xt[row * ldx + c];
                float d = load_grad1(gt + row * ldg + c);
                if (kOpt) {
                    d = d + ex.weight_decay * x;
                    if (kHasV) {
                        d = ex.momentum * ex.v[row * ex.ldv + c] + d;
                        ex.v[row * ex.ldv + c] = d;
                    }
                }
                acc += x - lr * d;
            }
            acc = acc / nf;
            tail_out = acc;
            for (int m = first; m < end; ++m) {
                const int64_t row = packed_byte(part.perm, m);
                xt[row * ldx + c] = acc;
                if (kHasS) ex.s[row * ex.lds + c] = ex.factor * ex.s[row * ex.lds + c] + (1.0f - ex.factor) * acc;
            }
        }
    }
}

template <typename GT, bool kRagged, bool kTiled, bool kOpt, bool kHasV, bool kHasS>
__global__ void __launch_bounds__(kSyncThreads)
group_sync_kernel(float* __restrict__ X, const GT* __restrict__ G, int64_t ldx, int64_t ldg,
                  int64_t P, const Tile* __restrict__ tiles, uint64_t plan_id, int32_t plan_entries,
                  PartitionArg part, float lr, Extras ex, TileWalk walk) {
    static_assert(kOpt || (!kHasV && !kHasS), "extra state implies the extended step");
    static_assert(!(kRagged && kTiled), "segment lists address row-major stacks");
    constexpr int kTileCols = kSyncTileCols;
    uint32_t tile_id = blockIdx.x, group_id = blockIdx.y;
    if (kTiled) {
        group_id = blockIdx.x % static_cast<uint32_t>(walk.tile_major);
        tile_id = blockIdx.x / static_cast<uint32_t>(walk.tile_major);
    }
    int64_t start;
    int32_t len;
    if (kRagged) {
        // a plan entry covers up to kPlanTileCols columns: kSub workgroups share it
        constexpr uint32_t kSub = kPlanTileCols / kTileCols;
        // Entry 0 says which plan this is: a buffer that holds another plan (or none) is left alone.
        // The header and this workgroup's entry are fetched together and judged afterwards (one wait
        // for memory instead of one per check): the entry lies inside the buffer whatever it holds,
        // because the host sized the grid and checked the buffer's size against the same list.
        const PlanHeader hd = *reinterpret_cast<const PlanHeader*>(tiles);
        const Tile tl = tiles[1 + tile_id / kSub];
        const int32_t done = static_cast<int32_t>(tile_id % kSub) * kTileCols;
        // a table that does not belong to these stacks must not become a wild access
        int64_t ld_min = ldx < ldg ? ldx : ldg;
        if (kHasV && ex.ldv < ld_min) ld_min = ex.ldv;
        if (kHasS && ex.lds < ld_min) ld_min = ex.lds;
        bool ok = (hd.id == plan_id) & (hd.n_entries == plan_entries);
        ok &= (tl.start >= 0) & ((tl.start & 7) == 0) & (tl.len >= 0) & (tl.len <= kPlanTileCols);
        ok &= (tl.start <= ld_min - tl.len) & (done < tl.len);
        if (!ok) return;
        start = tl.start + done;
        len = tl.len - done < kTileCols ? tl.len - done : kTileCols;
    } else {
        start = static_cast<int64_t>(tile_id) * kTileCols;
        const int64_t left = P - start;
        len = left < kTileCols ? static_cast<int32_t>(left) : kTileCols;
    }
    float* xt;
    const GT* gt;
    if (!kTiled) {
        xt = X + start;
        gt = G + start;
        if (kHasV) ex.v += start;
        if (kHasS) ex.s += start;
    } else {
        xt = X + static_cast<int64_t>(tile_id) * walk.tsx;
        gt = G + static_cast<int64_t>(tile_id) * walk.tsg;
        if (kHasV) ex.v += static_cast<int64_t>(tile_id) * ex.tsv;
        if (kHasS) ex.s += static_cast<int64_t>(tile_id) * ex.tss;
    }
    const int first = packed_byte(part.off, static_cast<int>(group_id));
    const int n = packed_byte(part.off, static_cast<int>(group_id) + 1) - first;
    f32x4 mean;
    float tail;
    if (len == kTileCols)
        sync_tile<GT, true, kOpt, kHasV, kHasS>(xt, gt, len, ldx, ldg, ex, part, first, n, lr, mean, tail);
    else
        sync_tile<GT, false, kOpt, kHasV, kHasS>(xt, gt, len, ldx, ldg, ex, part, first, n, lr, mean, tail);
}

// ---------------------------------------------------------------- step and consensus norms in one pass
//
// Right after a step every member of a group holds the group's mean, so the
// consensus norms (Sec. IV-B2, left side of Lemma 1) follow from the means the
// step has in registers anyway: with m_k the mean of group k and n_k its size,
//     xbar[p] = (1/W) sum_k n_k m_k[p],    d_i = || m_{g(i)} - xbar ||_2 .
// A wavefront owns a tile of 256 columns of ALL groups: it takes the step group
// after group exactly as above, parks each group's means in LDS (each lane
// reads back only what it wrote, so no barrier is needed), then forms xbar per
// column in fp64, splits it into an fp32 pair and sums ((m_k - hi) - lo)^2 over
// its columns - the arithmetic of the consensus kernel - reduces that across
// the lanes in fp64 and writes one partial sum per (group, tile).  A second,
// small kernel adds the partial sums of each group in a fixed order, takes the
// square root and hands the norm to every member.  The replica stack is not
// read a second time.
// What it costs: a wavefront takes its groups one after the other, each a round
// of loads, the arithmetic and a round of stores, and the loads of the next
// group queue behind those stores in the in-order memory counter.  At best
// 5.3-5.4 TB/s (3 to 5 wavefronts per CU) against 6.4 for the plain step on
// 32 x 25.6 M fp32 stacks.  The number of row streams open at once (2W in this
// tile-major walk against 2|g| in the group-major step) is not what holds it
// back: on tiled stacks, where the walk reads two sequential streams, it runs
// at the same 5.4 TB/s.  Also measured: the loads of group k+1 issued ahead of
// the stores of group k (no gain, 200 registers), and one wavefront per group
// in a workgroup that exchanges the means behind a barrier (30 % slower: the
// wavefronts of a workgroup move in lock step).  The fused pass therefore pays
// where launches and latency dominate (stacks that fit the last-level cache);
// on large stacks the plain step followed by ds_consensus_grouped is faster.
constexpr int kFusedLdsPerGroup = kSyncThreads * (16 + 4);   // bytes: a 4-vector and a tail value per lane

template <typename GT>
__global__ void __launch_bounds__(kSyncThreads)
group_sync_consensus_kernel(float* __restrict__ X, const GT* __restrict__ G, int64_t ldx, int64_t ldg, int64_t P,
                            PartitionArg part, int n_groups, int n_workers, float lr, int64_t n_tiles,
                            double* __restrict__ partial, TileWalk walk) {
    extern __shared__ __align__(16) unsigned char lds_raw[];
    f32x4* means = reinterpret_cast<f32x4*>(lds_raw);
    float* tails = reinterpret_cast<float*>(means + static_cast<size_t>(n_groups) * kSyncThreads);
    const int lane = static_cast<int>(threadIdx.x);
    const int64_t tile_id = blockIdx.x;
    const int64_t start = tile_id * kSyncTileCols;
    const int64_t left = P - start;
    const int len = left < kSyncTileCols ? static_cast<int>(left) : kSyncTileCols;
    const Extras none = {nullptr, nullptr, 0, 0, 0, 0, 0.f, 0.f, 0.f};
    float* xt = X + tile_id * walk.tsx;
    const GT* gt = G + tile_id * walk.tsg;
    for (int k = 0; k < n_groups; ++k) {
        const int first = packed_byte(part.off, k);
        const int n = packed_byte(part.off, k + 1) - first;
        f32x4 mean;
        float tail;
        if (len == kSyncTileCols)
            sync_tile<GT, true, false, false, false>(xt, gt, len, ldx, ldg, none, part, first, n, lr, mean, tail);
        else
            sync_tile<GT, false, false, false, false>(xt, gt, len, ldx, ldg, none, part, first, n, lr, mean, tail);
        means[k * kSyncThreads + lane] = mean;
        tails[k * kSyncThreads + lane] = tail;
    }
    // column means over all workers, fp64: the 4 vector columns and the tail column of this lane
    double xbar[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
    for (int k = 0; k < n_groups; ++k) {
        const double w = static_cast<double>(packed_byte(part.off, k + 1) - packed_byte(part.off, k));
        const f32x4 m = means[k * kSyncThreads + lane];
#pragma unroll
        for (int e = 0; e < 4; ++e) xbar[e] += w * static_cast<double>(m[e]);
        xbar[4] += w * static_cast<double>(tails[k * kSyncThreads + lane]);
    }
    float hi[5], lo[5];
#pragma unroll
    for (int e = 0; e < 5; ++e) {
        const double m = xbar[e] / static_cast<double>(n_workers);
        hi[e] = static_cast<float>(m);
        lo[e] = static_cast<float>(m - static_cast<double>(hi[e]));
    }
    for (int k = 0; k < n_groups; ++k) {
        const f32x4 m = means[k * kSyncThreads + lane];
        float sq = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float d = (m[e] - hi[e]) - lo[e];
            sq = __builtin_fmaf(d, d, sq);
        }
        const float dt = (tails[k * kSyncThreads + lane] - hi[4]) - lo[4];
        sq = __builtin_fmaf(dt, dt, sq);
        double v = static_cast<double>(sq);
#pragma unroll
        for (int mask = 32; mask >= 1; mask >>= 1) v += __shfl_xor(v, mask, 64);
        if (lane == 0) partial[static_cast<int64_t>(k) * n_tiles + tile_id] = v;
    }
}

constexpr int kNormThreads = 256;

// One workgroup per group: fixed-order sum of the group's partial sums, square
// root, and the norm goes to every member of the group.
__global__ void __launch_bounds__(kNormThreads)
group_norm_kernel(const double* __restrict__ partial, int64_t n_tiles, PartitionArg part, double* __restrict__ out) {
    __shared__ double buf[kNormThreads];
    const int k = static_cast<int>(blockIdx.x);
    const double* mine = partial + static_cast<int64_t>(k) * n_tiles;
    double v = 0.0;
    for (int64_t t = threadIdx.x; t < n_tiles; t += kNormThreads) v += mine[t];
    buf[threadIdx.x] = v;
    __syncthreads();
    for (int half = kNormThreads / 2; half >= 1; half >>= 1) {
        if (static_cast<int>(threadIdx.x) < half) buf[threadIdx.x] += buf[threadIdx.x + half];
        __syncthreads();
    }
    const int first = packed_byte(part.off, k);
    const int n = packed_byte(part.off, k + 1) - first;
    if (static_cast<int>(threadIdx.x) < n) out[packed_byte(part.perm, first + static_cast<int>(threadIdx.x))] = sqrt(buf[0]);
}

// ---------------------------------------------------------------- ragged plan

// Segments handed to one launch of the plan kernel, inside its kernel-argument
// block: the table is written on the device from arguments alone, so building
// a plan needs no host-to-device copy and no wait.
constexpr int kPlanBatch = 96;
struct PlanBatch {
    int64_t offset[kPlanBatch];
    int64_t length[kPlanBatch];
    int64_t first_entry[kPlanBatch];   // position of the segment's first entry among all entries
    int32_t count;
    int32_t with_header;               // this launch also writes entry 0
    PlanHeader header;
};
constexpr int kPlanThreads = 256;

// One workgroup per segment of the batch: entry k of the segment covers its
// columns k*kPlanTileCols .. and is written by thread k mod 256.
__global__ void __launch_bounds__(kPlanThreads) plan_fill_kernel(Tile* __restrict__ plan, PlanBatch b) {
    const int s = static_cast<int>(blockIdx.x);
    if (b.with_header && s == 0 && threadIdx.x == 0) *reinterpret_cast<PlanHeader*>(plan) = b.header;
    const int64_t off = b.offset[s], len = b.length[s];
    const int64_t n = (len + kPlanTileCols - 1) / kPlanTileCols;
    Tile* out = plan + 1 + b.first_entry[s];
    for (int64_t k = threadIdx.x; k < n; k += kPlanThreads) {
        const int64_t done = k * kPlanTileCols;
        const int64_t left = len - done;
        Tile tl;
        tl.start = off + done;
        tl.len = static_cast<int32_t>(left < kPlanTileCols ? left : kPlanTileCols);
        tl.pad = 0;
        out[k] = tl;
    }
}

struct SegmentScan {
    int status;
    int64_t n_entries;     // plan entries (runs of up to kPlanTileCols columns)
    int64_t n_live_tiles;  // workgroups that find columns to process
    int64_t end;           // one past the last column of any segment
    uint64_t id;           // identity of the list: 0 if it has no columns
};

inline uint64_t fold(uint64_t h, uint64_t word) {
    h = (h ^ word) * 0x100000001B3ull;   // FNV-1a step on a whole word ...
    return h ^ (h >> 29);                // ... with the high bits folded back
}

// Validates a segment list, counts the entries it is cut into and fingerprints it.
SegmentScan scan_segments(const ds_segment* segs, int32_t S, int64_t ldx, int64_t ldg, bool have_ld) {
    SegmentScan sc = {DS_OK, 0, 0, 0, 0};
    if (S < 0) return {DS_ERR_BAD_SHAPE, 0, 0, 0, 0};
    if (S > 0 && !segs) return {DS_ERR_NULL, 0, 0, 0, 0};
    uint64_t h = fold(0xCBF29CE484222325ull, static_cast<uint64_t>(S));
    for (int32_t s = 0; s < S; ++s) {
        const int64_t o = segs[s].offset, l = segs[s].length;
        if (o < 0 || l < 0 || l > INT64_MAX - o) return {DS_ERR_BAD_SHAPE, 0, 0, 0, 0};
        if (o % 8 != 0) return {DS_ERR_ALIGN, 0, 0, 0, 0};
        if (have_ld && (o + l > ldx || o + l > ldg)) return {DS_ERR_BAD_SHAPE, 0, 0, 0, 0};
        // bounded before it is added, so the sums below cannot overflow
        if (l > DS_MAX_COLUMNS) return {DS_ERR_BAD_SHAPE, 0, 0, 0, 0};
        sc.n_entries += (l + kPlanTileCols - 1) / kPlanTileCols;
        sc.n_live_tiles += (l + kSyncTileCols - 1) / kSyncTileCols;
        // every entry is launched as kPlanTileCols / kSyncTileCols workgroups along x
        if (sc.n_entries * (kPlanTileCols / kSyncTileCols) > ds::kMaxSyncGridX) return {DS_ERR_BAD_SHAPE, 0, 0, 0, 0};
        if (o + l > sc.end) sc.end = o + l;
        h = fold(fold(h, static_cast<uint64_t>(o)), static_cast<uint64_t>(l));
    }
    sc.id = sc.n_entries == 0 ? 0 : (h != 0 ? h : 1);
    return sc;
}

// Pairwise disjointness of the non-empty segments (sort by offset, compare
// neighbours).  DS_OK, DS_ERR_BAD_SHAPE for an overlap, DS_ERR_HOST_MEMORY.
int check_disjoint(const ds_segment* segs, int32_t S) {
    try {
        std::vector<std::pair<int64_t, int64_t>> v;
        v.reserve(static_cast<size_t>(S));
        for (int32_t s = 0; s < S; ++s)
            if (segs[s].length > 0) v.emplace_back(segs[s].offset, segs[s].offset + segs[s].length);
        std::sort(v.begin(), v.end());
        for (size_t i = 1; i < v.size(); ++i)
            if (v[i].first < v[i - 1].second) return DS_ERR_BAD_SHAPE;
    } catch (...) {
        return DS_ERR_HOST_MEMORY;
    }
    return DS_OK;
}

// ---------------------------------------------------------------- launch

int check_stacks(const void* X, const void* G, int32_t g_dtype, int64_t ldx, int64_t ldg) {
    if (!X || !G) return DS_ERR_NULL;
    if (g_dtype != DS_F32 && g_dtype != DS_BF16) return DS_ERR_DTYPE;
    if (ldx < 0 || ldg < 0) return DS_ERR_BAD_SHAPE;
    if (!ds::aligned16(X) || !ds::aligned16(G) || ldx % 4 != 0 || ldg % 4 != 0) return DS_ERR_ALIGN;
    return DS_OK;
}

// Dynamic LDS request (bytes) for a division whose largest group has `largest`
// members.  A round loads min(largest, 8) members, each 1 KiB of x, 1 KiB (fp32)
// or 0.5 KiB (bf16) of g and, with momentum, 1 KiB of v per wavefront; the SWA
// rows are loaded in a later round and do not count.  n_workgroups counts the
// workgroups that have columns to process.
unsigned occupancy_pad(int32_t largest, bool bf16, bool has_v, int64_t n_workgroups, const ds::DeviceInfo& dev) {
    // a launch that fits the chip in one go (cache-resident, latency-bound) is better off uncapped
    if (n_workgroups <= static_cast<int64_t>(dev.compute_units) * kUncappedWorkgroupsPerCu) return 0;
    const int round = largest < kSyncLoadsPerLane / 2 ? largest : kSyncLoadsPerLane / 2;
    const int half_kib = round * (2 + (bf16 ? 1 : 2) + (has_v ? 2 : 0));
    const int target = !bf16 ? kInFlightHalfKiB : has_v ? kInFlightHalfKiBBf16V : kInFlightHalfKiBBf16 + 4 * round;
    int waves = target / half_kib;
    if (waves < kMinWavesPerCu) waves = kMinWavesPerCu;
    if (waves >= kUncappedWavesPerCu) return 0;
    return dev.lds_per_cu / static_cast<unsigned>(waves) / kLdsGranule * kLdsGranule;
}

// What a launch needs beyond the stacks.
struct LaunchShape {
    int64_t P;               // flat: columns
    const Tile* plan;        // ragged: plan buffer (header + entries), else NULL
    uint64_t plan_id;
    int64_t plan_entries;
    int64_t n_live_tiles;    // workgroups along x that find columns
    int32_t largest;         // largest group
    int32_t n_groups;
    TileWalk walk;           // flat: where the tiles are and in which order they are walked
};

template <typename GT, bool kRagged, bool kTiled, bool kOpt, bool kHasV, bool kHasS>
int launch_one(float* X, const GT* G, int64_t ldx, int64_t ldg, const LaunchShape& sh, const PartitionArg& part,
               float lr, const Extras& ex, hipStream_t st) {
    ds::DeviceInfo dev;
    const int rc = ds::device_info(&dev);
    if (rc != DS_OK) return rc;
    const int64_t grid_x = kRagged ? sh.plan_entries * (kPlanTileCols / kSyncTileCols)
                                   : (sh.P + kSyncTileCols - 1) / kSyncTileCols;
    const bool tile_major = kTiled;
    const dim3 grid(static_cast<uint32_t>(tile_major ? grid_x * sh.n_groups : grid_x),
                    static_cast<uint32_t>(tile_major ? 1 : sh.n_groups), 1);
    const unsigned lds_pad = occupancy_pad(sh.largest, sizeof(GT) == 2, kHasV, sh.n_live_tiles * sh.n_groups, dev);
    const hipError_t err = ds::launch_kernel(group_sync_kernel<GT, kRagged, kTiled, kOpt, kHasV, kHasS>, grid,
                                             dim3(kSyncThreads, 1, 1), lds_pad, st, X, G, ldx, ldg, sh.P, sh.plan,
                                             sh.plan_id, static_cast<int32_t>(sh.plan_entries), part, lr, ex, sh.walk);
    return err == hipSuccess ? DS_OK : DS_ERR_HIP;
}

template <typename GT, bool kRagged, bool kTiled>
int launch_state(float* X, const GT* G, int64_t ldx, int64_t ldg, const LaunchShape& sh, const PartitionArg& part,
                 float lr, bool opt, const Extras& ex, hipStream_t st) {
    const bool has_v = ex.v != nullptr, has_s = ex.s != nullptr;
    if (!opt) return launch_one<GT, kRagged, kTiled, false, false, false>(X, G, ldx, ldg, sh, part, lr, ex, st);
    if (has_v && has_s) return launch_one<GT, kRagged, kTiled, true, true, true>(X, G, ldx, ldg, sh, part, lr, ex, st);
    if (has_v) return launch_one<GT, kRagged, kTiled, true, true, false>(X, G, ldx, ldg, sh, part, lr, ex, st);
    if (has_s) return launch_one<GT, kRagged, kTiled, true, false, true>(X, G, ldx, ldg, sh, part, lr, ex, st);
    return launch_one<GT, kRagged, kTiled, true, false, false>(X, G, ldx, ldg, sh, part, lr, ex, st);
}

template <bool kRagged, bool kTiled>
int launch(void* X, const void* G, int32_t g_dtype, int64_t ldx, int64_t ldg, const LaunchShape& sh,
           const PartitionArg& part, float lr, bool opt, const Extras& ex, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (g_dtype == DS_F32)
        return launch_state<float, kRagged, kTiled>(static_cast<float*>(X), static_cast<const float*>(G), ldx, ldg, sh, part,
                                            lr, opt, ex, st);
    return launch_state<uint16_t, kRagged, kTiled>(static_cast<float*>(X), static_cast<const uint16_t*>(G), ldx, ldg, sh, part,
                                           lr, opt, ex, st);
}

// Checks the optional state of the extended step and turns it into kernel arguments.
// *opt_out says whether the extended arithmetic is needed at all.
// With tiled stacks ldv / lds are tile strides and min_ld the smallest one allowed.
int read_opt(const ds_local_opt* opt, int64_t min_ld, Extras* ex, bool* opt_out, bool tiled = false) {
    *ex = Extras{nullptr, nullptr, 0, 0, kSyncTileCols, kSyncTileCols, 0.f, 0.f, 0.f};
    *opt_out = false;
    if (!opt) return DS_OK;
    const int64_t unit = tiled ? kSyncTileCols : 4;
    if (opt->V) {
        if (!ds::aligned16(opt->V) || opt->ldv % unit != 0) return DS_ERR_ALIGN;
        if (opt->ldv < min_ld) return DS_ERR_BAD_SHAPE;
        ex->v = static_cast<float*>(opt->V);
        ex->ldv = tiled ? kSyncTileCols : opt->ldv;
        ex->tsv = tiled ? opt->ldv : kSyncTileCols;
        ex->momentum = opt->momentum;
    }
    if (opt->S) {
        if (!ds::aligned16(opt->S) || opt->lds % unit != 0) return DS_ERR_ALIGN;
        if (opt->lds < min_ld) return DS_ERR_BAD_SHAPE;
        ex->s = static_cast<float*>(opt->S);
        ex->lds = tiled ? kSyncTileCols : opt->lds;
        ex->tss = tiled ? opt->lds : kSyncTileCols;
        ex->factor = opt->swa_factor;
    }
    ex->weight_decay = opt->weight_decay;
    *opt_out = opt->V || opt->S || opt->weight_decay != 0.f;
    return DS_OK;
}

int group_sync_flat(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx, int64_t ldg, int32_t W,
                    const int32_t* perm, const int32_t* off, int32_t n_groups, float lr, const ds_local_opt* opt,
                    void* stream) {
    int rc = check_stacks(X, G, g_dtype, ldx, ldg);
    if (rc != DS_OK) return rc;
    if (P < 0 || ldx < P || ldg < P || P > DS_MAX_COLUMNS) return DS_ERR_BAD_SHAPE;
    Extras ex;
    bool extended = false;
    rc = read_opt(opt, P, &ex, &extended);
    if (rc != DS_OK) return rc;
    PartitionArg part;
    int32_t max_size = 0;
    rc = ds::pack_partition(W, perm, off, n_groups, &part, &max_size);
    if (rc != DS_OK) return rc;
    if (P == 0) return DS_OK;
    const LaunchShape sh = {P, nullptr, 0, 0, (P + kSyncTileCols - 1) / kSyncTileCols, max_size, n_groups,
                            TileWalk{kSyncTileCols, kSyncTileCols, 0}};
    return launch<false, false>(X, G, g_dtype, ldx, ldg, sh, part, lr, extended, ex, stream);
}

// Tiled stacks: tile strides instead of leading dimensions, tile-major walk.
int check_tiled(const void* X, const void* G, int32_t g_dtype, int64_t P, int64_t tsx, int64_t tsg, int32_t W) {
    if (!X || !G) return DS_ERR_NULL;
    if (g_dtype != DS_F32 && g_dtype != DS_BF16) return DS_ERR_DTYPE;
    if (W < 1 || W > DS_MAX_W) return DS_ERR_BAD_W;
    const int64_t block = static_cast<int64_t>(W) * kSyncTileCols;
    if (P < 0 || P > DS_MAX_COLUMNS || tsx < block || tsg < block) return DS_ERR_BAD_SHAPE;
    if (!ds::aligned16(X) || !ds::aligned16(G) || tsx % kSyncTileCols != 0 || tsg % kSyncTileCols != 0) return DS_ERR_ALIGN;
    return DS_OK;
}

int group_sync_tiled(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t tsx, int64_t tsg, int32_t W,
                     const int32_t* perm, const int32_t* off, int32_t n_groups, float lr, const ds_local_opt* opt,
                     void* stream) {
    int rc = check_tiled(X, G, g_dtype, P, tsx, tsg, W);
    if (rc != DS_OK) return rc;
    Extras ex;
    bool extended = false;
    rc = read_opt(opt, static_cast<int64_t>(W) * kSyncTileCols, &ex, &extended, true);
    if (rc != DS_OK) return rc;
    PartitionArg part;
    int32_t max_size = 0;
    rc = ds::pack_partition(W, perm, off, n_groups, &part, &max_size);
    if (rc != DS_OK) return rc;
    const int64_t n_tiles = (P + kSyncTileCols - 1) / kSyncTileCols;
    if (n_tiles * n_groups > ds::kMaxSyncGridX) return DS_ERR_BAD_SHAPE;   // the 1-D grid tiles * groups
    if (P == 0) return DS_OK;
    const LaunchShape sh = {P, nullptr, 0, 0, n_tiles, max_size, n_groups, TileWalk{tsx, tsg, n_groups}};
    return launch<false, true>(X, G, g_dtype, kSyncTileCols, kSyncTileCols, sh, part, lr, extended, ex, stream);
}

int group_sync_ragged(void* X, const void* G, int32_t g_dtype, const ds_segment* segs, int32_t S, int64_t ldx,
                      int64_t ldg, int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups, float lr,
                      const ds_local_opt* opt, const void* plan, size_t plan_bytes, uint64_t plan_id, void* stream) {
    int rc = check_stacks(X, G, g_dtype, ldx, ldg);
    if (rc != DS_OK) return rc;
    const SegmentScan sc = scan_segments(segs, S, ldx, ldg, true);
    if (sc.status != DS_OK) return sc.status;
    Extras ex;
    bool extended = false;
    rc = read_opt(opt, sc.end, &ex, &extended);
    if (rc != DS_OK) return rc;
    PartitionArg part;
    int32_t max_size = 0;
    rc = ds::pack_partition(W, perm, off, n_groups, &part, &max_size);
    if (rc != DS_OK) return rc;
    if (sc.n_entries == 0) return DS_OK;
    if (!plan || !ds::aligned16(plan) || plan_bytes < static_cast<size_t>(sc.n_entries + 1) * sizeof(Tile))
        return DS_ERR_WORKSPACE;
    if (plan_id != sc.id) return DS_ERR_WORKSPACE;   // the plan was built from another list
    const LaunchShape sh = {0, static_cast<const Tile*>(plan), plan_id, sc.n_entries, sc.n_live_tiles, max_size,
                            n_groups, TileWalk{kSyncTileCols, kSyncTileCols, 0}};
    return launch<true, false>(X, G, g_dtype, ldx, ldg, sh, part, lr, extended, ex, stream);
}

}  // namespace

extern "C" int ds_group_sync(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx,
                             int64_t ldg, int32_t W, const int32_t* perm, const int32_t* off,
                             int32_t n_groups, float lr, void* stream) {
    return group_sync_flat(X, G, g_dtype, P, ldx, ldg, W, perm, off, n_groups, lr, nullptr, stream);
}

extern "C" int ds_group_sync_opt(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx,
                                 int64_t ldg, int32_t W, const int32_t* perm, const int32_t* off,
                                 int32_t n_groups, float lr, const ds_local_opt* opt, void* stream) {
    return group_sync_flat(X, G, g_dtype, P, ldx, ldg, W, perm, off, n_groups, lr, opt, stream);
}

extern "C" size_t ds_group_sync_consensus_workspace_bytes(int64_t P, int32_t n_groups) {
    if (P < 0 || P > DS_MAX_COLUMNS || n_groups < 1 || n_groups > DS_MAX_W) return 0;
    const int64_t n_tiles = (P + kSyncTileCols - 1) / kSyncTileCols;
    const int64_t entries = n_tiles * n_groups;
    return static_cast<size_t>(entries < 2 ? 2 : entries) * sizeof(double);   // never 0 for valid arguments
}

namespace {

// Launches of the one-pass step+norms; every argument has been checked.
int launch_sync_consensus(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t rsx, int64_t rsg,
                          const TileWalk& walk, int32_t W, const PartitionArg& part, int32_t max_size, int32_t n_groups,
                          float lr, double* dev_out, void* workspace, void* stream) {
    ds::DeviceInfo dev;
    const int rc = ds::device_info(&dev);
    if (rc != DS_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t n_tiles = (P + kSyncTileCols - 1) / kSyncTileCols;
    double* partial = static_cast<double*>(workspace);
    if (n_tiles > 0) {
        // LDS: the parked means, or more if the occupancy rule asks for fewer wavefronts per CU
        unsigned lds = static_cast<unsigned>(n_groups) * kFusedLdsPerGroup;
        const unsigned pad = occupancy_pad(max_size, g_dtype == DS_BF16, false, n_tiles * n_groups, dev);
        if (pad > lds) lds = pad;
        const dim3 grid(static_cast<uint32_t>(n_tiles)), block(kSyncThreads);
        hipError_t err;
        if (g_dtype == DS_F32)
            err = ds::launch_kernel(group_sync_consensus_kernel<float>, grid, block, lds, st, static_cast<float*>(X),
                                    static_cast<const float*>(G), rsx, rsg, P, part, n_groups, W, lr, n_tiles, partial,
                                    walk);
        else
            err = ds::launch_kernel(group_sync_consensus_kernel<uint16_t>, grid, block, lds, st, static_cast<float*>(X),
                                    static_cast<const uint16_t*>(G), rsx, rsg, P, part, n_groups, W, lr, n_tiles,
                                    partial, walk);
        if (err != hipSuccess) return DS_ERR_HIP;
    }
    const hipError_t err = ds::launch_kernel(group_norm_kernel, dim3(static_cast<uint32_t>(n_groups)),
                                             dim3(kNormThreads), 0, st, partial, n_tiles, part, dev_out);
    return err == hipSuccess ? DS_OK : DS_ERR_HIP;
}

int check_norm_outputs(const double* dev_out, const void* workspace, size_t workspace_bytes, int64_t P, int32_t n_groups) {
    if (!dev_out) return DS_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(dev_out) & 7u) != 0) return DS_ERR_ALIGN;
    if (!workspace || !ds::aligned16(workspace) ||
        workspace_bytes < ds_group_sync_consensus_workspace_bytes(P, n_groups))
        return DS_ERR_WORKSPACE;
    return DS_OK;
}

}  // namespace

extern "C" int ds_group_sync_consensus(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx,
                                       int64_t ldg, int32_t W, const int32_t* perm, const int32_t* off,
                                       int32_t n_groups, float lr, double* dev_out, void* workspace,
                                       size_t workspace_bytes, void* stream) {
    int rc = check_stacks(X, G, g_dtype, ldx, ldg);
    if (rc != DS_OK) return rc;
    if (!dev_out) return DS_ERR_NULL;
    if (P < 0 || ldx < P || ldg < P || P > DS_MAX_COLUMNS) return DS_ERR_BAD_SHAPE;
    PartitionArg part;
    int32_t max_size = 0;
    rc = ds::pack_partition(W, perm, off, n_groups, &part, &max_size);
    if (rc != DS_OK) return rc;
    rc = check_norm_outputs(dev_out, workspace, workspace_bytes, P, n_groups);
    if (rc != DS_OK) return rc;
    return launch_sync_consensus(X, G, g_dtype, P, ldx, ldg, TileWalk{kSyncTileCols, kSyncTileCols, 0}, W, part, max_size,
                                 n_groups, lr, dev_out, workspace, stream);
}

extern "C" int64_t ds_tiled_elements(int64_t P, int32_t W) {
    if (P < 0 || P > DS_MAX_COLUMNS || W < 1 || W > DS_MAX_W) return 0;
    return (P + kSyncTileCols - 1) / kSyncTileCols * W * kSyncTileCols;
}

extern "C" int ds_group_sync_tiled(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t tile_stride_x,
                                   int64_t tile_stride_g, int32_t W, const int32_t* perm, const int32_t* off,
                                   int32_t n_groups, float lr, const ds_local_opt* opt, void* stream) {
    return group_sync_tiled(X, G, g_dtype, P, tile_stride_x, tile_stride_g, W, perm, off, n_groups, lr, opt, stream);
}

extern "C" int ds_group_sync_consensus_tiled(void* X, const void* G, int32_t g_dtype, int64_t P,
                                             int64_t tile_stride_x, int64_t tile_stride_g, int32_t W,
                                             const int32_t* perm, const int32_t* off, int32_t n_groups, float lr,
                                             double* dev_out, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_tiled(X, G, g_dtype, P, tile_stride_x, tile_stride_g, W);
    if (rc != DS_OK) return rc;
    PartitionArg part;
    int32_t max_size = 0;
    rc = ds::pack_partition(W, perm, off, n_groups, &part, &max_size);
    if (rc != DS_OK) return rc;
    rc = check_norm_outputs(dev_out, workspace, workspace_bytes, P, n_groups);
    if (rc != DS_OK) return rc;
    return launch_sync_consensus(X, G, g_dtype, P, kSyncTileCols, kSyncTileCols,
                                 TileWalk{tile_stride_x, tile_stride_g, n_groups}, W, part, max_size, n_groups, lr, dev_out,
                                 workspace, stream);
}

extern "C" size_t ds_ragged_plan_bytes(const ds_segment* segs, int32_t S) {
    const SegmentScan sc = scan_segments(segs, S, 0, 0, false);
    if (sc.status != DS_OK || sc.n_entries == 0) return 0;
    return static_cast<size_t>(sc.n_entries + 1) * sizeof(Tile);   // entry 0 is the header
}

extern "C" int ds_ragged_plan(const ds_segment* segs, int32_t S, int64_t ldx, int64_t ldg, void* plan,
                              size_t plan_bytes, uint64_t* plan_id_out, void* stream) {
    if (!plan_id_out) return DS_ERR_NULL;
    *plan_id_out = 0;
    if (ldx < 0 || ldg < 0) return DS_ERR_BAD_SHAPE;
    const SegmentScan sc = scan_segments(segs, S, ldx, ldg, true);
    if (sc.status != DS_OK) return sc.status;
    const int rc = check_disjoint(segs, S);
    if (rc != DS_OK) return rc;
    if (sc.n_entries == 0) return DS_OK;
    const size_t need = static_cast<size_t>(sc.n_entries + 1) * sizeof(Tile);
    if (!plan || !ds::aligned16(plan) || plan_bytes < need) return DS_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    PlanBatch batch;
    batch.header.id = sc.id;
    batch.header.n_segments = S;
    batch.header.n_entries = static_cast<int32_t>(sc.n_entries);
    int64_t first_entry = 0;
    for (int32_t s0 = 0; s0 < S; s0 += kPlanBatch) {
        batch.count = S - s0 < kPlanBatch ? S - s0 : kPlanBatch;
        batch.with_header = s0 == 0;
        for (int32_t j = 0; j < kPlanBatch; ++j) {
            const bool used = j < batch.count;
            batch.offset[j] = used ? segs[s0 + j].offset : 0;
            batch.length[j] = used ? segs[s0 + j].length : 0;
            batch.first_entry[j] = first_entry;
            if (used) first_entry += (segs[s0 + j].length + kPlanTileCols - 1) / kPlanTileCols;
        }
        const hipError_t err = ds::launch_kernel(plan_fill_kernel, dim3(static_cast<uint32_t>(batch.count)),
                                                 dim3(kPlanThreads), 0, st, static_cast<Tile*>(plan), batch);
        if (err != hipSuccess) return DS_ERR_HIP;
    }
    *plan_id_out = sc.id;
    return DS_OK;
}

extern "C" int ds_group_sync_ragged(void* X, const void* G, int32_t g_dtype, const ds_segment* segs,
                                    int32_t S, int64_t ldx, int64_t ldg, int32_t W, const int32_t* perm,
                                    const int32_t* off, int32_t n_groups, float lr, const void* plan,
                                    size_t plan_bytes, uint64_t plan_id, void* stream) {
    return group_sync_ragged(X, G, g_dtype, segs, S, ldx, ldg, W, perm, off, n_groups, lr, nullptr, plan, plan_bytes,
                             plan_id, stream);
}

extern "C" int ds_group_sync_ragged_opt(void* X, const void* G, int32_t g_dtype, const ds_segment* segs,
                                        int32_t S, int64_t ldx, int64_t ldg, int32_t W, const int32_t* perm,
                                        const int32_t* off, int32_t n_groups, float lr, const ds_local_opt* opt,
                                        const void* plan, size_t plan_bytes, uint64_t plan_id, void* stream) {
    return group_sync_ragged(X, G, g_dtype, segs, S, ldx, ldg, W, perm, off, n_groups, lr, opt, plan, plan_bytes,
                             plan_id, stream);
}
