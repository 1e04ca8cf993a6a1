// Group-sync kernels for gfx950: the local SGD update of every worker fused
// with the parameter average inside each group and the write-back of the mean
// to every member (Listing 1: optimizer.step() then Average(model, group);
// Sec. III-A step 4; Sec. IV-B2: X_{k+1} = W_k X_k, w_ij = 1/|group|).
//
// The step is a streaming reduction over the worker axis: 8 (or 6) bytes are
// read and 4 written per (worker, column) and about one FMA is spent on them,
// so the kernel is bound by HBM bandwidth and uses no matrix cores.  Mapping:
//   - a workgroup of 256 lanes owns one tile of kSyncTileCols consecutive
//     columns of ONE group; blockIdx.y is the group, blockIdx.x the tile, so
//     consecutive workgroups walk each member row sequentially;
//   - a lane owns kSyncVecPerLane vectors of 4 consecutive columns, 64 lanes
//     apart, so every wavefront load/store instruction covers 1 KiB of one
//     row (128-bit per lane, fully coalesced) and a wavefront owns
//     kSyncVecPerLane consecutive KiB of every member row;
//   - member rows are uniform across the workgroup: their indices come from
//     the kernel-argument block through scalar loads (which have their own
//     wait counter, so fetching an index never waits for data loads), and the
//     row base addresses live in scalar registers;
//   - members are accumulated kChunk at a time, which keeps
//     2 * kChunk * kSyncVecPerLane 128-bit loads in flight per lane; interior
//     tiles run a predicate-free body so that those loads issue back to back
//     (a load guarded by a lane predicate gets its own basic block and the
//     compiler then waits for it before issuing the next one);
//   - the reduction over members is sequential inside a lane (no cross-lane
//     traffic is needed: a column never leaves its lane), one mean is formed
//     per column and stored |group| times, so members end bit-identical;
//   - loads and stores carry the non-temporal hint: every byte is touched
//     exactly once per step;
//   - the launch asks for kSyncLdsPad bytes of dynamic LDS that the kernel
//     never touches.  Its only purpose is to hold the number of workgroups per
//     CU at two: measured on MI355X, about eight wavefronts per CU with a few
//     KiB of loads in flight each sustain more HBM bandwidth for this 2:1
//     read/write mix than full occupancy does (5.8 vs 5.4 TB/s), and one
//     workgroup per CU is too few (3.9 TB/s).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <utility>
#include <vector>

#include "ds_internal.h"

namespace {

using ds::kSyncThreads;
using ds::kSyncTileCols;
using ds::kSyncVecPerLane;
using ds::PartitionArg;
using ds::Tile;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Tuning constants, fixed at build time from measurements on MI355X.
#ifndef DS_SYNC_CHUNK
#define DS_SYNC_CHUNK 2
#endif
#ifndef DS_SYNC_NT_LOAD
#define DS_SYNC_NT_LOAD 1
#endif
#ifndef DS_SYNC_NT_STORE
#define DS_SYNC_NT_STORE 1
#endif
#ifndef DS_SYNC_BARRIER
#define DS_SYNC_BARRIER 1
#endif
#ifndef DS_SYNC_LDS_PAD
#define DS_SYNC_LDS_PAD 65536
#endif
#ifndef DS_TUNE_ENV
constexpr unsigned kSyncLdsPad = DS_SYNC_LDS_PAD;
#endif
constexpr int kChunk = DS_SYNC_CHUNK;  // members accumulated per round of loads

template <typename V>
__device__ __forceinline__ V stream_load(const V* p) {
#if DS_SYNC_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename V>
__device__ __forceinline__ void stream_store(V v, V* p) {
#if DS_SYNC_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

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

// Adds the locally updated parameters x - lr*g of kCount members (perm
// positions q .. q+kCount-1) to the lane's column sums.  All 2*kCount*VPL
// vector loads are issued back to back before the first use; with kFull
// nothing is predicated, so the loads sit in one basic block.
template <typename GT, int kCount, bool kFull>
__device__ __forceinline__ void add_members(f32x4 (&sum)[kSyncVecPerLane], const float* xt, const GT* gt,
                                            int64_t ldx, int64_t ldg, const PartitionArg& part, int q,
                                            const int (&col)[kSyncVecPerLane],
                                            const bool (&live)[kSyncVecPerLane], float lr) {
    f32x4 x[kCount][kSyncVecPerLane], g[kCount][kSyncVecPerLane];
#pragma unroll
    for (int j = 0; j < kCount; ++j) {
        const int64_t row = packed_byte(part.perm, q + j);
        const float* xr = xt + row * ldx;
        const GT* gr = gt + row * ldg;
#pragma unroll
        for (int v = 0; v < kSyncVecPerLane; ++v) {
            if (kFull || live[v]) {
                x[j][v] = stream_load(reinterpret_cast<const f32x4*>(xr + col[v]));
                g[j][v] = load_grad4(gr + col[v]);
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kCount; ++j) {
#pragma unroll
        for (int v = 0; v < kSyncVecPerLane; ++v)
            if (kFull || live[v]) sum[v] += x[j][v] - lr * g[j][v];
    }
}

// One tile of one group.  kFull: the tile has all kSyncTileCols columns.
template <typename GT, bool kFull>
__device__ __forceinline__ void sync_tile(float* xt, const GT* gt, int len, int64_t ldx, int64_t ldg,
                                          const PartitionArg& part, int first, int n, float lr) {
    int col[kSyncVecPerLane];
    bool live[kSyncVecPerLane];
    f32x4 sum[kSyncVecPerLane];
    const int lane = static_cast<int>(threadIdx.x) & 63, wave = static_cast<int>(threadIdx.x) >> 6;
#pragma unroll
    for (int v = 0; v < kSyncVecPerLane; ++v) {
        col[v] = ((wave * kSyncVecPerLane + v) * 64 + lane) * 4;   // a wavefront owns VPL consecutive KiB
        live[v] = kFull || col[v] + 4 <= len;
        sum[v] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    int q = first;
    const int end = first + n;
    for (; q + kChunk <= end; q += kChunk)
        add_members<GT, kChunk, kFull>(sum, xt, gt, ldx, ldg, part, q, col, live, lr);
    // remaining members (fewer than kChunk): one specialised, branch-free body each
    switch (end - q) {
#define DS_REST(k) case k: if (k < kChunk) add_members<GT, (k < kChunk ? k : 1), kFull>(sum, xt, gt, ldx, ldg, part, q, col, live, lr); break;
        DS_REST(1) DS_REST(2) DS_REST(3) DS_REST(4) DS_REST(5) DS_REST(6) DS_REST(7)
        DS_REST(8) DS_REST(9) DS_REST(10) DS_REST(11) DS_REST(12) DS_REST(13) DS_REST(14) DS_REST(15)
#undef DS_REST
        default: break;
    }
    const float nf = static_cast<float>(n);
#pragma unroll
    for (int v = 0; v < kSyncVecPerLane; ++v) sum[v] = sum[v] / nf;
#if DS_SYNC_BARRIER
    // all four wavefronts switch from reading to writing together
    __syncthreads();
#endif
    for (int m = first; m < end; ++m) {
        float* xr = xt + static_cast<int64_t>(packed_byte(part.perm, m)) * ldx;
#pragma unroll
        for (int v = 0; v < kSyncVecPerLane; ++v)
            if (kFull || live[v]) stream_store(sum[v], reinterpret_cast<f32x4*>(xr + col[v]));
    }
    if (!kFull) {
        // ragged end of the tile: fewer than 4 columns, one lane each
        const int c = (len & ~3) + static_cast<int>(threadIdx.x);
        if (threadIdx.x < 3 && c < len) {
            float s = 0.f;
            for (int m = first; m < end; ++m) {
                const int64_t row = packed_byte(part.perm, m);
                s += xt[row * ldx + c] - lr * load_grad1(gt + row * ldg + c);
            }
            s = s / nf;
            for (int m = first; m < end; ++m) xt[static_cast<int64_t>(packed_byte(part.perm, m)) * ldx + c] = s;
        }
    }
}

template <typename GT, bool kRagged>
__global__ void __launch_bounds__(kSyncThreads)
group_sync_kernel(float* __restrict__ X, const GT* __restrict__ G, int64_t ldx, int64_t ldg,
                  int64_t P, const Tile* __restrict__ tiles, PartitionArg part, float lr) {
    static_assert(kChunk >= 1 && kChunk <= 16, "remainder switch covers up to 15 members");
    int64_t start;
    int32_t len;
    const uint32_t tile_id = blockIdx.x, group_id = blockIdx.y;
    if (kRagged) {
        const Tile tl = tiles[tile_id];
        start = tl.start;
        len = tl.len;
        // a table that does not belong to these stacks must not become a wild access
        const int64_t ld_min = ldx < ldg ? ldx : ldg;
        if (start < 0 || (start & 7) != 0 || len < 0 || len > kSyncTileCols || start > ld_min - len) return;
    } else {
        start = static_cast<int64_t>(tile_id) * kSyncTileCols;
        const int64_t left = P - start;
        len = left < kSyncTileCols ? static_cast<int32_t>(left) : kSyncTileCols;
    }
    const int first = packed_byte(part.off, static_cast<int>(group_id));
    const int n = packed_byte(part.off, static_cast<int>(group_id) + 1) - first;
    if (len == kSyncTileCols)
        sync_tile<GT, true>(X + start, G + start, len, ldx, ldg, part, first, n, lr);
    else
        sync_tile<GT, false>(X + start, G + start, len, ldx, ldg, part, first, n, lr);
}

struct SegmentScan {
    int status;
    int64_t n_tiles;
};

// Validates a segment list and counts the tiles it is cut into.
SegmentScan scan_segments(const ds_segment* segs, int32_t S, int64_t ldx, int64_t ldg, bool have_ld) {
    if (S < 0) return {DS_ERR_BAD_SHAPE, 0};
    if (S > 0 && !segs) return {DS_ERR_NULL, 0};
    int64_t tiles = 0;
    for (int32_t s = 0; s < S; ++s) {
        const int64_t o = segs[s].offset, l = segs[s].length;
        if (o < 0 || l < 0 || l > INT64_MAX - o) return {DS_ERR_BAD_SHAPE, 0};
        if (o % 8 != 0) return {DS_ERR_ALIGN, 0};
        if (have_ld && (o + l > ldx || o + l > ldg)) return {DS_ERR_BAD_SHAPE, 0};
        tiles += (l + kSyncTileCols - 1) / kSyncTileCols;
        if (tiles > INT32_MAX) return {DS_ERR_BAD_SHAPE, 0};
    }
    return {DS_OK, tiles};
}

// Pairwise disjointness of the non-empty segments (sort by offset, compare neighbours).
bool segments_overlap(const ds_segment* segs, int32_t S) {
    std::vector<std::pair<int64_t, int64_t>> v;
    v.reserve(static_cast<size_t>(S));
    for (int32_t s = 0; s < S; ++s)
        if (segs[s].length > 0) v.emplace_back(segs[s].offset, segs[s].offset + segs[s].length);
    std::sort(v.begin(), v.end());
    for (size_t i = 1; i < v.size(); ++i)
        if (v[i].first < v[i - 1].second) return true;
    return false;
}

int check_stacks(const void* X, const void* G, int32_t g_dtype, int64_t ldx, int64_t ldg) {
    if (!X || !G) return DS_ERR_NULL;
    if (g_dtype != DS_F32 && g_dtype != DS_BF16) return DS_ERR_DTYPE;
    if (ldx < 0 || ldg < 0) return DS_ERR_BAD_SHAPE;
    if (!ds::aligned16(X) || !ds::aligned16(G) || ldx % 4 != 0 || ldg % 4 != 0) return DS_ERR_ALIGN;
    return DS_OK;
}

template <bool kRagged>
int launch(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx, int64_t ldg,
           int64_t n_tiles, const Tile* tiles, const PartitionArg& part, int32_t n_groups, float lr,
           void* stream) {
    const dim3 grid(static_cast<uint32_t>(n_tiles), static_cast<uint32_t>(n_groups), 1);
    const dim3 block(kSyncThreads, 1, 1);
    hipStream_t st = static_cast<hipStream_t>(stream);
#ifdef DS_TUNE_ENV
    const char* pad_env = getenv("DS_LDS_PAD");
    const unsigned kSyncLdsPad = pad_env ? static_cast<unsigned>(atoi(pad_env)) : 0u;
    if (kSyncLdsPad > 65536u) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&group_sync_kernel<float, kRagged>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kSyncLdsPad));
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&group_sync_kernel<uint16_t, kRagged>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kSyncLdsPad));
    }
#endif
    if (g_dtype == DS_F32) {
        hipLaunchKernelGGL((group_sync_kernel<float, kRagged>), grid, block, kSyncLdsPad, st, static_cast<float*>(X),
                           static_cast<const float*>(G), ldx, ldg, P, tiles, part, lr);
    } else {
        hipLaunchKernelGGL((group_sync_kernel<uint16_t, kRagged>), grid, block, kSyncLdsPad, st, static_cast<float*>(X),
                           static_cast<const uint16_t*>(G), ldx, ldg, P, tiles, part, lr);
    }
    return hipGetLastError() == hipSuccess ? DS_OK : DS_ERR_HIP;
}

}  // namespace

extern "C" int ds_group_sync(void* X, const void* G, int32_t g_dtype, int64_t P, int64_t ldx,
                             int64_t ldg, int32_t W, const int32_t* perm, const int32_t* off,
                             int32_t n_groups, float lr, void* stream) {
    int rc = check_stacks(X, G, g_dtype, ldx, ldg);
    if (rc != DS_OK) return rc;
    if (P < 0 || ldx < P || ldg < P) return DS_ERR_BAD_SHAPE;
    PartitionArg part;
    int32_t max_size = 0, equal_size = 0;
    rc = ds::pack_partition(W, perm, off, n_groups, &part, &max_size, &equal_size);
    if (rc != DS_OK) return rc;
    const int64_t n_tiles = (P + kSyncTileCols - 1) / kSyncTileCols;
    if (n_tiles > INT32_MAX) return DS_ERR_BAD_SHAPE;
    if (n_tiles == 0) return DS_OK;
    return launch<false>(X, G, g_dtype, P, ldx, ldg, n_tiles, nullptr, part, n_groups, lr, stream);
}

extern "C" size_t ds_ragged_plan_bytes(const ds_segment* segs, int32_t S) {
    const SegmentScan sc = scan_segments(segs, S, 0, 0, false);
    if (sc.status != DS_OK) return 0;
    return static_cast<size_t>(sc.n_tiles) * sizeof(Tile);
}

extern "C" int ds_ragged_plan(const ds_segment* segs, int32_t S, int64_t ldx, int64_t ldg, void* plan,
                              size_t plan_bytes, void* stream) {
    if (ldx < 0 || ldg < 0) return DS_ERR_BAD_SHAPE;
    const SegmentScan sc = scan_segments(segs, S, ldx, ldg, true);
    if (sc.status != DS_OK) return sc.status;
    if (segments_overlap(segs, S)) return DS_ERR_BAD_SHAPE;
    if (sc.n_tiles == 0) return DS_OK;
    const size_t need = static_cast<size_t>(sc.n_tiles) * sizeof(Tile);
    if (!plan || !ds::aligned16(plan) || plan_bytes < need) return DS_ERR_WORKSPACE;

    std::vector<Tile> table;
    table.reserve(static_cast<size_t>(sc.n_tiles));
    for (int32_t s = 0; s < S; ++s) {
        for (int64_t done = 0; done < segs[s].length; done += kSyncTileCols) {
            const int64_t left = segs[s].length - done;
            table.push_back(Tile{segs[s].offset + done,
                                 static_cast<int32_t>(left < kSyncTileCols ? left : kSyncTileCols), 0});
        }
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(plan, table.data(), need, hipMemcpyHostToDevice, st) != hipSuccess) return DS_ERR_HIP;
    // the host table dies with this call, so the copy must have finished
    if (hipStreamSynchronize(st) != hipSuccess) return DS_ERR_HIP;
    return DS_OK;
}

extern "C" int ds_group_sync_ragged(void* X, const void* G, int32_t g_dtype, const ds_segment* segs,
                                    int32_t S, int64_t ldx, int64_t ldg, int32_t W, const int32_t* perm,
                                    const int32_t* off, int32_t n_groups, float lr, const void* plan,
                                    size_t plan_bytes, void* stream) {
    int rc = check_stacks(X, G, g_dtype, ldx, ldg);
    if (rc != DS_OK) return rc;
    const SegmentScan sc = scan_segments(segs, S, ldx, ldg, true);
    if (sc.status != DS_OK) return sc.status;
    PartitionArg part;
    int32_t max_size = 0, equal_size = 0;
    rc = ds::pack_partition(W, perm, off, n_groups, &part, &max_size, &equal_size);
    if (rc != DS_OK) return rc;
    if (sc.n_tiles == 0) return DS_OK;
    if (!plan || !ds::aligned16(plan) || plan_bytes < static_cast<size_t>(sc.n_tiles) * sizeof(Tile))
        return DS_ERR_WORKSPACE;
    return launch<true>(X, G, g_dtype, 0, ldx, ldg, sc.n_tiles, static_cast<const Tile*>(plan), part,
                        n_groups, lr, stream);
}
