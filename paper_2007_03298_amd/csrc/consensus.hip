// Consensus-deviation kernels for gfx950: d_i = || x_i - mean_j x_j ||_2 for
// every worker i (Sec. IV-B2; the left-hand side of Lemma 1, un-squared).
//
// A read-only streaming pass, bound by HBM bandwidth (4 bytes per (worker,
// column), a handful of ALU operations on them).  Mapping:
//   - a lane loads its kVec consecutive columns of ALL W rows into registers
//     (one 128-bit load per row up to 16 rows, one 64-bit load per row above,
//     coalesced across the wavefront), so X is read exactly once;
//   - the column mean is formed in fp64 and split into an fp32 pair hi + lo;
//     the difference (x_i - hi) - lo is then plain fp32 work whose rounding
//     error is relative to the difference itself (and exactly zero for
//     identical replicas); it is squared and summed into one fp32 accumulator
//     per worker per lane;
//   - a workgroup walks a run of consecutive column tiles; at the end (and,
//     for runs longer than kLaneColumns / kVec tiles, every that many tiles)
//     the lane accumulators are widened to fp64, reduced across the wavefront
//     with lane shuffles and added to the wavefront's fp64 totals in LDS, so an
//     fp32 accumulator never holds more than 256 squares and the rounding
//     error of a norm does not grow with the number of columns.  A widening
//     in mid-run costs about 1 % of the pass each (the wavefront has no loads
//     in flight meanwhile); with at most 8192 workgroups none is needed up to
//     537 M columns; at the end the 4 wavefronts' totals are added and written
//     as one partial row per workgroup;
//   - a second kernel adds the partial rows in a fixed order and takes the
//     square root.  No floating-point atomics: the result is deterministic.
#include <hip/hip_runtime.h>

#include <atomic>

#include "ds_internal.h"
#include "launch.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxBlocks = 8192;  // upper bound of the grid of the partial kernel
// An fp32 lane accumulator takes the squares of at most this many columns per worker
// before it is widened; with kVec columns per lane and tile that is kLaneColumns / kVec tiles.
constexpr int kLaneColumns = 256;

// Partial rows of ds_consensus_static: the largest workspace ds_consensus ever
// asks for (kMaxBlocks rows of DS_MAX_W sums, 4 MiB), resident on every GPU
// the library runs on until the process ends.  In host code this name is only
// a handle: the memory is reached through the address hipGetSymbolAddress
// returns on each device.
static __device__ __align__(256) double scratch[static_cast<size_t>(kMaxBlocks) * DS_MAX_W];

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

template <int kVec> struct VecOf;
template <> struct VecOf<4> { typedef f32x4 type; };
template <> struct VecOf<2> { typedef f32x2 type; };

__host__ __device__ constexpr int padded_w(int W) { return W <= 8 ? 8 : W <= 16 ? 16 : W <= 32 ? 32 : 64; }

// Which rows of the stack stand for what.  Plain consensus: every worker's own
// row, weight 1.  Grouped consensus (rows of a group are known to be
// identical, as they are right after a group-sync): one row per group, weight
// = group size, and `src` says which group's total each worker receives.
// One byte per entry, four per 32-bit word, read with scalar loads.
struct RowTable {
    uint32_t row[DS_MAX_W / 4];
    uint32_t weight[DS_MAX_W / 4];
    uint32_t src[DS_MAX_W / 4];
};

__device__ __forceinline__ int table_byte(const uint32_t* words, int i) {
    return static_cast<int>((words[i >> 2] >> ((i & 3) * 8)) & 0xffu);
}

// Adds one tile's squared deviations to the lane accumulators.  kFull: every
// lane's kVec columns lie inside the row (no predicates, so the W loads issue
// back to back).
// n_rows rows take part; kGrouped: row i is tab.row[i] with weight tab.weight[i]
// and total_weight = number of workers, else row i with weight 1.
// kPow2: the number of workers is a power of two and inv_pow2 its reciprocal -
// the fp64 division is a long sequence (3 % of the pass at 64 workers) and
// multiplying is then exactly dividing; any other count is divided properly, so
// that the mean of identical replicas is the replica itself to the last bit.
// kExact: all kWPad row slots are rows (8, 16, 32 or 64 of them); the per-row
// guard, which otherwise costs a select per fp64 value, is compiled out.
template <int kWPad, int kVec, bool kFull, bool kGrouped, bool kPow2, bool kExact>
__device__ __forceinline__ void consensus_tile(float (&acc)[kWPad], const float* __restrict__ X, int64_t c,
                                               int64_t P, int64_t ld, int64_t tile_stride, int W, const RowTable& tab,
                                               int total_weight, double inv_pow2) {
    typedef typename VecOf<kVec>::type vec_t;
    vec_t row[kWPad];
    // column c of row r is at (c / 256) * tile_stride + r * ld + c % 256: row-major stacks pass
    // tile_stride = 256 (that is r * ld + c), tiled stacks ld = 256 and the stride of their blocks
    static_assert(256 % kVec == 0, "a lane's columns stay inside one 256-column tile");
    const float* base = X + (c >> 8) * tile_stride + (c & 255);
#pragma unroll
    for (int i = 0; i < kWPad; ++i) {
        if (kExact || i < W) {
            const int64_t r = kGrouped ? table_byte(tab.row, i) : i;
            if (kFull) {
                row[i] = __builtin_nontemporal_load(reinterpret_cast<const vec_t*>(base + r * ld));
            } else {
                // last, partial vector of the row: columns at or beyond P count as 0
                // in every row, which adds nothing to any deviation
#pragma unroll
                for (int e = 0; e < kVec; ++e) row[i][e] = (c + e < P) ? base[r * ld + e] : 0.f;
            }
        }
    }
    // every row's load is issued before the first value is used: left to itself the scheduler
    // trades loads in flight for registers and waits for memory several times per tile
    __builtin_amdgcn_sched_barrier(0);
    double mean[kVec];
#pragma unroll
    for (int e = 0; e < kVec; ++e) mean[e] = 0.0;
#pragma unroll
    for (int i = 0; i < kWPad; ++i) {
        if (kExact || i < W) {
            const double w = kGrouped ? static_cast<double>(table_byte(tab.weight, i)) : 1.0;
#pragma unroll
            for (int e = 0; e < kVec; ++e)
                mean[e] += kGrouped ? w * static_cast<double>(row[i][e]) : static_cast<double>(row[i][e]);
        }
    }
    // mean as an unevaluated fp32 pair hi + lo (|lo| <= ulp(hi)/2): subtracting
    // hi, then lo, in fp32 leaves an error that is relative to the difference
    // itself, and is exactly 0 when every row equals the mean
    // a power-of-two worker count divides exactly by multiplication (the fp64 division is a long
    // sequence: 3 % of the pass at 64 workers); any other count is divided properly, so that the mean
    // of identical replicas is the replica itself to the last bit
    const double wd = static_cast<double>(kGrouped ? total_weight : W);
    float hi[kVec], lo[kVec];
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        const double m = kPow2 ? mean[e] * inv_pow2 : mean[e] / wd;
        hi[e] = static_cast<float>(m);
        lo[e] = static_cast<float>(m - static_cast<double>(hi[e]));
    }
#pragma unroll
    for (int i = 0; i < kWPad; ++i) {
        if (kExact || i < W) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const float d = (row[i][e] - hi[e]) - lo[e];
                acc[i] = __builtin_fmaf(d, d, acc[i]);
            }
        }
    }
}

template <int kWPad, int kVec, bool kGrouped, bool kPow2, bool kExact>
__global__ void __launch_bounds__(kThreads)
consensus_partial_kernel(const float* __restrict__ X, int64_t P, int64_t ld, int64_t tile_stride, int W,
                         int tiles_per_block, double* __restrict__ partial, RowTable tab, int total_weight,
                         double inv_pow2) {
    constexpr int kTileCols = kThreads * kVec;
    float acc[kWPad];
#pragma unroll
    for (int i = 0; i < kWPad; ++i) acc[i] = 0.f;

    __shared__ double wave_sum[kWaves][kWPad];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    static_assert(kWPad <= 64, "one lane per worker clears the wavefront's totals");
    if (lane < kWPad) wave_sum[wave][lane] = 0.0;   // only this wavefront touches its row before the barrier

    // a workgroup owns tiles_per_block consecutive tiles
    const int64_t n_tiles = (P + kTileCols - 1) / kTileCols;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * tiles_per_block;
    const int64_t tile1 = tile0 + tiles_per_block < n_tiles ? tile0 + tiles_per_block : n_tiles;
    int since = 0;
    for (int64_t tile = tile0; tile < tile1; ++tile) {
        const int64_t c = tile * kTileCols + static_cast<int64_t>(threadIdx.x) * kVec;
        if ((tile + 1) * kTileCols <= P) {
            consensus_tile<kWPad, kVec, true, kGrouped, kPow2, kExact>(acc, X, c, P, ld, tile_stride, W, tab, total_weight, inv_pow2);
        } else if (c < P) {
            if (c + kVec <= P)
                consensus_tile<kWPad, kVec, true, kGrouped, kPow2, kExact>(acc, X, c, P, ld, tile_stride, W, tab, total_weight, inv_pow2);
            else
                consensus_tile<kWPad, kVec, false, kGrouped, kPow2, kExact>(acc, X, c, P, ld, tile_stride, W, tab, total_weight, inv_pow2);
        }
        if (++since == kLaneColumns / kVec || tile + 1 == tile1) {
            // lanes -> wavefront in fp64, added to the wavefront's totals; the fp32 sums start over
            since = 0;
#pragma unroll
            for (int i = 0; i < kWPad; ++i) {
                double v = static_cast<double>(acc[i]);
#pragma unroll
                for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
                if (lane == 0) wave_sum[wave][i] += v;
                acc[i] = 0.f;
            }
        }
    }

    // wavefronts -> workgroup -> partial row
    __syncthreads();
    if (threadIdx.x < kWPad) {
        double v = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) v += wave_sum[w][threadIdx.x];
        partial[static_cast<int64_t>(blockIdx.x) * kWPad + threadIdx.x] = v;
    }
}

// one workgroup per worker: fixed-order sum of its column (tab.src) of the partial rows
__global__ void __launch_bounds__(kThreads)
consensus_final_kernel(const double* __restrict__ partial, int n_rows, int w_pad, double* __restrict__ out,
                       RowTable tab) {
    __shared__ double buf[kThreads];
    const int i = table_byte(tab.src, static_cast<int>(blockIdx.x));
    double v = 0.0;
    for (int b = threadIdx.x; b < n_rows; b += kThreads) v += partial[static_cast<int64_t>(b) * w_pad + i];
    buf[threadIdx.x] = v;
    __syncthreads();
    for (int half = kThreads / 2; half >= 1; half >>= 1) {
        if (static_cast<int>(threadIdx.x) < half) buf[threadIdx.x] += buf[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[blockIdx.x] = sqrt(buf[0]);
}

}  // namespace

extern "C" size_t ds_consensus_workspace_bytes(int32_t W, int64_t P) {
    if (W < 1 || W > DS_MAX_W || P < 0) return 0;
    return static_cast<size_t>(kMaxBlocks) * static_cast<size_t>(padded_w(W)) * sizeof(double);
}

namespace {

void set_byte(uint32_t* words, int i, int value) { words[i >> 2] |= static_cast<uint32_t>(value) << ((i & 3) * 8); }

// n_rows rows are read (W for the plain norm, n_groups for the grouped one); W outputs.
template <bool kGrouped>
int launch_consensus(const float* x, int64_t P, int64_t ld, int64_t tile_stride, int32_t W, int32_t n_rows,
                     const RowTable& tab, double* dev_out, double* partial, hipStream_t st) {
    const int w_pad = padded_w(n_rows);
    const int vec = w_pad >= 32 ? 2 : 4;   // keeps the rows of one lane within 64 registers
    const int64_t tile_cols = static_cast<int64_t>(kThreads) * vec;
    const int64_t n_tiles = (P + tile_cols - 1) / tile_cols;
    // Workgroups come in rounds of two per CU, all resident at once (the 64-row kernel fits
    // two per CU, the smaller ones more): ONE round wherever a lane accumulator can take a
    // workgroup's whole run of tiles, else as many rounds as keep the runs that short.  Measured
    // against 4096 workgroups for everything: +2 % at 32 x 25.6 M columns, +4 % at 16 x 11.7 M,
    // +8 % at 8 x 1 M (fewer end-of-block reductions and partial rows), equal at 64 x 138 M.
    // Runs longer than a lane accumulator takes (more than kMaxBlocks of them would be needed)
    // are widened in mid-run by the kernel.
    ds::DeviceInfo dev;
    const int drc = ds::device_info(&dev);
    if (drc != DS_OK) return drc;
    const int64_t round = 2 * static_cast<int64_t>(dev.compute_units);
    const int64_t lane_tiles = kLaneColumns / vec;
    int64_t rounds = (n_tiles + lane_tiles * round - 1) / (lane_tiles * round);
    if (rounds < 1) rounds = 1;
    int64_t blocks = rounds * round;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    int64_t per_block = (n_tiles + blocks - 1) / blocks;
    if (per_block < 1) per_block = 1;
    if (per_block > INT32_MAX) return DS_ERR_BAD_SHAPE;
    // at least one workgroup, so that P == 0 still writes a (zero) partial row
    const int64_t want_blocks = (n_tiles + per_block - 1) / per_block;
    const int n_blocks = static_cast<int>(want_blocks < 1 ? 1 : want_blocks);
    const int tpb = static_cast<int>(per_block);
    // 1/W when W is a power of two (then multiplying is exactly dividing), else 0: the kernel divides
    const double inv_pow2 = (W & (W - 1)) == 0 ? 1.0 / static_cast<double>(W) : 0.0;
    const dim3 grid(static_cast<uint32_t>(n_blocks)), block(kThreads);
    hipError_t err;
    // exact: every one of the w_pad row slots is a row, so the kernel needs no per-row guard
    const bool exact = n_rows == w_pad;
#define DS_PARTIAL_E(WP, V, POW2, EXACT) \
    ds::launch_kernel(consensus_partial_kernel<WP, V, kGrouped, POW2, EXACT>, grid, block, 0, st, x, P, ld, tile_stride, \
                      n_rows, tpb, partial, tab, W, inv_pow2)
#define DS_PARTIAL(WP, V) \
    err = inv_pow2 != 0.0 ? (exact ? DS_PARTIAL_E(WP, V, true, true) : DS_PARTIAL_E(WP, V, true, false)) \
                          : (exact ? DS_PARTIAL_E(WP, V, false, true) : DS_PARTIAL_E(WP, V, false, false))
    switch (w_pad) {
        case 8: DS_PARTIAL(8, 4); break;
        case 16: DS_PARTIAL(16, 4); break;
        case 32: DS_PARTIAL(32, 2); break;
        default: DS_PARTIAL(64, 2); break;
    }
#undef DS_PARTIAL
#undef DS_PARTIAL_E
    if (err != hipSuccess) return DS_ERR_HIP;
    err = ds::launch_kernel(consensus_final_kernel, dim3(static_cast<uint32_t>(W)), block, 0, st, partial, n_blocks, w_pad,
                            dev_out, tab);
    return err == hipSuccess ? DS_OK : DS_ERR_HIP;
}

int check_consensus_stack(const void* X, int64_t P, int64_t ld, int32_t W, const double* dev_out) {
    if (!X || !dev_out) return DS_ERR_NULL;
    if (W < 1 || W > DS_MAX_W) return DS_ERR_BAD_W;
    if (P < 0 || ld < P || P > DS_MAX_COLUMNS) return DS_ERR_BAD_SHAPE;
    if (!ds::aligned16(X) || ld % 4 != 0 || (reinterpret_cast<uintptr_t>(dev_out) & 7u) != 0) return DS_ERR_ALIGN;
    return DS_OK;
}

int check_consensus_args(const void* X, int64_t P, int64_t ld, int32_t W, const double* dev_out, const void* workspace,
                         size_t workspace_bytes) {
    const int rc = check_consensus_stack(X, P, ld, W, dev_out);
    if (rc != DS_OK) return rc;
    if (!workspace || !ds::aligned16(workspace) || workspace_bytes < ds_consensus_workspace_bytes(W, P))
        return DS_ERR_WORKSPACE;
    return DS_OK;
}

}  // namespace

extern "C" int ds_consensus(const void* X, int64_t P, int64_t ld, int32_t W, double* dev_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_consensus_args(X, P, ld, W, dev_out, workspace, workspace_bytes);
    if (rc != DS_OK) return rc;
    RowTable tab = {};
    for (int32_t i = 0; i < W; ++i) set_byte(tab.src, i, i);
    return launch_consensus<false>(static_cast<const float*>(X), P, ld, 256, W, W, tab, dev_out,
                                   static_cast<double*>(workspace), static_cast<hipStream_t>(stream));
}

namespace {

int check_tiled_consensus_args(const void* X, int64_t P, int64_t tile_stride, int32_t W, const double* dev_out,
                               const void* workspace, size_t workspace_bytes) {
    if (!X || !dev_out) return DS_ERR_NULL;
    if (W < 1 || W > DS_MAX_W) return DS_ERR_BAD_W;
    if (P < 0 || P > DS_MAX_COLUMNS || tile_stride < static_cast<int64_t>(W) * 256) return DS_ERR_BAD_SHAPE;
    if (!ds::aligned16(X) || tile_stride % 256 != 0 || (reinterpret_cast<uintptr_t>(dev_out) & 7u) != 0)
        return DS_ERR_ALIGN;
    if (!workspace || !ds::aligned16(workspace) || workspace_bytes < ds_consensus_workspace_bytes(W, P))
        return DS_ERR_WORKSPACE;
    return DS_OK;
}

// Row table of the grouped norm: one row per group (its first member), weighted by the group's size.
int grouped_table(int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups, RowTable* tab) {
    ds::PartitionArg packed;
    int32_t max_size = 0;
    const int rc = ds::pack_partition(W, perm, off, n_groups, &packed, &max_size);
    if (rc != DS_OK) return rc;
    *tab = RowTable{};
    for (int32_t k = 0; k < n_groups; ++k) {
        set_byte(tab->row, k, perm[off[k]]);                // the group's first member stands for all of them
        set_byte(tab->weight, k, off[k + 1] - off[k]);
        for (int32_t q = off[k]; q < off[k + 1]; ++q) set_byte(tab->src, perm[q], k);
    }
    return DS_OK;
}

}  // namespace

extern "C" int ds_consensus_tiled(const void* X, int64_t P, int64_t tile_stride, int32_t W, double* dev_out,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_tiled_consensus_args(X, P, tile_stride, W, dev_out, workspace, workspace_bytes);
    if (rc != DS_OK) return rc;
    RowTable tab = {};
    for (int32_t i = 0; i < W; ++i) set_byte(tab.src, i, i);
    return launch_consensus<false>(static_cast<const float*>(X), P, 256, tile_stride, W, W, tab, dev_out,
                                   static_cast<double*>(workspace), static_cast<hipStream_t>(stream));
}

extern "C" int ds_consensus_grouped_tiled(const void* X, int64_t P, int64_t tile_stride, int32_t W,
                                          const int32_t* perm, const int32_t* off, int32_t n_groups, double* dev_out,
                                          void* workspace, size_t workspace_bytes, void* stream) {
    const int rc = check_tiled_consensus_args(X, P, tile_stride, W, dev_out, workspace, workspace_bytes);
    if (rc != DS_OK) return rc;
    RowTable tab;
    const int prc = grouped_table(W, perm, off, n_groups, &tab);
    if (prc != DS_OK) return prc;
    return launch_consensus<true>(static_cast<const float*>(X), P, 256, tile_stride, W, n_groups, tab, dev_out,
                                  static_cast<double*>(workspace), static_cast<hipStream_t>(stream));
}

namespace {

constexpr int kMaxDevices = 64;
// address of `scratch` on each device, resolved on the first call there
std::atomic<double*> g_scratch_ptr[kMaxDevices];

// The current device's copy of `scratch`, or NULL if its address cannot be had.
double* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    double* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        // `dev` is current, so this is that device's copy of the array
        if (hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch)) != hipSuccess || !ptr)
            return nullptr;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

}  // namespace

extern "C" int ds_consensus_static(const void* X, int64_t P, int64_t ld, int32_t W, double* dev_out,
                                   void* stream) {
    const int rc = check_consensus_stack(X, P, ld, W, dev_out);
    if (rc != DS_OK) return rc;
    static_assert(sizeof(scratch) >= static_cast<size_t>(kMaxBlocks) * 64 * sizeof(double),
                  "the array holds the largest workspace ds_consensus asks for");
    double* partial = scratch_on_current_device();
    if (!partial) return DS_ERR_HIP;
    RowTable tab = {};
    for (int32_t i = 0; i < W; ++i) set_byte(tab.src, i, i);
    return launch_consensus<false>(static_cast<const float*>(X), P, ld, 256, W, W, tab, dev_out, partial,
                                   static_cast<hipStream_t>(stream));
}

extern "C" int ds_consensus_grouped(const void* X, int64_t P, int64_t ld, int32_t W, const int32_t* perm,
                                    const int32_t* off, int32_t n_groups, double* dev_out, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    const int rc = check_consensus_args(X, P, ld, W, dev_out, workspace, workspace_bytes);
    if (rc != DS_OK) return rc;
    RowTable tab;
    const int prc = grouped_table(W, perm, off, n_groups, &tab);
    if (prc != DS_OK) return prc;
    return launch_consensus<true>(static_cast<const float*>(X), P, ld, 256, W, n_groups, tab, dev_out,
                                  static_cast<double*>(workspace), static_cast<hipStream_t>(stream));
}
