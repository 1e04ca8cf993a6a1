// Host side of libdssync: status strings, the worker division for one
// iteration (Listing 1: the group list entry for iteration t; Sec. IV-B2:
// disjoint groups covering all workers) and validation of a division handed
// to the GPU entry points.  Integer work only; nothing here calls HIP.
#include "ds_internal.h"

extern "C" const char* ds_status_string(int status) {
    switch (status) {
        case DS_OK: return "DS_OK";
        case DS_ERR_NULL: return "DS_ERR_NULL: required pointer is NULL";
        case DS_ERR_BAD_W: return "DS_ERR_BAD_W: worker count outside 1..DS_MAX_W";
        case DS_ERR_BAD_SIZES: return "DS_ERR_BAD_SIZES: group sizes do not divide the workers";
        case DS_ERR_BAD_PART: return "DS_ERR_BAD_PART: perm/off is not a division of the workers";
        case DS_ERR_BAD_SHAPE: return "DS_ERR_BAD_SHAPE: bad column count, leading dimension or segment";
        case DS_ERR_ALIGN: return "DS_ERR_ALIGN: pointer, leading dimension or segment offset misaligned";
        case DS_ERR_DTYPE: return "DS_ERR_DTYPE: unknown gradient element type";
        case DS_ERR_WORKSPACE: return "DS_ERR_WORKSPACE: workspace or plan buffer missing, misaligned or too small";
        case DS_ERR_HIP: return "DS_ERR_HIP: HIP call or kernel launch failed";
        case DS_ERR_TOPOLOGY: return "DS_ERR_TOPOLOGY: rack table is not a usable topology";
        case DS_ERR_HOST_MEMORY: return "DS_ERR_HOST_MEMORY: host allocation failed";
        default: return "unknown ds_status";
    }
}

extern "C" int64_t ds_padded_ld(int64_t P) {
    constexpr int64_t kPad = 256;   // elements: 1 KiB of fp32
    if (P < 0 || P > INT64_MAX - 2 * kPad) return 0;
    int64_t units = (P + kPad - 1) / kPad;
    if (units % 2 == 0) ++units;
    return units * kPad;
}

namespace {

constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

// splitmix64 output function
inline uint64_t finalize64(uint64_t v) {
    v = (v ^ (v >> 30)) * 0xBF58476D1CE4E5B9ull;
    v = (v ^ (v >> 27)) * 0x94D049BB133111EBull;
    return v ^ (v >> 31);
}

// high 64 bits of a*b, from 32-bit halves
inline uint64_t mul_high(uint64_t a, uint64_t b) {
    const uint64_t a0 = a & 0xffffffffull, a1 = a >> 32;
    const uint64_t b0 = b & 0xffffffffull, b1 = b >> 32;
    const uint64_t lo_lo = a0 * b0;
    const uint64_t hi_lo = a1 * b0;
    const uint64_t lo_hi = a0 * b1;
    const uint64_t hi_hi = a1 * b1;
    const uint64_t carry = ((lo_lo >> 32) + (hi_lo & 0xffffffffull) + (lo_hi & 0xffffffffull)) >> 32;
    return hi_hi + (hi_lo >> 32) + (lo_hi >> 32) + carry;
}

}  // namespace

extern "C" int ds_partition(uint64_t seed, uint64_t t, int32_t W, const int32_t* sizes,
                            int32_t n_groups, int32_t* perm_out, int32_t* off_out) {
    if (!sizes || !perm_out || !off_out) return DS_ERR_NULL;
    if (W < 1 || W > DS_MAX_W) return DS_ERR_BAD_W;
    if (n_groups < 1 || n_groups > W) return DS_ERR_BAD_SIZES;
    int64_t covered = 0;
    for (int32_t k = 0; k < n_groups; ++k) {
        if (sizes[k] < 1 || sizes[k] > W) return DS_ERR_BAD_SIZES;
        covered += sizes[k];
    }
    if (covered != W) return DS_ERR_BAD_SIZES;

    // Durstenfeld shuffle from the top; the stream of draws depends on (seed, t) only.
    uint64_t state = finalize64(finalize64(seed) + (t + 1) * kGolden);
    for (int32_t w = 0; w < W; ++w) perm_out[w] = w;
    for (int32_t hi = W - 1; hi > 0; --hi) {
        state += kGolden;
        const int32_t pick = static_cast<int32_t>(mul_high(finalize64(state), static_cast<uint64_t>(hi) + 1));
        const int32_t moved = perm_out[pick];
        perm_out[pick] = perm_out[hi];
        perm_out[hi] = moved;
    }
    int32_t edge = 0;
    for (int32_t k = 0; k < n_groups; ++k) {
        off_out[k] = edge;
        edge += sizes[k];
    }
    off_out[n_groups] = edge;
    return DS_OK;
}

int ds::pack_partition(int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups,
                       PartitionArg* out, int32_t* max_size) {
    if (!perm || !off) return DS_ERR_NULL;
    if (W < 1 || W > DS_MAX_W) return DS_ERR_BAD_W;
    if (n_groups < 1 || n_groups > W) return DS_ERR_BAD_SIZES;
    if (off[0] != 0 || off[n_groups] != W) return DS_ERR_BAD_PART;
    int32_t largest = 0;
    for (int32_t k = 0; k < n_groups; ++k) {
        const int64_t sz = static_cast<int64_t>(off[k + 1]) - off[k];
        if (sz < 1 || sz > W) return DS_ERR_BAD_PART;
        if (sz > largest) largest = static_cast<int32_t>(sz);
    }
    bool seen[DS_MAX_W] = {};
    for (int32_t q = 0; q < W; ++q) {
        const int32_t w = perm[q];
        if (w < 0 || w >= W || seen[w]) return DS_ERR_BAD_PART;
        seen[w] = true;
    }
    for (uint32_t& word : out->perm) word = 0;
    for (uint32_t& word : out->off) word = 0;
    for (int32_t q = 0; q < W; ++q) out->perm[q >> 2] |= static_cast<uint32_t>(perm[q]) << ((q & 3) * 8);
    for (int32_t k = 0; k < DS_MAX_W + 4; ++k) {
        const uint32_t edge = static_cast<uint32_t>(k <= n_groups ? off[k] : W);
        out->off[k >> 2] |= edge << ((k & 3) * 8);
    }
    *max_size = largest;
    return DS_OK;
}
