// Internal declarations shared by the translation units of libdssync.
#pragma once

#include <stdint.h>

#include "dssync.h"

namespace ds {

// Division of the workers as the kernels see it: member rows of group k are
// perm[off[k]] .. perm[off[k+1]-1], one byte per entry, four entries packed
// per 32-bit word (entry i in bits 8*(i%4) of word i/4).  Passed by value in
// the kernel-argument block (132 bytes), so no host-to-device copy is needed;
// packing into words lets the device fetch entries with scalar loads, which do
// not share a wait counter with the vector loads of the data.
struct PartitionArg {
    uint32_t perm[DS_MAX_W / 4];
    uint32_t off[DS_MAX_W / 4 + 1];  // n_groups+1 entries used
};


// Checks perm/off (host arrays) and packs them; returns DS_OK or the status to
// hand back to the caller.  max_size receives the largest group size and
// equal_size the common size if all groups are equal (else 0).
int pack_partition(int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups,
                   PartitionArg* out, int32_t* max_size, int32_t* equal_size);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Group-sync launch shape.  A workgroup is ONE wavefront; a lane owns one
// vector of 4 consecutive columns, so a workgroup covers 256 columns of every
// member row (1 KiB per row and load instruction) and loads up to
// kSyncLoadsPerLane/2 members (x and g each) per round.
constexpr int kSyncThreads = 64;
constexpr int kSyncTileCols = kSyncThreads * 4;
constexpr int kSyncLoadsPerLane = 16;
// Unit of the ragged plan: 2048 columns = 8 workgroups.
constexpr int kPlanTileCols = 2048;

// One entry of the ragged plan: a run of at most kPlanTileCols columns that
// lies inside one segment and starts on a multiple of 8 columns.
struct Tile {
    int64_t start;
    int32_t len;
    int32_t pad;
};

}  // namespace ds
