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
// hand back to the caller.  max_size receives the largest group size.
int pack_partition(int32_t W, const int32_t* perm, const int32_t* off, int32_t n_groups,
                   PartitionArg* out, int32_t* max_size);

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// What the launch rules need to know of the current device.  Read with
// hipDeviceGetAttribute on the first launch on a device and kept for the
// life of the process (no allocation).  Returns DS_OK or DS_ERR_HIP.
struct DeviceInfo {
    int compute_units;
    unsigned lds_per_cu;   // bytes
};
int device_info(DeviceInfo* out);

// Group-sync launch shape.  A workgroup is ONE wavefront; a lane owns one
// vector of 4 consecutive columns, so a workgroup covers 256 columns of every
// member row (1 KiB per row and load instruction) and loads up to
// kSyncLoadsPerLane/2 members (x and g each) per round.
constexpr int kSyncThreads = 64;
constexpr int kSyncTileCols = kSyncThreads * 4;
constexpr int kSyncLoadsPerLane = 16;
// Unit of the ragged plan: 2048 columns = 8 workgroups.
constexpr int kPlanTileCols = 2048;

// HIP refuses a launch whose gridDim.x * blockDim.x reaches 2^32; with
// one-wavefront workgroups that is 2^26 workgroups along x.
constexpr int64_t kMaxSyncGridX = (int64_t{1} << 32) / kSyncThreads - 1;

// One entry of the ragged plan: a run of at most kPlanTileCols columns that
// lies inside one segment and starts on a multiple of 8 columns.
struct Tile {
    int64_t start;
    int32_t len;
    int32_t pad;
};

// Entry 0 of a plan buffer: says which segment list the entries after it were
// cut from, so that a launch can tell a plan that belongs to another list.
struct PlanHeader {
    uint64_t id;        // ds_ragged_plan's plan_id_out: hash of the list, never 0
    int32_t n_segments;
    int32_t n_entries;  // Tile entries that follow
};
static_assert(sizeof(PlanHeader) == sizeof(Tile), "the header takes the place of one entry");

}  // namespace ds
