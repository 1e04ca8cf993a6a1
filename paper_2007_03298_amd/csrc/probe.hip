// Plain device-to-device copy kernel of known size.  Not a step of the method:
// it is the yardstick the measurements are held against -- the bandwidth a
// simple streaming kernel attains on this GPU, and the reference that scales
// the profiler's HBM counters (bytes fetched / written per launch are known
// exactly for a copy).
#include <hip/hip_runtime.h>

#include "ds_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kThreads = 256;
constexpr int kVecPerLane = 4;

__global__ void __launch_bounds__(kThreads)
probe_copy_kernel(f32x4* __restrict__ dst, const f32x4* __restrict__ src, int64_t n_vec) {
    const int64_t base = static_cast<int64_t>(blockIdx.x) * (kThreads * kVecPerLane) + threadIdx.x;
    f32x4 v[kVecPerLane];
#pragma unroll
    for (int k = 0; k < kVecPerLane; ++k) {
        const int64_t i = base + k * kThreads;
        if (i < n_vec) v[k] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int k = 0; k < kVecPerLane; ++k) {
        const int64_t i = base + k * kThreads;
        if (i < n_vec) __builtin_nontemporal_store(v[k], dst + i);
    }
}

}  // namespace

extern "C" int ds_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return DS_ERR_NULL;
    if (!ds::aligned16(dst) || !ds::aligned16(src) || bytes % 16 != 0) return DS_ERR_ALIGN;
    const int64_t n_vec = static_cast<int64_t>(bytes / 16);
    const int64_t per_block = kThreads * kVecPerLane;
    const int64_t n_blocks = (n_vec + per_block - 1) / per_block;
    if (n_blocks > INT32_MAX) return DS_ERR_BAD_SHAPE;
    if (n_blocks == 0) return DS_OK;
    hipLaunchKernelGGL(probe_copy_kernel, dim3(static_cast<uint32_t>(n_blocks)), dim3(kThreads), 0,
                       static_cast<hipStream_t>(stream), static_cast<f32x4*>(dst),
                       static_cast<const f32x4*>(src), n_vec);
    return hipGetLastError() == hipSuccess ? DS_OK : DS_ERR_HIP;
}
