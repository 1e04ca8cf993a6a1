// Measurement aid of bench.py, not part of the DS-Sync library: a plain
// device-to-device streaming copy whose traffic is known exactly (reads
// `bytes`, writes `bytes`).  bench.py uses it as the attainable-bandwidth
// yardstick and to scale the profiler's HBM byte counters.
// Built into libbench_probe.so by `bench.py --build-probe` and by the
// repository's build entry point.
#include <hip/hip_runtime.h>
#include <stdint.h>

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

// dst, src: device, 16-byte aligned, non-overlapping; bytes a multiple of 16.
// Returns 0, -1 for a bad argument, -2 if the launch failed.
extern "C" int bench_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return -1;
    if ((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src) | bytes) & 15u) return -1;
    const int64_t n_vec = static_cast<int64_t>(bytes / 16);
    const int64_t per_block = kThreads * kVecPerLane;
    const int64_t n_blocks = (n_vec + per_block - 1) / per_block;
    if (n_blocks > (int64_t{1} << 24) - 1) return -1;   // grid.x * 256 threads must stay below 2^32
    if (n_blocks == 0) return 0;
    probe_copy_kernel<<<dim3(static_cast<uint32_t>(n_blocks)), dim3(kThreads), 0, static_cast<hipStream_t>(stream)>>>(
        static_cast<f32x4*>(dst), static_cast<const f32x4*>(src), n_vec);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

// What the runtime reports of the current device's clocks and memory bus (kHz, kHz, bits);
// an attribute the runtime does not know is returned as 0.  Returns 0, or -2 if no device is current.
extern "C" int bench_probe_device_clocks(int* memory_khz, int* shader_khz, int* bus_bits) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return -2;
    if (hipDeviceGetAttribute(memory_khz, hipDeviceAttributeMemoryClockRate, dev) != hipSuccess) *memory_khz = 0;
    if (hipDeviceGetAttribute(shader_khz, hipDeviceAttributeClockRate, dev) != hipSuccess) *shader_khz = 0;
    if (hipDeviceGetAttribute(bus_bits, hipDeviceAttributeMemoryBusWidth, dev) != hipSuccess) *bus_bits = 0;
    return 0;
}
