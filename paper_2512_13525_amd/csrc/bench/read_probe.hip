// Measurement helper, not a step of the layer and not part of libmoe_janus: a plain streaming read
// of a device buffer, swept over launch shapes by bench.py, to show what read bandwidth a launch of
// a given size reaches on this GPU next to the weight stream of the grouped FFN (Janus Sec. 2.2).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "moe_bench.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Every thread keeps U independent 16-byte loads in flight per iteration of a grid-stride loop
// (consecutive threads read consecutive 16 bytes); the xor of everything read is stored under a
// condition that practically never holds, so that no load can be dropped.
template <int U>
__global__ __launch_bounds__(256)
void read_probe_kernel(const u32x4 *__restrict__ src, size_t n16, uint32_t *__restrict__ sink) {
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (U - 1) * stride < n16; i += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(&src[i + u * stride]);
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= src[i];
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9e3779b9u) sink[blockIdx.x & 63] = x;
}

}  // namespace

extern "C" int moe_read_probe(const void *src_dev, size_t bytes, void *sink_dev, int workgroups, int loads_in_flight,
                              void *stream) {
    if (!src_dev || !sink_dev) return -1;
    if (reinterpret_cast<uintptr_t>(src_dev) % 16 || reinterpret_cast<uintptr_t>(sink_dev) % 4) return -1;
    if (workgroups < 1 || workgroups > (1 << 20)) return -1;
    if (bytes < 16) return 0;
    const u32x4 *src = static_cast<const u32x4 *>(src_dev);
    uint32_t *sink = static_cast<uint32_t *>(sink_dev);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(workgroups), block(256);
    switch (loads_in_flight) {
        case 1: hipLaunchKernelGGL(read_probe_kernel<1>, grid, block, 0, st, src, bytes / 16, sink); break;
        case 2: hipLaunchKernelGGL(read_probe_kernel<2>, grid, block, 0, st, src, bytes / 16, sink); break;
        case 4: hipLaunchKernelGGL(read_probe_kernel<4>, grid, block, 0, st, src, bytes / 16, sink); break;
        case 8: hipLaunchKernelGGL(read_probe_kernel<8>, grid, block, 0, st, src, bytes / 16, sink); break;
        case 16: hipLaunchKernelGGL(read_probe_kernel<16>, grid, block, 0, st, src, bytes / 16, sink); break;
        default: return -1;
    }
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
