// Measurement helper, not a step of the layer: a plain streaming read of a device buffer, the
// practical ceiling the weight stream of the grouped FFN (Janus Sec. 2.2) is compared with.
#include "common.h"

namespace {

// Every thread keeps kUnroll independent 16-byte loads in flight per iteration of a grid-stride
// loop (consecutive threads read consecutive 16 bytes); the xor of everything read is stored
// under a condition that practically never holds, so that no load can be dropped.
constexpr int kUnroll = 8;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256)
void read_probe_kernel(const u32x4 *__restrict__ src, size_t n16, uint32_t *__restrict__ sink) {
    const size_t stride = static_cast<size_t>(gridDim.x) * blockDim.x;
    size_t i = blockIdx.x * static_cast<size_t>(blockDim.x) + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (kUnroll - 1) * stride < n16; i += kUnroll * stride) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(&src[i + u * stride]);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u];
    }
    for (; i < n16; i += stride) acc ^= src[i];
    const uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (x == 0x9e3779b9u) sink[blockIdx.x & 63] = x;
}

}  // namespace

extern "C" int moe_read_probe(const void *src_dev, size_t bytes, void *sink_dev, void *stream) {
    if (!src_dev || !sink_dev) return MOE_EINVAL;
    if (!moe::aligned(src_dev, 16) || !moe::aligned(sink_dev, 4)) return MOE_EINVAL;
    if (bytes < 16) return MOE_OK;
    hipLaunchKernelGGL(read_probe_kernel, dim3(512), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const u32x4 *>(src_dev), bytes / 16, static_cast<uint32_t *>(sink_dev));
    return moe::check_launch("moe_read_probe");
}
