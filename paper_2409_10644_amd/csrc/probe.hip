// Measurement aid, not part of the method: a plain read-only streaming kernel.  Its bandwidth on a buffer much
// larger than the caches is what this machine's HBM delivers to the simplest possible reader, the yardstick
// next to the datasheet peak for the tree-attention sweep's achieved bandwidth.
#include "mcsd_internal.h"

namespace {

typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));

// Every thread reads 16-byte words grid-strided, eight loads in flight, and folds them into one word that is
// stored only if it has an (impossible in practice) value, so the loads cannot be optimised away.  The loads are
// non-temporal, like the sweep's: read-once data that the caches need not keep.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4_t *__restrict__ src, size_t n16, u32x4_t *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    u32x4_t acc = {0, 0, 0, 0};
    for (; i + 7 * stride < n16; i += 8 * stride) {
        u32x4_t v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
        for (int k = 0; k < 8; ++k) acc ^= v[k];
    }
    for (; i < n16; i += stride) {
        acc ^= __builtin_nontemporal_load(src + i);
    }
    if (acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u && acc.z == 0x85ebca6bu && acc.w == 0xc2b2ae35u) *sink = acc;
}

}  // namespace

extern "C" int mcsd_stream_read(const void *src_dev, size_t bytes, void *sink_dev, int32_t workgroups, void *hip_stream)
{
    if (!src_dev || !sink_dev || bytes < 16 || ((uintptr_t)src_dev & 15) || ((uintptr_t)sink_dev & 15)) return MCSD_EINVAL;
    if (workgroups < 0 || workgroups > 65535) return MCSD_EINVAL;
    mcsd_launch(MCSD_KERNEL_STREAM_READ, stream_read_kernel, dim3(workgroups ? workgroups : 1024), dim3(256), (hipStream_t)hip_stream,
                (const u32x4_t *)src_dev, bytes / 16, (u32x4_t *)sink_dev);
    return mcsd_hip_status(hipGetLastError());
}
