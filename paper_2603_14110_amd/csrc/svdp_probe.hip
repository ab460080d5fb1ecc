// Measurement helpers declared in include/svdp_probe.h: the fixed costs and ceilings the decode
// step's time is set against.  Not part of the decode path.
#include "../../include/svdp_probe.h"

#include <hip/hip_runtime.h>

namespace {

__global__ void k_null() {}

__global__ void k_stamp(uint64_t *slot)
{
    if (threadIdx.x == 0) slot[0] = wall_clock64();
}

__global__ void k_handover(uint32_t *cell)
{
    if (threadIdx.x == 0) cell[0] = cell[0] + 1u;
}

__global__ __launch_bounds__(512) void k_stream_read(const uint4 *__restrict__ p, size_t n16, uint32_t *sink)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (; i < n16; i += stride) {
        const uint4 v = p[i];
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x12345678u) sink[0] = acc;      // keeps the loads; practically never true
}

__global__ void k_chase(const uint32_t *__restrict__ ring, uint32_t n, int hops, uint64_t *ticks)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    uint32_t i = 0;
    const uint64_t t0 = wall_clock64();
    for (int h = 0; h < hops; ++h) i = ring[i] % n;
    const uint64_t t1 = wall_clock64();
    ticks[0] = t1 - t0;
    ticks[1] = i;
}

inline int32_t status()
{
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

}  // namespace

extern "C" {

int32_t svdp_probe_null(int32_t blocks, int32_t threads, void *stream)
{
    if (blocks < 1 || threads < 1 || threads > 1024) return 1;
    hipLaunchKernelGGL(k_null, dim3(blocks), dim3(threads), 0, static_cast<hipStream_t>(stream));
    return status();
}

int32_t svdp_probe_stamp(uint64_t *slot, void *stream)
{
    if (slot == nullptr) return 1;
    hipLaunchKernelGGL(k_stamp, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), slot);
    return status();
}

int32_t svdp_probe_handover(uint32_t *cell, void *stream)
{
    if (cell == nullptr) return 1;
    hipLaunchKernelGGL(k_handover, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), cell);
    return status();
}

int32_t svdp_probe_stream_read(const void *src, size_t bytes, int32_t blocks, uint32_t *sink, void *stream)
{
    if (src == nullptr || sink == nullptr || bytes == 0 || bytes % 16 != 0 || blocks < 1 ||
        (reinterpret_cast<uintptr_t>(src) & 15u))
        return 1;
    hipLaunchKernelGGL(k_stream_read, dim3(blocks), dim3(512), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4 *>(src), bytes / 16, sink);
    return status();
}

int32_t svdp_probe_chase(const uint32_t *ring, uint32_t n, int32_t hops, uint64_t *ticks, void *stream)
{
    if (ring == nullptr || ticks == nullptr || n < 1 || hops < 1) return 1;
    hipLaunchKernelGGL(k_chase, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), ring, n, hops, ticks);
    return status();
}

}  // extern "C"
