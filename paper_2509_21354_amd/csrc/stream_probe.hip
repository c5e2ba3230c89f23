// Calibration kernel behind kvev_debug_stream_probe (include/kvev_test_hooks.h): a plain streaming reader with an
// optional small write stream, the memory pattern of chunk pooling without any of its arithmetic.  It exists to show
// what the machine gives a kernel of that shape (a pure read stream; the same stream with 1.5 % or 3 % of its bytes
// written back), next to which the pooling and attention kernels' rates are read.
#include "common.hpp"
#include "kernels.hpp"

namespace kvev {

// One workgroup per tile: reads tile16 16-byte words (one per lane and load, 8 loads in flight), folds them into one
// word, writes that word to w16 consecutive 16-byte words of the tile's own output slot.
__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst, int tile16, int w16)
{
    const int tid = threadIdx.x;
    const u32x4_t *p = src + (size_t)blockIdx.x * tile16;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (int i = tid; i < tile16; i += 256 * 8) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[min(i + 256 * u, tile16 - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    if (w16 == 0) {
        // nothing is written; a store that no data satisfies keeps the loads alive
        if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0f1e2d3cu) dst[0] = acc;
    } else {
        for (int i = tid; i < w16; i += 256) dst[(size_t)blockIdx.x * w16 + i] = acc;
    }
}

hipError_t launch_stream_probe(const void *src, size_t tiles, int tile_bytes, void *dst, int write_bytes, hipStream_t st)
{
    if (tiles == 0) return hipSuccess;
    hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)tiles), dim3(256), 0, st, static_cast<const u32x4_t *>(src),
                       static_cast<u32x4_t *>(dst), tile_bytes / 16, write_bytes / 16);
    return hipGetLastError();
}

}  // namespace kvev
