// Calibration kernel behind kvev_debug_stream_probe (include/kvev_test_hooks.h): a plain streaming reader with an
// optional small write stream, the memory pattern of chunk pooling without any of its arithmetic.  It exists to show
// what the machine gives a kernel of that shape (a pure read stream; the same stream with 1.5 % or 3 % of its bytes
// written back; each with plain accesses or with the non-temporal hint that the library's streaming kernels use),
// next to which the pooling and attention kernels' rates are read.
#include "common.hpp"
#include "kernels.hpp"
#include <algorithm>

namespace kvev {

// One workgroup per tile: reads tile16 16-byte words (one per lane and load, 8 loads in flight), folds them into one
// word, writes that word to w16 consecutive 16-byte words of the tile's own output slot.
template <bool NT_LOAD, bool NT_STORE>
__global__ __launch_bounds__(256) void stream_probe_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst, int tile16, int w16)
{
    const int tid = threadIdx.x;
    const u32x4_t *p = src + (size_t)blockIdx.x * tile16;
    u32x4_t acc = {0u, 0u, 0u, 0u};
    for (int i = tid; i < tile16; i += 256 * 8) {
        u32x4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const u32x4_t *q = p + min(i + 256 * u, tile16 - 1);
            v[u] = NT_LOAD ? __builtin_nontemporal_load(q) : *q;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
    }
    if (w16 == 0) {
        // nothing is written; a store that no data satisfies keeps the loads alive
        if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0f1e2d3cu) dst[0] = acc;
    } else {
        for (int i = tid; i < w16; i += 256) {
            u32x4_t *q = dst + (size_t)blockIdx.x * w16 + i;
            if (NT_STORE) __builtin_nontemporal_store(acc, q);
            else *q = acc;
        }
    }
}

// The same stream from persistent workgroups (two per compute unit) that hold their outputs back in LDS and write them
// when the chip-wide real-time counter (100 MHz) enters a new slot of 2^13 ticks, or when the `cap` slots are full: the
// write pattern of the pooling kernel at scale.
template <bool NT_LOAD, bool NT_STORE>
__global__ __launch_bounds__(256) void stream_probe_burst_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst,
                                                                  int tiles, int tile16, int w16, int cap)
{
    extern __shared__ u32x4_t stage[];          // cap * w16 words
    __shared__ long long s_now;
    __shared__ int s_tile[64];
    const int tid = threadIdx.x;
    int held = 0;
    long long slot = wall_clock64() >> 13;
    auto flush = [&]() {
        for (int t = 0; t < held; ++t) {
            u32x4_t *q = dst + (size_t)s_tile[t] * w16;
            for (int i = tid; i < w16; i += 256) {
                if (NT_STORE) __builtin_nontemporal_store(stage[t * w16 + i], q + i);
                else q[i] = stage[t * w16 + i];
            }
        }
        held = 0;
    };
    for (int tile = blockIdx.x; tile < tiles; tile += gridDim.x) {
        const u32x4_t *p = src + (size_t)tile * tile16;
        u32x4_t acc = {0u, 0u, 0u, 0u};
        for (int i = tid; i < tile16; i += 256 * 8) {
            u32x4_t v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const u32x4_t *q = p + min(i + 256 * u, tile16 - 1);
                v[u] = NT_LOAD ? __builtin_nontemporal_load(q) : *q;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += v[u];
        }
        for (int i = tid; i < w16; i += 256) stage[held * w16 + i] = acc;
        if (tid == 0) { s_tile[held] = tile; s_now = wall_clock64() >> 13; }
        ++held;
        __syncthreads();
        const long long now = s_now;
        if (now != slot || held == cap) { flush(); slot = now; }
        __syncthreads();
    }
    flush();
}

hipError_t launch_stream_probe(const void *src, size_t tiles, int tile_bytes, void *dst, int write_bytes, int hints, hipStream_t st)
{
    if (tiles == 0) return hipSuccess;
    const dim3 grid((unsigned)tiles), block(256);
    const u32x4_t *s = static_cast<const u32x4_t *>(src);
    u32x4_t *d = static_cast<u32x4_t *>(dst);
    const int t16 = tile_bytes / 16, w16 = write_bytes / 16;
    if ((hints & 4) && w16 > 0) {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            return hipErrorInvalidDevice;
        const int cap = std::min(64, (48 * 1024) / write_bytes);
        if (cap < 1) return hipErrorInvalidValue;
        const dim3 pgrid((unsigned)std::min<size_t>(tiles, 2 * (size_t)cus));
        const size_t lds = (size_t)cap * write_bytes;
        switch (hints & 3) {
        case 0: hipLaunchKernelGGL((stream_probe_burst_kernel<false, false>), pgrid, block, lds, st, s, d, (int)tiles, t16, w16, cap); break;
        case 1: hipLaunchKernelGGL((stream_probe_burst_kernel<true, false>), pgrid, block, lds, st, s, d, (int)tiles, t16, w16, cap); break;
        case 2: hipLaunchKernelGGL((stream_probe_burst_kernel<false, true>), pgrid, block, lds, st, s, d, (int)tiles, t16, w16, cap); break;
        default: hipLaunchKernelGGL((stream_probe_burst_kernel<true, true>), pgrid, block, lds, st, s, d, (int)tiles, t16, w16, cap); break;
        }
        return hipGetLastError();
    }
    switch (hints & 3) {
    case 0: hipLaunchKernelGGL((stream_probe_kernel<false, false>), grid, block, 0, st, s, d, t16, w16); break;
    case 1: hipLaunchKernelGGL((stream_probe_kernel<true, false>), grid, block, 0, st, s, d, t16, w16); break;
    case 2: hipLaunchKernelGGL((stream_probe_kernel<false, true>), grid, block, 0, st, s, d, t16, w16); break;
    default: hipLaunchKernelGGL((stream_probe_kernel<true, true>), grid, block, 0, st, s, d, t16, w16); break;
    }
    return hipGetLastError();
}

}  // namespace kvev
