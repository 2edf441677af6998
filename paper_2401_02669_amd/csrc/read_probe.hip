// Measurement probes, built into a library of their own (libdistattn_probe.so), not into the attention library.
//
// Read-ceiling probe: streams a device buffer once with the same 16-byte-per-lane loads the
// MicroAttention kernels use and only adds the words up.  It measures the HBM read rate this GPU
// sustains for a pure streaming kernel, the practical ceiling the attention kernels are compared to.
// Copy probe: a plain copy of a known size, against which hardware traffic counters are scaled.
#include <hip/hip_runtime.h>

#include "../../include/distattn_probe.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Each workgroup owns consecutive `seg_bytes` segments (round-robin over the grid); a wavefront reads
// 1 KiB per load instruction, UNROLL loads in flight.
template <int UNROLL, bool NT>
__global__ __launch_bounds__(512) void read_probe_kernel(const u32x4 *src, size_t n16, size_t seg16, uint32_t *sink)
{
    const size_t nseg = (n16 + seg16 - 1) / seg16;
    uint32_t acc = 0;
    for (size_t seg = blockIdx.x; seg < nseg; seg += gridDim.x) {
        const size_t lo = seg * seg16;
        const size_t hi = lo + seg16 < n16 ? lo + seg16 : n16;
        for (size_t i = lo + threadIdx.x; i < hi; i += (size_t)512 * UNROLL) {
            u32x4 v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const size_t k = i + (size_t)u * 512;
                v[u] = u32x4{0u, 0u, 0u, 0u};
                if (k < hi) v[u] = NT ? __builtin_nontemporal_load(src + k) : src[k];
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;  // keeps the loads alive; practically never taken
}

// Plain grid-stride copy, 16 bytes per lane and step: reads n16 * 16 bytes and writes as many, each once.
__global__ __launch_bounds__(256) void copy_probe_kernel(const u32x4 *src, u32x4 *dst, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Streaming reads with small writes mixed in.  Wavefront g of the launch reads items g, g + waves, ... of
// `item16` 16-byte words each (as a wavefront that owns whole splits reads its requests) and, after every
// `burst` items (staggered != 0: at a phase of its own instead of together with all other wavefronts), writes
// burst x frag16 words of "results" to its own region of dst.  burst == 0: no writes at all.
__global__ __launch_bounds__(256) void read_write_probe_kernel(const u32x4 *src, u32x4 *dst, size_t item16, int items_per_wave,
                                                               int frag16, int burst, int staggered, uint32_t *sink)
{
    const int lane = threadIdx.x & 63;
    const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int nw = gridDim.x * 4;
    const int phase = (staggered && burst > 0) ? gw % burst : 0;
    uint32_t acc = 0;
    int pending = 0;
    for (int it = 0; it < items_per_wave; ++it) {
        const u32x4 *p = src + ((size_t)it * nw + gw) * item16;
        for (size_t i = lane; i < item16; i += 64 * 16) {
            u32x4 v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                v[u] = u32x4{0u, 0u, 0u, 0u};
                if (i + u * 64 < item16) v[u] = __builtin_nontemporal_load(p + i + u * 64);
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
        }
        ++pending;
        if (burst > 0 && ((it + 1 + phase) % burst == 0 || it + 1 == items_per_wave)) {
            const u32x4 val = {acc, acc, acc, acc};
            u32x4 *d = dst + ((size_t)gw * items_per_wave + (it + 1 - pending)) * frag16;
            for (int i = lane; i < frag16 * pending; i += 64) d[i] = val;
            pending = 0;
        }
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;
}

}  // namespace

extern "C" da_status da_probe_read_write(const void *src, size_t bytes, void *dst, size_t dst_bytes, size_t item_bytes,
                                         size_t frag_bytes, int32_t workgroups, int32_t burst, int32_t staggered,
                                         void *sink, void *stream)
{
    if (!src || !dst || !sink || workgroups < 1 || burst < 0 || item_bytes < 16 || (item_bytes & 15) || frag_bytes < 16 ||
        (frag_bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
        return DA_ERR_INVALID_ARG;
    const size_t waves = (size_t)workgroups * 4;
    const size_t items_per_wave = bytes / item_bytes / waves;
    if (items_per_wave < 1 || items_per_wave > (1u << 20)) return DA_ERR_INVALID_ARG;
    if (dst_bytes < waves * items_per_wave * frag_bytes) return DA_ERR_INVALID_ARG;  // every wavefront's region fits
    hipLaunchKernelGGL(read_write_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4 *)src, (u32x4 *)dst, item_bytes / 16, (int)items_per_wave, (int)(frag_bytes / 16), burst,
                       staggered, (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}

extern "C" da_status da_probe_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst || bytes < 16 || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return DA_ERR_INVALID_ARG;
    hipLaunchKernelGGL(copy_probe_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream, (const u32x4 *)src, (u32x4 *)dst,
                       bytes / 16);
    return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}

extern "C" da_status da_probe_read(const void *src, size_t bytes, size_t segment_bytes, int32_t workgroups,
                                   int32_t variant, void *sink, void *stream)
{
    if (!src || !sink || bytes < 16 || segment_bytes < 16 || workgroups < 1 || ((uintptr_t)src & 15)) return DA_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16, seg16 = segment_bytes / 16;
    hipStream_t s = (hipStream_t)stream;
    dim3 grid((unsigned)workgroups), block(512);
    switch (variant) {
    case 0: hipLaunchKernelGGL((read_probe_kernel<4, false>), grid, block, 0, s, (const u32x4 *)src, n16, seg16, (uint32_t *)sink); break;
    case 1: hipLaunchKernelGGL((read_probe_kernel<8, false>), grid, block, 0, s, (const u32x4 *)src, n16, seg16, (uint32_t *)sink); break;
    case 2: hipLaunchKernelGGL((read_probe_kernel<16, false>), grid, block, 0, s, (const u32x4 *)src, n16, seg16, (uint32_t *)sink); break;
    case 3: hipLaunchKernelGGL((read_probe_kernel<8, true>), grid, block, 0, s, (const u32x4 *)src, n16, seg16, (uint32_t *)sink); break;
    case 4: hipLaunchKernelGGL((read_probe_kernel<16, true>), grid, block, 0, s, (const u32x4 *)src, n16, seg16, (uint32_t *)sink); break;
    default: return DA_ERR_INVALID_ARG;
    }
    return hipGetLastError() == hipSuccess ? DA_OK : DA_ERR_HIP;
}
