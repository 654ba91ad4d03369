// Streaming-read yardstick: what a kernel that does nothing but read contiguous slabs reaches
// on this GPU with the attention kernel's launch shape.  It gives the bench a measured ceiling to
// set beside the nominal HBM peak, so "the kernel is at the memory system's practical limit" is
// a number and not a claim.  Not part of the method; no arithmetic of the paper lives here.
#include "polar_internal.h"

namespace polar {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
constexpr int kProbeWaves = 8;    // waves per workgroup, as in the per-head streaming kernel
constexpr int kProbeLoads = 16;   // 16-byte loads in flight per lane (K and V rows there: 8 + 8)

// Workgroup w reads slab w (slab_vecs 16-byte units, contiguous), wave-wide loads of 1 KiB,
// kProbeLoads of them in flight per wave; every loaded word is folded into one value per
// workgroup, stored to sink[w], so that no load can be dropped.
template <bool NT>
__global__ __launch_bounds__(kProbeWaves * 64) void read_probe_kernel(const u32x4 *__restrict__ src,
                                                                     size_t slab_vecs,
                                                                     uint32_t *__restrict__ sink)
{
    const u32x4 *p = src + (size_t)blockIdx.x * slab_vecs;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    constexpr size_t kWaveStep = (size_t)kProbeLoads * 64;          // units one wave takes per step
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (size_t i0 = (size_t)wave * kWaveStep; i0 < slab_vecs; i0 += (size_t)kProbeWaves * kWaveStep) {
        u32x4 v[kProbeLoads];
#pragma unroll
        for (int u = 0; u < kProbeLoads; ++u) {
            size_t i = i0 + (size_t)u * 64 + lane;
            if (i >= slab_vecs) i = slab_vecs - 1;                   // clamp: stays inside the slab
            v[u] = NT ? __builtin_nontemporal_load(p + i) : p[i];
        }
#pragma unroll
        for (int u = 0; u < kProbeLoads; ++u) acc ^= v[u];
    }
    uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x ^= __shfl_xor(x, off);
    __shared__ uint32_t sh[kProbeWaves];
    if (lane == 0) sh[wave] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t y = 0;
        for (int w = 0; w < kProbeWaves; ++w) y ^= sh[w];
        sink[blockIdx.x] = y;
    }
}

}  // namespace

hipError_t launch_read_probe(const void *src, size_t slabs, size_t slab_bytes, int nontemporal,
                             uint32_t *sink, hipStream_t stream)
{
    const u32x4 *p = static_cast<const u32x4 *>(src);
    const dim3 grid((unsigned)slabs), block(kProbeWaves * 64);
    if (nontemporal)
        hipLaunchKernelGGL(read_probe_kernel<true>, grid, block, 0, stream, p, slab_bytes / 16, sink);
    else
        hipLaunchKernelGGL(read_probe_kernel<false>, grid, block, 0, stream, p, slab_bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace polar
