// Streaming-read yardstick: what a kernel that does nothing but read contiguous slabs reaches
// on this GPU with the attention kernel's launch shape.  It gives the bench a measured ceiling to
// set beside the nominal HBM peak, so "the kernel is at the memory system's practical limit" is
// a number and not a claim.  A second probe reads gathered weight rows the way the selective
// GEMMs do.  Not part of the method; no arithmetic of the paper lives here.  Built into a library
// of its own (libpolar_probe.so, polar_probe.h) so the product library holds operations only.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "polar_probe.h"

namespace polar {
namespace {

thread_local int g_probe_hip_error = 0;

int record(hipError_t e)
{
    if (e == hipSuccess) return POLAR_OK;
    g_probe_hip_error = (int)e;
    return POLAR_EHIP;
}

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

// The selective GEMMs' access pattern and nothing else: workgroup (tile, slice) of two waves reads
// K / slices values of each of 64 gathered rows, wave w rows 32 w ..., in 256-byte pieces (16 lanes
// per piece, 4 rows per wave-wide load, 8 loads per 128-value block), `depth` blocks in flight per
// wave (1 or 4); every word is folded into sink[2 * workgroup + wave].
template <bool NT, int DEPTH>
__global__ __launch_bounds__(128) void gather_probe_kernel(const uint16_t *__restrict__ W,
                                                          const int32_t *__restrict__ idx, int n_idx, int N,
                                                          int K, int slices, uint32_t *__restrict__ sink)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int tile = (int)blockIdx.x / slices, slice = (int)blockIdx.x % slices;
    const int first = tile * 64 + wave * 32;
    if (first >= n_idx) return;
    const int per_slice = K / slices;                               // values; a multiple of 128
    const u32x4 *rows[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        int j = first + (lane >> 4) + 4 * i;
        j = j < n_idx ? j : n_idx - 1;
        int id = idx[j];
        id = (id >= 0 && id < N) ? id : 0;
        rows[i] = reinterpret_cast<const u32x4 *>(W + (size_t)id * K + (size_t)slice * per_slice) + (lane & 15);
    }
    const int blocks = per_slice / 128;
    u32x4 q[DEPTH][8];
    u32x4 acc = {0u, 0u, 0u, 0u};
    // blocks is a multiple of DEPTH (checked by the host): the loop has no conditional part
#pragma unroll
    for (int r = 0; r < DEPTH; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const u32x4 *p = rows[i] + (size_t)r * 16;
            q[r][i] = NT ? __builtin_nontemporal_load(p) : *p;
        }
    for (int b = 0; b < blocks; b += DEPTH) {
#pragma unroll
        for (int r = 0; r < DEPTH; ++r) {
#pragma unroll
            for (int i = 0; i < 8; ++i) acc ^= q[r][i];
            // the last pass refills with the last block again (from cache); that data is not folded
            const int nx = b + r + DEPTH < blocks ? b + r + DEPTH : blocks - 1;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const u32x4 *p = rows[i] + (size_t)nx * 16;
                q[r][i] = NT ? __builtin_nontemporal_load(p) : *p;
            }
        }
    }
    uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x ^= __shfl_xor(x, off);
    if (lane == 0) sink[2 * blockIdx.x + wave] = x;
}

hipError_t launch_gather_probe(const void *W, const int32_t *idx, int n_idx, int N, int K, int slices,
                               int depth, int nontemporal, uint32_t *sink, hipStream_t stream)
{
    const uint16_t *w = static_cast<const uint16_t *>(W);
    const dim3 grid((unsigned)((n_idx + 63) / 64 * slices)), block(128);
#define POLAR_GATHER_PROBE(NT, D) \
    hipLaunchKernelGGL((gather_probe_kernel<NT, D>), grid, block, 0, stream, w, idx, n_idx, N, K, slices, sink)
    if (nontemporal) {
        if (depth == 1) POLAR_GATHER_PROBE(true, 1);
        else POLAR_GATHER_PROBE(true, 4);
    } else {
        if (depth == 1) POLAR_GATHER_PROBE(false, 1);
        else POLAR_GATHER_PROBE(false, 4);
    }
#undef POLAR_GATHER_PROBE
    return hipGetLastError();
}

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

}  // namespace
}  // namespace polar

using namespace polar;

extern "C" {

int polar_probe_last_hip_error(void) { return g_probe_hip_error; }

int polar_probe_read(const void *src, size_t slabs, size_t slab_bytes, int nontemporal, uint32_t *sink,
                     void *stream)
{
    if (slab_bytes < 16 || slab_bytes % 16 != 0 || slabs > 0x7fffffffu) return POLAR_EINVAL;
    if (slabs == 0) return POLAR_OK;
    if (!src || !sink || ((uintptr_t)src & 15u) != 0) return POLAR_EINVAL;
    return record(launch_read_probe(src, slabs, slab_bytes, nontemporal, sink,
                                    static_cast<hipStream_t>(stream)));
}

int polar_probe_gather_read(const void *W, const int32_t *idx, int n_idx, int N, int K, int slices, int depth,
                            int nontemporal, uint32_t *sink, void *stream)
{
    if (n_idx < 0 || N < 1 || K < 1 || slices < 1) return POLAR_EINVAL;
    if (depth != 1 && depth != 4) return POLAR_EINVAL;
    if (K % (128 * slices * depth) != 0 || (long long)N * K > (1ll << 40)) return POLAR_EUNSUPPORTED;
    if ((long long)((n_idx + 63) / 64) * slices > (1ll << 30)) return POLAR_EUNSUPPORTED;
    if (n_idx == 0) return POLAR_OK;
    if (!W || !idx || !sink || ((uintptr_t)W & 15u)) return POLAR_EINVAL;
    return record(launch_gather_probe(W, idx, n_idx, N, K, slices, depth, nontemporal, sink,
                                      static_cast<hipStream_t>(stream)));
}

}  // extern "C"
