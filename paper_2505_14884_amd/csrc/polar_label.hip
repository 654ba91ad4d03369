// Head-importance labeller for gfx950 (Section 3.2, head-sparsity study: heads are ranked by
// the L2 norm of their attention output; Section 4.2: the k heads with the highest output
// norms of each input are the supervision targets of the attention router).
//
// Input is the dense decode-attention output (polar_sha_decode with head_idx = NULL).  One
// workgroup per request; each wave takes KV groups g = wave, wave + 4, ...; its lanes add the
// squares of the group's G*d output values (a float squared is exact in double; accumulation
// in double), the 64 lane sums are combined by an xor butterfly, and the groups are ranked by
// that sum of squares with the router's ordering rule (larger first, ties to the lower id,
// NaN last).  Ranking uses the sum of squares itself, not its square root, so no rounding of
// the root can create or break a tie.
#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kLabelThreads = 256;

__device__ __forceinline__ double shfl_xor_f64(double x, int mask)
{
    int lo = __shfl_xor(__double2loint(x), mask);
    int hi = __shfl_xor(__double2hiint(x), mask);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ bool precedes(double va, int a, double vb, int b)
{
    const bool an = va != va, bn = vb != vb;
    if (an || bn) return (an && bn) ? (a < b) : bn;
    return va > vb || (va == vb && a < b);
}

__global__ __launch_bounds__(kLabelThreads) void head_norm_topk_kernel(
    const float *__restrict__ attn_out, int Hkv, int group_elems, int k,
    int32_t *__restrict__ head_idx, float *__restrict__ norms_out)
{
    __shared__ double sh_ss[POLAR_MAX_ROUTER_H];
    __shared__ int sh_rank[POLAR_MAX_ROUTER_H];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *row = attn_out + (size_t)b * Hkv * group_elems;
    for (int g = wave; g < Hkv; g += kLabelThreads / 64) {
        const float *src = row + (size_t)g * group_elems;
        double ss = 0.0;
        for (int e = lane; e < group_elems; e += 64) {
            const double v = (double)src[e];
            ss = fma(v, v, ss);
        }
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) ss += shfl_xor_f64(ss, m);
        if (lane == 0) {
            sh_ss[g] = ss;
            sh_rank[g] = 0;
            if (norms_out) norms_out[(size_t)b * Hkv + g] = (float)sqrt(ss);
        }
    }
    __syncthreads();
    const int parts = kLabelThreads / Hkv;            // >= 1: Hkv <= 256
    if (tid < parts * Hkv) {
        const int part = tid / Hkv, h = tid - part * Hkv;
        const double mine = sh_ss[h];
        int cnt = 0;
        for (int j = part; j < Hkv; j += parts) cnt += precedes(sh_ss[j], j, mine, h) ? 1 : 0;
        if (cnt) atomicAdd(&sh_rank[h], cnt);
    }
    __syncthreads();
    if (tid < Hkv && sh_rank[tid] < k) head_idx[(size_t)b * k + sh_rank[tid]] = tid;
}

}  // namespace

hipError_t launch_head_norm_topk(const float *attn_out, int B, int Hq, int Hkv, int d, int k,
                                 int32_t *head_idx, float *norms_out, hipStream_t stream)
{
    const int group_elems = (Hq / Hkv) * d;
    hipLaunchKernelGGL(head_norm_topk_kernel, dim3((unsigned)B), dim3(kLabelThreads), 0, stream,
                       attn_out, Hkv, group_elems, k, head_idx, norms_out);
    return hipGetLastError();
}

}  // namespace polar
