// Attention-head router and per-request top-k for gfx950 (Section 4.2: a single fully
// connected layer gives one scalar logit per head; the k highest-logit heads of each
// request form that request's row of the batch head index).
//
// One workgroup of 1024 threads per request.  The [D, H] weight matrix is H-innermost, so a
// thread that owns VEC adjacent columns (VEC = 8, 4, 2 or 1, the largest that divides H and
// the pointer alignment) reads them with one load, and thread tid = slice*(H/VEC) + cg walks
// a contiguous stream of Wr: in pass it, the threads together read rows it*nslice ..
// it*nslice+nslice-1 of the matrix back to back.  Every wave load is therefore fully
// coalesced, and each thread stays on its own columns for rows slice, slice+nslice, ...
//
// Arithmetic: products of two 16-bit values are exact in double and the sum is accumulated
// in double, in an order that depends on D, H and VEC only: two interleaved chains per
// thread, added, then the slices are summed in two fixed levels (ascending order inside
// each).  Identical columns therefore give bit-identical logits, and any disagreement with
// a double-precision reference is confined to ~1e-13 of summation-order rounding, far below
// the gaps between distinct logits, which is what lets the selected ids be compared bit for
// bit.
//
// Top-k is rank counting in LDS (H <= 256): the rank of head h is the number of heads that
// precede it in the order "larger logit first, equal logits by lower id, NaN last"; heads
// of rank < k write their id at position rank.
#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kRouterThreads = 1024;

template <bool BF> __device__ __forceinline__ double widen_one(uint32_t bits16)
{
    if (BF) return (double)__uint_as_float(bits16 << 16);
    return (double)(float)__builtin_bit_cast(_Float16, (uint16_t)bits16);
}

template <int VEC> struct VecOf;
template <> struct VecOf<8> { typedef uint4 type; };
template <> struct VecOf<4> { typedef uint2 type; };
template <> struct VecOf<2> { typedef uint32_t type; };
template <> struct VecOf<1> { typedef uint16_t type; };

// The VEC 16-bit patterns of a loaded vector, element v in ascending address order.
__device__ __forceinline__ uint32_t lane16(const uint4 &x, int v)
{
    const uint32_t w = v < 2 ? x.x : v < 4 ? x.y : v < 6 ? x.z : x.w;
    return (v & 1) ? (w >> 16) : (w & 0xffffu);
}
__device__ __forceinline__ uint32_t lane16(const uint2 &x, int v)
{
    const uint32_t w = v < 2 ? x.x : x.y;
    return (v & 1) ? (w >> 16) : (w & 0xffffu);
}
__device__ __forceinline__ uint32_t lane16(const uint32_t &x, int v)
{
    return (v & 1) ? (x >> 16) : (x & 0xffffu);
}
__device__ __forceinline__ uint32_t lane16(const uint16_t &x, int) { return x; }

// true when head a precedes head b in the selection order
__device__ __forceinline__ bool precedes(double va, int a, double vb, int b)
{
    const bool an = va != va, bn = vb != vb;
    if (an || bn) return (an && bn) ? (a < b) : bn;
    return va > vb || (va == vb && a < b);
}

// dynamic LDS: uint16 hidden[Dpad] | double part[nslice*H] | double part2[J*H] | double logit[H]
template <bool BF, int VEC>
__global__ __launch_bounds__(kRouterThreads) void router_topk_kernel(
    const uint16_t *__restrict__ hidden, const uint16_t *__restrict__ Wr, int D, int H, int k,
    int nslice, int J, int Dpad, int32_t *__restrict__ head_idx, float *__restrict__ logits_out)
{
    typedef typename VecOf<VEC>::type vec_t;
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *sh_hidden = reinterpret_cast<uint16_t *>(smem);
    double *sh_part = reinterpret_cast<double *>(smem + (size_t)Dpad * sizeof(uint16_t));
    double *sh_part2 = sh_part + (size_t)nslice * H;
    double *sh_logit = sh_part2 + (size_t)J * H;

    const int b = blockIdx.x, tid = threadIdx.x;
    const uint16_t *hrow = hidden + (size_t)b * D;
    for (int i = tid; i < D; i += kRouterThreads) sh_hidden[i] = hrow[i];
    __syncthreads();

    const int CG = H / VEC;                    // column groups per row of Wr
    if (tid < nslice * CG) {
        const int slice = tid / CG, cg = tid - slice * CG;
        const vec_t *w = reinterpret_cast<const vec_t *>(Wr) + cg;
        double a0[VEC], a1[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) a0[v] = a1[v] = 0.0;
        int i = slice;
        for (; i + 3 * nslice < D; i += 4 * nslice) {
            const vec_t w0 = w[(size_t)i * CG];
            const vec_t w1 = w[(size_t)(i + nslice) * CG];
            const vec_t w2 = w[(size_t)(i + 2 * nslice) * CG];
            const vec_t w3 = w[(size_t)(i + 3 * nslice) * CG];
            const double h0 = widen_one<BF>(sh_hidden[i]);
            const double h1 = widen_one<BF>(sh_hidden[i + nslice]);
            const double h2 = widen_one<BF>(sh_hidden[i + 2 * nslice]);
            const double h3 = widen_one<BF>(sh_hidden[i + 3 * nslice]);
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                a0[v] = fma(h0, widen_one<BF>(lane16(w0, v)), a0[v]);
                a1[v] = fma(h1, widen_one<BF>(lane16(w1, v)), a1[v]);
                a0[v] = fma(h2, widen_one<BF>(lane16(w2, v)), a0[v]);
                a1[v] = fma(h3, widen_one<BF>(lane16(w3, v)), a1[v]);
            }
        }
        for (; i < D; i += nslice) {
            const vec_t w0 = w[(size_t)i * CG];
            const double h0 = widen_one<BF>(sh_hidden[i]);
#pragma unroll
            for (int v = 0; v < VEC; ++v) a0[v] = fma(h0, widen_one<BF>(lane16(w0, v)), a0[v]);
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) sh_part[(size_t)slice * H + cg * VEC + v] = a0[v] + a1[v];
    }
    __syncthreads();

    // level 1: group j adds slices j, j+J, j+2J, ... in ascending order
    if (tid < J * H) {
        const int j = tid / H, h = tid - j * H;
        double sum = 0.0;
        for (int s = j; s < nslice; s += J) sum += sh_part[(size_t)s * H + h];
        sh_part2[tid] = sum;
    }
    __syncthreads();
    // level 2: the J group sums in ascending order
    if (tid < H) {
        double sum = 0.0;
        for (int j = 0; j < J; ++j) sum += sh_part2[j * H + tid];
        sh_logit[tid] = sum;
        if (logits_out) logits_out[(size_t)b * H + tid] = (float)sum;
    }
    __syncthreads();

    if (tid < H) {
        const double mine = sh_logit[tid];
        int rank = 0;
        for (int j = 0; j < H; ++j) rank += precedes(sh_logit[j], j, mine, tid) ? 1 : 0;
        if (rank < k) head_idx[(size_t)b * k + rank] = tid;
    }
}

template <bool BF, int VEC>
hipError_t launch_vec(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k,
                      int32_t *head_idx, float *logits_out, hipStream_t stream)
{
    const int CG = H / VEC;
    int nslice = kRouterThreads / CG;
    if (nslice > D) nslice = D;
    int J = 1;
    while (J * J < nslice) ++J;                       // about sqrt(nslice) groups
    if (J > kRouterThreads / H) J = kRouterThreads / H;
    if (J < 1) J = 1;
    const int Dpad = (D + 7) & ~7;                    // keeps the double arrays 16-byte aligned
    const size_t lds = (size_t)Dpad * sizeof(uint16_t) +
                       ((size_t)nslice * H + (size_t)J * H + H) * sizeof(double);
    auto kern = router_topk_kernel<BF, VEC>;
    if (lds > 48 * 1024) {
        // above the default dynamic-LDS allowance; the CU has 160 KB
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)B), dim3(kRouterThreads), lds, stream, hidden, Wr, D, H,
                       k, nslice, J, Dpad, head_idx, logits_out);
    return hipGetLastError();
}

template <bool BF>
hipError_t launch_dt(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k,
                     int32_t *head_idx, float *logits_out, hipStream_t stream)
{
    const uintptr_t addr = reinterpret_cast<uintptr_t>(Wr);
    if (H % 8 == 0 && addr % 16 == 0)
        return launch_vec<BF, 8>(hidden, Wr, B, D, H, k, head_idx, logits_out, stream);
    if (H % 4 == 0 && addr % 8 == 0)
        return launch_vec<BF, 4>(hidden, Wr, B, D, H, k, head_idx, logits_out, stream);
    if (H % 2 == 0 && addr % 4 == 0)
        return launch_vec<BF, 2>(hidden, Wr, B, D, H, k, head_idx, logits_out, stream);
    return launch_vec<BF, 1>(hidden, Wr, B, D, H, k, head_idx, logits_out, stream);
}

}  // namespace

hipError_t launch_router_topk(const void *hidden, const void *Wr, int B, int D, int H, int k,
                              polar_dtype dt, int32_t *head_idx, float *logits_out,
                              hipStream_t stream)
{
    const uint16_t *h16 = static_cast<const uint16_t *>(hidden);
    const uint16_t *w16 = static_cast<const uint16_t *>(Wr);
    if (dt == POLAR_BF16) return launch_dt<true>(h16, w16, B, D, H, k, head_idx, logits_out, stream);
    return launch_dt<false>(h16, w16, B, D, H, k, head_idx, logits_out, stream);
}

}  // namespace polar
