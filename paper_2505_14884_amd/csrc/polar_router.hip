// Attention-head router and per-request top-k for gfx950 (Section 4.2: a single fully
// connected layer gives one scalar logit per head; the k highest-logit heads of each
// request form that request's row of the batch head index).
//
// One workgroup per request.  The [D, H] weight matrix is H-innermost, so thread
// tid = slice*H + h simply walks a contiguous stream of Wr (element it*T + tid of the
// matrix is row it*nslice + slice, column h): every wave load is fully coalesced and each
// thread stays on one column.  Products of two 16-bit values are exact in double and the
// sum is accumulated in double, in an order that depends on D and H only: four
// interleaved chains per thread, combined pairwise, then the slices added in ascending
// order.  Identical columns therefore give bit-identical logits, and any disagreement
// with a double-precision reference is confined to ~1e-13 of summation-order rounding,
// far below the gaps between distinct logits, which is what lets the selected ids be
// compared bit for bit.
//
// Top-k is rank counting in LDS (H <= 256): the rank of head h is the number of heads
// that precede it in the order "larger logit first, equal logits by lower id, NaN last";
// heads of rank < k write their id at position rank.
#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kRouterThreads = 1024;

template <bool BF> __device__ __forceinline__ double widen_one(uint16_t bits)
{
    if (BF) return (double)__uint_as_float((uint32_t)bits << 16);
    return (double)(float)__builtin_bit_cast(_Float16, bits);
}

// true when head a precedes head b in the selection order
__device__ __forceinline__ bool precedes(double va, int a, double vb, int b)
{
    const bool an = va != va, bn = vb != vb;
    if (an || bn) return (an && bn) ? (a < b) : bn;
    return va > vb || (va == vb && a < b);
}

// dynamic LDS: uint16 hidden[Dpad] | double partial[nslice*H] | double logit[H]
template <bool BF>
__global__ __launch_bounds__(kRouterThreads) void router_topk_kernel(
    const uint16_t *__restrict__ hidden, const uint16_t *__restrict__ Wr, int D, int H, int k,
    int nslice, int Dpad, int32_t *__restrict__ head_idx, float *__restrict__ logits_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *sh_hidden = reinterpret_cast<uint16_t *>(smem);
    double *sh_partial = reinterpret_cast<double *>(smem + (size_t)Dpad * sizeof(uint16_t));
    double *sh_logit = sh_partial + (size_t)nslice * H;

    const int b = blockIdx.x, tid = threadIdx.x;
    const uint16_t *hrow = hidden + (size_t)b * D;
    for (int i = tid; i < D; i += kRouterThreads) sh_hidden[i] = hrow[i];
    __syncthreads();

    const int T = nslice * H;
    if (tid < T) {
        const int slice = tid / H, h = tid - slice * H;
        const uint16_t *w = Wr + h;
        double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
        int i = slice;
        for (; i + 3 * nslice < D; i += 4 * nslice) {
            const uint16_t w0 = w[(size_t)i * H];
            const uint16_t w1 = w[(size_t)(i + nslice) * H];
            const uint16_t w2 = w[(size_t)(i + 2 * nslice) * H];
            const uint16_t w3 = w[(size_t)(i + 3 * nslice) * H];
            a0 = fma(widen_one<BF>(sh_hidden[i]), widen_one<BF>(w0), a0);
            a1 = fma(widen_one<BF>(sh_hidden[i + nslice]), widen_one<BF>(w1), a1);
            a2 = fma(widen_one<BF>(sh_hidden[i + 2 * nslice]), widen_one<BF>(w2), a2);
            a3 = fma(widen_one<BF>(sh_hidden[i + 3 * nslice]), widen_one<BF>(w3), a3);
        }
        for (; i < D; i += nslice)
            a0 = fma(widen_one<BF>(sh_hidden[i]), widen_one<BF>(w[(size_t)i * H]), a0);
        sh_partial[tid] = (a0 + a1) + (a2 + a3);
    }
    __syncthreads();

    if (tid < H) {
        double sum = 0.0;
        for (int s = 0; s < nslice; ++s) sum += sh_partial[s * H + tid];
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

}  // namespace

hipError_t launch_router_topk(const void *hidden, const void *Wr, int B, int D, int H, int k,
                              polar_dtype dt, int32_t *head_idx, float *logits_out,
                              hipStream_t stream)
{
    int nslice = kRouterThreads / H;
    if (nslice > D) nslice = D;
    const int Dpad = (D + 7) & ~7;   // keeps the double arrays 16-byte aligned
    const size_t lds = (size_t)Dpad * sizeof(uint16_t) + ((size_t)nslice * H + H) * sizeof(double);
    const uint16_t *h16 = static_cast<const uint16_t *>(hidden);
    const uint16_t *w16 = static_cast<const uint16_t *>(Wr);
    if (dt == POLAR_BF16)
        hipLaunchKernelGGL((router_topk_kernel<true>), dim3((unsigned)B), dim3(kRouterThreads), lds,
                           stream, h16, w16, D, H, k, nslice, Dpad, head_idx, logits_out);
    else
        hipLaunchKernelGGL((router_topk_kernel<false>), dim3((unsigned)B), dim3(kRouterThreads), lds,
                           stream, h16, w16, D, H, k, nslice, Dpad, head_idx, logits_out);
    return hipGetLastError();
}

}  // namespace polar
