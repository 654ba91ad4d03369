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
#include <atomic>

#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kRouterThreads = 1024;
constexpr int kStageBatch = 8;   // hidden elements a thread stages per batch of loads
constexpr int kRowBatch = 8;     // rows of Wr a thread loads before consuming any

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

// Rank counting spread over the whole workgroup: with `nthreads` threads, head h is handled
// by nthreads / H threads that each compare it with a strided share of the other heads and
// add their counts in LDS.  sh_rank[0..H) must be zero on entry (and visible to all threads).
__device__ __forceinline__ void rank_and_emit(const double *sh_logit, int *sh_rank, int H, int k,
                                              int nthreads, int tid, int32_t *row_out)
{
    const int parts = nthreads / H;            // >= 1: H never exceeds the workgroup size
    if (tid < parts * H) {
        const int part = tid / H, h = tid - part * H;
        const double mine = sh_logit[h];
        int cnt = 0;
#pragma unroll 4
        for (int j = part; j < H; j += parts) cnt += precedes(sh_logit[j], j, mine, h) ? 1 : 0;
        if (cnt) atomicAdd(&sh_rank[h], cnt);
    }
    __syncthreads();
    if (tid < H && sh_rank[tid] < k) row_out[sh_rank[tid]] = tid;
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
    __shared__ int sh_rank[POLAR_MAX_ROUTER_H];

    const int b = blockIdx.x, tid = threadIdx.x;
    const uint16_t *hrow = hidden + (size_t)b * D;
    // Stage the request's hidden row.  Every load of a batch is issued before any is used:
    // a dependent round trip to memory costs about a microsecond, so the kernel's time is
    // the number of such rounds, not its arithmetic.
    for (int base = 0; base < D; base += kStageBatch * kRouterThreads) {
        uint16_t v[kStageBatch];
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int i = base + u * kRouterThreads + tid;
            v[u] = i < D ? hrow[i] : (uint16_t)0;
        }
#pragma unroll
        for (int u = 0; u < kStageBatch; ++u) {
            const int i = base + u * kRouterThreads + tid;
            if (i < D) sh_hidden[i] = v[u];
        }
    }
    __syncthreads();

    const int CG = H / VEC;                    // column groups per row of Wr
    if (tid < nslice * CG) {
        const int slice = tid / CG, cg = tid - slice * CG;
        const vec_t *w = reinterpret_cast<const vec_t *>(Wr) + cg;
        double a0[VEC], a1[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) a0[v] = a1[v] = 0.0;
        // rows slice, slice + nslice, ...: kRowBatch loads in flight, then their multiply-adds,
        // even rows of the batch into chain a0 and odd rows into a1
        for (int i = slice; i < D; i += kRowBatch * nslice) {
            vec_t wv[kRowBatch];
#pragma unroll
            for (int u = 0; u < kRowBatch; ++u) {
                const int row = i + u * nslice;
                wv[u] = w[(size_t)(row < D ? row : i) * CG];
            }
#pragma unroll
            for (int u = 0; u < kRowBatch; ++u) {
                const int row = i + u * nslice;
                const double hv = row < D ? widen_one<BF>(sh_hidden[row]) : 0.0;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    if (u & 1)
                        a1[v] = fma(hv, widen_one<BF>(lane16(wv[u], v)), a1[v]);
                    else
                        a0[v] = fma(hv, widen_one<BF>(lane16(wv[u], v)), a0[v]);
                }
            }
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
        sh_rank[tid] = 0;
        if (logits_out) logits_out[(size_t)b * H + tid] = (float)sum;
    }
    __syncthreads();
    rank_and_emit(sh_logit, sh_rank, H, k, kRouterThreads, tid, head_idx + (size_t)b * k);
}

// Dynamic LDS beyond the default allowance has to be requested per kernel.  The request is made
// only when a launch needs more than any earlier launch of the same kernel did, so steady-state
// calls (and calls recorded into a HIP graph after one warm-up call) issue launches only.
template <class Kern> hipError_t ensure_dynamic_lds(Kern kern, size_t lds, std::atomic<size_t> &granted)
{
    if (lds <= 48 * 1024 || lds <= granted.load(std::memory_order_acquire)) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess) granted.store(lds, std::memory_order_release);
    return e;
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
    static std::atomic<size_t> granted{0};
    if (hipError_t e = ensure_dynamic_lds(kern, lds, granted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)B), dim3(kRouterThreads), lds, stream, hidden, Wr, D, H,
                       k, nslice, J, Dpad, head_idx, logits_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Split-D path (used when the caller supplies a workspace).  One workgroup per request keeps
// at most B compute units busy and pays two conversions per multiply-add; here a workgroup
// takes a tile of kTileR requests and one of P slices of the D axis, so a converted Wr
// element feeds kTileR multiply-adds and the grid (P x ceil(B / kTileR)) covers the chip.
// Phase 1 leaves, per (request tile, D slice), the kTileR x H partial sums in the workspace;
// phase 2 adds the P partials of each request in ascending slice order and ranks.
// The order of additions again depends on (D, H, VEC, P) only, never on the column.
#ifndef POLAR_ROUTER_TILE_R
#define POLAR_ROUTER_TILE_R 2
#endif
constexpr int kTileR = POLAR_ROUTER_TILE_R;
constexpr int kSplitThreads = 256;
constexpr int kSplitStageBatch = 2;   // hidden elements per request a thread stages per batch
#ifndef POLAR_ROUTER_DP_MAX
#define POLAR_ROUTER_DP_MAX 512
#endif
constexpr int kDpMax = POLAR_ROUTER_DP_MAX;
constexpr int kFinishBatch = 32;

// dynamic LDS: double h[kTileR][Dp] | double part[nslice][kTileR*H] | double part2[J][kTileR*H]
template <bool BF, int VEC>
__global__ __launch_bounds__(kSplitThreads) void router_partial_kernel(
    const uint16_t *__restrict__ hidden, const uint16_t *__restrict__ Wr, int B, int D, int H,
    int Dp, int nslice, int J, double *__restrict__ ws)
{
    typedef typename VecOf<VEC>::type vec_t;
    extern __shared__ __align__(16) unsigned char smem[];
    double *sh_h = reinterpret_cast<double *>(smem);
    double *sh_part = sh_h + (size_t)kTileR * Dp;
    const int RH = kTileR * H;
    double *sh_part2 = sh_part + (size_t)nslice * RH;

    const int p = blockIdx.x, rt = blockIdx.y, P = gridDim.x, tid = threadIdx.x;
    const int i0 = p * Dp;
    const int rows = min(Dp, D - i0);

    // The first batch of Wr rows is requested before the hidden rows are staged, and each
    // later batch before the previous one is consumed: the loads do not depend on the staging,
    // and a dependent round trip to memory is what this kernel's time is made of.
    const int CG = H / VEC;
    const bool active = tid < nslice * CG;
    const int slice = tid / CG, cg = tid - slice * CG;
    const vec_t *w = reinterpret_cast<const vec_t *>(Wr) + (size_t)i0 * CG + cg;
    vec_t wv[kRowBatch];
    if (active && slice < rows) {
#pragma unroll
        for (int u = 0; u < kRowBatch; ++u) {
            const int row = slice + u * nslice;
            wv[u] = w[(size_t)(row < rows ? row : slice) * CG];
        }
    }

    // stage (and widen once) the tile's hidden rows; all loads of a batch before any use
    for (int base = 0; base < rows; base += kSplitStageBatch * kSplitThreads) {
        uint16_t v[kTileR][kSplitStageBatch];
#pragma unroll
        for (int r = 0; r < kTileR; ++r) {
            const int b = rt * kTileR + r;
            const uint16_t *hrow = hidden + (size_t)(b < B ? b : 0) * D + i0;
#pragma unroll
            for (int u = 0; u < kSplitStageBatch; ++u) {
                const int i = base + u * kSplitThreads + tid;
                v[r][u] = (i < rows && b < B) ? hrow[i] : (uint16_t)0;
            }
        }
#pragma unroll
        for (int r = 0; r < kTileR; ++r)
#pragma unroll
            for (int u = 0; u < kSplitStageBatch; ++u) {
                const int i = base + u * kSplitThreads + tid;
                if (i < rows) sh_h[r * Dp + i] = widen_one<BF>(v[r][u]);
            }
    }
    __syncthreads();

    if (active) {
        double acc[kTileR][VEC];
#pragma unroll
        for (int r = 0; r < kTileR; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[r][v] = 0.0;
        for (int i = slice; i < rows; i += kRowBatch * nslice) {
            const int inext = i + kRowBatch * nslice;
            vec_t wn[kRowBatch];
            if (inext < rows) {
#pragma unroll
                for (int u = 0; u < kRowBatch; ++u) {
                    const int row = inext + u * nslice;
                    wn[u] = w[(size_t)(row < rows ? row : inext) * CG];
                }
            }
#pragma unroll
            for (int u = 0; u < kRowBatch; ++u) {
                const int row = i + u * nslice;
                if (row < rows) {
                    double wd[VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) wd[v] = widen_one<BF>(lane16(wv[u], v));
#pragma unroll
                    for (int r = 0; r < kTileR; ++r) {
                        const double hr = sh_h[r * Dp + row];
#pragma unroll
                        for (int v = 0; v < VEC; ++v) acc[r][v] = fma(hr, wd[v], acc[r][v]);
                    }
                }
            }
            if (inext < rows) {
#pragma unroll
                for (int u = 0; u < kRowBatch; ++u) wv[u] = wn[u];
            }
        }
#pragma unroll
        for (int r = 0; r < kTileR; ++r)
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                sh_part[(size_t)slice * RH + r * H + cg * VEC + v] = acc[r][v];
    }
    __syncthreads();

    for (int e = tid; e < J * RH; e += kSplitThreads) {      // level 1: slices j, j+J, ...
        const int j = e / RH, x = e - j * RH;
        double sum = 0.0;
        for (int s2 = j; s2 < nslice; s2 += J) sum += sh_part[(size_t)s2 * RH + x];
        sh_part2[e] = sum;
    }
    __syncthreads();
    double *dst = ws + ((size_t)rt * P + p) * RH;
    for (int x = tid; x < RH; x += kSplitThreads) {          // level 2: the J group sums
        double sum = 0.0;
        for (int j = 0; j < J; ++j) sum += sh_part2[j * RH + x];
        dst[x] = sum;
    }
}

// Phase 2: one workgroup per request; thread h adds the P slice partials in ascending order,
// then the same rank counting as the single-kernel path.
__global__ __launch_bounds__(POLAR_MAX_ROUTER_H) void router_finish_kernel(
    const double *__restrict__ ws, int H, int k, int P, int32_t *__restrict__ head_idx,
    float *__restrict__ logits_out)
{
    __shared__ double sh_logit[POLAR_MAX_ROUTER_H];
    __shared__ int sh_rank[POLAR_MAX_ROUTER_H];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int rt = b / kTileR, r = b - rt * kTileR;
    if (tid < H) {
        const double *src = ws + ((size_t)rt * P * kTileR + r) * H + tid;
        double sum = 0.0;
        for (int p0 = 0; p0 < P; p0 += kFinishBatch) {      // a batch of loads, then ordered adds
            double v[kFinishBatch];
#pragma unroll
            for (int u = 0; u < kFinishBatch; ++u)
                v[u] = p0 + u < P ? src[(size_t)(p0 + u) * kTileR * H] : 0.0;
#pragma unroll
            for (int u = 0; u < kFinishBatch; ++u)
                if (p0 + u < P) sum += v[u];
        }
        sh_logit[tid] = sum;
        sh_rank[tid] = 0;
        if (logits_out) logits_out[(size_t)b * H + tid] = (float)sum;
    }
    __syncthreads();
    rank_and_emit(sh_logit, sh_rank, H, k, POLAR_MAX_ROUTER_H, tid, head_idx + (size_t)b * k);
}

template <bool BF, int VEC>
hipError_t launch_split_vec(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k,
                            const RouterPlan &plan, int32_t *head_idx, float *logits_out, double *ws,
                            hipStream_t stream)
{
    const int CG = H / VEC;
    int nslice = kSplitThreads / CG;
    if (nslice < 1) nslice = 1;
    int J = 1;
    while (J * J < nslice) ++J;
    const int RH = kTileR * H;
    const size_t lds = ((size_t)kTileR * plan.Dp + (size_t)nslice * RH + (size_t)J * RH) * sizeof(double);
    auto kern = router_partial_kernel<BF, VEC>;
    static std::atomic<size_t> granted{0};
    if (hipError_t e = ensure_dynamic_lds(kern, lds, granted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)plan.P, (unsigned)plan.RT), dim3(kSplitThreads), lds, stream,
                       hidden, Wr, B, D, H, plan.Dp, nslice, J, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(router_finish_kernel, dim3((unsigned)B), dim3(POLAR_MAX_ROUTER_H), 0, stream, ws, H,
                       k, plan.P, head_idx, logits_out);
    return hipGetLastError();
}

template <bool BF>
hipError_t launch_split_dt(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k,
                           const RouterPlan &plan, int32_t *head_idx, float *logits_out, double *ws,
                           hipStream_t stream)
{
    const uintptr_t addr = reinterpret_cast<uintptr_t>(Wr);
    if (H % 8 == 0 && addr % 16 == 0)
        return launch_split_vec<BF, 8>(hidden, Wr, B, D, H, k, plan, head_idx, logits_out, ws, stream);
    if (H % 4 == 0 && addr % 8 == 0)
        return launch_split_vec<BF, 4>(hidden, Wr, B, D, H, k, plan, head_idx, logits_out, ws, stream);
    if (H % 2 == 0 && addr % 4 == 0)
        return launch_split_vec<BF, 2>(hidden, Wr, B, D, H, k, plan, head_idx, logits_out, ws, stream);
    return launch_split_vec<BF, 1>(hidden, Wr, B, D, H, k, plan, head_idx, logits_out, ws, stream);
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

hipError_t launch_router_split(const void *hidden, const void *Wr, int B, int D, int H, int k,
                               polar_dtype dt, const RouterPlan &plan, int32_t *head_idx,
                               float *logits_out, void *workspace, hipStream_t stream)
{
    const uint16_t *h16 = static_cast<const uint16_t *>(hidden);
    const uint16_t *w16 = static_cast<const uint16_t *>(Wr);
    double *ws = static_cast<double *>(workspace);
    if (dt == POLAR_BF16)
        return launch_split_dt<true>(h16, w16, B, D, H, k, plan, head_idx, logits_out, ws, stream);
    return launch_split_dt<false>(h16, w16, B, D, H, k, plan, head_idx, logits_out, ws, stream);
}

int make_router_plan(int B, int D, int H, RouterPlan *plan)
{
    if (B < 0 || D < 1 || H < 1) return POLAR_EINVAL;
    if (H > POLAR_MAX_ROUTER_H || D > POLAR_MAX_ROUTER_D || B > 0x7fffffff / 2)
        return POLAR_EUNSUPPORTED;
    plan->RT = (B + kTileR - 1) / kTileR;
    if (plan->RT > 65535) return POLAR_EUNSUPPORTED;             // grid.y limit
    const int rt = plan->RT > 0 ? plan->RT : 1;
    int P = (512 + rt - 1) / rt;                                 // aim at ~512 workgroups
    const int p_max = (D + 127) / 128, p_min = (D + kDpMax - 1) / kDpMax;  // 128..kDpMax rows of Wr per workgroup
    if (P > p_max) P = p_max;
    if (P < p_min) P = p_min;
    plan->Dp = (D + P - 1) / P;
    plan->P = (D + plan->Dp - 1) / plan->Dp;
    plan->bytes = ((size_t)plan->RT * plan->P * kTileR * H * sizeof(double) + 255) / 256 * 256;
    if (plan->bytes == 0) plan->bytes = 256;
    return POLAR_OK;
}

}  // namespace polar
