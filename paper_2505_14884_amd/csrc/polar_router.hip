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
//
// Further down: the split-D pair of kernels (partial sums per slice of D into a workspace, then
// a finish kernel that adds the slices and ranks), whose first phase runs on the vector ALU
// for batches under 16 requests and on the fp64 matrix cores (v_mfma_f64_16x16x4_f64, tiles of
// 16 requests) otherwise.  All paths share the arithmetic contract above.
#include <stdlib.h>

#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kRouterThreads = 1024;
constexpr int kRowBatch = 8;     // rows of Wr a thread of the split-D kernels loads before consuming any

// Timing-only build switches for the one-launch kernel (results are wrong with any of them set; every
// access stays in bounds): bit 0 drops the global loads, bit 1 the multiply-adds, bit 2 the two
// LDS reduction levels and the ranking.  They exist to measure what each part of the kernel's few
// microseconds costs on the machine; the product is built without them.
#ifndef POLAR_ROUTER_ABLATE
#define POLAR_ROUTER_ABLATE 0
#endif
constexpr int kAblate = POLAR_ROUTER_ABLATE;

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

__device__ __forceinline__ double shfl_xor_f64(double x, int mask)
{
    const int lo = __shfl_xor(__double2loint(x), mask), hi = __shfl_xor(__double2hiint(x), mask);
    return __hiloint2double(hi, lo);
}

// Sum over the slices of one wave, in registers.  Lane = slice_in_wave * CG + cg (CG a power of
// two), every lane holds VEC column sums.  The slice bits of the lane id are taken in ascending
// order: while a lane still holds more than one column, the two lanes of a pair split the columns
// between them (each sends the half it gives up and adds the half it receives to the half it keeps:
// the lane whose bit is set keeps the upper half), after that they exchange and add the one value
// left.  Every column is thus added up over the same binary tree of slices (pairs, pairs of pairs,
// ...), and a + b == b + a bit for bit, so identical columns still give identical sums.  On return
// x[0 .. n) holds the wave's sums of columns first .. first + n - 1 of the lane's column group.
template <int VEC>
__device__ __forceinline__ void wave_slice_sums(double (&x)[VEC], int lane, int cg_bits, int &first, int &n)
{
    first = 0;
    const int steps = 6 - cg_bits;               // slice bits of the lane id (wave-uniform)
#pragma unroll
    for (int j = 0; j < 6; ++j) {                // step j works on lane bit cg_bits + j
        const int held = (VEC >> j) > 1 ? (VEC >> j) : 1;   // columns a lane holds before step j (a constant once unrolled)
        if (j < steps) {
            const int s = cg_bits + j;
            const bool upper = (lane >> s) & 1;
            if (held > 1) {
                const int half = held / 2;
#pragma unroll
                for (int i = 0; i < VEC / 2; ++i) {
                    if (i < half) {
                        const double give = upper ? x[i] : x[i + half];
                        const double keep = upper ? x[i + half] : x[i];
                        x[i] = keep + shfl_xor_f64(give, 1 << s);
                    }
                }
                first += upper ? half : 0;
            } else {
                x[0] += shfl_xor_f64(x[0], 1 << s);
            }
        }
    }
    n = (VEC >> steps) > 1 ? (VEC >> steps) : 1;
}

// RB = rows of Wr a thread loads before it consumes any (even, so that a row's chain, a0 or a1, and
// with it every sum, is the same for every RB): the host picks the smallest of 4, 8, 16 that covers
// a thread's rows in one batch, since a batch is a dependent round trip to memory and those round
// trips, not the arithmetic, are what the kernel's time is made of.
// WAVE_SUMS (H / VEC a power of two up to 64): the slices of a wave are added in registers
// (wave_slice_sums), only the 16 waves' sums go through LDS (part2[16][H]) and one thread per head
// adds them in ascending order.  Otherwise the threads' sums go to LDS and are added in two levels.
// The two long serial LDS loops of that form cost about 2 us of the kernel's 7 to 9.
template <bool BF, int VEC, int RB, bool WAVE_SUMS>
__global__ __launch_bounds__(kRouterThreads) void router_topk_kernel(
    const uint16_t *__restrict__ hidden, const uint16_t *__restrict__ Wr, int D, int H, int k,
    int nslice, int J, int cg_bits, int32_t *__restrict__ head_idx, float *__restrict__ logits_out)
{
    typedef typename VecOf<VEC>::type vec_t;
    extern __shared__ __align__(16) unsigned char smem[];
    // dynamic LDS: [part: nslice x H] [part2: J x H] [logit: H]; with WAVE_SUMS only [part2: 16 x H] [logit: H]
    double *sh_part = reinterpret_cast<double *>(smem);
    double *sh_part2 = WAVE_SUMS ? sh_part : sh_part + (size_t)nslice * H;
    double *sh_logit = sh_part2 + (size_t)(WAVE_SUMS ? kRouterThreads / 64 : J) * H;
    __shared__ int sh_rank[POLAR_MAX_ROUTER_H];

    const int b = blockIdx.x, tid = threadIdx.x;
    const uint16_t *hrow = hidden + (size_t)b * D;
    // The request's hidden row is not staged: a thread needs only the elements of its own rows,
    // and their loads go out together with the rows' (one round trip to memory, not two with a
    // barrier in between).  A dependent round trip costs about a microsecond, so the kernel's
    // time is the number of such rounds, not its arithmetic.
    const int CG = H / VEC;                    // column groups per row of Wr
    const int slice = tid / CG, cg = tid - slice * CG;
    double a0[VEC], a1[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) a0[v] = a1[v] = 0.0;
    if (tid < nslice * CG) {
        const vec_t *w = reinterpret_cast<const vec_t *>(Wr) + cg;
        // rows slice, slice + nslice, ...: RB loads in flight, then their multiply-adds,
        // even rows of the batch into chain a0 and odd rows into a1
        for (int i = slice; i < D; i += RB * nslice) {
            vec_t wv[RB];
            uint16_t hq[RB];
#pragma unroll
            for (int u = 0; u < RB; ++u) {
                const int row = i + u * nslice;
                if (kAblate & 1) {
                    wv[u] = vec_t{};
                    hq[u] = (uint16_t)(row + tid);
                } else {
                    wv[u] = w[(size_t)(row < D ? row : i) * CG];
                    hq[u] = hrow[row < D ? row : i];
                }
            }
            if (kAblate & 2) {
#pragma unroll
                for (int u = 0; u < RB; ++u) a0[0] += (double)(lane16(wv[u], 0) + hq[u]);
                continue;
            }
#pragma unroll
            for (int u = 0; u < RB; ++u) {
                const int row = i + u * nslice;
                const double hv = row < D ? widen_one<BF>(hq[u]) : 0.0;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    if (u & 1)
                        a1[v] = fma(hv, widen_one<BF>(lane16(wv[u], v)), a1[v]);
                    else
                        a0[v] = fma(hv, widen_one<BF>(lane16(wv[u], v)), a0[v]);
                }
            }
        }
    }
    if (kAblate & 4) {
        if (tid < k) head_idx[(size_t)b * k + tid] = (int)(a0[0] + a1[0]) & 1;
        return;
    }
    if (WAVE_SUMS) {
        double x[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) x[v] = a0[v] + a1[v];    // threads without rows hold zeros
        int first, n;
        wave_slice_sums<VEC>(x, tid & 63, cg_bits, first, n);
        // after the splitting steps the columns of a group are spread over its lanes; every lane
        // stores what it holds (lanes that went through exchange-and-add steps hold equal values
        // and store the same bits)
        const int wave = tid >> 6;
        const int cgw = (tid & 63) & (CG - 1);
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            if (i < n) sh_part2[wave * H + cgw * VEC + first + i] = x[i];
        __syncthreads();
        if (tid < H) {
            double part[kRouterThreads / 64];
#pragma unroll
            for (int w = 0; w < kRouterThreads / 64; ++w) part[w] = sh_part2[w * H + tid];   // all loads, then
            double sum = 0.0;
#pragma unroll
            for (int w = 0; w < kRouterThreads / 64; ++w) sum += part[w];                    // the adds in order
            sh_logit[tid] = sum;
            sh_rank[tid] = 0;
            if (logits_out) logits_out[(size_t)b * H + tid] = (float)sum;
        }
        __syncthreads();
    } else {
        if (tid < nslice * CG) {
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
    }
    rank_and_emit(sh_logit, sh_rank, H, k, kRouterThreads, tid, head_idx + (size_t)b * k);
}

template <bool BF, int VEC, int RB, bool WAVE_SUMS>
hipError_t launch_vec_ws(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k, int nslice, int J,
                         int cg_bits, size_t lds, int32_t *head_idx, float *logits_out, hipStream_t stream)
{
    auto kern = router_topk_kernel<BF, VEC, RB, WAVE_SUMS>;
    static LdsGrant granted;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, granted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)B), dim3(kRouterThreads), lds, stream, hidden, Wr, D, H,
                       k, nslice, J, cg_bits, head_idx, logits_out);
    return hipGetLastError();
}

template <bool BF, int VEC, int RB>
hipError_t launch_vec_rb(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k, int nslice, int J,
                         size_t lds, int32_t *head_idx, float *logits_out, hipStream_t stream)
{
    const int CG = H / VEC;
    int cg_bits = 0;
    while ((1 << cg_bits) < CG) ++cg_bits;
#ifndef POLAR_ROUTER_LDS_SUMS                    // (timing comparisons: build with it to keep the two-level LDS form)
    if ((1 << cg_bits) == CG && CG <= 64)        // the slices of a wave can be added in registers
        return launch_vec_ws<BF, VEC, RB, true>(hidden, Wr, B, D, H, k, nslice, J, cg_bits,
                                                (size_t)(kRouterThreads / 64 + 1) * H * sizeof(double), head_idx,
                                                logits_out, stream);
#endif
    return launch_vec_ws<BF, VEC, RB, false>(hidden, Wr, B, D, H, k, nslice, J, 0, lds, head_idx, logits_out, stream);
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
    const size_t lds = ((size_t)nslice * H + (size_t)J * H + H) * sizeof(double);
    const int rows_per_thread = (D + nslice - 1) / nslice;
    if (rows_per_thread <= 4)
        return launch_vec_rb<BF, VEC, 4>(hidden, Wr, B, D, H, k, nslice, J, lds, head_idx, logits_out, stream);
    if (rows_per_thread <= 8 || VEC < 8)              // 16 rows of 16-byte vectors is what the registers hold
        return launch_vec_rb<BF, VEC, 8>(hidden, Wr, B, D, H, k, nslice, J, lds, head_idx, logits_out, stream);
    return launch_vec_rb<BF, VEC, 16>(hidden, Wr, B, D, H, k, nslice, J, lds, head_idx, logits_out, stream);
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
    const double *__restrict__ ws, int H, int k, int P, int tile, int32_t *__restrict__ head_idx,
    float *__restrict__ logits_out)
{
    __shared__ double sh_logit[POLAR_MAX_ROUTER_H];
    __shared__ int sh_rank[POLAR_MAX_ROUTER_H];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int rt = b / tile, r = b - rt * tile;       // workspace: [request tile][slice][row of tile][H]
    if (tid < H) {
        const double *src = ws + ((size_t)rt * P * tile + r) * H + tid;
        double sum = 0.0;
        for (int p0 = 0; p0 < P; p0 += kFinishBatch) {      // a batch of loads, then ordered adds
            double v[kFinishBatch];
#pragma unroll
            for (int u = 0; u < kFinishBatch; ++u)
                v[u] = p0 + u < P ? src[(size_t)(p0 + u) * tile * H] : 0.0;
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
    static LdsGrant granted;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, granted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)plan.P, (unsigned)plan.RT), dim3(kSplitThreads), lds, stream,
                       hidden, Wr, B, D, H, plan.Dp, nslice, J, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(router_finish_kernel, dim3((unsigned)B), dim3(POLAR_MAX_ROUTER_H), 0, stream, ws, H,
                       k, plan.P, kTileR, head_idx, logits_out);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Matrix-core form of phase 1 (batches of at least kMmTileR requests).  The same partial sums,
// logit[b, h] over one slice of D, are a [16 requests x Dp] by [Dp x H] product in double, which
// is what v_mfma_f64_16x16x4_f64 computes: a converted Wr element then feeds 16 multiply-adds
// instead of 2, and the vector ALU is left with two conversions per operand element.  The
// slice of Wr (one contiguous block of Dp*H values, H innermost) and the tile's hidden rows are
// staged in LDS as raw 16-bit patterns; a lane reads and widens the one A element and the one
// B element it supplies to each instruction: lane 16*kk + lo gives A[request lo][row 4t + kk]
// and B[row 4t + kk][column 16*tile + lo], and receives D[request kk + 4r][column lo] in
// register r.  The four waves take the 4-row steps t = wave, wave + 4, ... and their sums are
// added in the fixed order ((w3 + w2) + w1) + w0, so the result depends on (D, H, Dp) only and
// every column goes through the same sequence of operations (identical columns of Wr give
// bit-identical logits, as in the other paths).
constexpr int kMmTileR = 16;
constexpr int kMmWaves = 4;
constexpr int kMmThreads = kMmWaves * 64;
constexpr int kMmGroupMax = 5;      // 16-column tiles accumulated together (up to 80 columns)
constexpr int kMmHiddenBatch = 16;  // hidden elements a thread stages per batch
constexpr int kMmSlabBatch = 12;    // 16-byte pieces of the Wr slice a thread stages per batch
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));

__host__ __device__ inline int mm_hidden_pitch(int Dp) { return Dp + 2; }   // odd number of dwords per row
// tiles per group for H columns: all of them when they fit one group, else the maximum
__host__ __device__ inline int mm_group(int H)
{
    const int nt = (H + 15) / 16;
    return nt < kMmGroupMax ? nt : kMmGroupMax;
}
// columns of the LDS copy of the Wr slice: whole groups of tiles, zero beyond H, so the inner
// loop needs no bounds test
__host__ __device__ inline int mm_slab_pitch(int H)
{
    const int grp = mm_group(H);
    const int groups = ((H + 15) / 16 + grp - 1) / grp;
    return groups * grp * 16;
}

template <bool BF, int kMmGroup>
__global__ __launch_bounds__(kMmThreads) void router_partial_mfma_kernel(
    const uint16_t *__restrict__ hidden, const uint16_t *__restrict__ Wr, int B, int D, int H,
    int Dp, double *__restrict__ ws)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int p = blockIdx.x, rt = blockIdx.y, P = gridDim.x, tid = threadIdx.x;
    // the wave number as a scalar: the loop over this wave's steps is then uniform and its
    // accumulators stay in the matrix cores' registers instead of being moved every iteration
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i0 = p * Dp;
    const int rows = min(Dp, D - i0);
    const int Dp4 = (Dp + 3) & ~3;

    // LDS: slab[Dp4][Hp] (16-bit) | hd[16][pitch] (16-bit) | red[kMmGroup][4][64] (double)
    const int Hp = mm_slab_pitch(H);
    uint16_t *slab = reinterpret_cast<uint16_t *>(smem);
    const size_t slab_bytes = (size_t)Dp4 * Hp * 2;                 // Hp is a multiple of 16
    const int pitch = mm_hidden_pitch(Dp);
    uint16_t *hd = reinterpret_cast<uint16_t *>(smem + slab_bytes);
    const size_t hd_bytes = ((size_t)kMmTileR * pitch * 2 + 15) / 16 * 16;
    double *red = reinterpret_cast<double *>(smem + slab_bytes + hd_bytes);

    // Stage the tile's hidden rows (zeros for requests beyond B and rows beyond the slice) and the
    // slice of Wr, row by row into the padded pitch (zeros beyond the slice and beyond H).  All
    // loads of a batch are issued before any store, and the hidden rows travel with the first
    // batch of the slice: a dependent round trip per piece would cost more than everything else.
    const int hd_elems = kMmTileR * Dp4;
    const uint16_t *src = Wr + (size_t)i0 * H;
    const bool vec = H % 8 == 0 && (reinterpret_cast<uintptr_t>(Wr) & 15u) == 0;
    const int h8 = H / 8, hp8 = Hp / 8, nv = vec ? Dp4 * hp8 : 0;   // 16-byte pieces of the padded slab
    const u32x4v *sv = reinterpret_cast<const u32x4v *>(src);
    u32x4v *dv = reinterpret_cast<u32x4v *>(slab);
    for (int base = 0, sbase = 0; base < hd_elems || sbase < nv;
         base += kMmHiddenBatch * kMmThreads, sbase += kMmSlabBatch * kMmThreads) {
        uint16_t hv[kMmHiddenBatch];
        u32x4v wv[kMmSlabBatch];
#pragma unroll
        for (int u = 0; u < kMmHiddenBatch; ++u) {
            const int e = base + u * kMmThreads + tid;
            const int r = e / Dp4, i = e - r * Dp4, b = rt * kMmTileR + r;
            const bool live = e < hd_elems && b < B && i < rows;
            const uint16_t x = hidden[live ? (size_t)b * D + i0 + i : 0];
            hv[u] = live ? x : (uint16_t)0;
        }
#pragma unroll
        for (int u = 0; u < kMmSlabBatch; ++u) {
            const int i = sbase + u * kMmThreads + tid;
            const int row = i / hp8, c8 = i - row * hp8;
            const bool live = i < nv && row < rows && c8 < h8;
            const u32x4v x = sv[live ? row * h8 + c8 : 0];
            wv[u] = live ? x : u32x4v{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kMmHiddenBatch; ++u) {
            const int e = base + u * kMmThreads + tid;
            if (e < hd_elems) {
                const int r = e / Dp4, i = e - r * Dp4;
                hd[r * pitch + i] = hv[u];
            }
        }
#pragma unroll
        for (int u = 0; u < kMmSlabBatch; ++u) {
            const int i = sbase + u * kMmThreads + tid;
            if (i < nv) dv[i] = wv[u];
        }
    }
    if (!vec) {
        const int ne = Dp4 * Hp;
        for (int e = tid; e < ne; e += kMmThreads) {
            const int row = e / Hp, col = e - row * Hp;
            slab[e] = (row < rows && col < H) ? src[(size_t)row * H + col] : (uint16_t)0;
        }
    }
    __syncthreads();

    const int lo = lane & 15, kk = lane >> 4;
    const int NT = (H + 15) / 16;
    const int steps = Dp4 / 4;                                       // 4-row steps of the slice
    double *dst = ws + ((size_t)rt * P + p) * kMmTileR * H;          // [16][H]
    for (int g0 = 0; g0 < NT; g0 += kMmGroup) {
        f64x4 acc[kMmGroup];
#pragma unroll
        for (int u = 0; u < kMmGroup; ++u) acc[u] = f64x4{0.0, 0.0, 0.0, 0.0};
        const uint16_t *a_ptr = hd + lo * pitch + kk;                // + 4t
        const uint16_t *b_ptr = slab + (size_t)kk * Hp + 16 * g0 + lo;   // + 4t*Hp + 16u
        // operands of the next step are read from LDS while this step's products run
        uint16_t an = 0, wn[kMmGroup];
        if (wave < steps) {
            an = a_ptr[4 * wave];
#pragma unroll
            for (int u = 0; u < kMmGroup; ++u) wn[u] = b_ptr[(size_t)4 * wave * Hp + 16 * u];
        }
        for (int t = wave; t < steps; t += kMmWaves) {
            const uint16_t ab = an;
            uint16_t wb[kMmGroup];
#pragma unroll
            for (int u = 0; u < kMmGroup; ++u) wb[u] = wn[u];
            const int tn = min(t + kMmWaves, steps - 1);             // clamped: always a valid step
            an = a_ptr[4 * tn];
#pragma unroll
            for (int u = 0; u < kMmGroup; ++u) wn[u] = b_ptr[(size_t)4 * tn * Hp + 16 * u];
            const double a = widen_one<BF>(ab);
#pragma unroll
            for (int u = 0; u < kMmGroup; ++u)
                acc[u] = __builtin_amdgcn_mfma_f64_16x16x4f64(a, widen_one<BF>(wb[u]), acc[u], 0, 0, 0);
        }
        // add the waves' sums in a fixed order: ((w3 + w2) + w1) + w0
        for (int w = kMmWaves - 1; w >= 0; --w) {
            if (w != kMmWaves - 1) __syncthreads();
            if (wave == w) {
#pragma unroll
                for (int u = 0; u < kMmGroup; ++u)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        double *slot = red + ((size_t)u * 4 + r) * 64 + lane;
                        if (w == kMmWaves - 1) {
                            *slot = acc[u][r];
                        } else if (w > 0) {
                            *slot = *slot + acc[u][r];
                        } else {
                            const int col = 16 * (g0 + u) + lo;
                            if (col < H) dst[(size_t)(kk + 4 * r) * H + col] = *slot + acc[u][r];
                        }
                    }
            }
        }
        __syncthreads();      // red is reused by the next group of columns
    }
}

size_t mm_lds_bytes(int Dp, int H)
{
    const size_t slab = (size_t)((Dp + 3) / 4 * 4) * mm_slab_pitch(H) * 2;
    const size_t hd = ((size_t)kMmTileR * mm_hidden_pitch(Dp) * 2 + 15) / 16 * 16;
    return slab + hd + (size_t)kMmGroupMax * 4 * 64 * sizeof(double);
}

template <bool BF, int GRP>
hipError_t launch_split_mfma_grp(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k,
                                 const RouterPlan &plan, int32_t *head_idx, float *logits_out,
                                 double *ws, hipStream_t stream)
{
    const size_t lds = mm_lds_bytes(plan.Dp, H);
    auto kern = router_partial_mfma_kernel<BF, GRP>;
    static LdsGrant granted;
    if (hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(kern), lds, granted); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)plan.P, (unsigned)plan.RT), dim3(kMmThreads), lds, stream,
                       hidden, Wr, B, D, H, plan.Dp, ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(router_finish_kernel, dim3((unsigned)B), dim3(POLAR_MAX_ROUTER_H), 0, stream, ws, H,
                       k, plan.P, kMmTileR, head_idx, logits_out);
    return hipGetLastError();
}

template <bool BF>
hipError_t launch_split_mfma(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k,
                             const RouterPlan &plan, int32_t *head_idx, float *logits_out, double *ws,
                             hipStream_t stream)
{
#define POLAR_MM_ARGS hidden, Wr, B, D, H, k, plan, head_idx, logits_out, ws, stream
    switch (mm_group(H)) {
    case 1: return launch_split_mfma_grp<BF, 1>(POLAR_MM_ARGS);
    case 2: return launch_split_mfma_grp<BF, 2>(POLAR_MM_ARGS);
    case 3: return launch_split_mfma_grp<BF, 3>(POLAR_MM_ARGS);
    case 4: return launch_split_mfma_grp<BF, 4>(POLAR_MM_ARGS);
    default: return launch_split_mfma_grp<BF, 5>(POLAR_MM_ARGS);
    }
#undef POLAR_MM_ARGS
}

template <bool BF>
hipError_t launch_split_dt(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H, int k,
                           const RouterPlan &plan, int32_t *head_idx, float *logits_out, double *ws,
                           hipStream_t stream)
{
    if (plan.mfma)
        return launch_split_mfma<BF>(hidden, Wr, B, D, H, k, plan, head_idx, logits_out, ws, stream);
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
    plan->mfma = B >= kMmTileR;
    if (const int forced = option(POLAR_OPT_ROUTER_PHASE1)) plan->mfma = forced == 2;   // tests, sweeps
    if (plan->mfma) {
        // 16 requests per workgroup.  The slice length Dp (rows of Wr per workgroup, a multiple of
        // 32 whose padded 16-bit copy fits 80 KiB of LDS) is the one that minimises
        //   rounds of the 256 compute units x rows per workgroup   (the matrix-core time: an fp64
        //                                                           tile product takes ~110 cycles)
        //   + 40 rows' worth per 32 slices                          (the finish kernel adds the
        //                                                           slices of a request 32 at a time).
        // OPT-66B-shaped router (B=128, D=9216): Dp = 288, 32 slices x 8 tiles = 256 workgroups.
        plan->RT = (B + kMmTileR - 1) / kMmTileR;
        if (plan->RT > 65535) return POLAR_EUNSUPPORTED;         // grid.y limit
        const long rt = plan->RT > 0 ? plan->RT : 1;
        int dp_max = 320;
        while (dp_max > 32 && (size_t)dp_max * mm_slab_pitch(H) * 2 > 81920) dp_max -= 32;
        int dp = 32;
        long best = -1;
        for (int cand = 32; cand <= dp_max; cand += 32) {
            const long slices = (D + cand - 1) / cand;
            const long rounds = (rt * slices + 255) / 256;
            const long cost = rounds * cand + 40 * ((slices + 31) / 32);
            if (best < 0 || cost < best) {
                best = cost;
                dp = cand;
            }
        }
        plan->Dp = dp;
        plan->P = (D + dp - 1) / dp;
        plan->bytes = ((size_t)plan->RT * plan->P * kMmTileR * H * sizeof(double) + 255) / 256 * 256;
        if (plan->bytes == 0) plan->bytes = 256;
        return POLAR_OK;
    }
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
