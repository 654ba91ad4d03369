// Selective Head Attention, decode step, for gfx950 (CDNA4): split-KV streaming kernel for
// one query head per KV head (also grouped heads at d = 64; grouped heads at d = 128 take the
// matrix-core kernel in polar_sha_gqa.hip) and the merge / zero-fill kernel both share.
//
// What is computed (Section 3.2, per-head attention equation; Algorithm 1, Selective Head
// FlashAttention (decode)): for every request b and selected KV head g, one query row per
// query head of the group attends rows [0, n_b) of K[b,g] and V[b,g].  The head is
// gathered into the grid from the batch head index, so unselected K/V is never addressed.
//
// How it is laid out on the machine (differs from the paper's one-program-per-(b, slot)
// Triton kernel, which was shaped for its GPUs' shared memory):
//   * Decode attention is a memory-bound GEMV, so there is no MFMA and no LDS staging on
//     the streaming path: K and V rows go global -> VGPR with 16-byte loads.  A row of d
//     16-bit values is shared by d/8 adjacent lanes, so one wave-wide load covers 64*16
//     contiguous bytes (4 rows at d = 128, 8 rows at d = 64).
//   * Each lane holds its 8-element slice of q (per query head of the group) in registers;
//     the row dot product is 4 packed dot2 instructions per lane followed by a DPP
//     butterfly over the d/8 lanes of the row, which leaves the score in all of them.
//   * Every (wave, row-slot) pair runs its own online softmax (running max, sum and an
//     8-wide slice of the output per lane) over the rows it sees, in base-2 exponent space
//     (scores are pre-multiplied by scale*log2 e).  At the end of a chunk the row-slots of
//     a wave are merged with cross-lane shuffles, the waves through LDS, and one
//     (max, sum, unnormalised output) record per query head goes to the workspace.
//   * Long sequences are split across workgroups in chunks of rows (occupancy: the number
//     of (request, head) units alone does not fill 256 compute units); the merge kernel
//     applies the same max/sum rescale across chunks, normalises, and stores zeros for
//     the heads that were not selected.  A cache that is not split can skip the merge: the
//     streaming kernel then finishes the rows and zero-fills by itself (DIRECT below).
#include "polar_internal.h"

namespace polar {
namespace {

// Launch shape of the streaming kernel, per group size G (measured on MI355X; overridable at
// build time for sweeps).  WAVES = waves per workgroup, LOADS = 16-byte loads of K (and of V)
// a lane issues before consuming any.  For G = 1 the kernel needs few registers, so 8 waves x
// 8 loads (16 KiB in flight per wave) makes a lone workgroup fast, which shortens the tail of
// the grid; larger groups hold G output slices per lane and take fewer loads per step.
template <int G> struct Shape {
#if defined(POLAR_SHA_WAVES) && defined(POLAR_SHA_LOADS)
    static constexpr int kWaves = POLAR_SHA_WAVES, kLoads = POLAR_SHA_LOADS;
#else
    static constexpr int kWaves = G <= 4 ? 8 : 4;
    static constexpr int kLoads = G == 1 ? 8 : 4;
#endif
};
constexpr float kNegBig = -1.0e30f;       // "no row seen yet": finite, so exp2(x - max) never sees inf - inf

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct F16 {};
struct BF16 {};

template <class DT> __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc);
template <> __device__ __forceinline__ float dot2<F16>(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, a), __builtin_bit_cast(f16x2, b), acc,
                                  false);
}
template <> __device__ __forceinline__ float dot2<BF16>(uint32_t a, uint32_t b, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a),
                                           __builtin_bit_cast(bf16x2, b), acc, false);
}

// Two packed 16-bit values -> two floats (exact).
template <class DT> __device__ __forceinline__ void widen2(uint32_t w, float &lo, float &hi);
template <> __device__ __forceinline__ void widen2<F16>(uint32_t w, float &lo, float &hi)
{
    f16x2 h = __builtin_bit_cast(f16x2, w);
    lo = (float)h.x;
    hi = (float)h.y;
}
template <> __device__ __forceinline__ void widen2<BF16>(uint32_t w, float &lo, float &hi)
{
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xffff0000u);
}

template <int CTRL> __device__ __forceinline__ float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false);
    return x + __int_as_float(y);
}

// Sum over the LPR (8 or 16) adjacent lanes that share a row; result in every one of them.
// quad_perm [1,0,3,2], quad_perm [2,3,0,1], row_half_mirror, row_mirror.
template <int LPR> __device__ __forceinline__ float row_allreduce(float x)
{
    x = dpp_add<0xB1>(x);
    x = dpp_add<0x4E>(x);
    x = dpp_add<0x141>(x);
    if (LPR == 16) x = dpp_add<0x140>(x);
    return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16-byte load of cache rows, marked non-temporal: every K/V byte is used exactly once, and
// telling the memory system so (no retention in L2 or the memory-side cache) is worth about
// 9 % of bandwidth on this part (746 -> 682 us on the OPT-66B-shaped layer).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_row16(const uint4 *p)
{
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// One step of a row-slot's online softmax: kLoads rows of K and V already in registers.
template <class DT, int D, int G, int kLoads, bool MASKED>
__device__ __forceinline__ void consume(const uint4 (&kr)[kLoads], const uint4 (&vr)[kLoads],
                                        const bool (&ok)[kLoads], const uint4 (&qr)[G], float c,
                                        float (&m)[G], float (&l)[G], float (&o)[G][8])
{
    constexpr int LPR = D / 8;
    float p[G][kLoads];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float s[kLoads];
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            float a = dot2<DT>(kr[u].x, qr[g].x, 0.0f);
            a = dot2<DT>(kr[u].y, qr[g].y, a);
            a = dot2<DT>(kr[u].z, qr[g].z, a);
            a = dot2<DT>(kr[u].w, qr[g].w, a);
            a = row_allreduce<LPR>(a) * c;
            s[u] = (MASKED && !ok[u]) ? -INFINITY : a;
        }
        float mx = m[g];
#pragma unroll
        for (int u = 0; u < kLoads; ++u) mx = fmaxf(mx, s[u]);
        const float alpha = fast_exp2(m[g] - mx);
        float psum = 0.0f;
#pragma unroll
        for (int u = 0; u < kLoads; ++u) {
            p[g][u] = fast_exp2(s[u] - mx);
            psum += p[g][u];
        }
        l[g] = l[g] * alpha + psum;
        m[g] = mx;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] *= alpha;
    }
#pragma unroll
    for (int u = 0; u < kLoads; ++u) {
        float v[8];
        widen2<DT>(vr[u].x, v[0], v[1]);
        widen2<DT>(vr[u].y, v[2], v[3]);
        widen2<DT>(vr[u].z, v[4], v[5]);
        widen2<DT>(vr[u].w, v[6], v[7]);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int e = 0; e < 8; ++e) o[g][e] = fmaf(p[g][u], v[e], o[g][e]);
    }
}

// Streaming kernel.  1-D grid of B*nsplit*k workgroups; block = Shape<G>::kWaves waves.
// Workgroup L works on slot = L % k, split = (L / k) % nsplit, b = L / (k * nsplit).  The slot
// varies fastest on purpose: the hardware deals consecutive workgroups round-robin over the 8
// XCDs, and the k workgroups of one (request, split) all have the same amount of work, so every
// XCD gets an equal share of each request however ragged the lengths are.  (With the split
// fastest, XCD j would get exactly the splits congruent to j, and late splits are mostly empty.)
// Workspace record of unit u = ((b*k + slot)*G + gi)*nsplit + split:
//   ws_o[u*D .. u*D+D)   unnormalised output, ws_ml[2u] running max (base-2), ws_ml[2u+1] sum.
// A workgroup whose chunk starts at or beyond n_b, or whose head id is out of range, writes
// nothing; the merge kernel never reads those records.
// ROW_MAJOR_SEQ selects the cache layout: false = [B, Hkv, S, d] (a head's rows are contiguous),
// true = [B, S, Hkv, d] (a row of one head is d contiguous values, consecutive rows of that
// head are Hkv*d apart).
// DIRECT (only launched with nsplit == 1, where a workgroup sees all rows of its (request, slot)):
// the epilogue divides by the sum and stores the final rows to `out`, and one wave of the
// workgroup zero-fills this slot's share of the unselected heads, so no merge kernel runs.
template <class DT, int D, int G, bool ROW_MAJOR_SEQ, bool DIRECT>
__global__ __launch_bounds__(Shape<G>::kWaves * 64) void sha_partial_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int32_t *__restrict__ seqlens, const int32_t *__restrict__ head_idx,
    float *__restrict__ ws_o, float *__restrict__ ws_ml, float *__restrict__ out, int Hq, int Hkv,
    int S, int k, int chunk, int nsplit, float c)
{
    constexpr int kWaves = Shape<G>::kWaves, kLoads = Shape<G>::kLoads;
    constexpr int LPR = D / 8;             // lanes per row
    constexpr int RPL = 64 / LPR;          // rows per wave-wide load
    constexpr int ROWS_WAVE = kLoads * RPL;
    constexpr int ROWS_WG = kWaves * ROWS_WAVE;

    const int slot = blockIdx.x % k;
    const int rest = blockIdx.x / k;
    const int split = rest % nsplit, b = rest / nsplit;
    // both index loads are issued before either is tested: one round trip instead of two
    int n = seqlens[b];
    const int g_kv = head_idx ? head_idx[(size_t)b * k + slot] : slot;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int id0 = -1;
    if (DIRECT && head_idx && wave == kWaves - 1 && lane < k) id0 = head_idx[(size_t)b * k + lane];
    n = n < 0 ? 0 : (n > S ? S : n);
    // The zero fill is left to the last wave, after the workgroup's barrier, while the first
    // waves finish the output rows (its index loads are issued here, with the others): any
    // earlier and the whole workgroup would wait for it.
#define POLAR_DIRECT_ZERO_FILL()                                                                   \
    if (DIRECT && wave == kWaves - 1 && (head_idx || n == 0))                                      \
        direct_zero_fill(head_idx ? head_idx + (size_t)b * k : nullptr, id0, head_idx && n > 0,    \
                         slot, k, Hkv, G * D, out + (size_t)b * Hq * D, lane)
    const int row_begin = split * chunk;
    if (row_begin >= n || (unsigned)g_kv >= (unsigned)Hkv) {
        POLAR_DIRECT_ZERO_FILL();
        return;
    }
    const int row_end = min(row_begin + chunk, n);

    const int r = lane / LPR, cl = lane % LPR;

    // first row of this (request, head), and the distance between its rows in 16-byte units
    const size_t slab = ROW_MAJOR_SEQ ? ((size_t)b * S * Hkv + g_kv) * D
                                      : ((size_t)b * Hkv + g_kv) * (size_t)S * D;
    const size_t row_stride = ROW_MAJOR_SEQ ? (size_t)Hkv * LPR : (size_t)LPR;
    const uint4 *__restrict__ Kp = reinterpret_cast<const uint4 *>(K + slab) + cl;
    const uint4 *__restrict__ Vp = reinterpret_cast<const uint4 *>(V + slab) + cl;

    uint4 qr[G];
#pragma unroll
    for (int g = 0; g < G; ++g)
        qr[g] = reinterpret_cast<const uint4 *>(q + ((size_t)b * Hq + (size_t)g_kv * G + g) * D)[cl];

    float m[G], l[G], o[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegBig;
        l[g] = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[g][e] = 0.0f;
    }

    for (int row0 = row_begin + wave * ROWS_WAVE; row0 < row_end; row0 += ROWS_WG) {
        uint4 kr[kLoads], vr[kLoads];
        bool ok[kLoads];
        if (row0 + ROWS_WAVE <= row_end) {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                kr[u] = load_row16(Kp + (size_t)(row0 + u * RPL + r) * row_stride);
                ok[u] = true;
            }
#pragma unroll
            for (int u = 0; u < kLoads; ++u) vr[u] = load_row16(Vp + (size_t)(row0 + u * RPL + r) * row_stride);
            consume<DT, D, G, kLoads, false>(kr, vr, ok, qr, c, m, l, o);
        } else {
#pragma unroll
            for (int u = 0; u < kLoads; ++u) {
                const int row = row0 + u * RPL + r;
                ok[u] = row < row_end;
                kr[u] = make_uint4(0u, 0u, 0u, 0u);
                vr[u] = make_uint4(0u, 0u, 0u, 0u);
                if (ok[u]) {
                    kr[u] = load_row16(Kp + (size_t)row * row_stride);
                    vr[u] = load_row16(Vp + (size_t)row * row_stride);
                }
            }
            consume<DT, D, G, kLoads, true>(kr, vr, ok, qr, c, m, l, o);
        }
    }

    // Merge the RPL row-slots of this wave: butterfly over lane distances LPR, 2*LPR, ... 32.
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m2 = __shfl_xor(m[g], off);
            const float l2 = __shfl_xor(l[g], off);
            const float mx = fmaxf(m[g], m2);
            const float a1 = fast_exp2(m[g] - mx), a2 = fast_exp2(m2 - mx);
            l[g] = l[g] * a1 + l2 * a2;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float o2 = __shfl_xor(o[g][e], off);
                o[g][e] = o[g][e] * a1 + o2 * a2;
            }
            m[g] = mx;
        }
    }

    __shared__ float sm_o[kWaves][G][D];
    __shared__ float sm_ml[kWaves][G][2];
    if (r == 0) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float4 *dst = reinterpret_cast<float4 *>(&sm_o[wave][g][cl * 8]);
            dst[0] = make_float4(o[g][0], o[g][1], o[g][2], o[g][3]);
            dst[1] = make_float4(o[g][4], o[g][5], o[g][6], o[g][7]);
            if (cl == 0) {
                sm_ml[wave][g][0] = m[g];
                sm_ml[wave][g][1] = l[g];
            }
        }
    }
    __syncthreads();
    static_assert(D <= (kWaves - 1) * 64, "the last wave must be free of the final merge");
    POLAR_DIRECT_ZERO_FILL();
#undef POLAR_DIRECT_ZERO_FILL

    // Merge the waves: thread t owns output column t of every query head of the group.
    const int t = threadIdx.x;
    if (t < D) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mx = sm_ml[0][g][0];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, sm_ml[w][g][0]);
            float acc = 0.0f, lsum = 0.0f;
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float a = fast_exp2(sm_ml[w][g][0] - mx);
                acc = fmaf(a, sm_o[w][g][t], acc);
                lsum = fmaf(a, sm_ml[w][g][1], lsum);
            }
            if (DIRECT) {
                out[((size_t)b * Hq + (size_t)g_kv * G + g) * D + t] = lsum > 0.0f ? acc / lsum : 0.0f;
            } else {
                const size_t unit = (((size_t)b * k + slot) * G + g) * nsplit + split;
                ws_o[unit * D + t] = acc;
                if (t == 0) {
                    ws_ml[unit * 2 + 0] = mx;
                    ws_ml[unit * 2 + 1] = lsum;
                }
            }
        }
    }
}

// Merge / zero-fill kernel.  grid = (ceil(Hq / kMergeHeads), B); block = 256 threads.
// A workgroup owns kMergeHeads consecutive query heads of one request.  It first finds, with
// one parallel pass over the request's row of the batch head index, the slot that selected
// each of the (at most kMergeHeads) KV groups those heads belong to (lowest slot wins, so
// duplicate ids are harmless); then D threads per head combine that head's chunk records
// with the max/sum rescale of Algorithm 1 and normalise.  Heads whose group has no slot, and
// requests of length 0, are stored as +0.0.
constexpr int kMergeHeads = 8;
constexpr int kMergeThreads = 256;
constexpr int kNoSlot = 0x7fffffff;

// Element t of one query head's output from its chunk records unit0 .. unit0 + used - 1: one pass
// with a running max (the recurrence of Algorithm 1 over chunks), then the division by the sum.
// The loads of different chunks are independent of the arithmetic, so unrolling puts several
// records in flight at once.
template <int D>
__device__ __forceinline__ float fold_chunks(const float *__restrict__ ws_o, const float *__restrict__ ws_ml,
                                             size_t unit0, int used, int t)
{
    const float2 *ml = reinterpret_cast<const float2 *>(ws_ml) + unit0;
    const float *oc = ws_o + unit0 * D + t;
    float mx = kNegBig, acc = 0.0f, lsum = 0.0f;
#pragma unroll 4
    for (int c = 0; c < used; ++c) {
        const float2 rec = ml[c];
        const float part = oc[(size_t)c * D];
        const float m_new = fmaxf(mx, rec.x);
        const float a_old = fast_exp2(mx - m_new), a_new = fast_exp2(rec.x - m_new);
        lsum = fmaf(a_new, rec.y, lsum * a_old);
        acc = fmaf(a_new, part, acc * a_old);
        mx = m_new;
    }
    return lsum > 0.0f ? acc / lsum : 0.0f;
}

template <int D>
__global__ __launch_bounds__(kMergeThreads) void sha_merge_kernel(
    const int32_t *__restrict__ seqlens, const int32_t *__restrict__ head_idx,
    const float *__restrict__ ws_o, const float *__restrict__ ws_ml, float *__restrict__ out,
    int Hq, int Hkv, int S, int k, int G, int chunk, int nsplit)
{
    constexpr int HEADS_PER_PASS = kMergeThreads / D;
    __shared__ int slot_of[kMergeHeads];
    const int b = blockIdx.y, tid = threadIdx.x;
    const int h0 = blockIdx.x * kMergeHeads;
    const int h_last = min(h0 + kMergeHeads, Hq) - 1;
    const int g_first = h0 / G, g_last = h_last / G;

    if (tid < kMergeHeads) slot_of[tid] = kNoSlot;
    __syncthreads();
    if (head_idx) {
        for (int s = tid; s < k; s += kMergeThreads) {
            const int id = head_idx[(size_t)b * k + s];
            if (id >= g_first && id <= g_last) atomicMin(&slot_of[id - g_first], s);
        }
    } else if (tid <= g_last - g_first) {
        slot_of[tid] = g_first + tid;               // dense: slot == KV head
    }
    __syncthreads();

    int n = seqlens[b];
    n = n < 0 ? 0 : (n > S ? S : n);
    const int used = (n + chunk - 1) / chunk;
    const int t = tid % D;
#pragma unroll
    for (int pass = 0; pass < kMergeHeads / HEADS_PER_PASS; ++pass) {
        const int h = h0 + pass * HEADS_PER_PASS + tid / D;
        if (h > h_last) continue;
        const int slot = slot_of[h / G - g_first];
        float result = 0.0f;
        if (slot != kNoSlot && used > 0)
            result = fold_chunks<D>(ws_o, ws_ml, (((size_t)b * k + slot) * G + (h % G)) * nsplit, used, t);
        out[((size_t)b * Hq + h) * D + t] = result;
    }
}

// Merge kernel of the head-importance labeller (Section 3.2: heads ranked by the L2 norm of
// their attention output; Section 4.2: the k best are the router's training targets): the dense
// run's merge with the norm and the ranking as its epilogue, so the labels need no pass over the
// stored output.  grid = B, block = 256: one workgroup folds the chunk records of ALL query heads
// of its request (dense: slot == KV head), 256 / D heads at a time, exactly as sha_merge_kernel
// does (same fold, same bits), optionally stores them, and adds the squares of each group's
// G * D values in double (a float squared is exact in double): the D values of a head through an
// xor butterfly per wave and a fixed-order sum over the head's waves, the G heads of a group in
// ascending order (one thread does those few additions, so the order never varies).  The groups are then ranked by that sum of squares with the router's rule
// (larger first, equal by ascending id, NaN last).
template <int D>
__global__ __launch_bounds__(kMergeThreads) void sha_merge_label_kernel(
    const int32_t *__restrict__ seqlens, const float *__restrict__ ws_o, const float *__restrict__ ws_ml,
    float *__restrict__ out, int32_t *__restrict__ labels, float *__restrict__ norms_out, int Hq, int Hkv,
    int S, int G, int chunk, int nsplit, int k_label)
{
    constexpr int HEADS_PER_PASS = kMergeThreads / D, WAVES_PER_HEAD = D / 64;
    __shared__ double sh_ss[POLAR_MAX_ROUTER_H];
    __shared__ double sh_part[kMergeThreads / 64];
    __shared__ int sh_rank[POLAR_MAX_ROUTER_H];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int g = tid; g < Hkv; g += kMergeThreads) {
        sh_ss[g] = 0.0;
        sh_rank[g] = 0;
    }
    int n = seqlens[b];
    n = n < 0 ? 0 : (n > S ? S : n);
    const int used = (n + chunk - 1) / chunk;
    const int t = tid % D;
    for (int h0 = 0; h0 < Hq; h0 += HEADS_PER_PASS) {
        const int h = h0 + tid / D;
        float result = 0.0f;
        if (h < Hq && used > 0)       // dense: unit0 = ((b * Hkv + h / G) * G + h % G) * nsplit = (b * Hq + h) * nsplit
            result = fold_chunks<D>(ws_o, ws_ml, ((size_t)b * Hq + h) * nsplit, used, t);
        if (h < Hq && out) out[((size_t)b * Hq + h) * D + t] = result;
        double sq = (double)result * (double)result;
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            const int lo = __shfl_xor(__double2loint(sq), m), hi = __shfl_xor(__double2hiint(sq), m);
            sq += __hiloint2double(hi, lo);
        }
        __syncthreads();                       // sh_part of the previous pass has been consumed
        if (lane == 0) sh_part[wave] = sq;
        __syncthreads();
        if (tid == 0)                          // one thread, fixed order: waves of a head, heads ascending
            for (int i = 0; i < HEADS_PER_PASS && h0 + i < Hq; ++i) {
                double head_ss = 0.0;
#pragma unroll
                for (int w = 0; w < WAVES_PER_HEAD; ++w) head_ss += sh_part[i * WAVES_PER_HEAD + w];
                sh_ss[(h0 + i) / G] += head_ss;
            }
    }
    __syncthreads();
    for (int g = tid; g < Hkv; g += kMergeThreads)
        if (norms_out) norms_out[(size_t)b * Hkv + g] = (float)sqrt(sh_ss[g]);
    const int parts = kMergeThreads / Hkv;            // >= 1: Hkv <= 256
    if (tid < parts * Hkv) {
        const int part = tid / Hkv, g = tid - part * Hkv;
        const double mine = sh_ss[g];
        int cnt = 0;
        for (int j = part; j < Hkv; j += parts) {
            const double other = sh_ss[j];
            const bool on = other != other, mn = mine != mine;
            const bool first = (on || mn) ? ((on && mn) ? j < g : mn) : (other > mine || (other == mine && j < g));
            cnt += first ? 1 : 0;
        }
        if (cnt) atomicAdd(&sh_rank[g], cnt);
    }
    __syncthreads();
    if (tid < Hkv && sh_rank[tid] < k_label) labels[(size_t)b * k_label + sh_rank[tid]] = tid;
}

template <class DT, int D, bool RMS>
hipError_t launch_partial_g(int G, dim3 grid, hipStream_t st, const uint16_t *q, const uint16_t *K,
                            const uint16_t *V, const int32_t *seqlens, const int32_t *head_idx,
                            float *ws_o, float *ws_ml, float *out, int Hq, int Hkv, int S, int k,
                            int chunk, int nsplit, float c)
{
#define POLAR_LAUNCH(GG)                                                                          \
    if (out)                                                                                      \
        hipLaunchKernelGGL((sha_partial_kernel<DT, D, GG, RMS, true>), grid,                      \
                           dim3(Shape<GG>::kWaves * 64), 0, st, q, K, V, seqlens, head_idx, ws_o, \
                           ws_ml, out, Hq, Hkv, S, k, chunk, nsplit, c);                          \
    else                                                                                          \
        hipLaunchKernelGGL((sha_partial_kernel<DT, D, GG, RMS, false>), grid,                     \
                           dim3(Shape<GG>::kWaves * 64), 0, st, q, K, V, seqlens, head_idx, ws_o, \
                           ws_ml, out, Hq, Hkv, S, k, chunk, nsplit, c)
    switch (G) {
    case 1: POLAR_LAUNCH(1); break;
    case 2: POLAR_LAUNCH(2); break;
    case 4: POLAR_LAUNCH(4); break;
    case 8: POLAR_LAUNCH(8); break;
    default: return hipErrorInvalidValue;
    }
#undef POLAR_LAUNCH
    return hipGetLastError();
}

template <class DT, int D>
hipError_t launch_partial_layout(polar_kv_layout layout, int G, dim3 grid, hipStream_t st,
                                 const uint16_t *q, const uint16_t *K, const uint16_t *V,
                                 const int32_t *seqlens, const int32_t *head_idx, float *ws_o,
                                 float *ws_ml, float *out, int Hq, int Hkv, int S, int k, int chunk,
                                 int nsplit, float c)
{
    if (layout == POLAR_KV_BSHD)
        return launch_partial_g<DT, D, true>(G, grid, st, q, K, V, seqlens, head_idx, ws_o, ws_ml, out,
                                             Hq, Hkv, S, k, chunk, nsplit, c);
    return launch_partial_g<DT, D, false>(G, grid, st, q, K, V, seqlens, head_idx, ws_o, ws_ml, out,
                                          Hq, Hkv, S, k, chunk, nsplit, c);
}

}  // namespace

hipError_t launch_sha_partial(const void *q, const void *K, const void *V, const int32_t *seqlens,
                              const int32_t *head_idx, float *ws, float *direct_out,
                              const ShaPlan &plan, int B, int Hq, int Hkv, int S, int d, int k,
                              polar_dtype dt, polar_kv_layout layout, float scale_log2e,
                              hipStream_t stream)
{
    if (direct_out && plan.nsplit != 1) return hipErrorInvalidValue;
    if (plan.grouped_mfma)
        return launch_sha_partial_gqa(q, K, V, seqlens, head_idx, ws, direct_out, plan, B, Hq, Hkv, S,
                                      k, dt, layout, scale_log2e, stream);
    const dim3 grid((unsigned)((size_t)B * plan.nsplit * k));
    float *ws_o = ws, *ws_ml = ws + plan.o_floats;
    const uint16_t *q16 = static_cast<const uint16_t *>(q);
    const uint16_t *K16 = static_cast<const uint16_t *>(K);
    const uint16_t *V16 = static_cast<const uint16_t *>(V);
#define POLAR_ARGS layout, plan.G, grid, stream, q16, K16, V16, seqlens, head_idx, ws_o, ws_ml, direct_out, Hq, \
                   Hkv, S, k, plan.chunk, plan.nsplit, scale_log2e
    if (dt == POLAR_F16) {
        if (d == 128) return launch_partial_layout<F16, 128>(POLAR_ARGS);
        if (d == 64) return launch_partial_layout<F16, 64>(POLAR_ARGS);
    } else {
        if (d == 128) return launch_partial_layout<BF16, 128>(POLAR_ARGS);
        if (d == 64) return launch_partial_layout<BF16, 64>(POLAR_ARGS);
    }
#undef POLAR_ARGS
    return hipErrorInvalidValue;
}

hipError_t launch_sha_merge(const int32_t *seqlens, const int32_t *head_idx, float *out,
                            const float *ws, const ShaPlan &plan, int B, int Hq, int Hkv, int S,
                            int d, int k, hipStream_t stream)
{
    const dim3 grid((unsigned)((Hq + kMergeHeads - 1) / kMergeHeads), (unsigned)B);
    const float *ws_o = ws, *ws_ml = ws + plan.o_floats;
    if (d == 128)
        hipLaunchKernelGGL((sha_merge_kernel<128>), grid, dim3(kMergeThreads), 0, stream, seqlens,
                           head_idx, ws_o, ws_ml, out, Hq, Hkv, S, k, plan.G, plan.chunk,
                           plan.nsplit);
    else if (d == 64)
        hipLaunchKernelGGL((sha_merge_kernel<64>), grid, dim3(kMergeThreads), 0, stream, seqlens, head_idx,
                           ws_o, ws_ml, out, Hq, Hkv, S, k, plan.G, plan.chunk, plan.nsplit);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t launch_sha_merge_label(const int32_t *seqlens, float *out, int32_t *labels, float *norms_out,
                                  const float *ws, const ShaPlan &plan, int B, int Hq, int Hkv, int S, int d,
                                  int k_label, hipStream_t stream)
{
    const float *ws_o = ws, *ws_ml = ws + plan.o_floats;
    if (d == 128)
        hipLaunchKernelGGL((sha_merge_label_kernel<128>), dim3((unsigned)B), dim3(kMergeThreads), 0, stream, seqlens,
                           ws_o, ws_ml, out, labels, norms_out, Hq, Hkv, S, plan.G, plan.chunk, plan.nsplit, k_label);
    else if (d == 64)
        hipLaunchKernelGGL((sha_merge_label_kernel<64>), dim3((unsigned)B), dim3(kMergeThreads), 0, stream, seqlens,
                           ws_o, ws_ml, out, labels, norms_out, Hq, Hkv, S, plan.G, plan.chunk, plan.nsplit, k_label);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace polar
