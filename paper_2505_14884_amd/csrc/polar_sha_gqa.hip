// Selective Head Attention, decode step, grouped-query variant for gfx950 (CDNA4): the
// streaming kernel for G = Hq / Hkv > 1 at head dimension 128, with both contractions on the
// matrix cores.
//
// What is computed is the same as in the per-head kernel (Section 3.2, per-head attention
// equation; Algorithm 1; Section 4.2, last sentence, for grouped heads: the selection unit is a
// KV group, and a selected group serves all G query heads of the group from one read of its K
// and V rows): per (request, selected group, chunk
// of rows) one record (running max, sum, unnormalised output) per query head.
//
// Why a second kernel: with G query rows per K/V row the vector-ALU formulation needs G dot
// products, G cross-lane reductions and G*d multiply-adds per cache row, and at G = 4 and 8
// that arithmetic, not HBM, sets the time.  A G x d by d x rows product is a (thin) matrix
// product, so here S = K Q^T runs on v_mfma_f32_16x16x32 and O^T = V^T P^T on
// v_mfma_f32_16x16x16, with the G heads padded to the 16 columns of a tile; the vector ALU is
// left with the softmax of 4 scores per lane and a few shifts per 16 rows, the same for every
// G <= 16.
//
// Register layouts (lane = 16*hi + lo, one wave handles blocks of 16 consecutive rows):
//   * K and V are both loaded with wave-wide reads of four whole 256-byte rows: lane (lo, hi),
//     load u reads row 4hi + u of the block, 16-byte piece lo (dims 8lo .. 8lo+7).
//     (Loading K straight into the operand layout below would read 64-byte pieces of 16 rows
//     per instruction, i.e. every 128-byte line twice; under load the second request often
//     misses and K is fetched twice from HBM: 828 -> 721 us on a ragged 128/32-head layer.)
//   * S = K Q^T: the K rows go through a wave-private LDS tile (no workgroup barrier) into
//     the operand layout: step s: lane holds row lo, dims 32s + 8hi .. +7.  Q^T operand: lane
//     holds head lo (zero for lo >= G), same dims.  Result: lane holds the scores of head lo
//     for rows 4hi + i, i = 0..3.
//   * Those 4 scores are exactly the 4 contraction slots a lane must supply to the second
//     product (slot u = row 4hi + u, the row that load u brought into this lane's group).  V is
//     transposed *inside each lane* with shifts and masks: for dim e of the piece, the operand
//     is {V[4hi + u][8lo + e]}, u = 0..3.  O^T tile e = (V^T)_e P^T: lane holds head lo, dims
//     8(4hi + i) + e, i = 0..3.
//   * P is fed as two 16-bit terms (the rounded value and the rounded remainder), so the
//     probabilities keep ~17 (bf16) or ~22 (fp16) significant bits; the products with the
//     16-bit V values are exact and accumulate in fp32.
//   * One running max per head, shared by the 4 lanes (hi = 0..3) of the head through two
//     cross-lane exchanges per block; sums are kept per lane and added at the end.
//   * Blocks of 16 rows rather than 32 keep the register stages (K: one, V: two) small enough
//     for three waves per SIMD, i.e. three workgroups per compute unit: one that is starting or
//     finishing then idles a third of the unit instead of half (LLaMA-3-8B GQA layer: 82.4 ->
//     79.7 us; ragged 128/32-head layer in chunks of 4096: 719 -> 697 us).
#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kD = 128;                 // head dimension this kernel is written for
#if defined(POLAR_GQA_WAVES)
constexpr int kGqaWaves = POLAR_GQA_WAVES;   // build-time override for sweeps
#else
constexpr int kGqaWaves = 4;            // waves per workgroup
#endif
constexpr int kBlockRows = 16;          // cache rows one wave consumes per iteration
constexpr int kTilePitch = 2 * kD + 16; // bytes between rows of a wave's K tile in LDS: the 16
                                        // lanes of an operand read then fall in distinct banks
constexpr int kTileBytes = kBlockRows * kTilePitch;
constexpr float kNegBig = -1.0e30f;     // "no row seen yet" (finite on purpose)

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// D[i][j] += sum_k A[i][k] * B[k][j]; lane 16*hi + lo supplies A[lo][8hi..8hi+7] and
// B[8hi..8hi+7][lo], and receives D[4hi + 0..3][lo].
template <bool BF> __device__ __forceinline__ f32x4 mfma(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ u32x4 load_nt(const u32x4 *p) { return __builtin_nontemporal_load(p); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Round a probability to the 16-bit type and return its bit pattern; `back` is the rounded value.
template <bool BF> __device__ __forceinline__ uint32_t round16(float x, float &back)
{
    if constexpr (BF) {
        const __bf16 h = (__bf16)x;
        back = (float)h;
        return (uint32_t)__builtin_bit_cast(unsigned short, h);
    } else {
        const _Float16 h = (_Float16)x;
        back = (float)h;
        return (uint32_t)__builtin_bit_cast(unsigned short, h);
    }
}

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// D[i][j] += sum_k A[i][k] * B[k][j] with k = 16: lane 16*hi + lo supplies A[lo][4hi..4hi+3] and
// B[4hi..4hi+3][lo] (four 16-bit values each) and receives D[4hi + 0..3][lo].
template <bool BF> __device__ __forceinline__ f32x4 mfma_k16(const u32x2 &a, const u32x2 &b, f32x4 c)
{
    if constexpr (BF)
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(i16x4, a),
                                                         __builtin_bit_cast(i16x4, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4, a),
                                                     __builtin_bit_cast(f16x4, b), c, 0, 0, 0);
}

// Four wave-wide loads of four whole rows each: lane (lo, hi), load u reads row 4hi + u of the
// 16-row block at `rb`, 16-byte piece lo; rows clamped to `last`.
__device__ __forceinline__ void load_rows16(u32x4 (&x)[4], const u32x4 *__restrict__ p, int rb, int last,
                                            int row_stride, int lo, int hi)
{
#pragma unroll
    for (int u = 0; u < 4; ++u)
        x[u] = load_nt(p + (size_t)min(rb + 4 * hi + u, last) * row_stride + lo);
}

__device__ __forceinline__ void stash_k16(unsigned char *tile, const u32x4 (&kx)[4], int lo, int hi)
{
#pragma unroll
    for (int u = 0; u < 4; ++u)
        *reinterpret_cast<u32x4 *>(tile + (4 * hi + u) * kTilePitch + 16 * lo) = kx[u];
    __builtin_amdgcn_wave_barrier();
}

// One 16-row block: K already in the wave's LDS tile, V rows in registers.
template <bool BF>
__device__ __forceinline__ void consume_block16(const unsigned char *tile, const u32x4 (&vx)[4],
                                                const u32x4 (&qs)[4], int rb, int last, int lo, int hi,
                                                float c, float &m, float &l, f32x4 (&o)[8])
{
    f32x4 s0 = {0.0f, 0.0f, 0.0f, 0.0f};
    const unsigned char *rd = tile + lo * kTilePitch + 16 * hi;
#pragma unroll
    for (int s = 0; s < 4; ++s)
        s0 = mfma<BF>(*reinterpret_cast<const u32x4 *>(rd + 64 * s), qs[s], s0);
    __builtin_amdgcn_wave_barrier();

    float sc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) sc[i] = (rb + 4 * hi + i > last) ? -INFINITY : s0[i] * c;
    float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    const float alpha = fast_exp2(m - m_new);
    m = m_new;

    float psum = 0.0f;
    uint32_t ph[4], pl[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const float p = fast_exp2(sc[u] - m_new);
        psum += p;
        float back, unused;
        ph[u] = round16<BF>(p, back);
        pl[u] = round16<BF>(p - back, unused);
    }
    l = l * alpha + psum;
    const u32x2 bh = {ph[0] | (ph[1] << 16), ph[2] | (ph[3] << 16)};
    const u32x2 bl = {pl[0] | (pl[1] << 16), pl[2] | (pl[3] << 16)};

#pragma unroll
    for (int e = 0; e < 8; ++e) {
        u32x2 a;
#pragma unroll
        for (int t = 0; t < 2; ++t)
            a[t] = (e & 1) ? ((vx[2 * t][e / 2] >> 16) | (vx[2 * t + 1][e / 2] & 0xffff0000u))
                           : ((vx[2 * t][e / 2] & 0xffffu) | (vx[2 * t + 1][e / 2] << 16));
        f32x4 acc = o[e] * alpha;
        acc = mfma_k16<BF>(a, bh, acc);
        o[e] = mfma_k16<BF>(a, bl, acc);
    }
}

// Streaming kernel for grouped heads.  1-D grid of B*nsplit*k workgroups decoded as in the
// per-head kernel (slot fastest, so the equal-sized workgroups of one (request, chunk) spread
// over the XCDs); block = 4 waves.  Wave w takes blocks w, w+4, ... of the chunk; the loads of
// the next block are in flight while the current one is consumed.
// Workspace records as in the per-head kernel: unit = ((b*k + slot)*G + g)*nsplit + split.
// DIRECT (only with nsplit == 1): final normalised rows go to `out` and one wave zero-fills this
// slot's share of the unselected heads, as in the per-head kernel; no merge kernel runs.
template <bool BF, bool ROW_MAJOR_SEQ, bool DIRECT>
__global__ __launch_bounds__(kGqaWaves * 64) __attribute__((amdgpu_waves_per_eu(2, 3))) void sha_partial_gqa_kernel(
    const uint16_t *__restrict__ q, const uint16_t *__restrict__ K, const uint16_t *__restrict__ V,
    const int32_t *__restrict__ seqlens, const int32_t *__restrict__ head_idx,
    float *__restrict__ ws_o, float *__restrict__ ws_ml, float *__restrict__ out, int Hq, int Hkv,
    int S, int k, int G, int chunk, int nsplit, float c)
{
    const int slot = blockIdx.x % k;
    const int rest = blockIdx.x / k;
    const int split = rest % nsplit, b = rest / nsplit;
    int n = seqlens[b];
    const int g_kv = head_idx ? head_idx[(size_t)b * k + slot] : slot;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int id0 = -1;
    if (DIRECT && head_idx && wave == kGqaWaves - 1 && lane < k) id0 = head_idx[(size_t)b * k + lane];
    n = n < 0 ? 0 : (n > S ? S : n);
    // The zero fill runs last (one wave, after the output rows), so that no wave waits for it.
#define POLAR_DIRECT_ZERO_FILL()                                                                   \
    if (DIRECT && wave == kGqaWaves - 1 && (head_idx || n == 0))                                   \
        direct_zero_fill(head_idx ? head_idx + (size_t)b * k : nullptr, id0, head_idx && n > 0,    \
                         slot, k, Hkv, G * kD, out + (size_t)b * Hq * kD, lane)
    const int row_begin = split * chunk;
    if (row_begin >= n || (unsigned)g_kv >= (unsigned)Hkv) {
        POLAR_DIRECT_ZERO_FILL();
        return;
    }
    const int row_end = min(row_begin + chunk, n);
    const int last = row_end - 1;

    const int lo = lane & 15, hi = lane >> 4;

    const size_t slab = ROW_MAJOR_SEQ ? ((size_t)b * S * Hkv + g_kv) * kD
                                      : ((size_t)b * Hkv + g_kv) * (size_t)S * kD;
    const int row_stride = ROW_MAJOR_SEQ ? Hkv * (kD / 8) : (kD / 8);   // in 16-byte units
    const u32x4 *__restrict__ Kp = reinterpret_cast<const u32x4 *>(K + slab);
    const u32x4 *__restrict__ Vp = reinterpret_cast<const u32x4 *>(V + slab);

    // one buffer: the waves' K tiles during the loop, their partial results after it
    constexpr int kMergeBytes = kGqaWaves * POLAR_MAX_GROUP * kD * (int)sizeof(float);
    constexpr int kSmemBytes = kGqaWaves * kTileBytes > kMergeBytes ? kGqaWaves * kTileBytes : kMergeBytes;
    __shared__ __align__(16) unsigned char smem[kSmemBytes];
    unsigned char *tile = smem + wave * kTileBytes;

    u32x4 qs[4];
    {
        const u32x4 *qp = reinterpret_cast<const u32x4 *>(
            q + ((size_t)b * Hq + (size_t)g_kv * G + (lo < G ? lo : 0)) * kD);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const u32x4 v = qp[4 * s + hi];
            qs[s] = lo < G ? v : u32x4{0u, 0u, 0u, 0u};
        }
    }

    float m = kNegBig, l = 0.0f;
    f32x4 o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};

    // Blocks of 16 rows: wave w takes blocks w, w+4, ... of the chunk.  K has one register stage
    // (its rows go to the wave's LDS tile first thing, which frees the registers for the next
    // block's loads), V two.  Blocks are taken in pairs so that the body has no branch between a
    // load and its use (the compiler would otherwise sink the loads below the branch, next to the
    // use); the scheduling fences keep the next block's loads ahead of the waits on this one.
    const int rows = row_end - row_begin;
    constexpr int kStep = kBlockRows * kGqaWaves;
    const int n_blocks = (rows + kBlockRows - 1) / kBlockRows;
    const int n_it = n_blocks > wave ? (n_blocks - wave + kGqaWaves - 1) / kGqaWaves : 0;
    const int rb0 = row_begin + kBlockRows * wave;
    if (n_it > 0) {
        u32x4 kr[4], va[4], vb[4];
        load_rows16(kr, Kp, rb0, last, row_stride, lo, hi);
        load_rows16(va, Vp, rb0, last, row_stride, lo, hi);
        int it = 0;
        for (; it + 2 <= n_it; it += 2) {
            const int rb = rb0 + it * kStep;
            stash_k16(tile, kr, lo, hi);
            load_rows16(kr, Kp, rb + kStep, last, row_stride, lo, hi);
            load_rows16(vb, Vp, rb + kStep, last, row_stride, lo, hi);
            __builtin_amdgcn_sched_barrier(0);
            consume_block16<BF>(tile, va, qs, rb, last, lo, hi, c, m, l, o);
            __builtin_amdgcn_sched_barrier(0);
            stash_k16(tile, kr, lo, hi);
            load_rows16(kr, Kp, rb + 2 * kStep, last, row_stride, lo, hi);
            load_rows16(va, Vp, rb + 2 * kStep, last, row_stride, lo, hi);
            __builtin_amdgcn_sched_barrier(0);
            consume_block16<BF>(tile, vb, qs, rb + kStep, last, lo, hi, c, m, l, o);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (it < n_it) {
            stash_k16(tile, kr, lo, hi);
            consume_block16<BF>(tile, va, qs, rb0 + it * kStep, last, lo, hi, c, m, l, o);
        }
    }
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);

    // the per-wave partial results reuse the K tiles' memory once every wave has left the loop
    __syncthreads();
    float (*sm_o)[POLAR_MAX_GROUP][kD] = reinterpret_cast<float (*)[POLAR_MAX_GROUP][kD]>(smem);
    __shared__ float sm_ml[kGqaWaves][POLAR_MAX_GROUP][2];
    if (lo < G) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float4 *dst = reinterpret_cast<float4 *>(&sm_o[wave][lo][32 * hi + 8 * i]);
            dst[0] = make_float4(o[0][i], o[1][i], o[2][i], o[3][i]);
            dst[1] = make_float4(o[4][i], o[5][i], o[6][i], o[7][i]);
        }
        if (hi == 0) {
            sm_ml[wave][lo][0] = m;
            sm_ml[wave][lo][1] = l;
        }
    }
    __syncthreads();

    // Merge the waves: thread t owns output column t % 128 of every second query head.
    const int t = threadIdx.x % kD;
    for (int g = threadIdx.x / kD; g < G; g += kGqaWaves * 64 / kD) {
        float mx = sm_ml[0][g][0];
#pragma unroll
        for (int w = 1; w < kGqaWaves; ++w) mx = fmaxf(mx, sm_ml[w][g][0]);
        float acc = 0.0f, lsum = 0.0f;
#pragma unroll
        for (int w = 0; w < kGqaWaves; ++w) {
            const float a = fast_exp2(sm_ml[w][g][0] - mx);
            acc = fmaf(a, sm_o[w][g][t], acc);
            lsum = fmaf(a, sm_ml[w][g][1], lsum);
        }
        if (DIRECT) {
            out[((size_t)b * Hq + (size_t)g_kv * G + g) * kD + t] = lsum > 0.0f ? acc / lsum : 0.0f;
        } else {
            const size_t unit = (((size_t)b * k + slot) * G + g) * nsplit + split;
            ws_o[unit * kD + t] = acc;
            if (t == 0) {
                ws_ml[unit * 2 + 0] = mx;
                ws_ml[unit * 2 + 1] = lsum;
            }
        }
    }
    POLAR_DIRECT_ZERO_FILL();
#undef POLAR_DIRECT_ZERO_FILL
}

}  // namespace

hipError_t launch_sha_partial_gqa(const void *q, const void *K, const void *V, const int32_t *seqlens,
                                  const int32_t *head_idx, float *ws, float *direct_out,
                                  const ShaPlan &plan, int B, int Hq, int Hkv, int S, int k,
                                  polar_dtype dt, polar_kv_layout layout, float scale_log2e,
                                  hipStream_t stream)
{
    if (plan.G > POLAR_MAX_GROUP) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((size_t)B * plan.nsplit * k)), block(kGqaWaves * 64);
    float *ws_o = ws, *ws_ml = ws + plan.o_floats;
    const uint16_t *q16 = static_cast<const uint16_t *>(q);
    const uint16_t *K16 = static_cast<const uint16_t *>(K);
    const uint16_t *V16 = static_cast<const uint16_t *>(V);
#define POLAR_GQA_LAUNCH3(BF, RMS, DIR)                                                             \
    hipLaunchKernelGGL((sha_partial_gqa_kernel<BF, RMS, DIR>), grid, block, 0, stream, q16, K16, V16,  \
                       seqlens, head_idx, ws_o, ws_ml, direct_out, Hq, Hkv, S, k, plan.G, plan.chunk, \
                       plan.nsplit, scale_log2e)
#define POLAR_GQA_LAUNCH(BF, RMS)                                                                   \
    if (direct_out) {                                                                               \
        POLAR_GQA_LAUNCH3(BF, RMS, true);                                                           \
    } else {                                                                                        \
        POLAR_GQA_LAUNCH3(BF, RMS, false);                                                          \
    }
    const bool bf = dt == POLAR_BF16, rms = layout == POLAR_KV_BSHD;
    if (bf && rms) {
        POLAR_GQA_LAUNCH(true, true);
    } else if (bf) {
        POLAR_GQA_LAUNCH(true, false);
    } else if (rms) {
        POLAR_GQA_LAUNCH(false, true);
    } else {
        POLAR_GQA_LAUNCH(false, false);
    }
#undef POLAR_GQA_LAUNCH
#undef POLAR_GQA_LAUNCH3
    return hipGetLastError();
}

}  // namespace polar
