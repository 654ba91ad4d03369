// Second factor of the sparsified MLP for gfx950 (Section 3.1: MLP_{S_B}(x) =
// sigma(x W_{1,S_B}) W_{2,S_B}^T, the sum running over the selected neurons only; Section 4.1 and
// Appendix "Sparse Kernels": the index is applied inside the kernel, the weights are stored one
// contiguous row per neuron).
//
//   Y[m, c] = sum_{j < live} h16(H[m, j]) * W2[idx[j], c]       H [M,cap] float, W2 [N,Kout]
//
// Here the gather runs along the contraction axis: every selected neuron contributes one row of
// Kout weights, read once and used for M <= 128 multiply-adds per element, so the kernel is bound
// by HBM like the first factor and is organised around streaming those rows:
//   * (up to 64 rows; the kernel for 65 to 128 rows is described where it stands) a wave owns 128
//     output columns and all M rows (MT * 8 accumulator tiles of 16 x 16) and walks
//     the selected neurons 32 at a time: 8 loads of 16 bytes per lane fetch 32 row pieces of 256
//     bytes (16 lanes per piece, 4 pieces per load: whole cache lines).  A lane then holds an
//     8 x 8 block (8 neurons x 8 columns) of 16-bit weights; transposed inside the lane (shifts
//     and masks, no LDS) it is the B operand of 8 matrix-core steps, one per column e of the block:
//     lane (x, kg) feeds column 8x + e with the neurons 8kg .. 8kg + 7 of the block.
//   * the activations are the A operand.  A first, small kernel rounds them to the storage type
//     (the matrix cores take 16-bit operands; a 16-bit model holds them so), zeroes the entries
//     whose id is invalid or beyond the live count, and pads the rows to a multiple of 32: every
//     column block needs the same values, so doing it once takes the conversions, the masking and
//     the row-end special case out of the streaming loop.  The workgroup stages the prepared
//     values through LDS, a chunk of 8 blocks at a time (whole cache lines, each once; the next
//     chunk travels in registers while the current one is multiplied), and lane (x, kg) reads
//     H16[m = 16t + x, 8 consecutive j] with one 16-byte LDS read.
//   * apart from one barrier per chunk the waves of a workgroup do not talk to each other while
//     they stream.  A workgroup is a pair of column blocks times four neuron parities: wave (c, p)
//     takes the 32-neuron blocks p, p + 4, ... of the workgroup's range, and the four add their
//     accumulators through LDS at the end.  Eight waves per compute unit, two per SIMD, are what
//     keeps the matrix cores and the vector ALU fed: with one wave per SIMD every dependent
//     instruction waits out its full latency.
//   * the launch is Kout/256 column blocks times NS contraction ranges, NS chosen so that the
//     grid fills the compute units once; range s covers an NS-th of the live blocks, whatever the
//     live count is (it stays on the device), and leaves its sums in the workspace; a second
//     kernel adds the NS sums of every output element in ascending range order and stores Y.
#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kDownParities = 4;                 // waves that share a column block
constexpr int kDownThreads = 64 * 2 * kDownParities;
constexpr int kPrepThreads = 256;
constexpr int kDownWaveCols = 128;               // output columns per wave
constexpr int kDownGroupCols = 2 * kDownWaveCols;    // per workgroup (two column blocks x four parities)
constexpr int kDownBlock = 32;                   // neurons per step (the contraction depth of one MFMA)
constexpr int kDownMaxIds = 8192;                // ids of a workgroup's range kept in LDS
constexpr int kDownTargetGroups = 256;           // one workgroup per compute unit
constexpr int kDownMaxRows = 64;                 // rows of the batch the kernel with two column blocks per workgroup takes
constexpr int kDownPassRows = 128;               // rows of the batch per pass (65 to 128: the row-split kernel)
constexpr int kChunkBlocks = 8;                  // blocks of activations staged in LDS at a time
constexpr int kChunkPitch = kChunkBlocks * kDownBlock * 2 + 16;   // bytes per row of a chunk, padded

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
// vectors that need only 4-byte alignment (a row of H starts wherever cap puts it)
typedef float f32x4u __attribute__((ext_vector_type(4), aligned(4)));
typedef int i32x4u __attribute__((ext_vector_type(4), aligned(4)));

template <bool BF> __device__ __forceinline__ f32x4 mfma16x16x32(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    if (BF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// bit pattern of x rounded to the storage type (nearest, ties to even)
template <bool BF> __device__ __forceinline__ unsigned int to_storage(float x)
{
    if constexpr (BF)
        return (unsigned int)__builtin_bit_cast(unsigned short, (__bf16)x);
    else
        return (unsigned int)__builtin_bit_cast(unsigned short, (_Float16)x);
}

// The blocks of 32 neurons are dealt to the NS ranges as evenly as whole blocks allow.
__device__ __forceinline__ int range_bound(int blocks, int NS, int s) { return (int)((long)blocks * s / NS); }

// H16[m, j] = the storage-type bit pattern of H[m, j] rounded to nearest even, or 0 where position j
// is at or beyond the live count or its id lies outside [0, N); rows have room for cap32 (cap
// rounded up to a multiple of 32) values and are written, zero-padded, up to the live count
// rounded up likewise.  One thread per (row, 8 positions).
template <bool BF>
__global__ __launch_bounds__(kPrepThreads) void select_gemm_down_prepare_kernel(
    const float *__restrict__ H, const int32_t *__restrict__ idx, const int32_t *__restrict__ count_ptr,
    uint16_t *__restrict__ H16, int M, int N, int cap)
{
    int count = cap;
    if (count_ptr) {
        const int c = *count_ptr;
        count = c < 0 ? 0 : (c < cap ? c : cap);
    }
    const int cap32 = (cap + kDownBlock - 1) / kDownBlock * kDownBlock;
    const int groups = cap32 / 8;
    const long item = (long)blockIdx.x * kPrepThreads + threadIdx.x;
    if (item >= (long)M * groups) return;
    const int m = (int)(item / groups), j0 = (int)(item % groups) * 8;
    // the streaming kernel reads whole blocks of 32 up to the live count and nothing beyond
    if (j0 >= (count + kDownBlock - 1) / kDownBlock * kDownBlock) return;
    unsigned int v[8];
    if (j0 + 8 <= count) {                       // eight live positions: vector loads
        const i32x4u id_lo = *reinterpret_cast<const i32x4u *>(idx + j0);
        const i32x4u id_hi = *reinterpret_cast<const i32x4u *>(idx + j0 + 4);
        const f32x4u h_lo = *reinterpret_cast<const f32x4u *>(H + (size_t)m * cap + j0);
        const f32x4u h_hi = *reinterpret_cast<const f32x4u *>(H + (size_t)m * cap + j0 + 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int id = i < 4 ? id_lo[i & 3] : id_hi[i & 3];
            const float h = i < 4 ? h_lo[i & 3] : h_hi[i & 3];
            v[i] = (id >= 0 && id < N) ? to_storage<BF>(h) : 0u;
        }
    } else {                                     // the group that holds the live count's end, and the padding
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = j0 + i;
            unsigned int bits = 0u;
            if (j < count) {
                const int id = idx[j];
                if (id >= 0 && id < N) bits = to_storage<BF>(H[(size_t)m * cap + j]);
            }
            v[i] = bits;
        }
    }
    const u32x4 packed = {v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
    *reinterpret_cast<u32x4 *>(H16 + (size_t)m * cap32 + j0) = packed;
}

// grid = (Kout / 256) * NS workgroups; block = 512 threads (8 waves).
// part holds, per (range, column block of 128), MT * 8 accumulator tiles of 64 lanes x 16 bytes.
template <bool BF, int MT>
__global__ __launch_bounds__(kDownThreads) void select_gemm_down_kernel(
    const uint16_t *__restrict__ H16, const uint16_t *__restrict__ W2, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_ptr, float *__restrict__ part, int M, int Kout, int N, int cap,
    int NS)
{
    // LDS: two buffers for chunks of the activations (16 * MT rows x 256 positions, padded rows:
    // conflict-free 16-byte operand reads), which the waves' accumulators reuse at the end, then
    // the ids of the range
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kChunkBytes = 16 * MT * kChunkPitch;
    int *sh_id = reinterpret_cast<int *>(smem + 2 * kChunkBytes);

    int count = cap;
    if (count_ptr) {
        const int c = *count_ptr;
        count = c < 0 ? 0 : (c < cap ? c : cap);
    }
    const int groups = Kout / kDownGroupCols;
    const int cg = (int)blockIdx.x % groups, s = (int)blockIdx.x / groups;
    const int blocks = (count + kDownBlock - 1) / kDownBlock;
    const int b_begin = range_bound(blocks, NS, s), b_end = range_bound(blocks, NS, s + 1);
    const int j_begin = b_begin * kDownBlock;

    // the wave index is the same in every lane: kept scalar, so that the loop below and its
    // branches are scalar too and the compiler's count of outstanding loads stays exact
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 15, kg = lane >> 4;
    const int cw = wave & 1, parity = wave >> 1;
    const int col0 = cg * kDownGroupCols + cw * kDownWaveCols;

    // ids of the range, -1 for an id outside [0, N) or a position at or beyond the live count
    for (int e = tid; e < (b_end - b_begin) * kDownBlock; e += kDownThreads) {
        const int j = j_begin + e;
        const int id = j < count ? idx[j] : -1;
        sh_id[e] = (id >= 0 && id < N) ? id : -1;
    }
    __syncthreads();

    f32x4 acc[MT][8];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t][e] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // Activations: the workgroup stages them through LDS a chunk of 8 blocks (256 positions) at
    // a time, whole cache lines, each once; chunk c + 1 is fetched into registers while chunk c is
    // multiplied.  (Read straight into operand layout, 16 rows x 64 bytes per load, they took as
    // many places among the compute unit's outstanding misses as the weights did.)  Thread tid
    // moves the 16-byte pieces tid + 512 i of a chunk: 32 pieces per row.
    const int cap32 = (cap + kDownBlock - 1) / kDownBlock * kDownBlock;
    constexpr int kPieces = 16 * MT * 32 / kDownThreads;            // per thread: 1, 2 or 4
    const uint16_t *hsrc[kPieces];
    int hdst[kPieces];
#pragma unroll
    for (int i = 0; i < kPieces; ++i) {
        const int e = tid + kDownThreads * i;
        int m = e >> 5;
        m = m < M ? m : M - 1;                   // rows m >= M are computed and never stored
        hsrc[i] = H16 + (size_t)m * cap32 + 8 * (e & 31);
        hdst[i] = (e >> 5) * kChunkPitch + 16 * (e & 31);
    }
    u32x4 hp[kPieces];
    // positions of chunk `first_block`, clamped so that every piece lies inside its row
    auto fetch_chunk = [&](int first_block) {
#pragma unroll
        for (int i = 0; i < kPieces; ++i) {
            int pos = first_block * kDownBlock;
            const int piece = 8 * ((tid + kDownThreads * i) & 31);
            pos = pos + piece + 8 <= cap32 ? pos : cap32 - 8 - piece;
            hp[i] = *reinterpret_cast<const u32x4 *>(hsrc[i] + pos);
        }
    };
    auto store_chunk = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kPieces; ++i)
            *reinterpret_cast<u32x4 *>(smem + buf * kChunkBytes + hdst[i]) = hp[i];
    };
    const int lds_a = x * kChunkPitch + 16 * kg;                    // + 16 t rows, + 64 bytes per block of the chunk
    const uint16_t *wcol = W2 + col0 + 8 * x;

    // Ring of two blocks: slot r holds this wave's block b (weights: 8 row pieces; the 8 row pieces
    // of its 32 neurons).  A block index beyond the range is
    // clamped for the loads and skipped for the arithmetic.
    u32x4 wq[2][8];
    const int last = b_end - 1;
#define POLAR_DOWN_FETCH(r, block)                                                                 \
    {                                                                                              \
        const int bb = (block) < last ? (block) : last;                                            \
        const int e0 = (bb - b_begin) * kDownBlock + 8 * kg;      /* this lane's 8 neurons */       \
        const i32x4 id_lo = *reinterpret_cast<const i32x4 *>(sh_id + e0);                          \
        const i32x4 id_hi = *reinterpret_cast<const i32x4 *>(sh_id + e0 + 4);                      \
        __builtin_amdgcn_sched_barrier(0);                                                         \
        _Pragma("unroll") for (int i = 0; i < 8; ++i)                                              \
        {                                                                                          \
            const int id = i < 4 ? id_lo[i & 3] : id_hi[i & 3];                                    \
            wq[r][i] = *reinterpret_cast<const u32x4 *>(wcol + (size_t)(id < 0 ? 0 : id) * Kout);  \
        }                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
#define POLAR_DOWN_MULTIPLY(r, abase)                                                                   \
    {                                                                                              \
        u32x4 ha[MT];                            /* A operands: 8 positions of 16 * MT rows */     \
        _Pragma("unroll") for (int t = 0; t < MT; ++t)                                             \
            ha[t] = *reinterpret_cast<const u32x4 *>((abase) + lds_a + 16 * t * kChunkPitch);      \
        /* B operand of column e of the lane's 8 x 8 block: its 8 neurons packed in pairs */        \
        _Pragma("unroll") for (int e = 0; e < 8; ++e)                                              \
        {                                                                                          \
            u32x4 o;                                                                               \
            _Pragma("unroll") for (int p = 0; p < 4; ++p)                                          \
            {                                                                                      \
                const unsigned int lo = wq[r][2 * p][e >> 1], hi = wq[r][2 * p + 1][e >> 1];       \
                o[p] = (e & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16)); \
            }                                                                                      \
            _Pragma("unroll") for (int t = 0; t < MT; ++t)                                         \
                acc[t][e] = mfma16x16x32<BF>(ha[t], o, acc[t][e]);                                 \
        }                                                                                          \
    }

    // A chunk is 2 * P blocks: each wave's two ring slots.  Every wave runs the same number of
    // chunks (one barrier each); a block beyond the range is skipped for the arithmetic.
    constexpr int P = kDownParities;             // this wave takes every P-th block of the range
    static_assert(kChunkBlocks == 2 * P, "a chunk is one pass of the two-slot ring of every wave");
    const int chunks = (b_end - b_begin + kChunkBlocks - 1) / kChunkBlocks;
    if (chunks > 0) {
        fetch_chunk(b_begin);
        store_chunk(0);
        POLAR_DOWN_FETCH(0, b_begin + parity)
        POLAR_DOWN_FETCH(1, b_begin + parity + P)
        __syncthreads();
    }
    for (int c = 0; c < chunks; ++c) {
        const int b = b_begin + c * kChunkBlocks + parity;
        const unsigned char *abuf = smem + (c & 1) * kChunkBytes;
        if (c + 1 < chunks) fetch_chunk(b_begin + (c + 1) * kChunkBlocks);
        if (b < b_end) POLAR_DOWN_MULTIPLY(0, abuf + 64 * parity)
        POLAR_DOWN_FETCH(0, b + 2 * P)
        if (b + P < b_end) POLAR_DOWN_MULTIPLY(1, abuf + 64 * (parity + P))
        POLAR_DOWN_FETCH(1, b + 3 * P)
        if (c + 1 < chunks) store_chunk((c + 1) & 1);
        __syncthreads();
    }
#undef POLAR_DOWN_MULTIPLY
#undef POLAR_DOWN_FETCH

    // The four waves of a column block add their sums through LDS, (p0 + p2) + (p1 + p3), in two
    // rounds: parities 2 and 3 hand theirs to 0 and 1; then 0 and 1 exchange halves (1 gives its
    // tiles e < 4, 0 its tiles e >= 4), so that each finishes and stores one half of the range's
    // sums.  (Addition commutes, so both halves carry the sum in the order above.)  A region
    // holds one wave's accumulators; there are two per column block.
    constexpr int kRegion = MT * 8 * 64;         // f32x4 entries
    f32x4 *region0 = reinterpret_cast<f32x4 *>(smem) + (size_t)(cw * 2 + 0) * kRegion + lane;
    f32x4 *region1 = reinterpret_cast<f32x4 *>(smem) + (size_t)(cw * 2 + 1) * kRegion + lane;
    __syncthreads();                             // the activation chunks are no longer read
    if (parity >= 2) {
        f32x4 *to = parity == 2 ? region0 : region1;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) to[(t * 8 + e) * 64] = acc[t][e];
    }
    __syncthreads();
    if (parity < 2) {
        const f32x4 *from = parity == 0 ? region0 : region1;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[t][e] += from[(t * 8 + e) * 64];
    }
    __syncthreads();                             // both regions have been read
    if (parity == 1) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) region0[(t * 8 + e) * 64] = acc[t][e];
    } else if (parity == 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 4; e < 8; ++e) region1[(t * 8 + e) * 64] = acc[t][e];
    }
    __syncthreads();
    if (parity < 2) {
        const f32x4 *from = parity == 0 ? region0 : region1;
        const int e0 = parity == 0 ? 0 : 4;      // the half this wave finishes
        f32x4 *dst = reinterpret_cast<f32x4 *>(part) +
                     ((size_t)s * (Kout / kDownWaveCols) + (size_t)cg * 2 + cw) * (MT * 8) * 64 + lane;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // parity 0: (p0 + p2) + (p1 + p3); parity 1: (p1 + p3) + (p0 + p2), the same sum
                const f32x4 other = from[(t * 8 + e0 + e) * 64];
                dst[(t * 8 + e0 + e) * 64] = parity == 0 ? acc[t][e0 + e] + other : other + acc[t][e0 + e];
            }
    }
}

// Batches of 65 to 128 rows: the same streaming scheme with the workgroup cut the other way.  A
// workgroup owns ONE column block of 128; wave (h, p) takes rows 64 h .. 64 h + 63 and the
// 32-neuron blocks p, p + 4, ... of the range, so the two waves of a parity load the same weight
// pieces (the second request finds them in the compute unit's cache or in flight) and the gathered
// rows leave HBM once, not once per 64 rows.  Activations of all 128 rows are staged per chunk
// (two buffers of 66 KB), which leaves no room for the ids of a whole range: the ids travel with
// the chunks instead, two chunks ahead (the weight loads of chunk c + 1 are issued during chunk c).
// grid = (Kout / 128) * NS workgroups; block = 512 threads; part holds, per (range, column block),
// 64 accumulator tiles (row tile 4 h + t, column tile e).
constexpr int kSplitRowTiles = 4;                // 16-row tiles per wave
constexpr int kSplitRows = 2 * 16 * kSplitRowTiles;
constexpr int kChunkIds = kChunkBlocks * kDownBlock;

template <bool BF>
__global__ __launch_bounds__(kDownThreads) void select_gemm_down_split_kernel(
    const uint16_t *__restrict__ H16, const uint16_t *__restrict__ W2, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_ptr, float *__restrict__ part, int M, int Kout, int N, int cap,
    int NS)
{
    constexpr int MT = kSplitRowTiles;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kChunkBytes = kSplitRows * kChunkPitch;
    int *sh_id = reinterpret_cast<int *>(smem + 2 * kChunkBytes);   // two buffers of kChunkIds ids

    int count = cap;
    if (count_ptr) {
        const int c = *count_ptr;
        count = c < 0 ? 0 : (c < cap ? c : cap);
    }
    const int groups = Kout / kDownWaveCols;
    const int cg = (int)blockIdx.x % groups, s = (int)blockIdx.x / groups;
    const int blocks = (count + kDownBlock - 1) / kDownBlock;
    const int b_begin = range_bound(blocks, NS, s), b_end = range_bound(blocks, NS, s + 1);

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int x = lane & 15, kg = lane >> 4;
    const int mh = wave & 1, parity = wave >> 1;
    const int col0 = cg * kDownWaveCols;

    f32x4 acc[MT][8];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[t][e] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // id of position e of chunk c (first block b_begin + 8 c), -1 for an id outside [0, N) or a
    // position at or beyond the live count
    auto chunk_id = [&](int c, int e) -> int {
        const int j = (b_begin + c * kChunkBlocks) * kDownBlock + e;      // at most count + 3 chunks: fits an int
        const int id = j < count ? idx[j] : -1;
        return (id >= 0 && id < N) ? id : -1;
    };
    // Activations: a chunk is 128 rows x 256 positions = 4096 pieces of 16 bytes, 8 per thread,
    // moved in four steps of 2 so that fewer registers are held than in the 64-row kernel.
    // Thread tid moves piece tid % 32 of the rows tid / 32 + 16 j: one base address and a fixed
    // stride.  All 128 rows are read whatever M is (the buffer has room for 128; rows m >= M hold
    // anything, are multiplied and never stored).
    const int cap32 = (cap + kDownBlock - 1) / kDownBlock * kDownBlock;
    constexpr int kHalf = 2;                     // pieces per step
    const int piece = 8 * (tid & 31);
    const uint16_t *hbase = H16 + (size_t)(tid >> 5) * cap32 + piece;
    const size_t hstride = (size_t)16 * cap32;
    unsigned char *sbase = smem + (tid >> 5) * kChunkPitch + 16 * (tid & 31);
    u32x4 hp[kHalf];
    auto fetch_half = [&](int first_block, int half) {
        int pos = first_block * kDownBlock;
        pos = pos + piece + 8 <= cap32 ? pos : cap32 - 8 - piece;       // every piece inside its row
#pragma unroll
        for (int i = 0; i < kHalf; ++i)
            hp[i] = *reinterpret_cast<const u32x4 *>(hbase + (size_t)(half * kHalf + i) * hstride + pos);
    };
    auto store_half = [&](int buf, int half) {
#pragma unroll
        for (int i = 0; i < kHalf; ++i)
            *reinterpret_cast<u32x4 *>(sbase + buf * kChunkBytes + (half * kHalf + i) * 16 * kChunkPitch) = hp[i];
    };
    const int lds_a = (64 * mh + x) * kChunkPitch + 16 * kg;        // + 16 t rows, + 64 bytes per block of the chunk
    const uint16_t *wcol = W2 + col0 + 8 * x;

    // ring of two blocks per wave, as in the 64-row kernel; block `block` lies in chunk `ch`
    u32x4 wq[2][8];
    const int last = b_end - 1;
#define POLAR_SPLIT_FETCH(r, block, ch)                                                            \
    {                                                                                              \
        const int bb = (block) < last ? (block) : last;                                            \
        int e0 = (bb - b_begin - (ch) * kChunkBlocks) * kDownBlock + 8 * kg;                       \
        e0 = e0 < 0 ? 0 : (e0 > kChunkIds - 8 ? kChunkIds - 8 : e0);  /* a clamped block: any ids */ \
        const int *ids = sh_id + ((ch) & 1) * kChunkIds + e0;                                      \
        const i32x4 id_lo = *reinterpret_cast<const i32x4 *>(ids);                                 \
        const i32x4 id_hi = *reinterpret_cast<const i32x4 *>(ids + 4);                             \
        __builtin_amdgcn_sched_barrier(0);                                                         \
        _Pragma("unroll") for (int i = 0; i < 8; ++i)                                              \
        {                                                                                          \
            const int id = i < 4 ? id_lo[i & 3] : id_hi[i & 3];                                    \
            wq[r][i] = *reinterpret_cast<const u32x4 *>(wcol + (size_t)(id < 0 ? 0 : id) * Kout);  \
        }                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
#define POLAR_SPLIT_MULTIPLY(r, abase)                                                             \
    {                                                                                              \
        u32x4 ha[MT];                                                                              \
        _Pragma("unroll") for (int t = 0; t < MT; ++t)                                             \
            ha[t] = *reinterpret_cast<const u32x4 *>((abase) + lds_a + 16 * t * kChunkPitch);      \
        _Pragma("unroll") for (int e = 0; e < 8; ++e)                                              \
        {                                                                                          \
            u32x4 o;                                                                               \
            _Pragma("unroll") for (int p = 0; p < 4; ++p)                                          \
            {                                                                                      \
                const unsigned int lo = wq[r][2 * p][e >> 1], hi = wq[r][2 * p + 1][e >> 1];       \
                o[p] = (e & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16)); \
            }                                                                                      \
            _Pragma("unroll") for (int t = 0; t < MT; ++t)                                         \
                acc[t][e] = mfma16x16x32<BF>(ha[t], o, acc[t][e]);                                 \
        }                                                                                          \
    }

    constexpr int P = kDownParities;
    const int chunks = (b_end - b_begin + kChunkBlocks - 1) / kChunkBlocks;
    if (chunks > 0) {
        // ids of chunks 0 and 1, activations of chunk 0
        if (tid < kChunkIds) {
            sh_id[tid] = chunk_id(0, tid);
            sh_id[kChunkIds + tid] = chunk_id(1, tid);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            fetch_half(b_begin, q);
            store_half(0, q);
        }
        __syncthreads();
        POLAR_SPLIT_FETCH(0, b_begin + parity, 0)
        POLAR_SPLIT_FETCH(1, b_begin + parity + P, 0)
    }
    for (int c = 0; c < chunks; ++c) {
        const int b = b_begin + c * kChunkBlocks + parity;
        const unsigned char *abuf = smem + (c & 1) * kChunkBytes;
        const int next_first = b_begin + (c + 1) * kChunkBlocks;
        const int id_next = tid < kChunkIds ? chunk_id(c + 2, tid) : -1;    // consumed during chunk c + 1
        fetch_half(next_first, 0);
        if (b < b_end) POLAR_SPLIT_MULTIPLY(0, abuf + 64 * parity)
        store_half((c + 1) & 1, 0);
        fetch_half(next_first, 1);
        POLAR_SPLIT_FETCH(0, b + 2 * P, c + 1)
        store_half((c + 1) & 1, 1);
        fetch_half(next_first, 2);
        if (b + P < b_end) POLAR_SPLIT_MULTIPLY(1, abuf + 64 * (parity + P))
        store_half((c + 1) & 1, 2);
        fetch_half(next_first, 3);
        POLAR_SPLIT_FETCH(1, b + 3 * P, c + 1)
        store_half((c + 1) & 1, 3);
        // buffer c & 1 held the ids of chunk c, last read while chunk c - 1 was multiplied
        if (tid < kChunkIds) sh_id[(c & 1) * kChunkIds + tid] = id_next;
        __syncthreads();
    }
#undef POLAR_SPLIT_MULTIPLY
#undef POLAR_SPLIT_FETCH

    // The four waves of a row half add their sums through LDS as in the 64-row kernel:
    // (p0 + p2) + (p1 + p3), two rounds, parities 0 and 1 each storing one half of the tiles.
    constexpr int kRegion = MT * 8 * 64;         // f32x4 entries
    f32x4 *region0 = reinterpret_cast<f32x4 *>(smem) + (size_t)(mh * 2 + 0) * kRegion + lane;
    f32x4 *region1 = reinterpret_cast<f32x4 *>(smem) + (size_t)(mh * 2 + 1) * kRegion + lane;
    __syncthreads();                             // chunks and ids are no longer read
    if (parity >= 2) {
        f32x4 *to = parity == 2 ? region0 : region1;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) to[(t * 8 + e) * 64] = acc[t][e];
    }
    __syncthreads();
    if (parity < 2) {
        const f32x4 *from = parity == 0 ? region0 : region1;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[t][e] += from[(t * 8 + e) * 64];
    }
    __syncthreads();
    if (parity == 1) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) region0[(t * 8 + e) * 64] = acc[t][e];
    } else if (parity == 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 4; e < 8; ++e) region1[(t * 8 + e) * 64] = acc[t][e];
    }
    __syncthreads();
    if (parity < 2) {
        const f32x4 *from = parity == 0 ? region0 : region1;
        const int e0 = parity == 0 ? 0 : 4;
        f32x4 *dst = reinterpret_cast<f32x4 *>(part) +
                     (((size_t)s * groups + cg) * (2 * MT) + (size_t)mh * MT) * 8 * 64 + lane;
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const f32x4 other = from[(t * 8 + e0 + e) * 64];
                dst[(t * 8 + e0 + e) * 64] = parity == 0 ? acc[t][e0 + e] + other : other + acc[t][e0 + e];
            }
    }
}

// grid = (Kout / 128) * MT workgroups of 64 threads: workgroup (column block, row tile t) adds the
// NS sums of its 16 x 128 outputs in ascending range order.  Accumulator layout: lane (x, kg)
// holds rows 16t + 4kg + i (i < 4) of column 8x + e for each of its 8 tiles e, so per row it
// owns 8 consecutive columns: two 16-byte stores.
template <int MT>
__global__ __launch_bounds__(64) void select_gemm_down_reduce_kernel(const float *__restrict__ part,
                                                                    float *__restrict__ Y, int M, int Kout,
                                                                    int NS)
{
    const int cb = (int)blockIdx.x / MT, t = (int)blockIdx.x % MT;
    const int lane = threadIdx.x, x = lane & 15, kg = lane >> 4;
    const size_t per_range = (size_t)(Kout / kDownWaveCols) * (MT * 8) * 64;
    const f32x4 *src = reinterpret_cast<const f32x4 *>(part) + ((size_t)cb * (MT * 8) + t * 8) * 64 + lane;
    f32x4 sum[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) sum[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // four ranges' loads in flight at a time (one range per round trip would make the kernel a chain
    // of NS memory latencies); the additions stay in ascending range order
    for (int s0 = 0; s0 < NS; s0 += 4) {
        f32x4 v[4][8];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                v[q][e] = s0 + q < NS ? src[(size_t)(s0 + q) * per_range + e * 64] : (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (s0 + q < NS) {
#pragma unroll
                for (int e = 0; e < 8; ++e) sum[e] += v[q][e];
            }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = 16 * t + 4 * kg + i;
        if (m >= M) continue;
        f32x4 *dst = reinterpret_cast<f32x4 *>(Y + (size_t)m * Kout + cb * kDownWaveCols + 8 * x);
        dst[0] = (f32x4){sum[0][i], sum[1][i], sum[2][i], sum[3][i]};
        dst[1] = (f32x4){sum[4][i], sum[5][i], sum[6][i], sum[7][i]};
    }
}

int down_mt(int M) { return M <= 16 ? 1 : (M <= 32 ? 2 : 4); }

// contraction ranges: enough to fill the compute units once, and never more ids per range than
// the kernel keeps in LDS
int down_ranges(int Kout, int cap)
{
    const int groups = Kout / kDownGroupCols;
    int ns = kDownTargetGroups / groups;
    if (ns < 1) ns = 1;
    const long blocks = ((long)cap + kDownBlock - 1) / kDownBlock;
    const long max_blocks = kDownMaxIds / kDownBlock - 1;     // a range holds at most blocks / ns + 1 blocks
    if (blocks / ns > max_blocks) ns = (int)((blocks + max_blocks - 1) / max_blocks);
    if (ns > blocks && blocks > 0) ns = (int)blocks;          // no empty ranges beyond the live blocks' count
    return ns < 1 ? 1 : ns;
}

// contraction ranges of the row-split kernel (one column block per workgroup; the ids travel
// with the chunks, so a range may be of any length)
int down_split_ranges(int Kout, int cap)
{
    const int groups = Kout / kDownWaveCols;
    int ns = kDownTargetGroups / groups;
    const long blocks = ((long)cap + kDownBlock - 1) / kDownBlock;
    if (ns > blocks && blocks > 0) ns = (int)blocks;
    return ns < 1 ? 1 : ns;
}

}  // namespace

// partial sums of one pass of `rows` rows
static size_t down_partial_bytes(int rows, int Kout, int cap)
{
    if (rows > kDownMaxRows)
        return (size_t)down_split_ranges(Kout, cap) * (Kout / kDownWaveCols) * (2 * kSplitRowTiles) * 8 * 64 * sizeof(f32x4);
    return (size_t)down_ranges(Kout, cap) * (Kout / kDownWaveCols) * down_mt(rows) * 8 * 64 * sizeof(f32x4);
}

// room for the partial sums of every pass a batch of M rows goes through: passes of 128 rows, a
// remainder of up to 128
size_t select_gemm_down_partial_region(int M, int Kout, int cap)
{
    const size_t small = down_partial_bytes(M < kDownMaxRows ? M : kDownMaxRows, Kout, cap);
    const size_t large = M > kDownMaxRows ? down_partial_bytes(kDownPassRows, Kout, cap) : 0;
    return small > large ? small : large;
}

// the ranges' sums, then the prepared activations of one pass
size_t select_gemm_down_workspace_bytes(int M, int Kout, int cap)
{
    // (the row-split kernel reads 128 rows of them whatever the batch size is)
    const size_t rows = M <= kDownMaxRows ? M : kDownPassRows;
    const size_t cap32 = ((size_t)cap + kDownBlock - 1) / kDownBlock * kDownBlock;
    return select_gemm_down_partial_region(M, Kout, cap) + rows * cap32 * sizeof(uint16_t);
}

template <bool BF>
static hipError_t launch_down_mt(int mt, int NS, hipStream_t st, const float *H, const uint16_t *W2,
                                 const int32_t *idx, const int32_t *count, float *Y, float *part,
                                 uint16_t *H16, int M, int Kout, int N, int cap)
{
    const dim3 grid((unsigned)(Kout / kDownGroupCols * NS)), block(kDownThreads);
    const dim3 rgrid((unsigned)(Kout / kDownWaveCols * mt)), rblock(64);
    // H == nullptr: H16 already holds the prepared activations
    const long items = H ? (long)M * ((cap + kDownBlock - 1) / kDownBlock * kDownBlock / 8) : 0;
    if (items > 0)
        hipLaunchKernelGGL((select_gemm_down_prepare_kernel<BF>), dim3((unsigned)((items + kPrepThreads - 1) / kPrepThreads)),
                           dim3(kPrepThreads), 0, st, H, idx, count, H16, M, N, cap);
    // dynamic LDS: two activation chunks and the ids of a range; above 64 KB it has to be granted
    size_t lds = (size_t)2 * 16 * mt * kChunkPitch + (size_t)kDownMaxIds * sizeof(int);
    const size_t regions = (size_t)4 * mt * 8 * 64 * sizeof(f32x4);      // the epilogue's exchange buffers
    if (lds < regions) lds = regions;
    static LdsGrant granted[3];                  // one set per instantiation of this launcher
    const void *kernels[3] = {reinterpret_cast<const void *>(select_gemm_down_kernel<BF, 1>),
                              reinterpret_cast<const void *>(select_gemm_down_kernel<BF, 2>),
                              reinterpret_cast<const void *>(select_gemm_down_kernel<BF, 4>)};
    const int ki = mt == 1 ? 0 : (mt == 2 ? 1 : 2);
    if (const hipError_t e = ensure_dynamic_lds(kernels[ki], lds, granted[ki]); e != hipSuccess) return e;
    switch (mt) {
    case 1:
        hipLaunchKernelGGL((select_gemm_down_kernel<BF, 1>), grid, block, lds, st, H16, W2, idx, count, part, M, Kout, N, cap, NS);
        hipLaunchKernelGGL((select_gemm_down_reduce_kernel<1>), rgrid, rblock, 0, st, part, Y, M, Kout, NS);
        break;
    case 2:
        hipLaunchKernelGGL((select_gemm_down_kernel<BF, 2>), grid, block, lds, st, H16, W2, idx, count, part, M, Kout, N, cap, NS);
        hipLaunchKernelGGL((select_gemm_down_reduce_kernel<2>), rgrid, rblock, 0, st, part, Y, M, Kout, NS);
        break;
    default:
        hipLaunchKernelGGL((select_gemm_down_kernel<BF, 4>), grid, block, lds, st, H16, W2, idx, count, part, M, Kout, N, cap, NS);
        hipLaunchKernelGGL((select_gemm_down_reduce_kernel<4>), rgrid, rblock, 0, st, part, Y, M, Kout, NS);
        break;
    }
    return hipGetLastError();
}

template <bool BF>
static hipError_t launch_down_split(int NS, hipStream_t st, const float *H, const uint16_t *W2, const int32_t *idx,
                                    const int32_t *count, float *Y, float *part, uint16_t *H16, int M, int Kout,
                                    int N, int cap)
{
    const dim3 grid((unsigned)(Kout / kDownWaveCols * NS)), block(kDownThreads);
    const dim3 rgrid((unsigned)(Kout / kDownWaveCols * 2 * kSplitRowTiles)), rblock(64);
    const long items = H ? (long)M * ((cap + kDownBlock - 1) / kDownBlock * kDownBlock / 8) : 0;
    if (items > 0)
        hipLaunchKernelGGL((select_gemm_down_prepare_kernel<BF>), dim3((unsigned)((items + kPrepThreads - 1) / kPrepThreads)),
                           dim3(kPrepThreads), 0, st, H, idx, count, H16, M, N, cap);
    // dynamic LDS: two activation chunks of 128 rows and two chunks' ids (the epilogue's four
    // exchange buffers fit inside)
    const size_t lds = (size_t)2 * kSplitRows * kChunkPitch + (size_t)2 * kChunkIds * sizeof(int);
    static_assert((size_t)2 * kSplitRows * kChunkPitch >= (size_t)4 * kSplitRowTiles * 8 * 64 * sizeof(f32x4), "exchange buffers");
    static LdsGrant granted;
    const void *kernel = reinterpret_cast<const void *>(select_gemm_down_split_kernel<BF>);
    if (const hipError_t e = ensure_dynamic_lds(kernel, lds, granted); e != hipSuccess) return e;
    hipLaunchKernelGGL((select_gemm_down_split_kernel<BF>), grid, block, lds, st, H16, W2, idx, count, part, M, Kout, N, cap, NS);
    hipLaunchKernelGGL((select_gemm_down_reduce_kernel<2 * kSplitRowTiles>), rgrid, rblock, 0, st, part, Y, M, Kout, NS);
    return hipGetLastError();
}

// one pass of at most 128 rows; H == nullptr: H16 is already prepared
static hipError_t down_pass(const float *H, const uint16_t *W16, const int32_t *idx, const int32_t *count,
                            float *Y, int rows, int Kout, int N, int cap, polar_dtype dt, float *part,
                            uint16_t *H16, hipStream_t stream)
{
    if (rows > kDownMaxRows) {
        const int NS = down_split_ranges(Kout, cap);
        return dt == POLAR_BF16 ? launch_down_split<true>(NS, stream, H, W16, idx, count, Y, part, H16, rows, Kout, N, cap)
                                : launch_down_split<false>(NS, stream, H, W16, idx, count, Y, part, H16, rows, Kout, N, cap);
    }
    const int mt = down_mt(rows), NS = down_ranges(Kout, cap);
    return dt == POLAR_BF16
               ? launch_down_mt<true>(mt, NS, stream, H, W16, idx, count, Y, part, H16, rows, Kout, N, cap)
               : launch_down_mt<false>(mt, NS, stream, H, W16, idx, count, Y, part, H16, rows, Kout, N, cap);
}

hipError_t launch_select_gemm_down(const float *H, const void *W2, const int32_t *idx, const int32_t *count,
                                   float *Y, int M, int Kout, int N, int cap, polar_dtype dt, void *workspace,
                                   hipStream_t stream)
{
    const uint16_t *W16 = static_cast<const uint16_t *>(W2);
    // batches beyond 128 rows are processed 128 rows at a time (the gathered rows are re-read; the
    // passes share the workspace, which the stream's order makes safe)
    float *part = static_cast<float *>(workspace);
    uint16_t *H16 = reinterpret_cast<uint16_t *>(static_cast<unsigned char *>(workspace) +
                                                 select_gemm_down_partial_region(M, Kout, cap));
    for (int m0 = 0; m0 < M; m0 += kDownPassRows) {
        const int rows = M - m0 < kDownPassRows ? M - m0 : kDownPassRows;
        const hipError_t e = down_pass(H + (size_t)m0 * cap, W16, idx, count, Y + (size_t)m0 * Kout, rows, Kout,
                                       N, cap, dt, part, H16, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Workspace of the two-factor call, four regions that do not overlap: the first factor's partial
// sums, the second factor's partial sums, the 16-bit hidden activations of one pass of the first
// factor, and room for the hidden activations of one pass as floats, used only where the first
// factor's evenly split form cannot run.  Each region starts on a multiple of 256 bytes.
static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }
struct MlpRegions {
    int up_rows;                                 // rows of the batch one pass of the first factor takes
    size_t gemm_bytes, down_offset, h16_offset, hidden_offset, total;
};
static MlpRegions mlp_regions(int M, int D, int cap)
{
    const int down_rows = M < kDownPassRows ? M : kDownPassRows;
    const size_t cap32 = ((size_t)cap + kDownBlock - 1) / kDownBlock * kDownBlock;
    MlpRegions r;
    r.up_rows = M < select_gemm_ws_max_rows() ? M : select_gemm_ws_max_rows();
    r.gemm_bytes = select_gemm_workspace_bytes(r.up_rows);
    r.down_offset = align256(r.gemm_bytes);
    r.h16_offset = r.down_offset + align256(select_gemm_down_partial_region(M, D, cap));
    r.hidden_offset = r.h16_offset + align256((size_t)(M <= kDownMaxRows ? M : kDownPassRows) * cap32 * sizeof(uint16_t));
    r.total = r.hidden_offset + align256((size_t)down_rows * cap * sizeof(float));
    return r;
}

size_t sparse_mlp_workspace_bytes(int M, int D, int cap) { return mlp_regions(M, D, cap).total; }

hipError_t launch_sparse_mlp(const void *X, const void *W1, const void *W2, const int32_t *idx,
                             const int32_t *count, float *Y, int M, int D, int N, int cap, polar_dtype dt,
                             int relu, void *workspace, hipStream_t stream)
{
    const MlpRegions r = mlp_regions(M, D, cap);
    unsigned char *base = static_cast<unsigned char *>(workspace);
    float *part = reinterpret_cast<float *>(base + r.down_offset);
    uint16_t *H16 = reinterpret_cast<uint16_t *>(base + r.h16_offset);
    float *hidden = reinterpret_cast<float *>(base + r.hidden_offset);
    const size_t cap32 = ((size_t)cap + kDownBlock - 1) / kDownBlock * kDownBlock;
    const uint16_t *X16 = static_cast<const uint16_t *>(X);
    const uint16_t *W216 = static_cast<const uint16_t *>(W2);
    // Both factors take up to 128 rows of the batch at a time (larger batches
    // re-read the gathered rows).
    for (int m0 = 0; m0 < M; m0 += r.up_rows) {
        const int rows = M - m0 < r.up_rows ? M - m0 : r.up_rows;
        // its reduction writes what the second factor's kernel reads
        const bool fused = cap > 0 && select_gemm_h16_applicable(rows, D, cap, r.gemm_bytes);
        if (fused) {
            const hipError_t e = launch_select_gemm_h16(X16 + (size_t)m0 * D, W1, idx, count, H16, rows, D, N, cap,
                                                        dt, relu, base, r.gemm_bytes, stream);
            if (e != hipSuccess) return e;
        }
        for (int r0 = 0; r0 < rows; r0 += kDownPassRows) {
            const int drows = rows - r0 < kDownPassRows ? rows - r0 : kDownPassRows;
            float *Yp = Y + (size_t)(m0 + r0) * D;
            hipError_t e = hipSuccess;
            if (fused) {
                e = down_pass(nullptr, W216, idx, count, Yp, drows, D, N, cap, dt, part, H16 + (size_t)r0 * cap32, stream);
            } else {
                if (cap > 0) {
                    e = launch_select_gemm(X16 + (size_t)(m0 + r0) * D, W1, idx, count, hidden, drows, D, N, cap, dt,
                                           relu, stream);
                    if (e != hipSuccess) return e;
                }
                e = down_pass(hidden, W216, idx, count, Yp, drows, D, N, cap, dt, part, H16, stream);
            }
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace polar
