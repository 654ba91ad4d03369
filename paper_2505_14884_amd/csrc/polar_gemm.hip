// Selective (fused-gather) GEMM and the batch neuron index for gfx950 (Section 3.1: the
// sparsified MLP sigma(x W_{1,S_B}) over the union S_B of the requests' active neurons;
// Section 4.1: the neuron index tensor and the kernel that fuses indexing with the matrix
// product; Appendix "Sparse Kernels", Algorithm 3: gather the indexed rows, multiply, apply
// the activation, store).
//
//   C[m, j] = act( sum_k A[m, k] * W[idx[j], k] )       A [M,K], W [N,K] (one row per neuron)
//
// At decode batch sizes this is bound by HBM, not by the matrix cores: every gathered weight
// row (K 16-bit values) is read once and used for only M <= 256 multiply-adds per element,
// far below the ~300 flop/byte ridge of the part, but above what the vector ALUs sustain at
// HBM speed, so the contraction runs on MFMA (v_mfma_f32_16x16x32) while the kernel is
// organised around streaming the gathered rows.  Two forms: the one-launch kernel described
// here, and, further down, an evenly split form that needs a workspace and is faster:
//   * a workgroup owns 32 selected neurons and walks K in blocks of 128 values; per block it
//     loads its 32 x 256-byte row pieces with fully coalesced 16-byte loads (16 lanes per
//     piece), parks them in LDS (padded rows, conflict-free 16-byte reads) and every wave
//     reads them back as B operands.  A register ring keeps the next 8 blocks' loads in
//     flight while the current one is multiplied (registers -> LDS double buffer, one
//     barrier per block).
//   * the activations are small (M x K), shared by all workgroups and served by L2: each wave
//     fetches its 16 rows x 256 bytes per block with the same row-piece loads and turns them
//     into operand layout through a wave-private LDS tile (no barrier: one wave writes and
//     reads it).  Within a block, MFMA step s contracts the k values {32*kg + 8*s + j}; A and
//     B use the same assignment, which is all the contraction needs.
//   * wave w owns rows [16*MT*w, 16*MT*(w+1)) of the output tile (MT = 1, 2 or 4 for M up to
//     64, 128, 256) and both 16-column halves of the 32 neurons: 2*MT accumulators.
// The gather costs nothing extra: a row index only changes the base address of a contiguous
// 2K-byte stream, which is why the weights are stored one contiguous row per neuron.
#include <cstdlib>

#include "polar_internal.h"

namespace polar {
namespace {

constexpr int kGemmThreads = 256;
constexpr int kTileN = 32;                       // selected neurons per workgroup
constexpr int kBlockK = 128;                     // K values per step (256 bytes of a row)
constexpr int kRowBytes = kBlockK * 2 + 16;      // padded LDS row: 16-lane reads hit 64 banks
#ifndef POLAR_GEMM_RING
#define POLAR_GEMM_RING 8
#endif
constexpr int kRingW = POLAR_GEMM_RING;          // K blocks of weights in flight per workgroup (even)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// 16 bytes as a native vector (not HIP's uint4 struct: arrays of the struct are copied with
// memcpy, which keeps the register rings below from being promoted out of scratch memory)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <bool BF> __device__ __forceinline__ f32x4 mfma16x16x32(const u32x4 &a, const u32x4 &b, f32x4 c)
{
    if (BF)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// bit pattern of v rounded to the 16-bit storage type (nearest, ties to even)
__device__ __forceinline__ uint16_t to_storage(float v, bool bf)
{
    return bf ? __builtin_bit_cast(uint16_t, (__bf16)v) : __builtin_bit_cast(uint16_t, (_Float16)v);
}

// grid = ceil(cap / kTileN) workgroups; block = 256 threads (4 waves).
// Rows m >= M of the tile are computed on clamped addresses and never stored; columns at or
// beyond the live count are never stored; an id outside [0, N) yields a zero column.
template <bool BF, int MT>
__global__ __launch_bounds__(kGemmThreads) void select_gemm_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_ptr, float *__restrict__ C, int M, int K, int N, int cap,
    int relu)
{
    __shared__ __align__(16) unsigned char sh_w[2][kTileN * kRowBytes];
    __shared__ __align__(16) unsigned char sh_a[kGemmThreads / 64][16 * kRowBytes];   // per wave
    __shared__ int sh_row[kTileN];               // weight row to stream, -1 for an invalid id

    int count = cap;
    if (count_ptr) {
        const int c = *count_ptr;
        count = c < 0 ? 0 : (c < cap ? c : cap);
    }
    const int n0 = blockIdx.x * kTileN;
    if (n0 >= count) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < kTileN) {
        const int id = n0 + tid < count ? idx[n0 + tid] : -1;
        sh_row[tid] = (id >= 0 && id < N) ? id : -1;
    }
    __syncthreads();

    // global -> LDS assignment: 16 lanes per 256-byte row piece, two pieces per thread
    const int g_chunk = tid & 15, g_row = tid >> 4;                 // rows g_row and g_row + 16
    const int r0 = sh_row[g_row], r1 = sh_row[g_row + 16];
    const u32x4 *w0 = reinterpret_cast<const u32x4 *>(W + (size_t)(r0 < 0 ? 0 : r0) * K) + g_chunk;
    const u32x4 *w1 = reinterpret_cast<const u32x4 *>(W + (size_t)(r1 < 0 ? 0 : r1) * K) + g_chunk;
    const int lds_w0 = g_row * kRowBytes + g_chunk * 16, lds_w1 = lds_w0 + 16 * kRowBytes;

    // operand layout: lane (x = lane % 16, kg = lane / 16)
    const int x = lane & 15, kg = lane >> 4;
    // Activations are fetched like cache rows (16 lanes per 256-byte row piece, 4 rows per
    // wave-wide load: full cache lines per request) and turned into operand layout through a
    // wave-private LDS tile; fetching them directly in operand layout (16 bytes from each of
    // 16 rows per quarter-wave) made the L2 -> CU path the bottleneck at M >= 64.
    const u32x4 *a_src[MT][4];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int row = (wave * MT + t) * 16 + 4 * u + kg;
            row = row < M ? row : M - 1;
            a_src[t][u] = reinterpret_cast<const u32x4 *>(A + (size_t)row * K) + x;   // chunk x of the block
        }
    unsigned char *a_tile = sh_a[wave];
    const int lds_a_wr = kg * kRowBytes + x * 16;                   // + 4*u rows
    const int lds_a_rd = x * kRowBytes + kg * 64;                   // + 16*s
    const int lds_b = x * kRowBytes + kg * 64;                      // + 16*s, + 16*kRowBytes for half 1

    f32x4 acc[MT][2];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t][0] = acc[t][1] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // Register rings keep several K blocks in flight: kRingW blocks of this workgroup's weight
    // rows (8 KiB each: what hides HBM latency when only one or two workgroups fit a compute
    // unit's share of the grid) and RA blocks of activations (L2 latency).  The main loop is
    // unrolled by the ring length so every ring slot is a fixed register, and its body has no
    // branches: a slot is refilled kRingW blocks ahead with the block index clamped to the last
    // block (the few repeated requests near the end hit in cache), which lets the compiler
    // count outstanding loads instead of draining them at every join.
    constexpr int RA = MT == 1 ? 4 : 2;
    static_assert(kRingW % RA == 0 && kRingW % 2 == 0, "ring lengths");
    const int nblk = K / kBlockK, last = nblk - 1;

    // K blocks that do not fill a whole ring are done first, one at a time (plain loads, no
    // ring); model widths are multiples of 1024, so this loop normally runs zero times.
    const int head = nblk % kRingW;
    for (int kb = 0; kb < head; ++kb) {
        unsigned char *buf = sh_w[0];
        const u32x4 h0 = w0[(size_t)kb * 16], h1 = w1[(size_t)kb * 16];
        u32x4 ah[MT][4];
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int u = 0; u < 4; ++u) ah[t][u] = a_src[t][u][(size_t)kb * 16];
        __syncthreads();                                   // previous block's readers are done
        *reinterpret_cast<u32x4 *>(buf + lds_w0) = h0;
        *reinterpret_cast<u32x4 *>(buf + lds_w1) = h1;
        __syncthreads();
#pragma unroll
        for (int t = 0; t < MT; ++t) {
#pragma unroll
            for (int u = 0; u < 4; ++u)
                *reinterpret_cast<u32x4 *>(a_tile + lds_a_wr + 4 * u * kRowBytes) = ah[t][u];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const u32x4 a = *reinterpret_cast<const u32x4 *>(a_tile + lds_a_rd + 16 * s);
                const u32x4 b0 = *reinterpret_cast<const u32x4 *>(buf + lds_b + 16 * s);
                const u32x4 b1 = *reinterpret_cast<const u32x4 *>(buf + lds_b + 16 * kRowBytes + 16 * s);
                acc[t][0] = mfma16x16x32<BF>(a, b0, acc[t][0]);
                acc[t][1] = mfma16x16x32<BF>(a, b1, acc[t][1]);
            }
        }
    }
    if (head) __syncthreads();

    if (head < nblk) {
    u32x4 wq[kRingW][2];
    u32x4 aq[RA][MT][4];
    // Prologue: fill the rings in the order in which the steady-state loop leaves its loads
    // pending at the top of an iteration (weight slots 0..R-RA, then activation slot i after
    // weight slot R-RA+i), so that the compiler's count of outstanding loads at the loop
    // header is the same on entry and on the back edge and nothing is drained there.
#pragma unroll
    for (int j = 0; j < kRingW; ++j) {
        const size_t blk = (size_t)min(head + j, last) * 16;
        wq[j][0] = w0[blk];
        wq[j][1] = w1[blk];
        if (j >= kRingW - RA) {
            const int ja = j - (kRingW - RA);
            const size_t ablk = (size_t)min(head + ja, last) * 16;
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int u = 0; u < 4; ++u) aq[ja][t][u] = a_src[t][u][ablk];
        }
    }

    // one K block: ring slot j (a compile-time constant after unrolling) holds block kb
#define POLAR_GEMM_STEP(j, kb)                                                                     \
    {                                                                                              \
        unsigned char *buf = sh_w[(j) & 1]; /* ring starts are even, so kb & 1 == j & 1 */          \
        *reinterpret_cast<u32x4 *>(buf + lds_w0) = wq[j][0];                                       \
        *reinterpret_cast<u32x4 *>(buf + lds_w1) = wq[j][1];                                       \
        __syncthreads();                                                                           \
        const size_t nw = (size_t)min((kb) + kRingW, last) * 16;                                   \
        wq[j][0] = w0[nw];                                                                         \
        wq[j][1] = w1[nw];                                                                         \
        _Pragma("unroll") for (int t = 0; t < MT; ++t)                                             \
        {                                                                                          \
            _Pragma("unroll") for (int u = 0; u < 4; ++u)                                          \
                *reinterpret_cast<u32x4 *>(a_tile + lds_a_wr + 4 * u * kRowBytes) =                \
                    aq[(j) % RA][t][u];                                                            \
            _Pragma("unroll") for (int s = 0; s < 4; ++s)                                          \
            {                                                                                      \
                const u32x4 a = *reinterpret_cast<const u32x4 *>(a_tile + lds_a_rd + 16 * s);      \
                const u32x4 b0 = *reinterpret_cast<const u32x4 *>(buf + lds_b + 16 * s);           \
                const u32x4 b1 =                                                                   \
                    *reinterpret_cast<const u32x4 *>(buf + lds_b + 16 * kRowBytes + 16 * s);       \
                acc[t][0] = mfma16x16x32<BF>(a, b0, acc[t][0]);                                    \
                acc[t][1] = mfma16x16x32<BF>(a, b1, acc[t][1]);                                    \
            }                                                                                      \
        }                                                                                          \
        const size_t na = (size_t)min((kb) + RA, last) * 16;                                       \
        _Pragma("unroll") for (int t = 0; t < MT; ++t)                                             \
            _Pragma("unroll") for (int u = 0; u < 4; ++u) aq[(j) % RA][t][u] = a_src[t][u][na];    \
    }

    static_assert(kRingW == 8, "the ring loop below is written out for 8 slots");
    for (int kb0 = head; kb0 < nblk; kb0 += kRingW) {      // nblk - head is a multiple of the ring
        POLAR_GEMM_STEP(0, kb0 + 0)
        POLAR_GEMM_STEP(1, kb0 + 1)
        POLAR_GEMM_STEP(2, kb0 + 2)
        POLAR_GEMM_STEP(3, kb0 + 3)
        POLAR_GEMM_STEP(4, kb0 + 4)
        POLAR_GEMM_STEP(5, kb0 + 5)
        POLAR_GEMM_STEP(6, kb0 + 6)
        POLAR_GEMM_STEP(7, kb0 + 7)
    }
#undef POLAR_GEMM_STEP
    }

    // accumulator layout: lane holds rows 4*kg + i (i = 0..3) of column x
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int col = n0 + 16 * h + x;
            if (col >= count) continue;
            const bool valid = sh_row[16 * h + x] >= 0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = (wave * MT + t) * 16 + kg * 4 + i;
                if (row < M) {
                    float v = acc[t][h][i];
                    if (relu) v = v > 0.0f ? v : 0.0f;
                    C[(size_t)row * cap + col] = valid ? v : 0.0f;
                }
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Evenly split form with a caller-supplied workspace (up to 128 rows of the batch per pass).
//
// In the kernel above the number of workgroups follows the live count, which the host does not
// know (it stays on the device): at a 29 % union 332 workgroups land on 256 compute units, one
// or two each, and the machine waits for the doubly loaded ones; and with every wave owning
// other rows of the batch, each weight byte drags M/32 activation bytes through L2 and LDS.
// Here the work is cut the other way round.  A workgroup's tile is 128 neurons; wave w of its
// eight loads 16 of them and multiplies them with all M rows (from 33 rows up, two waves share
// their 32 neurons and take half the rows each: see the kernel), and the activation block
// is staged once per workgroup and shared (M/128 activation bytes per weight byte: the
// activations come from L2, and every line of them in flight takes a place among the compute
// unit's outstanding misses that a weight line from HBM could have).  The launch has a fixed
// number G of workgroups, one per compute unit; each reads the live count, lays all
// (tile, K unit) pairs out in one line, tile-major, and takes the g-th of G equal spans of that
// line, so every compute unit streams the same number of bytes whatever the count is.  A span
// covers the end of one tile and the start of the next (or, for short K, whole tiles in
// between): a segment that covers all of a tile's K is finished in place (activation, store to
// C); any other is stored as raw accumulators in one of the workgroup's two workspace slots
// (slot 0: the span's first tile, slot 1: its last), and a second kernel adds each tile's
// segments in ascending workgroup order, applies the activation and stores.  The order of the
// additions depends only on (count, K, G), so results are reproducible.
constexpr int kStreamWaves = 8;                  // waves per workgroup
constexpr int kStreamGrid = 256;                 // workgroups per launch: one per compute unit
constexpr int kStreamThreads = 64 * kStreamWaves;
constexpr int kStreamWaveN = 16;                 // neurons a wave loads per tile
constexpr int NH = kStreamWaveN / 16;            // 16-neuron halves per wave
constexpr int NR = kStreamWaveN / 4;             // row loads per wave and block (4 rows each)
constexpr int kStreamTileN = kStreamWaveN * kStreamWaves;  // neurons per workgroup tile

// units * G < 2^31 (checked by the host), so 32-bit arithmetic is exact
__device__ __forceinline__ int span_bound(int units, int G, int g) { return (int)((unsigned)units * (unsigned)g / (unsigned)G); }

// A unit is a pair of K blocks (K a multiple of 256), so every segment is a whole number of
// passes of the two-slot ring below.  The span is walked as one stream: the loads for the next
// unit are issued while the current one is multiplied, also when that unit belongs to the next
// tile (its row addresses are fetched a tile ahead), so the memory pipeline is filled once per
// workgroup, not once per tile.
constexpr int kUnitBlocks = 2;                   // K blocks per unit = ring slots
// Timing-only build switches for the streaming kernel below (results are wrong with any of them set; no
// access leaves its bounds and no wait is left without its signal): bit 0 no matrix instructions (the
// operands are still read), bit 1 no operand reads from LDS either, bit 2 no workgroup barrier per block,
// bit 3 no activation loads and stores, bit 4 no weight loads, bit 5 one value per thread stored in place of a
// segment.  They exist to measure where the kernel's
// time goes at a given batch size; the product is built without them.
#ifndef POLAR_STREAM_ABLATE
#define POLAR_STREAM_ABLATE 0
#endif
constexpr int kStreamAblate = POLAR_STREAM_ABLATE;
constexpr int kSpanTiles = 8;                    // tiles a span may touch (row ids kept in LDS)

template <bool BF, int MT>
__global__ __launch_bounds__(kStreamThreads) void select_gemm_stream_kernel(
    const uint16_t *__restrict__ A, const uint16_t *__restrict__ W, const int32_t *__restrict__ idx,
    const int32_t *__restrict__ count_ptr, float *__restrict__ C, uint16_t *__restrict__ H16,
    float *__restrict__ part, int M, int K, int N, int cap, int relu)
{
    // From 33 rows up (MT = 4, 8) the waves pair up.  Wave 2g + r takes the row half r (TW row
    // tiles) and the neurons of BOTH waves of pair g (HW = 2 groups of 16): each wave reads half
    // the activation rows for twice the neurons, which takes a sixth (MT = 4) to a quarter
    // (MT = 8) off the workgroup's LDS traffic: 51.5 -> 48 us at 64 rows, 80 -> 73 us at 128; at
    // 32 rows it changes nothing.  A wave still loads and parks its own 16 weight rows; the
    // pair's tile is then read by both, so it is double-buffered like the activations and
    // ordered by the same barrier.
    constexpr bool kSplit = MT >= 4;
    constexpr int TW = kSplit ? MT / 2 : MT;     // 16-row tiles per wave
    constexpr int HW = kSplit ? 2 * NH : NH;     // 16-neuron groups per wave
    constexpr int kTileBytes = kStreamTileN * kRowBytes;
    __shared__ __align__(16) unsigned char sh_wt[(kSplit ? 2 : 1) * kTileBytes];
    __shared__ __align__(16) unsigned char sh_at[2][16 * MT * kRowBytes];
    __shared__ int sh_id[kSpanTiles * kStreamTileN];

    int count = cap;
    if (count_ptr) {
        const int c = *count_ptr;
        count = c < 0 ? 0 : (c < cap ? c : cap);
    }
    const int upt = K / (kBlockK * kUnitBlocks);                    // units per tile
    const int units = (count + kStreamTileN - 1) / kStreamTileN * upt;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int x = lane & 15, kg = lane >> 4;

    // Workgroup g takes span g.  (Sorting the spans by the K position they start at, so that the
    // workgroups of one die walk K side by side, was built and measured: the activations of up to
    // 128 rows fit every die's L2 whole, and the sort's own barriers cost more than it gained.)
    const int G = (int)gridDim.x;
    const int span = (int)blockIdx.x;
    int u = span_bound(units, G, span);
    const int u0 = u, u1 = span_bound(units, G, span + 1);
    if (u0 >= u1) return;
    const int first_tile = u0 / upt;

    // activation block: 16 lanes per 256-byte row piece, rows a_row + kARows*i
    // (staged by the first kAThreads threads: all of them unless the block has only 16 rows)
    constexpr int kAThreads = 16 * MT * 16 < kStreamThreads ? 16 * MT * 16 : kStreamThreads;
    constexpr int kARows = kAThreads / 16, AP = 16 * MT / kARows;
    const bool stages_a = !(kStreamAblate & 8) && (kAThreads == kStreamThreads || wave < kAThreads / 64);
    const int a_row = tid >> 4;
    const u32x4 *ap[AP];
#pragma unroll
    for (int i = 0; i < AP; ++i) {
        int row = a_row + kARows * i;
        row = row < M ? row : M - 1;
        ap[i] = reinterpret_cast<const u32x4 *>(A + (size_t)row * K) + x;
    }
    unsigned char *wt = sh_wt + wave * kStreamWaveN * kRowBytes;                       // where this wave parks its rows
    const int ncol0 = kSplit ? (wave >> 1) * 2 * kStreamWaveN : wave * kStreamWaveN;   // first neuron it multiplies
    const int row_tile0 = kSplit ? (wave & 1) * TW : 0;                                // first row tile it multiplies
    const unsigned char *wop = sh_wt + ncol0 * kRowBytes;                              // its B operands' rows
    const int lds_w_wr = kg * kRowBytes + x * 16;                   // + 4*i rows
    const int lds_a_wr = a_row * kRowBytes + x * 16;                // + kARows*i rows
    const int lds_op = x * kRowBytes + kg * 64;                     // operand reads: + 16*s, + 16 rows per tile

    // Row ids of every tile the span can touch (the host keeps that below kSpanTiles), fetched
    // once: after this, the ring's loads are the only global loads in the loop, so waiting for
    // the oldest of them never has to wait for anything else.  An id outside [0, N) or beyond
    // the live count is kept as -1: it streams row 0 and its column is zeroed when stored.
    for (int e = tid; e < kSpanTiles * kStreamTileN; e += kStreamThreads) {
        const long col = (long)first_tile * kStreamTileN + e;
        const int id = col < count ? idx[col] : -1;
        sh_id[e] = (id >= 0 && id < N) ? id : -1;
    }
    __syncthreads();
    // this wave's kStreamWaveN weight rows of a tile: 16 lanes per 256-byte row piece, rows kg + 4*i
    const int my_first = wave * kStreamWaveN + kg;
    auto row_id = [&](int tile_in_span, int i) -> int {
        const int id = sh_id[(tile_in_span % kSpanTiles) * kStreamTileN + my_first + 4 * i];
        return id < 0 ? 0 : id;
    };
    // rows of the tile being multiplied and of the tile after it (ids: the address is formed at
    // the load, from W, so that every load is known to be a global one)
    int cur[NR], nxt[NR];
    int tile = first_tile;
    int tile_base = tile * upt, tile_end = tile_base + upt;         // its units
#pragma unroll
    for (int i = 0; i < NR; ++i) {
        cur[i] = row_id(0, i);
        nxt[i] = row_id(1, i);
    }

    // Loads of block j of unit v (past the span's end: one piece that every workgroup shares, so
    // that the loop needs no branch and the memory system no traffic).  The weights come from HBM
    // and are fetched two blocks ahead, into ring slot j; the activations come from L2, need
    // less lead and are fetched one block ahead, into a single slot: every line in flight takes
    // one of the compute unit's outstanding misses, and the fewer of them the activations hold,
    // the more are left for the weights (41.7 -> 39.2 us at 128 rows in a stand-alone model of
    // this pipeline).  The loads are fenced so that the compiler keeps their order
    // (activations of the next block before weights of the block after it): the wave's loads
    // complete in order, so what a step waits for is always the oldest of what is in flight,
    // and the count of outstanding loads at the loop header is the same on entry and on the
    // back edge, so nothing is drained there.
    u32x4 wq[kUnitBlocks][NR], aq[AP];
    if (kStreamAblate & 16)
        for (int j = 0; j < kUnitBlocks; ++j)
            for (int i = 0; i < NR; ++i) wq[j][i] = (u32x4){0u, 0u, 0u, 0u};
#define POLAR_STREAM_BLOCK_OFFSET(j, unit)                                                         \
    const int v = (unit);                                                                          \
    const bool past = v >= u1, ahead = v >= tile_end;                                              \
    const size_t blk = past ? 0 : (size_t)((v - (ahead ? tile_end : tile_base)) * kUnitBlocks + (j)) * 16;
#define POLAR_STREAM_FETCH_W(j, unit)                                                              \
    {                                                                                              \
        POLAR_STREAM_BLOCK_OFFSET(j, unit)                                                         \
        __builtin_amdgcn_sched_barrier(0);                                                         \
        _Pragma("unroll") for (int i = 0; i < NR; ++i)                                             \
        {                                                                                          \
            const u32x4 *p = reinterpret_cast<const u32x4 *>(W + (size_t)(past ? 0 : (ahead ? nxt[i] : cur[i])) * K) + x; \
            if (!(kStreamAblate & 16))                                                             \
                wq[j][i] = __builtin_nontemporal_load(p + blk); /* read once: leave the caches to */ \
                                                              /* the activations and the partials */ \
        }                                                                                          \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
#define POLAR_STREAM_FETCH_A(j, unit)                                                              \
    {                                                                                              \
        POLAR_STREAM_BLOCK_OFFSET(j, unit)                                                         \
        (void)ahead;                                                                               \
        __builtin_amdgcn_sched_barrier(0);                                                         \
        if (stages_a) _Pragma("unroll") for (int i = 0; i < AP; ++i) aq[i] = ap[i][blk];          \
        __builtin_amdgcn_sched_barrier(0);                                                         \
    }
    // block j of unit u: the weights in ring slot j and the activations go to LDS, the loads of
    // the blocks ahead are issued, and the block is multiplied; the wave's B operands (NH groups
    // of 16 neurons, four k steps) stay in registers while the M rows go by, 16 at a time
#define POLAR_STREAM_STEP(j)                                                                       \
    {                                                                                              \
        unsigned char *abuf = sh_at[j];                                                            \
        _Pragma("unroll") for (int i = 0; i < NR; ++i)                                             \
            *reinterpret_cast<u32x4 *>(wt + (kSplit ? (j) * kTileBytes : 0) + lds_w_wr + 4 * i * kRowBytes) = wq[j][i]; \
        if (stages_a) _Pragma("unroll") for (int i = 0; i < AP; ++i)                               \
            *reinterpret_cast<u32x4 *>(abuf + lds_a_wr + kARows * i * kRowBytes) = aq[i];          \
        POLAR_STREAM_FETCH_A(1 - (j), u + (j))                                                     \
        POLAR_STREAM_FETCH_W(j, u + 1)                                                             \
        if (!(kStreamAblate & 4)) __syncthreads();                                                 \
        if (!(kStreamAblate & 2)) {                                                                \
        u32x4 bq[HW][4];                                                                           \
        _Pragma("unroll") for (int h = 0; h < HW; ++h)                                             \
            _Pragma("unroll") for (int s = 0; s < 4; ++s) bq[h][s] = *reinterpret_cast<const u32x4 *>( \
                wop + (kSplit ? (j) * kTileBytes : 0) + lds_op + 16 * h * kRowBytes + 16 * s);     \
        _Pragma("unroll") for (int t = 0; t < TW; ++t)                                             \
        {                                                                                          \
            u32x4 a[4];                                                                            \
            _Pragma("unroll") for (int s = 0; s < 4; ++s) a[s] =                                   \
                *reinterpret_cast<const u32x4 *>(abuf + lds_op + 16 * (row_tile0 + t) * kRowBytes + 16 * s); \
            _Pragma("unroll") for (int s = 0; s < 4; ++s)                                          \
            {                                                                                      \
                _Pragma("unroll") for (int h = 0; h < HW; ++h)                                     \
                    if (kStreamAblate & 1) asm volatile("" ::"v"(a[s]), "v"(bq[h][s]));            \
                    else acc[t][h] = mfma16x16x32<BF>(a[s], bq[h][s], acc[t][h]);                  \
            }                                                                                      \
        }                                                                                          \
        }                                                                                          \
    }

    // a finished segment of `tile`: the whole contraction is finished in place, a part of it goes
    // to the workspace as raw accumulators
    auto store_segment = [&](const f32x4 (&sum)[TW][HW], int of_tile, bool whole) {
        if (kStreamAblate & 32) {                // one value per thread, so that the sums stay live
            float v = 0.0f;
#pragma unroll
            for (int t = 0; t < TW; ++t)
#pragma unroll
                for (int h = 0; h < HW; ++h) v += sum[t][h][0] + sum[t][h][1] + sum[t][h][2] + sum[t][h][3];
            part[((size_t)span * 2 + (of_tile == first_tile ? 0 : 1)) * kStreamThreads + tid] = v;
            return;
        }
        if (whole) {
            // accumulator layout: this lane holds rows 16*t + 4*kg + i of column x of each group
            // of 16 neurons
#pragma unroll
            for (int h = 0; h < HW; ++h) {
                const int col = of_tile * kStreamTileN + ncol0 + 16 * h + x;
                const bool valid = sh_id[(of_tile - first_tile) * kStreamTileN + ncol0 + 16 * h + x] >= 0;
                if (H16) {                       // rounded to the storage type, rows padded with zeros
                    if (col >= (count + 31) / 32 * 32) continue;
                    const size_t pitch = ((size_t)cap + 31) / 32 * 32;
#pragma unroll
                    for (int t = 0; t < TW; ++t)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int row = 16 * (row_tile0 + t) + 4 * kg + i;
                            if (row < M) {
                                float val = sum[t][h][i];
                                if (relu) val = val > 0.0f ? val : 0.0f;
                                H16[(size_t)row * pitch + col] = (col < count && valid) ? to_storage(val, BF) : (uint16_t)0;
                            }
                        }
                    continue;
                }
                if (col >= count) continue;
#pragma unroll
                for (int t = 0; t < TW; ++t)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int row = 16 * (row_tile0 + t) + 4 * kg + i;
                        if (row < M) {
                            float val = sum[t][h][i];
                            if (relu) val = val > 0.0f ? val : 0.0f;
                            C[(size_t)row * cap + col] = valid ? val : 0.0f;
                        }
                    }
            }
        } else {
            const int slot = of_tile == first_tile ? 0 : 1;          // slot 0: the span's first tile
            f32x4 *dst = reinterpret_cast<f32x4 *>(part) +
                         (((size_t)span * 2 + slot) * kStreamWaves + wave) * (TW * HW) * 64 + lane;
#pragma unroll
            for (int t = 0; t < TW; ++t)
#pragma unroll
                for (int h = 0; h < HW; ++h) dst[(t * HW + h) * 64] = sum[t][h];
        }
    };
    constexpr bool kDefer = MT <= 4;             // at 128 rows it fits (254 registers) and gains nothing measurable
    f32x4 held[TW][HW];
    int held_tile = -1;
    bool held_whole = false;

    POLAR_STREAM_FETCH_W(0, u)
    POLAR_STREAM_FETCH_A(0, u)
    POLAR_STREAM_FETCH_W(1, u)
    while (u < u1) {
        const int seg_begin = u, seg_end = tile_end < u1 ? tile_end : u1;
        f32x4 acc[TW][HW];
#pragma unroll
        for (int t = 0; t < TW; ++t)
#pragma unroll
            for (int h = 0; h < HW; ++h) acc[t][h] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (; u < seg_end; ++u) {
            POLAR_STREAM_STEP(0)
            POLAR_STREAM_STEP(1)
        }

        // A segment's stores are counted with the loads in flight, and the loads issued after
        // them cannot be waited for before the stores are acknowledged: the first segment that is
        // followed by more work is therefore kept in registers and stored when the span is done.
        const bool whole = seg_end - seg_begin == upt;
        if (kDefer && u < u1 && held_tile < 0) {
            held_tile = tile;
            held_whole = whole;
#pragma unroll
            for (int t = 0; t < TW; ++t)
#pragma unroll
                for (int h = 0; h < HW; ++h) held[t][h] = acc[t][h];
        } else {
            store_segment(acc, tile, whole);
        }
        if (u < u1) {                            // on to the next tile; fetch the row ids of the one after it
            ++tile;
            tile_base = tile_end;
            tile_end += upt;
#pragma unroll
            for (int i = 0; i < NR; ++i) {
                cur[i] = nxt[i];
                nxt[i] = row_id(tile + 1 - first_tile, i);
            }
        }
    }
    if (kDefer && held_tile >= 0) store_segment(held, held_tile, held_whole);
#undef POLAR_STREAM_STEP
#undef POLAR_STREAM_FETCH_A
#undef POLAR_STREAM_FETCH_W
#undef POLAR_STREAM_BLOCK_OFFSET
}

// grid = tiles * waves per tile * ceil(MT * NH / 4) workgroups: workgroup (tile, w, q) adds four of
// the MT * NH accumulator tiles that wave w of the kernel above left for that tile (thread
// (j, lane) owns entry e = 4 * q + j = t * NH + h); G is that kernel's grid.
template <int MT>
__global__ __launch_bounds__(kGemmThreads) void select_gemm_reduce_kernel(
    const float *__restrict__ part, const int32_t *__restrict__ idx, const int32_t *__restrict__ count_ptr,
    float *__restrict__ C, uint16_t *__restrict__ H16, int bf, int M, int K, int N, int cap, int relu, int G)
{
    int count = cap;
    if (count_ptr) {
        const int c = *count_ptr;
        count = c < 0 ? 0 : (c < cap ? c : cap);
    }
    const int nblk = K / (kBlockK * kUnitBlocks);            // units per tile
    const int tiles = (count + kStreamTileN - 1) / kStreamTileN;
    constexpr bool kSplit = MT >= 4;              // the streaming kernel's pairing of waves
    constexpr int TW = kSplit ? MT / 2 : MT, HW = kSplit ? 2 * NH : NH;
    constexpr int kQuads = (TW * HW + 3) / 4;
    const int tile = blockIdx.x / (kStreamWaves * kQuads), wave = blockIdx.x / kQuads % kStreamWaves;
    const int e = (blockIdx.x % kQuads) * 4 + (threadIdx.x >> 6);
    if (tile >= tiles || e >= TW * HW) return;
    const int units = tiles * nblk, lo = tile * nblk, hi = lo + nblk;
    // the workgroup whose span holds unit lo
    int g0 = (int)((unsigned)lo * (unsigned)G / (unsigned)units);
    while (g0 + 1 < G && span_bound(units, G, g0 + 1) <= lo) ++g0;
    while (g0 > 0 && span_bound(units, G, g0) > lo) --g0;
    if (span_bound(units, G, g0 + 1) >= hi) return;      // one workgroup did the whole tile in place
    // and the one whose span holds the tile's last unit
    int g1 = (int)((unsigned)(hi - 1) * (unsigned)G / (unsigned)units);
    while (g1 + 1 < G && span_bound(units, G, g1 + 1) <= hi - 1) ++g1;
    while (g1 > 0 && span_bound(units, G, g1) > hi - 1) --g1;

    const int lane = threadIdx.x & 63, x = lane & 15, kg = lane >> 4;
    const int n0 = tile * kStreamTileN;
    {
        const int t = (kSplit ? (wave & 1) * TW : 0) + e / HW, h = e % HW;
        const int ncol0 = kSplit ? (wave >> 1) * 2 * kStreamWaveN : wave * kStreamWaveN;
        f32x4 sum = (f32x4){0.f, 0.f, 0.f, 0.f};
        // segments in ascending workgroup order (g0 .. g1, empty spans skipped: adding +0.0
        // leaves the sum as it is), loads issued four at a time
        for (int gb = g0; gb <= g1; gb += 4) {
            f32x4 v[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int g = gb + q;
                v[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
                if (g > g1) continue;
                const int b = span_bound(units, G, g);
                if (span_bound(units, G, g + 1) <= b) continue;
                const int slot = b / nblk == tile ? 0 : 1;
                v[q] = *(reinterpret_cast<const f32x4 *>(part) +
                         ((((size_t)g * 2 + slot) * kStreamWaves + wave) * (TW * HW) + e) * 64 + lane);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) sum += v[q];
        }
        const int col = n0 + ncol0 + 16 * h + x;
        if (col >= (H16 ? (count + 31) / 32 * 32 : count)) return;
        const int id = col < count ? idx[col] : -1;
        const bool valid = id >= 0 && id < N;
        const size_t pitch = ((size_t)cap + 31) / 32 * 32;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 16 * t + 4 * kg + i;
            if (row < M) {
                float v = sum[i];
                if (relu) v = v > 0.0f ? v : 0.0f;
                if (H16)
                    H16[(size_t)row * pitch + col] = valid ? to_storage(v, bf != 0) : (uint16_t)0;
                else
                    C[(size_t)row * cap + col] = valid ? v : 0.0f;
            }
        }
    }
}

// Batch union of predicted neuron ids (Section 4.1: one index tensor for the whole batch).
// An LDS bitmap of N bits is cleared, every valid id of topk sets its bit, then each thread
// counts the bits of its contiguous share of the bitmap, an exclusive scan over the threads gives
// its output offset, and it emits its ids in ascending order.  The result is the ascending list
// of distinct ids, whatever the order of the input.  One workgroup does all of it; with a
// workspace the bitmap is built by several workgroups instead, each over its share of the ids
// (the slow part: B * kn ids through one compute unit's LDS atomics), and the last kernel ORs
// their bitmaps together before it counts and emits.
constexpr int kUnionThreads = 1024;
constexpr int kUnionMaxWords = 16384;            // N <= 524288 neurons (64 KB of LDS)
constexpr int kUnionBuilders = 8;                // workgroups that build partial bitmaps (more: the emitters OR more maps)
constexpr int kUnionMinIdsPerBuilder = 2048;
constexpr long kUnionSplitFrom = 1l << 14;       // ids from which the split form (builders + emitters) pays
constexpr int kUnionScanSlots = 32;               // wave totals of the scan (16 used)
constexpr int kUnionEmitters = 16;               // workgroups of the split form's last launch (one wave's share each)

// sh_bits[0, words) cleared, then the bits of topk[begin, end) set; ends with a barrier
__device__ __forceinline__ void union_mark(unsigned int *sh_bits, int words, const int32_t *__restrict__ topk,
                                           long begin, long end, int N)
{
    const int tid = threadIdx.x;
    for (int wd = tid; wd < words; wd += kUnionThreads) sh_bits[wd] = 0u;
    __syncthreads();
    for (long i = begin + tid; i < end; i += kUnionThreads) {
        const int id = topk[i];
        if (id >= 0 && id < N) atomicOr(&sh_bits[id >> 5], 1u << (id & 31));
    }
    __syncthreads();
}

// thread t counts and emits the words [first(t), first(t + 1)): contiguous, in thread order, as
// even as it gets (at most one word apart)
__device__ __forceinline__ int union_first_word(int t, int words)
{
    return (int)((long)t * words / kUnionThreads);
}

// sh_bits[0, words) holds the union: count, scan, emit (sh_scan: kUnionScanSlots words)
// Workgroup `part` of `parts` emits the ids of the threads [part, part + 1) * kUnionThreads / parts
// (every workgroup does the whole count and scan; the bit loops with their scattered 4-byte
// stores, the slow part, are what is shared out); part 0 stores the count.
__device__ __forceinline__ void union_emit(const unsigned int *sh_bits, unsigned int *sh_scan, int words,
                                           int cap, int32_t *__restrict__ idx_out,
                                           int32_t *__restrict__ count_out, int part, int parts)
{
    const int tid = threadIdx.x;
    const int w_begin = union_first_word(tid, words), w_end = union_first_word(tid + 1, words);
    unsigned int mine = 0;
    for (int wd = w_begin; wd < w_end; ++wd) mine += __popc(sh_bits[wd]);
    // exclusive scan over the threads: shuffles inside a wave, then the 16 wave totals
    const int lane = tid & 63, wave = tid >> 6;
    unsigned int incl = mine;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const unsigned int up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (lane == 63) sh_scan[wave] = incl;
    __syncthreads();
    unsigned int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kUnionThreads / 64; ++w) {
        const unsigned int t = sh_scan[w];
        before += w < wave ? t : 0u;
        all += t;
    }
    unsigned int pos = before + incl - mine;
    if (tid == 0 && part == 0) count_out[0] = (int32_t)(all < (unsigned)cap ? all : (unsigned)cap);
    if (tid < part * kUnionThreads / parts || tid >= (part + 1) * kUnionThreads / parts) return;
    for (int wd = w_begin; wd < w_end; ++wd) {
        unsigned int bits = sh_bits[wd];
        while (bits) {
            const int bit = __ffs(bits) - 1;
            bits &= bits - 1;
            if (pos < (unsigned)cap) idx_out[pos] = wd * 32 + bit;
            ++pos;
        }
    }
}

// grid = parts (1 or kUnionEmitters): EVERY workgroup marks all the ids in a bitmap of its own, counts and
// scans it, and emits its share of the output (the bit loops with their scattered 4-byte stores are the
// slow part of a one-workgroup union: 12 to 19 us for ten thousand ids; marking is cheap to repeat).  No
// workgroup depends on another, so this is one launch with no workspace.
__global__ __launch_bounds__(kUnionThreads) void neuron_union_kernel(
    const int32_t *__restrict__ topk, long total, int N, int cap, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out)
{
    extern __shared__ unsigned int sh_bits[];     // words, then the scan slots
    const int words = (N + 31) / 32;
    union_mark(sh_bits, words, topk, 0, total, N);
    union_emit(sh_bits, sh_bits + words, words, cap, idx_out, count_out, (int)blockIdx.x, (int)gridDim.x);
}

// grid = builders: workgroup g marks its share of the ids and stores its bitmap to maps[g][words]
__global__ __launch_bounds__(kUnionThreads) void neuron_bitmap_kernel(
    const int32_t *__restrict__ topk, long total, int N, unsigned int *__restrict__ maps)
{
    extern __shared__ unsigned int sh_bits[];
    const int words = (N + 31) / 32;
    const long per = (total + gridDim.x - 1) / gridDim.x;
    const long begin = min((long)blockIdx.x * per, total), end = min(begin + per, total);
    union_mark(sh_bits, words, topk, begin, end, N);
    unsigned int *dst = maps + (size_t)blockIdx.x * words;
    for (int wd = threadIdx.x; wd < words; wd += kUnionThreads) dst[wd] = sh_bits[wd];
}

// grid = emitters: every workgroup ORs the builders' bitmaps, counts and scans; each emits its share
__global__ __launch_bounds__(kUnionThreads) void neuron_emit_kernel(
    const unsigned int *__restrict__ maps, int builders, int N, int cap, int32_t *__restrict__ idx_out,
    int32_t *__restrict__ count_out)
{
    extern __shared__ unsigned int sh_bits[];
    const int words = (N + 31) / 32;
    // each thread ORs the words it will count and emit itself, so no barrier is needed in between
    const int w_begin = union_first_word(threadIdx.x, words), w_end = union_first_word(threadIdx.x + 1, words);
    for (int wd = w_begin; wd < w_end; ++wd) {
        // all loads in flight at once (a plain loop would wait for each in turn)
        unsigned int v[kUnionBuilders];
#pragma unroll
        for (int g = 0; g < kUnionBuilders; ++g) v[g] = g < builders ? maps[(size_t)g * words + wd] : 0u;
        unsigned int bits = 0u;
#pragma unroll
        for (int g = 0; g < kUnionBuilders; ++g) bits |= v[g];
        sh_bits[wd] = bits;
    }
    union_emit(sh_bits, sh_bits + words, words, cap, idx_out, count_out, (int)blockIdx.x, (int)gridDim.x);
}

template <bool BF>
hipError_t launch_gemm_mt(int mt, dim3 grid, hipStream_t st, const uint16_t *A, const uint16_t *W,
                          const int32_t *idx, const int32_t *count, float *C, int M, int K, int N,
                          int cap, int relu)
{
    switch (mt) {
    case 1:
        hipLaunchKernelGGL((select_gemm_kernel<BF, 1>), grid, dim3(kGemmThreads), 0, st, A, W, idx,
                           count, C, M, K, N, cap, relu);
        break;
    case 2:
        hipLaunchKernelGGL((select_gemm_kernel<BF, 2>), grid, dim3(kGemmThreads), 0, st, A, W, idx,
                           count, C, M, K, N, cap, relu);
        break;
    default:
        hipLaunchKernelGGL((select_gemm_kernel<BF, 4>), grid, dim3(kGemmThreads), 0, st, A, W, idx,
                           count, C, M, K, N, cap, relu);
        break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_select_gemm(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                              float *C, int M, int K, int N, int cap, polar_dtype dt, int relu,
                              hipStream_t stream)
{
    const uint16_t *A16 = static_cast<const uint16_t *>(A);
    const uint16_t *W16 = static_cast<const uint16_t *>(W);
    const dim3 grid((unsigned)((cap + kTileN - 1) / kTileN));
    // batches beyond 256 rows are processed 256 rows at a time (the gathered rows are re-read)
    for (int m0 = 0; m0 < M; m0 += 256) {
        const int rows = M - m0 < 256 ? M - m0 : 256;
        const int mt = rows <= 64 ? 1 : (rows <= 128 ? 2 : 4);
        const uint16_t *Ap = A16 + (size_t)m0 * K;
        float *Cp = C + (size_t)m0 * cap;
        const hipError_t e =
            dt == POLAR_BF16
                ? launch_gemm_mt<true>(mt, grid, stream, Ap, W16, idx, count, Cp, rows, K, N, cap, relu)
                : launch_gemm_mt<false>(mt, grid, stream, Ap, W16, idx, count, Cp, rows, K, N, cap, relu);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Workspace of the wide-tile form: two slots of raw accumulators per workgroup.
static size_t stream_slot_bytes(int mt) { return (size_t)2 * kStreamWaves * mt * NH * 64 * sizeof(f32x4); }
constexpr int kStreamMaxRows = 128;              // rows of the batch the evenly split form takes
static int stream_mt(int M) { return M <= 16 ? 1 : (M <= 32 ? 2 : (M <= 64 ? 4 : 8)); }

int select_gemm_ws_max_rows() { return kStreamMaxRows; }

size_t select_gemm_workspace_bytes(int M)
{
    return (size_t)kStreamGrid * stream_slot_bytes(stream_mt(M < kStreamMaxRows ? M : kStreamMaxRows));
}

template <bool BF>
static hipError_t launch_stream_mt(int mt, int G, int tiles, hipStream_t st, const uint16_t *A,
                                   const uint16_t *W, const int32_t *idx, const int32_t *count, float *C,
                                   uint16_t *H16, float *part, int M, int K, int N, int cap, int relu)
{
    const dim3 grid((unsigned)G), rgrid((unsigned)tiles * kStreamWaves * ((mt * NH + 3) / 4)), block(kStreamThreads), rblock(kGemmThreads);
    const int bf = BF ? 1 : 0;
#define POLAR_STREAM_LAUNCH(MT_)                                                                                          \
    hipLaunchKernelGGL((select_gemm_stream_kernel<BF, MT_>), grid, block, 0, st, A, W, idx, count, C, H16, part, M, K, N, \
                       cap, relu);                                                                                        \
    hipLaunchKernelGGL((select_gemm_reduce_kernel<MT_>), rgrid, rblock, 0, st, part, idx, count, C, H16, bf, M, K, N, cap, \
                       relu, G)
    switch (mt) {
    case 1: POLAR_STREAM_LAUNCH(1); break;
    case 2: POLAR_STREAM_LAUNCH(2); break;
    case 4: POLAR_STREAM_LAUNCH(4); break;
    default: POLAR_STREAM_LAUNCH(8); break;
    }
#undef POLAR_STREAM_LAUNCH
    return hipGetLastError();
}

// Workgroups the evenly split form would launch for these sizes and this much workspace; 0: it
// cannot run (the caller takes the one-launch kernel).
static int stream_grid(int M, int K, int cap, bool have_workspace, size_t workspace_bytes)
{
    if (!have_workspace || M > kStreamMaxRows || K % (kBlockK * kUnitBlocks) != 0 ||
        option(POLAR_OPT_GEMM_FORM) == 1)                    // forced: always the 32-neuron one-launch kernel
        return 0;
    const int mt = stream_mt(M);
    const int tiles = (cap + kStreamTileN - 1) / kStreamTileN;
    const long units = (long)tiles * (K / (kBlockK * kUnitBlocks));
    long G = kStreamGrid;
    if (const int v = option(POLAR_OPT_GEMM_WORKGROUPS)) {
        if (v >= 1 && v <= kStreamGrid) G = v;
    }
    if (G > units) G = units;
    if ((size_t)G * stream_slot_bytes(mt) > workspace_bytes) G = (long)(workspace_bytes / stream_slot_bytes(mt));
    // a span of at most units / G + 1 units touches at most tiles / G + 2 tiles, whose row ids
    // the kernel keeps in LDS; the span arithmetic is 32-bit
    if (G < 1 || tiles / G + 2 > kSpanTiles || units * G >= (1l << 31)) return 0;
    return (int)G;
}

static hipError_t launch_stream(int G, const void *A, const void *W, const int32_t *idx, const int32_t *count,
                                float *C, uint16_t *H16, int M, int K, int N, int cap, polar_dtype dt, int relu,
                                void *workspace, hipStream_t stream)
{
    const int mt = stream_mt(M), tiles = (cap + kStreamTileN - 1) / kStreamTileN;
    const uint16_t *A16 = static_cast<const uint16_t *>(A);
    const uint16_t *W16 = static_cast<const uint16_t *>(W);
    float *part = static_cast<float *>(workspace);
    return dt == POLAR_BF16
               ? launch_stream_mt<true>(mt, G, tiles, stream, A16, W16, idx, count, C, H16, part, M, K, N, cap, relu)
               : launch_stream_mt<false>(mt, G, tiles, stream, A16, W16, idx, count, C, H16, part, M, K, N, cap, relu);
}

hipError_t launch_select_gemm_ws(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                                 float *C, int M, int K, int N, int cap, polar_dtype dt, int relu,
                                 void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    // batches beyond 128 rows are processed 128 rows at a time (the gathered rows are re-read; the
    // passes share the workspace, which the stream's order makes safe)
    for (int m0 = 0; m0 < M; m0 += kStreamMaxRows) {
        const int rows = M - m0 < kStreamMaxRows ? M - m0 : kStreamMaxRows;
        const uint16_t *Ap = static_cast<const uint16_t *>(A) + (size_t)m0 * K;
        float *Cp = C + (size_t)m0 * cap;
        const int G = stream_grid(rows, K, cap, workspace != nullptr, workspace_bytes);
        const hipError_t e =
            G < 1 ? launch_select_gemm(Ap, W, idx, count, Cp, rows, K, N, cap, dt, relu, stream)
                  : launch_stream(G, Ap, W, idx, count, Cp, nullptr, rows, K, N, cap, dt, relu, workspace, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

bool select_gemm_h16_applicable(int M, int K, int cap, size_t workspace_bytes)
{
    return stream_grid(M, K, cap, true, workspace_bytes) >= 1;
}

hipError_t launch_select_gemm_h16(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                                  uint16_t *H16, int M, int K, int N, int cap, polar_dtype dt, int relu,
                                  void *workspace, size_t workspace_bytes, hipStream_t stream)
{
    const int G = stream_grid(M, K, cap, true, workspace_bytes);
    if (G < 1) return hipErrorInvalidValue;      // callers ask select_gemm_h16_applicable first
    return launch_stream(G, A, W, idx, count, nullptr, H16, M, K, N, cap, dt, relu, workspace, stream);
}

int neuron_union_max_n() { return kUnionMaxWords * 32; }

hipError_t launch_neuron_union(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                               int32_t *count_out, hipStream_t stream)
{
    const int words = (N + 31) / 32;
    const size_t lds = ((size_t)words + kUnionScanSlots) * sizeof(unsigned int);
    static LdsGrant granted;                     // the bitmap and the scan slots
    const hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(neuron_union_kernel), lds, granted);
    if (e != hipSuccess) return e;
    // a handful of ids: one workgroup; otherwise kUnionEmitters of them share the emit phase
    const long total = (long)B * kn;
    const int parts = total < 1024 ? 1 : kUnionEmitters;
    hipLaunchKernelGGL(neuron_union_kernel, dim3(parts), dim3(kUnionThreads), lds, stream, topk, total, N, cap, idx_out,
                       count_out);
    return hipGetLastError();
}

// builders the split form would use for this input (0: the one-launch kernel is the faster one).  In the
// one-launch kernel every workgroup marks all the ids, total / 1024 LDS atomics per thread at about 6 ids per
// nanosecond and compute unit; from kUnionSplitFrom ids on, sharing the marking over builders and paying a
// second launch is faster (replayed from a graph, one launch / split: 8848 ids 5.8 / 7.4 us, 35392 ids 11.7 /
// 9.4 us, 117952 ids 25.7 / 11.8 us).  POLAR_OPT_UNION_FORM pins the choice.
static int union_builders(long total)
{
    const int form = option(POLAR_OPT_UNION_FORM);
    if (form == 1 || (form == 0 && total < kUnionSplitFrom)) return 0;
    const long want = total / kUnionMinIdsPerBuilder;
    return want < 2 ? 0 : (int)(want < kUnionBuilders ? want : kUnionBuilders);
}

size_t neuron_union_workspace_bytes(int B, int kn, int N)
{
    return (size_t)union_builders((long)B * kn) * ((N + 31) / 32) * sizeof(unsigned int);
}

hipError_t launch_neuron_union_ws(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                                  int32_t *count_out, void *workspace, size_t workspace_bytes,
                                  hipStream_t stream)
{
    const int words = (N + 31) / 32;
    const long total = (long)B * kn;
    int builders = union_builders(total);
    const size_t per = (size_t)words * sizeof(unsigned int);
    if (workspace && (size_t)builders * per > workspace_bytes) builders = (int)(workspace_bytes / per);
    if (!workspace || builders < 2) return launch_neuron_union(topk, B, kn, N, cap, idx_out, count_out, stream);
    static LdsGrant granted_build, granted_emit;
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(neuron_bitmap_kernel), per, granted_build);
    if (e != hipSuccess) return e;
    const size_t lds = ((size_t)words + kUnionScanSlots) * sizeof(unsigned int);
    e = ensure_dynamic_lds(reinterpret_cast<const void *>(neuron_emit_kernel), lds, granted_emit);
    if (e != hipSuccess) return e;
    unsigned int *maps = static_cast<unsigned int *>(workspace);
    hipLaunchKernelGGL(neuron_bitmap_kernel, dim3(builders), dim3(kUnionThreads), per, stream, topk, total, N, maps);
    hipLaunchKernelGGL(neuron_emit_kernel, dim3(kUnionEmitters), dim3(kUnionThreads), lds, stream, maps, builders, N, cap,
                       idx_out, count_out);
    return hipGetLastError();
}

}  // namespace polar
