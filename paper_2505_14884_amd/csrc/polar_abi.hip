// extern "C" boundary: host-side argument validation, launch planning, error codes.
// Every check below runs before the first HIP call, so invalid arguments are reported the
// same way with or without a GPU in the machine.
#include <math.h>

#include <mutex>

#include "polar_internal.h"

// Scratch of polar_sha_decode_static: part of the library's device image, one copy per GPU.  In
// host code this name is only a handle for hipGetSymbolAddress; kernels get the address it returns.
static __device__ __align__(256) unsigned char scratch[POLAR_STATIC_SCRATCH_BYTES];

namespace polar {
namespace {

// Device address of `scratch` on the current GPU, looked up once per GPU (each GPU holds its own
// copy at its own address) and kept for the life of the process.
hipError_t static_scratch(void **ptr)
{
    constexpr int kDevices = 64;
    static std::atomic<void *> known[kDevices];
    static std::mutex lookup;
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    if (dev < 0 || dev >= kDevices) return hipErrorInvalidDevice;
    void *p = known[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> guard(lookup);
        p = known[dev].load(std::memory_order_acquire);
        if (!p) {
            if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
            if (!p) return hipErrorInvalidSymbol;
            known[dev].store(p, std::memory_order_release);
        }
    }
    *ptr = p;
    return hipSuccess;
}

thread_local int g_last_hip_error = 0;

// Process-wide options: plain integers, 0 = the library's own choice.  Relaxed atomics: an option
// is a hint that each call reads once, not a synchronisation point.
std::atomic<int> g_options[POLAR_OPT_COUNT_];

bool option_value_ok(int opt, int v)
{
    switch (opt) {
    case POLAR_OPT_SHA_CHUNK_ROWS: return v == 0 || (v >= 128 && v <= (1 << 20));
    case POLAR_OPT_SHA_FORM: return v >= 0 && v <= 2;
    case POLAR_OPT_SHA_GROUPED_KERNEL: return v == 0 || v == 1;
    case POLAR_OPT_ROUTER_PATH: return v >= 0 && v <= 2;
    case POLAR_OPT_ROUTER_PHASE1: return v >= 0 && v <= 2;
    case POLAR_OPT_GEMM_FORM: return v == 0 || v == 1;
    case POLAR_OPT_GEMM_WORKGROUPS: return v >= 0 && v <= 256;
    case POLAR_OPT_UNION_FORM: return v >= 0 && v <= 2;
    default: return false;
    }
}

int record(hipError_t e)
{
    if (e == hipSuccess) return POLAR_OK;
    g_last_hip_error = (int)e;
    return POLAR_EHIP;
}

bool dtype_ok(int dt) { return dt == POLAR_F16 || dt == POLAR_BF16; }

// Rows of the cache one workgroup of the streaming kernel covers, i.e. into how many chunks a
// (request, head) unit is split.  Every workgroup pays a fixed few microseconds (index loads,
// first-load latency, the epilogue) and every split adds a record for the merge kernel, so the
// number of splits is the smallest one for which
//   (a) a chunk is short enough for the tail of the grid: a lone workgroup streams far below the
//       chip's bandwidth, so the rows one workgroup carries are capped (kMaxChunk; an unsplit
//       cache may be up to kMaxUnsplit rows: it saves the merge kernel and the workspace traffic),
//   (b) the grid fills the chip (kFill workgroups; kComputeUnits for an unsplit cache), and
//   (c) the workgroups fill whole rounds of the 256 compute units to at least 90 % (320 units on
//       256 compute units: 134 us unsplit against 117 us in 3 chunks);
// without (c) if no split count meets it.  Measured choices: LLaMA-2-7B-shaped layer, 512 units,
// unsplit: 93.1 -> 87.7 us per step; LLaMA-3-8B GQA layer, 256 units, unsplit: 96.6 -> 92.3 us.
// The grouped-query kernel has fewer, longer-lived workgroups per compute unit, so its fixed
// costs weigh more: chunks up to 4096 rows, and 256 workgroups already fill the chip (a
// 64-query-head / 8-group layer with 8192-row caches and 128 units: 84.6 us in chunks of 1024,
// 82.4 us in chunks of 4096).  Its unsplit limit stays at 4096 rows: with ragged lengths longer
// unsplit caches lose more to the grid's tail (770 against 697 us) than uniform ones gain.
// Chunks are multiples of 128 rows, which every kernel shape's per-wave step divides, so only a
// request's last chunk has a ragged tail.  POLAR_OPT_SHA_CHUNK_ROWS overrides the choice (sweeps).
constexpr long kComputeUnits = 256;
constexpr int kMinChunk = 256;
constexpr long kDirectMaxUnits = 2048;
struct ChunkPolicy {
    int max_chunk;     // rows per workgroup when the cache is split
    int max_unsplit;   // longest cache that may stay in one piece
    long fill;         // workgroups wanted in the grid when splitting
};
constexpr ChunkPolicy kPerHeadPolicy = {1024, 2048, 1024};
constexpr ChunkPolicy kGroupedPolicy = {4096, 4096, 256};

int choose_chunk(int B, int k, int S, const ChunkPolicy &pol)
{
    const int cap = (S + 127) / 128 * 128;
    if (const int forced = option(POLAR_OPT_SHA_CHUNK_ROWS)) {
        const long chunk = ((long)forced + 127) / 128 * 128;
        return chunk < cap ? (int)chunk : cap;
    }
    const long units = (long)(B > 0 ? B : 1) * k;
    int fallback = 0;
    for (int want = 1;; ++want) {
        int chunk = ((S + want - 1) / want + 127) / 128 * 128;
        if (chunk < kMinChunk) chunk = kMinChunk;
        if (chunk > cap) chunk = cap;
        const int nsplit = (S + chunk - 1) / chunk;
        const bool smallest = chunk <= kMinChunk;                    // no finer split exists
        if (nsplit < want && !smallest) continue;                    // same chunk as an earlier `want`
        const bool short_enough = nsplit == 1 ? S <= pol.max_unsplit : chunk <= pol.max_chunk;
        const long wgs = units * nsplit;
        const bool fills = wgs >= (nsplit == 1 ? kComputeUnits : pol.fill);
        if ((short_enough && fills) || smallest) {
            const long rounds = (wgs + kComputeUnits - 1) / kComputeUnits;
            const bool even = wgs * 10 >= rounds * kComputeUnits * 9;
            if (even || smallest) return fallback && !even ? fallback : chunk;
            if (!fallback) fallback = chunk;
            if (want - (S + fallback - 1) / fallback >= 8) return fallback;   // looked far enough
        }
    }
}

// Which router path is faster when the caller offers a workspace.  The one-workgroup-per-request
// kernel is a single launch whose time depends on D*H only while B fits the chip (256 compute
// units); the split-D pair spreads the work over the whole chip but pays a second launch.  The
// estimates are fits to event timings on MI355X over B = 1..1024, D*H = 32 K..2 M (microseconds):
//   single            = ceil(B/256) * max(7.5, 5.2 + D*H / 31e3)
//   split, B >= 16    = 11.5 + 2.6e-5 * ceil(B/16) * D * padded 16-column tiles   (fp64 matrix cores)
//   split, B <  16    = 10.5 + B*D*H / 8.5e6                                      (vector ALU)
// Examples (single vs split measured): B=64, D=4096, H=8: 8.4 vs 11.3; B=128, D=9216, H=72:
// 29.3 vs 20.4; B=256, D=4096, H=32: 9.8 vs 13.4; B=1024, D=8192, H=64: 89 vs 48.
// POLAR_OPT_ROUTER_PATH overrides the choice (tests use it to reach both paths).
bool router_split_pays(int B, int D, int H, const RouterPlan &plan)
{
    if (const int forced = option(POLAR_OPT_ROUTER_PATH)) return forced == 2;
    const double dh = (double)D * H;
    const double rounds = (double)((B + 255) / 256);
    double single_us = 5.2 + dh / 31.0e3;
    if (single_us < 7.5) single_us = 7.5;
    single_us *= rounds;
    double split_us;
    if (plan.mfma) {
        const int nt = (H + 15) / 16, grp = nt < 5 ? nt : 5;
        const double tiles = (double)((nt + grp - 1) / grp * grp);
        split_us = 11.5 + 2.6e-5 * (double)((B + 15) / 16) * D * tiles;
    } else {
        split_us = 10.5 + (double)B * dh / 8.5e6;
    }
    return split_us < single_us;
}

int check_sha_sizes(int B, int Hq, int Hkv, int S, int d, int k)
{
    if (B < 0 || Hq < 1 || Hkv < 1 || S < 1 || d < 1 || k < 1) return POLAR_EINVAL;
    if (k > Hkv || Hq % Hkv != 0) return POLAR_EINVAL;
    if (d != 64 && d != 128) return POLAR_EUNSUPPORTED;
    const int G = Hq / Hkv;
    if (G > POLAR_MAX_GROUP) return POLAR_EUNSUPPORTED;
    // d = 64 runs the vector-ALU kernel, instantiated for power-of-two groups up to 8
    if (d == 64 && G != 1 && G != 2 && G != 4 && G != 8) return POLAR_EUNSUPPORTED;
    // ... as is the same kernel when an option forces it on grouped heads at d = 128
    if (d == 128 && G > 1 && option(POLAR_OPT_SHA_GROUPED_KERNEL) == 1 && G != 2 && G != 4 && G != 8)
        return POLAR_EUNSUPPORTED;
    if (B > 65535 || Hq > 65535) return POLAR_EUNSUPPORTED;   // grid.y limit of the merge kernel
    return POLAR_OK;
}

}  // namespace

int option(polar_option opt)
{
    return (unsigned)opt < (unsigned)POLAR_OPT_COUNT_ ? g_options[opt].load(std::memory_order_relaxed) : 0;
}

int make_sha_plan(int B, int Hq, int Hkv, int S, int d, int k, ShaPlan *plan)
{
    const int rc = check_sha_sizes(B, Hq, Hkv, S, d, k);
    if (rc != POLAR_OK) return rc;
    plan->G = Hq / Hkv;
    plan->grouped_mfma = plan->G > 1 && d == 128 && option(POLAR_OPT_SHA_GROUPED_KERNEL) != 1;
    const bool grouped_mfma = plan->grouped_mfma;        // which streaming kernel will run
    plan->chunk = choose_chunk(B, k, S, grouped_mfma ? kGroupedPolicy : kPerHeadPolicy);
    plan->nsplit = (S + plan->chunk - 1) / plan->chunk;
    // One-kernel form: an unsplit cache needs no merge; the streaming kernel can normalise, store
    // the rows and zero-fill the unselected heads itself.  That saves a launch (4 to 6 us per step
    // on layers of 0.5 to 1.5 GB) but its scattered zero stores land in the middle of the read
    // stream and cost about 2.5 ns per workgroup (12 us at 4608 workgroups, where the merge
    // kernel takes 6), so it is used up to kDirectMaxUnits workgroups.  POLAR_OPT_SHA_FORM forces
    // the choice, for comparisons.
    plan->direct = plan->nsplit == 1 && (long)B * k <= kDirectMaxUnits;
    if (const int form = option(POLAR_OPT_SHA_FORM)) plan->direct = form == 1 && plan->nsplit == 1;
    if ((size_t)B * plan->nsplit * k > 0x7fffffffu) return POLAR_EUNSUPPORTED;   // 1-D grid limit
    const size_t units = (size_t)B * k * plan->G * plan->nsplit;
    plan->o_floats = (units * d + 63) / 64 * 64;   // keeps the (max, sum) region 256-byte aligned
    plan->ml_floats = units * 2;
    plan->bytes = ((plan->o_floats + plan->ml_floats) * sizeof(float) + 255) / 256 * 256;
    if (plan->bytes == 0) plan->bytes = 256;
    return POLAR_OK;
}

}  // namespace polar

using namespace polar;

extern "C" {

int polar_version(void) { return 2300; }

#ifndef POLAR_SOURCE_HASH
#define POLAR_SOURCE_HASH "unknown"
#endif
const char *polar_source_hash(void) { return POLAR_SOURCE_HASH; }

int polar_set_option(int opt, int value)
{
    if (!option_value_ok(opt, value)) return POLAR_EINVAL;
    g_options[opt].store(value, std::memory_order_relaxed);
    return POLAR_OK;
}

int polar_get_option(int opt, int *value)
{
    if ((unsigned)opt >= (unsigned)POLAR_OPT_COUNT_ || !value) return POLAR_EINVAL;
    *value = option(static_cast<polar_option>(opt));
    return POLAR_OK;
}

int polar_last_hip_error(void) { return g_last_hip_error; }

const char *polar_strerror(int status)
{
    switch (status) {
    case POLAR_OK: return "ok";
    case POLAR_EINVAL: return "invalid argument";
    case POLAR_EUNSUPPORTED: return "unsupported shape or dtype";
    case POLAR_EWORKSPACE: return "workspace missing, misaligned or too small";
    case POLAR_EHIP: return "HIP launch failed (see polar_last_hip_error)";
    default: return "unknown status";
    }
}

size_t polar_router_workspace_bytes(int B, int D, int H)
{
    RouterPlan plan;
    if (make_router_plan(B, D, H, &plan) != POLAR_OK) return 0;
    return plan.bytes;
}

int polar_router_topk(const void *hidden, const void *Wr, int B, int D, int H, int k,
                      int dt, int32_t *head_idx, float *logits_out, void *workspace,
                      size_t workspace_bytes, void *stream)
{
    if (B < 0 || D < 1 || H < 1 || k < 1 || k > H || !dtype_ok(dt)) return POLAR_EINVAL;
    RouterPlan plan;
    const int rc = make_router_plan(B, D, H, &plan);
    if (rc != POLAR_OK) return rc;
    if (B == 0) return POLAR_OK;
    if (!hidden || !Wr || !head_idx) return POLAR_EINVAL;
    if (!workspace)
        return record(launch_router_topk(hidden, Wr, B, D, H, k, (polar_dtype)dt, head_idx, logits_out,
                                         static_cast<hipStream_t>(stream)));
    if (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < plan.bytes) return POLAR_EWORKSPACE;
    if (!router_split_pays(B, D, H, plan))
        return record(launch_router_topk(hidden, Wr, B, D, H, k, (polar_dtype)dt, head_idx, logits_out,
                                         static_cast<hipStream_t>(stream)));
    return record(launch_router_split(hidden, Wr, B, D, H, k, (polar_dtype)dt, plan, head_idx, logits_out,
                                      workspace, static_cast<hipStream_t>(stream)));
}

size_t polar_sha_workspace_bytes(int B, int Hq, int Hkv, int S, int d, int k)
{
    ShaPlan plan;
    if (make_sha_plan(B, Hq, Hkv, S, d, k, &plan) != POLAR_OK) return 0;
    return plan.bytes;
}

int polar_sha_launches(int B, int Hq, int Hkv, int S, int d, int k)
{
    ShaPlan plan;
    if (make_sha_plan(B, Hq, Hkv, S, d, k, &plan) != POLAR_OK) return 0;
    return plan.direct ? 1 : 2;
}

int polar_sha_chunk_rows(int B, int Hq, int Hkv, int S, int d, int k)
{
    ShaPlan plan;
    if (make_sha_plan(B, Hq, Hkv, S, d, k, &plan) != POLAR_OK) return 0;
    return plan.chunk;
}

// The attention kernels read q, K, V and write `out` with 16-byte accesses.
static bool misaligned16(const void *p) { return ((uintptr_t)p & 15u) != 0; }

static int check_workspace(const ShaPlan &plan, const void *workspace, size_t workspace_bytes)
{
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < plan.bytes)
        return POLAR_EWORKSPACE;
    return POLAR_OK;
}

// `direct_out` non-NULL asks for the one-kernel form (the caller has checked plan.nsplit == 1).
static int sha_partial_impl(const void *q, const void *K, const void *V, const int32_t *seqlens,
                            const int32_t *head_idx, float *direct_out, int B, int Hq, int Hkv, int S,
                            int d, int k, int dt, int layout, float scale,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    ShaPlan plan;
    int rc = make_sha_plan(B, Hq, Hkv, S, d, k, &plan);
    if (rc != POLAR_OK) return rc;
    if (!dtype_ok(dt) || !(scale >= 0.0f) || isinf(scale)) return POLAR_EINVAL;
    if (layout != POLAR_KV_BHSD && layout != POLAR_KV_BSHD) return POLAR_EINVAL;
    if (B == 0) return POLAR_OK;
    if (!head_idx && k != Hkv) return POLAR_EINVAL;
    if (!q || !K || !V || !seqlens) return POLAR_EINVAL;
    if (misaligned16(q) || misaligned16(K) || misaligned16(V) || misaligned16(direct_out)) return POLAR_EINVAL;
    if ((rc = check_workspace(plan, workspace, workspace_bytes)) != POLAR_OK) return rc;
    const float s = scale == 0.0f ? 1.0f / sqrtf((float)d) : scale;
    const float log2e = 1.4426950408889634f;
    return record(launch_sha_partial(q, K, V, seqlens, head_idx, static_cast<float *>(workspace),
                                     direct_out, plan, B, Hq, Hkv, S, d, k, (polar_dtype)dt, (polar_kv_layout)layout, s * log2e,
                                     static_cast<hipStream_t>(stream)));
}

int polar_sha_partial(const void *q, const void *K, const void *V, const int32_t *seqlens,
                      const int32_t *head_idx, int B, int Hq, int Hkv, int S, int d, int k,
                      int dt, float scale, void *workspace, size_t workspace_bytes,
                      void *stream)
{
    return sha_partial_impl(q, K, V, seqlens, head_idx, nullptr, B, Hq, Hkv, S, d, k, dt, POLAR_KV_BHSD,
                            scale, workspace, workspace_bytes, stream);
}

int polar_sha_partial_layout(const void *q, const void *K, const void *V, const int32_t *seqlens,
                             const int32_t *head_idx, int B, int Hq, int Hkv, int S, int d, int k,
                             int dt, int layout, float scale, void *workspace,
                             size_t workspace_bytes, void *stream)
{
    return sha_partial_impl(q, K, V, seqlens, head_idx, nullptr, B, Hq, Hkv, S, d, k, dt, layout, scale,
                            workspace, workspace_bytes, stream);
}

int polar_sha_merge(const int32_t *seqlens, const int32_t *head_idx, float *out, int B, int Hq,
                    int Hkv, int S, int d, int k, const void *workspace, size_t workspace_bytes,
                    void *stream)
{
    ShaPlan plan;
    int rc = make_sha_plan(B, Hq, Hkv, S, d, k, &plan);
    if (rc != POLAR_OK) return rc;
    if (B == 0) return POLAR_OK;
    if (!head_idx && k != Hkv) return POLAR_EINVAL;
    if (!seqlens || !out || misaligned16(out)) return POLAR_EINVAL;
    if ((rc = check_workspace(plan, workspace, workspace_bytes)) != POLAR_OK) return rc;
    return record(launch_sha_merge(seqlens, head_idx, out, static_cast<const float *>(workspace),
                                   plan, B, Hq, Hkv, S, d, k, static_cast<hipStream_t>(stream)));
}

int polar_sha_decode_layout(const void *q, const void *K, const void *V, const int32_t *seqlens,
                            const int32_t *head_idx, float *out, int B, int Hq, int Hkv, int S,
                            int d, int k, int dt, int layout, float scale,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    ShaPlan plan;
    int rc = make_sha_plan(B, Hq, Hkv, S, d, k, &plan);   // size errors take precedence
    if (rc != POLAR_OK) return rc;
    if (B > 0 && (!out || misaligned16(out))) return POLAR_EINVAL;
    const bool direct = plan.direct;
    rc = sha_partial_impl(q, K, V, seqlens, head_idx, direct ? out : nullptr, B, Hq, Hkv, S, d, k, dt,
                          layout, scale, workspace, workspace_bytes, stream);
    if (rc != POLAR_OK || direct) return rc;
    return polar_sha_merge(seqlens, head_idx, out, B, Hq, Hkv, S, d, k, workspace, workspace_bytes,
                           stream);
}

int polar_sha_decode(const void *q, const void *K, const void *V, const int32_t *seqlens,
                     const int32_t *head_idx, float *out, int B, int Hq, int Hkv, int S, int d,
                     int k, int dt, float scale, void *workspace, size_t workspace_bytes,
                     void *stream)
{
    return polar_sha_decode_layout(q, K, V, seqlens, head_idx, out, B, Hq, Hkv, S, d, k, dt,
                                   POLAR_KV_BHSD, scale, workspace, workspace_bytes, stream);
}

int polar_sha_decode_static(const void *q, const void *K, const void *V, const int32_t *seqlens,
                            const int32_t *head_idx, float *out, int B, int Hq, int Hkv, int S, int d,
                            int k, int dt, float scale, void *stream)
{
    ShaPlan plan;
    const int rc = make_sha_plan(B, Hq, Hkv, S, d, k, &plan);      // size errors first, as in polar_sha_decode
    if (rc != POLAR_OK) return rc;
    if (plan.bytes > POLAR_STATIC_SCRATCH_BYTES) return POLAR_EWORKSPACE;
    if (B == 0) return polar_sha_decode(q, K, V, seqlens, head_idx, out, B, Hq, Hkv, S, d, k, dt, scale, nullptr, 0, stream);
    // polar_sha_decode's argument checks, made here so that a bad argument is reported before the
    // first HIP call (the address lookup below) as everywhere else in the library
    if (!dtype_ok(dt) || !(scale >= 0.0f) || isinf(scale)) return POLAR_EINVAL;
    if (!head_idx && k != Hkv) return POLAR_EINVAL;
    if (!q || !K || !V || !seqlens || !out) return POLAR_EINVAL;
    if (misaligned16(q) || misaligned16(K) || misaligned16(V) || misaligned16(out)) return POLAR_EINVAL;
    void *ws = nullptr;
    if (hipError_t e = static_scratch(&ws); e != hipSuccess) return record(e);
    return polar_sha_decode(q, K, V, seqlens, head_idx, out, B, Hq, Hkv, S, d, k, dt, scale, ws,
                            POLAR_STATIC_SCRATCH_BYTES, stream);
}

int polar_head_labels(const void *q, const void *K, const void *V, const int32_t *seqlens, int32_t *labels,
                      float *norms_out, float *attn_out, int B, int Hq, int Hkv, int S, int d, int k_label, int dt,
                      int layout, float scale, void *workspace, size_t workspace_bytes, void *stream)
{
    ShaPlan plan;
    int rc = make_sha_plan(B, Hq, Hkv, S, d, Hkv, &plan);        // the dense plan: every KV head is a unit
    if (rc != POLAR_OK) return rc;
    if (k_label < 1 || k_label > Hkv) return POLAR_EINVAL;
    if (Hkv > POLAR_MAX_ROUTER_H) return POLAR_EUNSUPPORTED;
    if (B > 0 && (!labels || misaligned16(attn_out))) return POLAR_EINVAL;
    // the streaming kernel in its record-writing form (argument checks as in polar_sha_partial) ...
    rc = sha_partial_impl(q, K, V, seqlens, nullptr, nullptr, B, Hq, Hkv, S, d, Hkv, dt, layout, scale, workspace,
                          workspace_bytes, stream);
    if (rc != POLAR_OK || B == 0) return rc;
    // ... and the merge whose epilogue takes the norms and ranks them
    return record(launch_sha_merge_label(seqlens, attn_out, labels, norms_out, static_cast<const float *>(workspace),
                                         plan, B, Hq, Hkv, S, d, k_label, static_cast<hipStream_t>(stream)));
}

int polar_head_norm_topk(const float *attn_out, int B, int Hq, int Hkv, int d, int k,
                         int32_t *head_idx, float *norms_out, void *stream)
{
    if (B < 0 || Hq < 1 || Hkv < 1 || d < 1 || k < 1 || k > Hkv || Hq % Hkv != 0) return POLAR_EINVAL;
    if (Hkv > POLAR_MAX_ROUTER_H || B > 0x7fffffff / 2 || (long long)(Hq / Hkv) * d > (1 << 20))
        return POLAR_EUNSUPPORTED;
    if (B == 0) return POLAR_OK;
    if (!attn_out || !head_idx) return POLAR_EINVAL;
    return record(launch_head_norm_topk(attn_out, B, Hq, Hkv, d, k, head_idx, norms_out,
                                        static_cast<hipStream_t>(stream)));
}

int polar_select_gemm(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                      float *C, int M, int K, int N, int cap, int dt, int relu, void *stream)
{
    if (M < 0 || K < 1 || N < 1 || cap < 0 || !dtype_ok(dt)) return POLAR_EINVAL;
    if (K % 128 != 0 || (long long)N * K > (1ll << 40)) return POLAR_EUNSUPPORTED;
    if (M == 0 || cap == 0) return POLAR_OK;
    if (!A || !W || !idx || !C) return POLAR_EINVAL;
    if (((uintptr_t)A & 15u) || ((uintptr_t)W & 15u)) return POLAR_EINVAL;   // 16-byte loads
    return record(launch_select_gemm(A, W, idx, count, C, M, K, N, cap, (polar_dtype)dt, relu,
                                     static_cast<hipStream_t>(stream)));
}

size_t polar_select_gemm_workspace_bytes(int M) { return M <= 0 ? 0 : select_gemm_workspace_bytes(M); }

int polar_select_gemm_ws(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                         float *C, int M, int K, int N, int cap, int dt, int relu,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    if (M < 0 || K < 1 || N < 1 || cap < 0 || !dtype_ok(dt)) return POLAR_EINVAL;
    if (K % 128 != 0 || (long long)N * K > (1ll << 40)) return POLAR_EUNSUPPORTED;
    if (M == 0 || cap == 0) return POLAR_OK;
    if (!A || !W || !idx || !C) return POLAR_EINVAL;
    if (((uintptr_t)A & 15u) || ((uintptr_t)W & 15u) || ((uintptr_t)workspace & 15u)) return POLAR_EINVAL;
    return record(launch_select_gemm_ws(A, W, idx, count, C, M, K, N, cap, (polar_dtype)dt, relu, workspace,
                                        workspace ? workspace_bytes : 0, static_cast<hipStream_t>(stream)));
}

int polar_neuron_union(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                       int32_t *count_out, void *stream)
{
    if (B < 0 || kn < 0 || N < 1 || cap < 0) return POLAR_EINVAL;
    if (N > neuron_union_max_n()) return POLAR_EUNSUPPORTED;
    if (!count_out || (cap > 0 && !idx_out) || ((long long)B * kn > 0 && !topk)) return POLAR_EINVAL;
    return record(launch_neuron_union(topk, B, kn, N, cap, idx_out, count_out,
                                      static_cast<hipStream_t>(stream)));
}

static int check_down_sizes(int M, int Kout, int N, int cap)
{
    if (M < 0 || Kout < 1 || N < 1 || cap < 0) return POLAR_EINVAL;
    if (Kout % 256 != 0 || (long long)N * Kout > (1ll << 40) || (long long)M * cap >= (1ll << 40))
        return POLAR_EUNSUPPORTED;
    return POLAR_OK;
}

size_t polar_select_gemm_down_workspace_bytes(int M, int Kout, int cap)
{
    if (check_down_sizes(M, Kout, 1, cap) != POLAR_OK || M == 0) return 0;
    return select_gemm_down_workspace_bytes(M, Kout, cap);
}

int polar_select_gemm_down(const float *H, const void *W2, const int32_t *idx, const int32_t *count,
                           float *Y, int M, int Kout, int N, int cap, int dt, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    if (!dtype_ok(dt)) return POLAR_EINVAL;
    const int rc = check_down_sizes(M, Kout, N, cap);
    if (rc != POLAR_OK) return rc;
    if (M == 0) return POLAR_OK;
    if (!W2 || !Y || !workspace || (cap > 0 && (!H || !idx))) return POLAR_EINVAL;
    if (((uintptr_t)W2 & 15u) || ((uintptr_t)Y & 15u) || ((uintptr_t)workspace & 15u) || ((uintptr_t)H & 3u))
        return POLAR_EINVAL;
    if (workspace_bytes < select_gemm_down_workspace_bytes(M, Kout, cap)) return POLAR_EWORKSPACE;
    return record(launch_select_gemm_down(H, W2, idx, count, Y, M, Kout, N, cap, (polar_dtype)dt, workspace,
                                          static_cast<hipStream_t>(stream)));
}

static int check_mlp_sizes(int M, int D, int N, int cap)
{
    if (M < 0 || D < 1 || N < 1 || cap < 0) return POLAR_EINVAL;
    if (D % 256 != 0 || (long long)N * D > (1ll << 40) || (long long)M * cap >= (1ll << 40))
        return POLAR_EUNSUPPORTED;
    return POLAR_OK;
}

size_t polar_sparse_mlp_workspace_bytes(int M, int D, int cap)
{
    if (check_mlp_sizes(M, D, 1, cap) != POLAR_OK || M == 0) return 0;
    return sparse_mlp_workspace_bytes(M, D, cap);
}

int polar_sparse_mlp(const void *X, const void *W1, const void *W2, const int32_t *idx, const int32_t *count,
                     float *Y, int M, int D, int N, int cap, int dt, int relu, void *workspace,
                     size_t workspace_bytes, void *stream)
{
    if (!dtype_ok(dt)) return POLAR_EINVAL;
    const int rc = check_mlp_sizes(M, D, N, cap);
    if (rc != POLAR_OK) return rc;
    if (M == 0) return POLAR_OK;
    if (!W2 || !Y || !workspace || (cap > 0 && (!X || !W1 || !idx))) return POLAR_EINVAL;
    if (((uintptr_t)X & 15u) || ((uintptr_t)W1 & 15u) || ((uintptr_t)W2 & 15u) || ((uintptr_t)Y & 15u) ||
        ((uintptr_t)workspace & 255u))
        return POLAR_EINVAL;
    if (workspace_bytes < sparse_mlp_workspace_bytes(M, D, cap)) return POLAR_EWORKSPACE;
    return record(launch_sparse_mlp(X, W1, W2, idx, count, Y, M, D, N, cap, (polar_dtype)dt, relu, workspace,
                                    static_cast<hipStream_t>(stream)));
}

size_t polar_neuron_union_workspace_bytes(int B, int kn, int N)
{
    if (B < 0 || kn < 0 || N < 1 || N > neuron_union_max_n()) return 0;
    return neuron_union_workspace_bytes(B, kn, N);
}

int polar_neuron_union_ws(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                          int32_t *count_out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (B < 0 || kn < 0 || N < 1 || cap < 0) return POLAR_EINVAL;
    if (N > neuron_union_max_n()) return POLAR_EUNSUPPORTED;
    if (!count_out || (cap > 0 && !idx_out) || ((long long)B * kn > 0 && !topk)) return POLAR_EINVAL;
    if ((uintptr_t)workspace & 3u) return POLAR_EINVAL;
    return record(launch_neuron_union_ws(topk, B, kn, N, cap, idx_out, count_out, workspace,
                                         workspace ? workspace_bytes : 0, static_cast<hipStream_t>(stream)));
}

}  // extern "C"
