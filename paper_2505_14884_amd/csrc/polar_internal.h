// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "polar.h"

namespace polar {

// Current value of a process-wide option (polar_set_option): one relaxed atomic load.
int option(polar_option opt);

// Launch geometry of the split-KV attention kernels, derived on the host from sizes only
// (device-side seqlens are never read on the host).
struct ShaPlan {
    int G;            // query heads per KV head
    bool grouped_mfma; // the grouped-head matrix-core streaming kernel runs (G > 1, d = 128)
    int chunk;        // cache rows one workgroup of the streaming kernel covers
    int nsplit;       // chunks per (request, slot): ceil(S / chunk)
    bool direct;      // polar_sha_decode runs the streaming kernel alone (it finishes the output)
    size_t o_floats;  // floats in the partial-output region of the workspace
    size_t ml_floats; // floats in the (max, sum) region
    size_t bytes;     // total workspace bytes, 256-aligned
};

// Fills `plan`; returns POLAR_OK or the status the public calls must return for these sizes.
int make_sha_plan(int B, int Hq, int Hkv, int S, int d, int k, ShaPlan *plan);

// Launch geometry of the split-D router path.
struct RouterPlan {
    bool mfma;     // phase 1 on the fp64 matrix cores (tiles of 16 requests) or on the vector ALU (tiles of 2)
    int RT;        // request tiles
    int P;         // slices of the D axis
    int Dp;        // rows of Wr per slice
    size_t bytes;  // workspace bytes, 256-aligned
};
int make_router_plan(int B, int D, int H, RouterPlan *plan);

// Dynamic LDS beyond the default allowance has to be requested per kernel, on the device the
// launch goes to.  The request is made only when a launch needs more than any earlier launch of
// the same kernel on that device did, so steady-state calls (and calls recorded into a HIP graph
// after one warm-up call) issue launches only.  One LdsGrant per kernel, with static storage.
struct LdsGrant {
    static constexpr int kDevices = 64;          // devices remembered; beyond that, every call asks
    std::atomic<size_t> bytes[kDevices];
};
inline hipError_t ensure_dynamic_lds(const void *kernel, size_t lds, LdsGrant &grant)
{
    if (lds <= 48 * 1024) return hipSuccess;
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    std::atomic<size_t> *slot = dev >= 0 && dev < LdsGrant::kDevices ? &grant.bytes[dev] : nullptr;
    if (slot && lds <= slot->load(std::memory_order_acquire)) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e == hipSuccess && slot) slot->store(lds, std::memory_order_release);
    return e;
}

// Kernel launchers.  Arguments were validated by the caller; each returns the hipError_t of
// its launch.
// `direct_out` non-NULL (allowed only when plan.nsplit == 1): the streaming kernel normalises and
// writes the final output itself, and zero-fills the unselected heads, instead of leaving records
// for the merge kernel; the workspace is then not touched.
hipError_t launch_sha_partial(const void *q, const void *K, const void *V, const int32_t *seqlens,
                              const int32_t *head_idx, float *ws, float *direct_out,
                              const ShaPlan &plan, int B, int Hq, int Hkv, int S, int d, int k,
                              polar_dtype dt, polar_kv_layout layout, float scale_log2e,
                              hipStream_t stream);
// Grouped-query variant of the streaming kernel (G > 1, d = 128): both contractions on MFMA.
hipError_t launch_sha_partial_gqa(const void *q, const void *K, const void *V, const int32_t *seqlens,
                                  const int32_t *head_idx, float *ws, float *direct_out,
                                  const ShaPlan &plan, int B, int Hq, int Hkv, int S, int k,
                                  polar_dtype dt, polar_kv_layout layout, float scale_log2e,
                                  hipStream_t stream);

hipError_t launch_sha_merge(const int32_t *seqlens, const int32_t *head_idx, float *out,
                            const float *ws, const ShaPlan &plan, int B, int Hq, int Hkv, int S,
                            int d, int k, hipStream_t stream);
// Dense run's merge with the labeller's norm and ranking as its epilogue (out and norms_out nullable).
hipError_t launch_sha_merge_label(const int32_t *seqlens, float *out, int32_t *labels, float *norms_out,
                                  const float *ws, const ShaPlan &plan, int B, int Hq, int Hkv, int S, int d,
                                  int k_label, hipStream_t stream);
hipError_t launch_router_topk(const void *hidden, const void *Wr, int B, int D, int H, int k,
                              polar_dtype dt, int32_t *head_idx, float *logits_out,
                              hipStream_t stream);
hipError_t launch_router_split(const void *hidden, const void *Wr, int B, int D, int H, int k,
                               polar_dtype dt, const RouterPlan &plan, int32_t *head_idx,
                               float *logits_out, void *workspace, hipStream_t stream);

hipError_t launch_head_norm_topk(const float *attn_out, int B, int Hq, int Hkv, int d, int k,
                                 int32_t *head_idx, float *norms_out, hipStream_t stream);

hipError_t launch_select_gemm(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                              float *C, int M, int K, int N, int cap, polar_dtype dt, int relu,
                              hipStream_t stream);
// Wide-tile form (workspace of select_gemm_workspace_bytes(M) bytes or less; up to 128 rows of the
// batch per pass; falls back to the form above when the workspace is absent).
size_t select_gemm_workspace_bytes(int M);
int select_gemm_ws_max_rows();                   // rows of the batch the wide-tile form takes in one pass
hipError_t launch_select_gemm_ws(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                                 float *C, int M, int K, int N, int cap, polar_dtype dt, int relu,
                                 void *workspace, size_t workspace_bytes, hipStream_t stream);
// The same product with the output rounded to the storage type and laid out as the second factor's
// kernel reads it (H16 [M][cap rounded up to 32], zero beyond the live count and for invalid ids),
// for sizes and a workspace with which the evenly split form can run (ask first).
bool select_gemm_h16_applicable(int M, int K, int cap, size_t workspace_bytes);
hipError_t launch_select_gemm_h16(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                                  uint16_t *H16, int M, int K, int N, int cap, polar_dtype dt, int relu,
                                  void *workspace, size_t workspace_bytes, hipStream_t stream);
// Second MLP factor: Y = h16(H) * W2[idx,:] (Kout % 256 == 0; the workspace is required; up to 128
// rows of the batch per pass).
size_t select_gemm_down_workspace_bytes(int M, int Kout, int cap);
hipError_t launch_select_gemm_down(const float *H, const void *W2, const int32_t *idx, const int32_t *count,
                                   float *Y, int M, int Kout, int N, int cap, polar_dtype dt, void *workspace,
                                   hipStream_t stream);
// Both factors in one call: Y = h16(act(X W1[idx,:]^T)) W2[idx,:]; the hidden activations stay in
// the workspace in 16-bit form (D % 256 == 0; the workspace is required).
size_t sparse_mlp_workspace_bytes(int M, int D, int cap);
hipError_t launch_sparse_mlp(const void *X, const void *W1, const void *W2, const int32_t *idx,
                             const int32_t *count, float *Y, int M, int D, int N, int cap, polar_dtype dt,
                             int relu, void *workspace, hipStream_t stream);
int neuron_union_max_n();
hipError_t launch_neuron_union(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                               int32_t *count_out, hipStream_t stream);

// With a workspace of neuron_union_workspace_bytes(B, kn, N) bytes (0: the input is too small to
// split) several workgroups build the bitmap; without one this is launch_neuron_union.
size_t neuron_union_workspace_bytes(int B, int kn, int N);
hipError_t launch_neuron_union_ws(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                                  int32_t *count_out, void *workspace, size_t workspace_bytes,
                                  hipStream_t stream);

#if defined(__HIPCC__)
// Direct mode's zero fill, run by one wave of the workgroup of (request b, slot): that workgroup
// owns the KV heads h = slot, slot + k, slot + 2k, ... and stores +0.0 to the G query heads of
// every one of them that no entry of the request's head_idx row names (all of them when the
// request is empty).  The k workgroups of a request cover every head exactly once, and a head
// that some slot selected is written by that slot's workgroup, never here.  `id0` is the lane's
// entry of the row (entry `lane`, or -1 beyond k), loaded by the caller together with its other
// index loads; longer rows are re-read in 64-entry pieces.  Control flow is wave-uniform.
__device__ __forceinline__ void direct_zero_fill(const int32_t *__restrict__ head_idx_row, int id0,
                                                 bool any_selected, int slot, int k, int Hkv,
                                                 int group_floats, float *__restrict__ out_request,
                                                 int lane)
{
    for (int h = slot; h < Hkv; h += k) {
        bool member = false;
        if (any_selected) {
            member = __builtin_amdgcn_ballot_w64(id0 == h) != 0;
            for (int c = 64; c < k && !member; c += 64) {
                const int id = (c + lane < k) ? head_idx_row[c + lane] : -1;
                member = __builtin_amdgcn_ballot_w64(id == h) != 0;
            }
        }
        if (!member) {
            float4 *dst = reinterpret_cast<float4 *>(out_request + (size_t)h * group_floats);
            for (int i = lane; i < group_floats / 4; i += 64) dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
}
#endif

}  // namespace polar
