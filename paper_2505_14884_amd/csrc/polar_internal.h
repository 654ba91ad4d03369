// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "polar.h"

namespace polar {

// Launch geometry of the split-KV attention kernels, derived on the host from sizes only
// (device-side seqlens are never read on the host).
struct ShaPlan {
    int G;            // query heads per KV head
    int chunk;        // cache rows one workgroup of the streaming kernel covers
    int nsplit;       // chunks per (request, slot): ceil(S / chunk)
    size_t o_floats;  // floats in the partial-output region of the workspace
    size_t ml_floats; // floats in the (max, sum) region
    size_t bytes;     // total workspace bytes, 256-aligned
};

// Fills `plan`; returns POLAR_OK or the status the public calls must return for these sizes.
int make_sha_plan(int B, int Hq, int Hkv, int S, int d, int k, ShaPlan *plan);

// Launch geometry of the split-D router path.
struct RouterPlan {
    int RT;        // request tiles (kTileR requests each)
    int P;         // slices of the D axis
    int Dp;        // rows of Wr per slice
    size_t bytes;  // workspace bytes, 256-aligned
};
int make_router_plan(int B, int D, int H, RouterPlan *plan);

// Kernel launchers.  Arguments were validated by the caller; each returns the hipError_t of
// its launch.
hipError_t launch_sha_partial(const void *q, const void *K, const void *V, const int32_t *seqlens,
                              const int32_t *head_idx, float *ws, const ShaPlan &plan, int B,
                              int Hq, int Hkv, int S, int d, int k, polar_dtype dt,
                              polar_kv_layout layout, float scale_log2e, hipStream_t stream);
// Grouped-query variant of the streaming kernel (G > 1, d = 128): both contractions on MFMA.
hipError_t launch_sha_partial_gqa(const void *q, const void *K, const void *V, const int32_t *seqlens,
                                  const int32_t *head_idx, float *ws, const ShaPlan &plan, int B,
                                  int Hq, int Hkv, int S, int k, polar_dtype dt,
                                  polar_kv_layout layout, float scale_log2e, hipStream_t stream);
hipError_t launch_sha_merge(const int32_t *seqlens, const int32_t *head_idx, float *out,
                            const float *ws, const ShaPlan &plan, int B, int Hq, int Hkv, int S,
                            int d, int k, hipStream_t stream);
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
int neuron_union_max_n();
hipError_t launch_neuron_union(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                               int32_t *count_out, hipStream_t stream);

}  // namespace polar
