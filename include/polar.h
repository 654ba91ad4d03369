/*
 * polar.h — C ABI of the MI355X (gfx950) Selective Head Attention decode path.
 *
 * The library implements the batched decode-step hot path of Polar Sparsity:
 * a per-request attention-head router followed by attention over the selected
 * heads only.  Conventions shared by every entry point:
 *
 *  - Every array pointer is a DEVICE pointer owned by the caller.  The library
 *    never allocates, frees, copies to the host or synchronises; it validates
 *    the scalar arguments on the host (before any HIP call) and enqueues kernels
 *    on the caller's stream.  `stream` is a hipStream_t passed as void*; NULL is
 *    the default stream.
 *  - Return value: POLAR_OK (0) or a negative polar_status.  Nothing is printed,
 *    no exception crosses the boundary.  B == 0 is a successful no-op.
 *  - 16-bit storage: `dt` says whether hidden/Wr/q/K/V hold IEEE binary16
 *    (POLAR_F16) or bfloat16 (POLAR_BF16).  Accumulation is wider (see each call).
 *  - Enumerated arguments (`dt`: a polar_dtype, `layout`: a polar_kv_layout, `opt`: a
 *    polar_option) are declared `int`: the size of an enum type is the compiler's choice, an
 *    int's is not, and a value outside the enumeration is then an ordinary bad argument
 *    (POLAR_EINVAL), never undefined behaviour.
 *  - Device-side contents are not validated on the hot path; the behaviour for
 *    out-of-range contents is defined below and never reads or writes out of
 *    bounds.
 *  - Calls that share a workspace, or the same output, must be ordered on one
 *    stream (or by events); the library keeps no global mutable state besides
 *    the last HIP error code.
 */
#ifndef POLAR_H
#define POLAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { POLAR_F16 = 0, POLAR_BF16 = 1 } polar_dtype;

/* Memory layout of the K and V caches (Section 3.2 gives both: the main-text layout and, in
 * its footnote, the sequence-major one some implementations use). */
typedef enum {
    POLAR_KV_BHSD = 0, /* [B, Hkv, S, d]: the rows of one head are contiguous */
    POLAR_KV_BSHD = 1  /* [B, S, Hkv, d]: the heads of one row are contiguous */
} polar_kv_layout;

typedef enum {
    POLAR_OK = 0,
    POLAR_EINVAL = -1,       /* NULL pointer, negative size, k outside [1,H], Hq % Hkv != 0 ... */
    POLAR_EUNSUPPORTED = -2, /* a shape or dtype this build has no kernel for */
    POLAR_EWORKSPACE = -3,   /* workspace NULL, misaligned or smaller than required */
    POLAR_EHIP = -4          /* a HIP launch failed; see polar_last_hip_error() */
} polar_status;

/* Limits of this build (host-checked, POLAR_EUNSUPPORTED beyond them). */
#define POLAR_MAX_ROUTER_H 256    /* selection units a router may score */
#define POLAR_MAX_ROUTER_D 16384  /* router input width */
#define POLAR_MAX_GROUP 16        /* query heads per KV head: any 1..16 at d = 128; 1, 2, 4, 8 at d = 64 */

/*
 * Process-wide options.  Every option starts at 0, "the library's own choice", which is what
 * a user wants; the other values pin a kernel or a split granularity so that tests and sweeps
 * can reach every code path.  The library reads no environment variable.  An option is a plain
 * integer read (atomically) by each call; changing one while calls that share a workspace are
 * being made (for instance between polar_sha_partial and polar_sha_merge) changes the layout
 * the workspace is read with and is a caller error.  Workspace queries answer for the options
 * in force when they are asked.
 */
typedef enum {
    POLAR_OPT_SHA_CHUNK_ROWS = 0,     /* cache rows per workgroup of the streaming kernel: 0 auto, else 128..2^20
                                         (rounded up to a multiple of 128) */
    POLAR_OPT_SHA_FORM = 1,           /* 0 auto, 1 one kernel wherever the cache is unsplit, 2 always streaming + merge */
    POLAR_OPT_SHA_GROUPED_KERNEL = 2, /* grouped heads at d = 128: 0 matrix-core kernel, 1 vector-ALU kernel
                                         (group sizes 2, 4, 8 only: others become POLAR_EUNSUPPORTED) */
    POLAR_OPT_ROUTER_PATH = 3,        /* with a workspace: 0 auto, 1 one-kernel path, 2 split-D path */
    POLAR_OPT_ROUTER_PHASE1 = 4,      /* split-D phase 1: 0 auto, 1 vector ALU, 2 fp64 matrix cores */
    POLAR_OPT_GEMM_FORM = 5,          /* polar_select_gemm_ws / polar_sparse_mlp: 0 auto, 1 one-launch kernel */
    POLAR_OPT_GEMM_WORKGROUPS = 6,    /* launch width of the evenly split GEMM: 0 auto, else 1..256 */
    POLAR_OPT_UNION_FORM = 7,         /* polar_neuron_union_ws: 0 auto, 1 one-launch kernel, 2 split form (builders + emitters) */
    POLAR_OPT_COUNT_ = 8
} polar_option;
/* POLAR_EINVAL for an unknown option or a value outside the ranges above (nothing is changed). */
int polar_set_option(int opt, int value);
/* Current value of an option; POLAR_EINVAL for an unknown option or value == NULL. */
int polar_get_option(int opt, int *value);

/*
 * Attention-head router and per-request top-k (Section 4.2: the router is one fully
 * connected layer producing a scalar logit per head; the k highest-logit heads of each
 * request form the batch head index).
 *
 *   logit[b,h]  = sum_{i<D} hidden[b,i] * Wr[i,h]          no bias, no activation
 *   head_idx[b] = ids of the k largest logits of row b, best first; equal logits
 *                 (-0.0 equals +0.0) are ordered by ascending id; NaN logits rank
 *                 after every number and among themselves by id.
 *
 *   hidden     in   [B, D]  dt, row-major
 *   Wr         in   [D, H]  dt, row-major (H innermost).  H is the number of
 *                   selection units: heads for MHA, KV groups for GQA.
 *   head_idx   out  [B, k]  int32
 *   logits_out out  [B, H]  float, nullable: the logits rounded to float, for inspection.
 *
 *   workspace  nullable.  NULL: one workgroup per request does the whole row (no scratch
 *                   needed; at most B compute units busy).  Otherwise at least
 *                   polar_router_workspace_bytes(B, D, H) bytes, 256-byte aligned, contents
 *                   need no initialisation: the library may then split the D axis over many
 *                   workgroups that leave partial sums there, with a second small kernel adding
 *                   and ranking them; it does so when that is the faster path for the shape
 *                   (small batches of wide routers) and otherwise runs the one-kernel path.
 *
 * Products are exact and the sum over D is accumulated in double precision in a fixed,
 * column-independent order (a different fixed order with and without a workspace), so
 * identical columns of Wr give bit-identical logits and the result does not depend on launch
 * timing.  1 <= k <= H <= POLAR_MAX_ROUTER_H, 1 <= D <= POLAR_MAX_ROUTER_D.
 */
int polar_router_topk(const void *hidden, const void *Wr, int B, int D, int H, int k,
                      int dt, int32_t *head_idx, float *logits_out, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * Workspace queries, one style for every operation: `size_t polar_<op>_workspace_bytes(sizes)`
 * returns the bytes of device scratch the operation wants for these sizes, and 0 where there is
 * nothing to allocate: sizes the operation rejects (its own call reports the status), an empty
 * batch, or an input too small for the workspace form to pay.
 */
/* Bytes of device workspace the split path of polar_router_topk needs; 0 for invalid sizes. */
size_t polar_router_workspace_bytes(int B, int D, int H);

/*
 * Bytes of device workspace polar_sha_decode needs for these sizes (split-KV partial
 * results).  Returns 0 for invalid or unsupported sizes.  The workspace must be
 * 256-byte aligned; its contents need no initialisation and are undefined afterwards.
 */
size_t polar_sha_workspace_bytes(int B, int Hq, int Hkv, int S, int d, int k);

/*
 * Selective Head Attention, decode step (Section 3.2, the per-head attention equation;
 * Section 4.2 and Algorithm 1, Selective Head FlashAttention (decode); group sparsity
 * for GQA as in the last sentence of Section 4.2).
 *
 * For every request b and every selected KV head g = head_idx[b,t], and every query
 * head h of that group (h in [g*G, (g+1)*G), G = Hq/Hkv):
 *
 *   out[b,h,:] = softmax_j( scale * q[b,h,:] . K[b,g,j,:] ) @ V[b,g,j,:],   j in [0, n_b)
 *
 * with n_b = clamp(seqlens[b], 0, S).  Every other out[b,h',:] is written as +0.0
 * (heads that are not activated are masked to zero).  Only rows j < n_b of the selected
 * heads' K and V are read; no other K/V byte is touched.
 *
 *   q        in   [B, Hq, d]      dt
 *   K, V     in   [B, Hkv, S, d]  dt, contiguous; S is the cache capacity in rows
 *   seqlens  in   [B] int32       rows in use per request (the current token included)
 *   head_idx in   [B, k] int32    KV-head (group) ids; entries outside [0,Hkv) are
 *                                 skipped; duplicates are harmless.  NULL means dense
 *                                 attention and requires k == Hkv.
 *   out      out  [B, Hq, d] float; every element is written on every call.
 *   scale         softmax scale; 0 selects 1/sqrt(d).
 *   workspace     at least polar_sha_workspace_bytes(...) bytes, 256-byte aligned.
 *
 * q, K, V and out must be 16-byte aligned (the kernels use 16-byte accesses), else POLAR_EINVAL.
 * Scores, softmax statistics and the output are accumulated in float.  A request with
 * n_b == 0 gets zeros.  Supported: d in {64, 128}; G = Hq / Hkv in 1..16 at d = 128, in
 * {1, 2, 4, 8} at d = 64; 1 <= k <= Hkv.
 *
 * Launches (polar_sha_launches tells which): for an unsplit cache of moderate size one
 * kernel streams the rows, normalises, stores `out` and zero-fills the unselected heads, and
 * the workspace is left untouched; otherwise the streaming kernel leaves per-chunk records in
 * the workspace and a second small kernel combines them.  Both forms give the same bits.
 */
int polar_sha_decode(const void *q, const void *K, const void *V, const int32_t *seqlens,
                     const int32_t *head_idx, float *out, int B, int Hq, int Hkv, int S, int d,
                     int k, int dt, float scale, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * polar_sha_decode for callers that cannot allocate and have no workspace to pass: code that
 * runs under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, checks, kernels and result (bit for bit) as polar_sha_decode, minus the workspace:
 * the split-KV partial results go to a scratch array of POLAR_STATIC_SCRATCH_BYTES that lives in
 * the library's own device image (one copy per GPU, held until the process ends).  The call
 * allocates and frees nothing.  Sizes whose polar_sha_workspace_bytes exceed
 * POLAR_STATIC_SCRATCH_BYTES are refused with POLAR_EWORKSPACE (use polar_sha_decode with a
 * workspace of your own).  The scratch needs no clearing (the streaming kernel writes every
 * record the merge kernel reads) and keeps the previous call's contents.  Every call on one GPU
 * shares that GPU's array: calls that may overlap in time on one GPU (different streams, or
 * different threads) race and must be ordered by the caller.  The first call on a GPU looks up
 * the array's device address (with that GPU current); make it outside any graph capture, like
 * the first launch of any kernel.
 */
#define POLAR_STATIC_SCRATCH_BYTES (32u << 20)
int polar_sha_decode_static(const void *q, const void *K, const void *V, const int32_t *seqlens,
                            const int32_t *head_idx, float *out, int B, int Hq, int Hkv, int S, int d,
                            int k, int dt, float scale, void *stream);

/*
 * polar_sha_decode for either cache layout (Section 3.2, footnote: K, V in R^{B x N x Hkv x d}).
 * Identical to polar_sha_decode except that K and V are laid out as `layout` says; with
 * POLAR_KV_BSHD a selected head's rows are d contiguous values every Hkv*d, so the kernel
 * gathers 2*d-byte rows instead of streaming a contiguous slab.  q and out are unchanged
 * ([B, Hq, d]; with one query row per request both of the paper's q layouts coincide).
 */
int polar_sha_decode_layout(const void *q, const void *K, const void *V, const int32_t *seqlens,
                            const int32_t *head_idx, float *out, int B, int Hq, int Hkv, int S,
                            int d, int k, int dt, int layout, float scale,
                            void *workspace, size_t workspace_bytes, void *stream);

/*
 * The two phases of the split form of polar_sha_decode as separate launches, with the same
 * arguments and checks (partial followed by merge on one stream gives polar_sha_decode's
 * result bit for bit, also where polar_sha_decode itself takes its one-kernel form).  They
 * exist so a harness can time the KV-streaming phase by itself.
 *   polar_sha_partial: streams K/V of the selected heads in chunks of rows and leaves a
 *     running (max, sum, unnormalised output) per chunk in the workspace (Algorithm 1's
 *     recurrence applied per chunk).
 *   polar_sha_partial_layout: the same for either cache layout.
 *   polar_sha_merge: combines the chunks of each selected head with the same max/sum
 *     rescale, normalises, and writes zeros for unselected heads.
 */
int polar_sha_partial(const void *q, const void *K, const void *V, const int32_t *seqlens,
                      const int32_t *head_idx, int B, int Hq, int Hkv, int S, int d, int k,
                      int dt, float scale, void *workspace, size_t workspace_bytes,
                      void *stream);
int polar_sha_partial_layout(const void *q, const void *K, const void *V, const int32_t *seqlens,
                             const int32_t *head_idx, int B, int Hq, int Hkv, int S, int d, int k,
                             int dt, int layout, float scale, void *workspace,
                             size_t workspace_bytes, void *stream);
int polar_sha_merge(const int32_t *seqlens, const int32_t *head_idx, float *out, int B, int Hq,
                    int Hkv, int S, int d, int k, const void *workspace, size_t workspace_bytes,
                    void *stream);

/*
 * Rows of the KV cache one workgroup of the streaming phase covers for these sizes
 * (the split granularity the workspace size is computed from).  0 for invalid sizes.
 */
int polar_sha_chunk_rows(int B, int Hq, int Hkv, int S, int d, int k);

/*
 * Kernels polar_sha_decode launches for these sizes: 1 (an unsplit cache finished by the
 * streaming kernel alone) or 2 (streaming kernel + merge kernel); 0 for invalid sizes.  For
 * harnesses that attribute time to kernels; results do not depend on it.
 */
int polar_sha_launches(int B, int Hq, int Hkv, int S, int d, int k);

/*
 * Head-importance labels (Section 3.2: heads ranked by the L2 norm of their attention output;
 * Section 4.2: the k heads with the highest output norms are the router's training targets).
 *
 *   attn_out   in   [B, Hq, d] float: dense decode attention output, e.g. from
 *                   polar_sha_decode(..., head_idx = NULL, k = Hkv, ...)
 *   head_idx   out  [B, k] int32: the k selection units (KV groups; heads when Hq == Hkv) of
 *                   each request with the largest output norm, best first
 *   norms_out  out  [B, Hkv] float, nullable: the L2 norms, for inspection
 *
 * A group's score is the sum of squares of the outputs of all its Hq/Hkv query heads
 * (accumulated in double; ranking by the sum of squares is ranking by the norm, without the
 * rounding of a square root); ordering and tie rules are those of polar_router_topk.
 * 1 <= k <= Hkv <= POLAR_MAX_ROUTER_H.
 */
int polar_head_norm_topk(const float *attn_out, int B, int Hq, int Hkv, int d, int k,
                         int32_t *head_idx, float *norms_out, void *stream);

/*
 * The same labels straight from the caches (Section 3.2: dense attention, heads ranked by the L2
 * norm of their output; Section 4.2: the k best are the router's targets): dense decode attention
 * whose merge step takes the norms and ranks them as its epilogue, so no pass over a stored
 * output is needed.  Two launches: the streaming kernel of polar_sha_decode (k = Hkv, per-chunk
 * records) and one merge kernel with one workgroup per request.
 *
 *   q, K, V, seqlens, S, d, dt, layout, scale   as for polar_sha_decode_layout (dense: every head)
 *   labels     out  [B, k_label] int32, as head_idx of polar_head_norm_topk
 *   norms_out  out  [B, Hkv] float, nullable
 *   attn_out   out  [B, Hq, d] float, nullable: the dense attention output, bit-identical to
 *                   polar_sha_decode's (head_idx = NULL); 16-byte aligned
 *   workspace       at least polar_sha_workspace_bytes(B, Hq, Hkv, S, d, Hkv) bytes, 256-byte aligned
 *
 * The norm of a group is taken over the float values attn_out holds (or would hold), squares
 * and sums in double in a fixed order; ordering and tie rules are those of polar_router_topk.
 * 1 <= k_label <= Hkv <= POLAR_MAX_ROUTER_H.
 */
int polar_head_labels(const void *q, const void *K, const void *V, const int32_t *seqlens, int32_t *labels,
                      float *norms_out, float *attn_out, int B, int Hq, int Hkv, int S, int d, int k_label, int dt,
                      int layout, float scale, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Selective (fused-gather) GEMM (Appendix "Sparse Kernels", Algorithm 3; Section 3.1, the
 * first factor sigma(x W_{1,S_B}) of the sparsified MLP; Section 4.1).
 *
 *   C[m, j] = act( sum_{k<K} A[m,k] * W[idx[j], k] )   for m < M, j < count
 *
 *   A      in   [M, K] dt      activations (one row per request)
 *   W      in   [N, K] dt      weights, one contiguous row of K values per neuron
 *   idx    in   [cap] int32    neuron index; ids outside [0,N) give a zero column
 *   count  in   [1] int32, nullable, DEVICE pointer: number of live entries of idx (clamped to
 *               [0, cap]); NULL means all cap entries are live.  Lets the index be built on
 *               the device (polar_neuron_union) without a host round trip.
 *   C      out  [M, cap] float, row-major with leading dimension cap; columns at or beyond
 *               the live count are not written.
 *   relu        non-zero: act = max(., 0); zero: identity.
 *
 * 16-bit inputs, float accumulation on the matrix cores, float output.  K must be a multiple
 * of 128; A and W 16-byte aligned.  M > 256 is processed 256 rows at a time.
 */
int polar_select_gemm(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                      float *C, int M, int K, int N, int cap, int dt, int relu, void *stream);

/*
 * The same operation with a workspace (Appendix "Sparse Kernels", Algorithm 3; same arguments,
 * same result up to the order of the float additions).  The library then runs a form built for
 * decode batches: 128-neuron tiles and a fixed-size launch whose workgroups split the (neuron
 * tile, K block) work evenly whatever the live count is, followed by a small kernel that adds
 * the pieces of each tile in a fixed order (two launches per 128 rows of the batch: M > 128 is
 * processed 128 rows at a time; results are reproducible for given sizes, count and workspace
 * size).  With workspace NULL, with K not a multiple of 256 or with cap beyond 196608 it runs
 * the kernel of polar_select_gemm.
 *   workspace        scratch, DEVICE pointer, 16-byte aligned, caller-owned; contents are
 *                    overwritten; calls that overlap in time need separate workspaces
 *   workspace_bytes  its size; polar_select_gemm_workspace_bytes(M) gives the size at which
 *                    the launch is as wide as the library wants it (it grows with M up to
 *                    128 rows; 0 for M <= 0); a smaller workspace narrows the launch, it is
 *                    not an error
 */
size_t polar_select_gemm_workspace_bytes(int M);
int polar_select_gemm_ws(const void *A, const void *W, const int32_t *idx, const int32_t *count,
                         float *C, int M, int K, int N, int cap, int dt, int relu,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * Second factor of the sparsified MLP (Section 3.1: MLP_{S_B}(x) = sigma(x W_{1,S_B}) W_{2,S_B}^T;
 * Section 4.1 and Appendix "Sparse Kernels": indexing fused into the product, weights stored one
 * contiguous row per neuron).  The gather runs along the contraction axis:
 *
 *   Y[m, c] = sum_{j < live} h16(Hact[m, j]) * W2[idx[j], c]
 *
 *   Hact   in   [M, cap] float, row-major with leading dimension cap: the selected neurons'
 *               activations, as polar_select_gemm[_ws] writes them.  h16: each value is rounded
 *               to dt (nearest, ties to even) before the multiply, as a 16-bit model holds it.
 *               Columns at or beyond the live count are not read.  4-byte aligned.
 *   W2     in   [N, Kout] dt: row n holds neuron n's Kout output weights.  16-byte aligned.
 *   idx    in   [cap] int32 neuron ids, position j pairs with column j of Hact; an id outside
 *               [0,N) contributes nothing
 *   count  in   [1] int32, nullable, DEVICE pointer: live entries of idx (clamped to [0, cap]);
 *               NULL means all cap
 *   Y      out  [M, Kout] float, row-major; every element is written (zeros when nothing is
 *               live).  16-byte aligned.
 *   workspace   required scratch, DEVICE pointer, 16-byte aligned, caller-owned, at least
 *               polar_select_gemm_down_workspace_bytes(M, Kout, cap) bytes (else POLAR_EWORKSPACE);
 *               contents are overwritten; calls that overlap in time need separate workspaces
 *
 * 16-bit operands, float accumulation on the matrix cores, float output.  Kout a multiple of
 * 256, else POLAR_EUNSUPPORTED.  Three launches per 128 rows of the batch (M > 128 is processed
 * 128 rows at a time; up to 64 rows and 65 to 128 rows run different kernels); the contraction
 * is cut into ranges whose sums are added in a fixed order, so results are reproducible for
 * given sizes and count.
 * Hact and idx may be NULL when cap == 0.
 */
size_t polar_select_gemm_down_workspace_bytes(int M, int Kout, int cap);
int polar_select_gemm_down(const float *Hact, const void *W2, const int32_t *idx, const int32_t *count,
                           float *Y, int M, int Kout, int N, int cap, int dt, void *workspace,
                           size_t workspace_bytes, void *stream);

/*
 * The sparsified MLP in one call (Section 3.1: MLP_{S_B}(x) = sigma(x W_{1,S_B}) W_{2,S_B}^T over
 * the batch's union S_B of active neurons; Section 4.1: both factors gather by the same index):
 *
 *   Y[m, c] = sum_{j < live} h16( act( sum_k X[m, k] * W1[idx[j], k] ) ) * W2[idx[j], c]
 *
 * i.e. polar_select_gemm_ws followed by polar_select_gemm_down, with the hidden activations kept
 * in the workspace in the 16-bit form the second factor reads (the first factor's reduction
 * writes them rounded, masked and padded; no float copy, no separate conversion launch).  The
 * result is bit-identical to that of the two calls made one after the other.
 *
 *   X      in   [M, D] dt, row-major.  16-byte aligned.
 *   W1     in   [N, D] dt: row n holds neuron n's D input weights.  16-byte aligned.
 *   W2     in   [N, D] dt: row n holds neuron n's D output weights.  16-byte aligned.
 *   idx    in   [cap] int32 neuron ids; an id outside [0,N) contributes nothing
 *   count  in   [1] int32, nullable, DEVICE pointer: live entries of idx (clamped to [0, cap]);
 *               NULL means all cap
 *   Y      out  [M, D] float, row-major; every element is written (zeros when nothing is live).
 *               16-byte aligned.
 *   relu        nonzero: act = max(., 0); zero: identity
 *   workspace   required scratch, DEVICE pointer, 256-byte aligned, caller-owned, at least
 *               polar_sparse_mlp_workspace_bytes(M, D, cap) bytes (else POLAR_EWORKSPACE);
 *               contents are overwritten; calls that overlap in time need separate workspaces
 *
 * D a multiple of 256, else POLAR_EUNSUPPORTED.  Four launches for up to 128 rows; larger
 * batches go through 128 rows at a time, re-reading the gathered rows.  Where the first factor's
 * evenly split form cannot run (see polar_select_gemm_ws) its one-launch kernel and the
 * conversion launch take its place, with the same result.  X, W1 and idx may be NULL when
 * cap == 0.
 */
size_t polar_sparse_mlp_workspace_bytes(int M, int D, int cap);
int polar_sparse_mlp(const void *X, const void *W1, const void *W2, const int32_t *idx, const int32_t *count,
                     float *Y, int M, int D, int N, int cap, int dt, int relu, void *workspace,
                     size_t workspace_bytes, void *stream);

/*
 * Batch neuron index (Section 4.1: the predicted activations of all requests are aggregated
 * into one index tensor; Section 3.1: the union set S_B).
 *
 *   topk       in   [B, kn] int32: each request's predicted neuron ids (any order; ids outside
 *                   [0,N) are ignored)
 *   idx_out    out  [cap] int32: the distinct ids in ascending order (first min(count, cap))
 *   count_out  out  [1] int32: number of distinct ids, clamped to cap
 *
 * N <= 524288.  One launch, deterministic, no workspace: from a thousand ids on, sixteen
 * workgroups each mark all the ids in a bitmap of their own (cheap to repeat) and emit a
 * sixteenth of the output (the slow part), so no workgroup waits for another.
 */
int polar_neuron_union(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                       int32_t *count_out, void *stream);

/*
 * The same index with a workspace (Section 4.1; same arguments, same result), for very large
 * inputs: several workgroups each mark their SHARE of the ids in a bitmap of their own, stored
 * to the workspace, and a last launch ORs the bitmaps, counts and emits (two launches,
 * deterministic).  Worth its second launch only where marking all ids in every workgroup gets
 * expensive (from about a hundred thousand ids); for smaller inputs, workspace NULL or a
 * workspace too small for two bitmaps it runs the one-launch kernel of polar_neuron_union.
 *   workspace        scratch, DEVICE pointer, 4-byte aligned, caller-owned; contents are
 *                    overwritten; calls that overlap in time need separate workspaces
 *   workspace_bytes  its size; polar_neuron_union_workspace_bytes(B, kn, N) gives the size the
 *                    library wants (0: the one-launch kernel is the faster one for this input)
 */
size_t polar_neuron_union_workspace_bytes(int B, int kn, int N);
int polar_neuron_union_ws(const int32_t *topk, int B, int kn, int N, int cap, int32_t *idx_out,
                          int32_t *count_out, void *workspace, size_t workspace_bytes, void *stream);

/* Text for a polar_status value; never NULL. */
const char *polar_strerror(int status);
/* The hipError_t (as int) recorded by the most recent POLAR_EHIP on this thread; 0 if none. */
int polar_last_hip_error(void);
/* ABI version: major * 1000 + minor.  2000: options (polar_set_option / polar_get_option) replace the
 * environment switches; every workspace query returns size_t; the read yardsticks moved to their own
 * library (polar_probe.h); q, K, V and out of the attention calls must be 16-byte aligned.
 * 2100: adds polar_sha_decode_static.  2200: adds polar_head_labels.  2300: POLAR_OPT_UNION_FORM. */
int polar_version(void);
/* Hash of the source files this binary was built from (set by the build script; "unknown" for a
 * build made without it).  Lets a loader refuse a binary older than the sources beside it. */
const char *polar_source_hash(void);

#ifdef __cplusplus
}
#endif
#endif /* POLAR_H */
