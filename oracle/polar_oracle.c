/*
 * polar_oracle.c — CPU oracle for batched decode-step Selective Head Attention.
 *
 * TEST INFRASTRUCTURE, NOT PRODUCT.  Only the tests, the smoke check and the
 * bench's cpu_baseline leg may call this.  It shares no code with the HIP
 * library: no common header, helper, table or conversion routine.
 *
 * Everything is the plain definition written out in double precision, reading
 * the same 16-bit (fp16 / bf16) input bits the GPU reads, widened exactly:
 *
 *   router      logit[b,h] = sum_i hidden[b,i] * Wr[i,h]              (Section 4.2: the
 *               attention router is one fully connected layer that emits a scalar per head)
 *   top-k       per request keep the k heads with the largest logits   (Section 4.2)
 *   attention   softmax(q K^T / sqrt(d_h)) V per (request, head)       (Section 3.2, the
 *               per-head attention equation), evaluated two-pass: all scores, their
 *               maximum, the exponentials, the weighted mean of V.  No tiling, no
 *               online update, no blocking.
 *   masking     heads that are not selected produce exactly +0.0       (Section 3.2, the
 *               head-sparsity study masks non-activated heads to zero; Algorithm 1 writes
 *               only the activated heads)
 *   GQA         the selection unit is a KV group; every query head of a selected group
 *               is computed against that group's K/V                   (Section 4.2, last
 *               sentence: group sparsity for grouped-query attention)
 *
 *   labels      the k heads (groups) whose attention output has the largest L2 norm
 *               (Section 3.2 study; Section 4.2, router supervision targets)
 *
 *   select GEMM C = act(A W[idx,:]^T) with the rows of W gathered by a neuron index, and the
 *               batch union of predicted neuron ids that forms that index (Section 3.1,
 *               Section 4.1, Appendix "Sparse Kernels" Algorithm 3)
 *
 * A second routine, oracle_alg1_tiled, evaluates one head tile by tile, as a
 * left fold of an associative "softmax state" combination over tiles of B_c
 * rows (what Algorithm 1, Selective Head FlashAttention (decode), does with its
 * running maximum and sum and its per-tile renormalised output), so a test can
 * show that the tiled evaluation and the two-pass definition agree.
 *
 * Readings where the paper is silent (kept in step with the design notes):
 *   - head ids come out ordered by descending logit; equal logits (-0.0 == +0.0)
 *     are ordered by ascending head id; NaN logits rank after every number and
 *     among themselves by id.
 *   - no bias and no sigmoid in the router (monotone, cannot change the top-k).
 *   - seqlens[b] is clamped to [0, S]; a request of length 0 yields zeros.
 *   - head_idx entries outside [0, Hkv) are ignored; duplicates are harmless.
 *   - the current token is already in the cache; one query row attends all
 *     n_b rows; no causal mask.
 *   - scale = 1/sqrt(d) when the caller passes 0.
 *
 * OpenMP, when compiled in, only spreads independent (request, slot) units
 * over threads; each unit's arithmetic is the same scalar loop.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* IEEE binary16 bit pattern -> double, exact. */
static double widen_f16(uint16_t bits)
{
    int sign = bits >> 15;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);              /* zero and subnormals */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp((double)(frac + 1024), expo - 25);
    return sign ? -v : v;
}

/* bfloat16 bit pattern -> double, exact: it is the top half of a binary32. */
static double widen_bf16(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double widen(uint16_t bits, int dt)
{
    return dt == ORACLE_BF16 ? widen_bf16(bits) : widen_f16(bits);
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* Widen n 16-bit values; lets a test check the decoders against numpy. */
int oracle_widen16(const uint16_t *in, long n, int dt, double *out)
{
    if (!in || !out || n < 0 || (dt != ORACLE_F16 && dt != ORACLE_BF16)) return -1;
    for (long i = 0; i < n; ++i) out[i] = widen(in[i], dt);
    return 0;
}

/* Router (Section 4.2): logits[b,h] = sum_{i<D} hidden[b,i] * Wr[i,h], i ascending.
 * hidden is [B,D] row-major, Wr is [D,H] row-major (H innermost). */
int oracle_router_logits(const uint16_t *hidden, const uint16_t *Wr, int B, int D, int H,
                         int dt, double *logits)
{
    if (!hidden || !Wr || !logits || B < 0 || D < 1 || H < 1) return -1;
    if (dt != ORACLE_F16 && dt != ORACLE_BF16) return -1;
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            double acc = 0.0;
            for (int i = 0; i < D; ++i)
                acc += widen(hidden[(size_t)b * D + i], dt) * widen(Wr[(size_t)i * H + h], dt);
            logits[(size_t)b * H + h] = acc;
        }
    return 0;
}

struct scored { double v; int id; };

/* Total order "a ranks before b": larger logit first, equal logits by lower id,
 * NaN after every number. */
static int rank_cmp(const void *pa, const void *pb)
{
    const struct scored *a = pa, *b = pb;
    int an = isnan(a->v), bn = isnan(b->v);
    if (an != bn) return an ? 1 : -1;
    if (!an) {
        if (a->v > b->v) return -1;
        if (a->v < b->v) return 1;
    }
    return (a->id > b->id) - (a->id < b->id);
}

/* Top-k (Section 4.2): sort each row's heads by (logit descending, id ascending)
 * and keep the first k ids, in that order. */
int oracle_topk(const double *logits, int B, int H, int k, int32_t *head_idx)
{
    if (!logits || !head_idx || B < 0 || H < 1 || k < 1 || k > H) return -1;
    struct scored *row = malloc(sizeof *row * (size_t)H);
    if (!row) return -2;
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            row[h].v = logits[(size_t)b * H + h];
            row[h].id = h;
        }
        qsort(row, (size_t)H, sizeof *row, rank_cmp);
        for (int t = 0; t < k; ++t) head_idx[(size_t)b * k + t] = row[t].id;
    }
    free(row);
    return 0;
}

/* One query row against n cached rows (the per-head attention equation of
 * Section 3.2): two passes over the scores, then the weighted mean of V. */
static void attend_one(const uint16_t *q, const uint16_t *K, const uint16_t *V, int n, int d,
                       int dt, double scale, double *score, double *out)
{
    double M = -INFINITY;
    for (int j = 0; j < n; ++j) {
        double s = 0.0;
        for (int e = 0; e < d; ++e)
            s += widen(q[e], dt) * widen(K[(size_t)j * d + e], dt);
        s *= scale;
        score[j] = s;
        if (s > M) M = s;
    }
    double denom = 0.0;
    for (int j = 0; j < n; ++j) {
        score[j] = exp(score[j] - M);
        denom += score[j];
    }
    for (int e = 0; e < d; ++e) {
        double acc = 0.0;
        for (int j = 0; j < n; ++j)
            acc += score[j] * widen(V[(size_t)j * d + e], dt);
        out[e] = acc / denom;
    }
}

/* Selective head attention for a batch (Sections 3.2 and 4.2).
 *   q [B,Hq,d], K and V [B,Hkv,S,d] 16-bit; seqlens [B]; head_idx [B,k] KV-head
 *   (group) ids, or NULL for dense attention with k == Hkv; out [B,Hq,d] double.
 * Every element of out is written: selected heads get attention, the rest +0.0. */
int oracle_sha_decode(const uint16_t *q, const uint16_t *K, const uint16_t *V,
                      const int32_t *seqlens, const int32_t *head_idx, double *out,
                      int B, int Hq, int Hkv, int S, int d, int k, int dt, double scale)
{
    if (!q || !K || !V || !seqlens || !out) return -1;
    if (B < 0 || Hq < 1 || Hkv < 1 || S < 1 || d < 1 || k < 1 || k > Hkv) return -1;
    if (Hq % Hkv != 0) return -1;
    if (!head_idx && k != Hkv) return -1;
    if (dt != ORACLE_F16 && dt != ORACLE_BF16) return -1;
    const int G = Hq / Hkv;
    if (scale == 0.0) scale = 1.0 / sqrt((double)d);
    for (size_t i = 0; i < (size_t)B * Hq * d; ++i) out[i] = 0.0;

    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel
#endif
    {
        double *score = malloc(sizeof *score * (size_t)S);
        if (!score) {
#ifdef _OPENMP
#pragma omp atomic write
#endif
            failed = 1;
        }
#ifdef _OPENMP
#pragma omp for collapse(2) schedule(dynamic, 1)
#endif
        for (int b = 0; b < B; ++b)
            for (int t = 0; t < k; ++t) {
                if (!score) continue;
                int n = seqlens[b];
                if (n < 0) n = 0;
                if (n > S) n = S;
                if (n == 0) continue;
                int g = head_idx ? head_idx[(size_t)b * k + t] : t;
                if (g < 0 || g >= Hkv) continue;
                /* A duplicate id recomputes the same values; skip all but its first slot
                 * so two threads never write one output row. */
                int first = 1;
                if (head_idx)
                    for (int u = 0; u < t; ++u)
                        if (head_idx[(size_t)b * k + u] == g) first = 0;
                if (!first) continue;
                const uint16_t *Kg = K + ((size_t)b * Hkv + g) * (size_t)S * d;
                const uint16_t *Vg = V + ((size_t)b * Hkv + g) * (size_t)S * d;
                for (int r = 0; r < G; ++r) {
                    int h = g * G + r;   /* query heads of group g are contiguous */
                    attend_one(q + ((size_t)b * Hq + h) * d, Kg, Vg, n, d, dt, scale, score,
                               out + ((size_t)b * Hq + h) * d);
                }
            }
        free(score);
    }
    return failed ? -2 : 0;
}

/* Head importance (Section 3.2: heads ranked by the L2 norm of their attention output;
 * Section 4.2: the k heads with the highest output norms are the router's labels).
 * attn [B,Hq,d] is dense attention output in double (oracle_sha_decode with head_idx NULL).
 * score[b,g] = sum of squares over the G = Hq/Hkv query heads of group g (the squared L2 norm
 * of the group's concatenated output); norms[b,g] = sqrt(score).  Ranking is done on the
 * scores (same order as the norms, no rounding of the root). */
int oracle_head_scores(const double *attn, int B, int Hq, int Hkv, int d, double *score,
                       double *norms)
{
    if (!attn || !score || B < 0 || Hq < 1 || Hkv < 1 || d < 1 || Hq % Hkv != 0) return -1;
    const int G = Hq / Hkv;
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g) {
            double ss = 0.0;
            for (int r = 0; r < G; ++r)
                for (int e = 0; e < d; ++e) {
                    double v = attn[((size_t)b * Hq + (size_t)g * G + r) * d + e];
                    ss += v * v;
                }
            score[(size_t)b * Hkv + g] = ss;
            if (norms) norms[(size_t)b * Hkv + g] = sqrt(ss);
        }
    return 0;
}

/* Neuron index tensor (Section 4.1: at inference the predicted activations are aggregated
 * across the batch into a single index of the neurons that are active for any request;
 * Section 3.1: the union set S_B).  topk [B,kn] holds each request's predicted neuron ids;
 * the result is the ascending list of distinct ids in [0,N) (others are ignored). */
int oracle_neuron_union(const int32_t *topk, int B, int kn, int N, int32_t *out, int32_t *count)
{
    if (!topk || !out || !count || B < 0 || kn < 0 || N < 1) return -1;
    unsigned char *seen = calloc((size_t)N, 1);
    if (!seen) return -2;
    for (size_t i = 0; i < (size_t)B * kn; ++i)
        if (topk[i] >= 0 && topk[i] < N) seen[topk[i]] = 1;
    int32_t c = 0;
    for (int n = 0; n < N; ++n)
        if (seen[n]) out[c++] = n;
    *count = c;
    free(seen);
    return 0;
}

/* Selective (fused-gather) GEMM (Appendix "Sparse Kernels", Algorithm 3; Section 3.1, the
 * first factor sigma(x W_{1,S_B}) of the sparsified MLP): the rows of the weight matrix named
 * by the index vector are gathered and multiplied with the activations, then the activation
 * function is applied.
 *   A [M,K] 16-bit activations; W [N,K] 16-bit, one contiguous row of K weights per neuron;
 *   idx [n_sel] neuron ids;  C [M,n_sel] double:
 *   C[m,j] = act( sum_{k<K} A[m,k] * W[idx[j],k] ),  act = ReLU when relu != 0, else identity.
 * An id outside [0,N) gives a zero column. */
int oracle_select_gemm(const uint16_t *A, const uint16_t *W, const int32_t *idx, int M, int K,
                       int N, int n_sel, int dt, int relu, double *C)
{
    if (!A || !W || !idx || !C || M < 0 || K < 1 || N < 1 || n_sel < 0) return -1;
    if (dt != ORACLE_F16 && dt != ORACLE_BF16) return -1;
    for (int m = 0; m < M; ++m)
        for (int j = 0; j < n_sel; ++j) {
            double acc = 0.0;
            int n = idx[j];
            if (n >= 0 && n < N) {
                for (int k = 0; k < K; ++k)
                    acc += widen(A[(size_t)m * K + k], dt) * widen(W[(size_t)n * K + k], dt);
                if (relu && !(acc > 0.0)) acc = 0.0;
            }
            C[(size_t)m * n_sel + j] = acc;
        }
    return 0;
}

/* Nearest value of the 16-bit storage type to v, ties to even, as a double (what a 16-bit
 * model holds after it stores an activation).  binary16 has 11 significant bits, exponents down
 * to 2^-14 and subnormals in steps of 2^-24; bfloat16 has 8 significant bits on binary32's
 * exponent range (subnormal step 2^-133).  rint() rounds to even in the default mode. */
static double round_to_storage(double v, int dt)
{
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    const int digits = dt == ORACLE_BF16 ? 8 : 11;
    const int min_step = dt == ORACLE_BF16 ? -133 : -24;
    const double largest = dt == ORACLE_BF16 ? ldexp(255.0, 120) : 65504.0;
    int e;
    (void)frexp(v, &e);                            /* |v| in [2^(e-1), 2^e) */
    int step = e - digits;                         /* spacing of the type's values there */
    if (step < min_step) step = min_step;
    double r = ldexp(rint(ldexp(v, -step)), step);
    if (fabs(r) > largest) r = copysign(INFINITY, v);
    return r;
}

/* Second factor of the sparsified MLP (Section 3.1: MLP_{S_B}(x) = sigma(x W_{1,S_B}) W_{2,S_B}^T,
 * the sum running over the neurons of S_B only):
 *   H [M,n_sel] float: the activations of the selected neurons (the first factor's output);
 *   W2 [N,Kout] 16-bit, one contiguous row of Kout weights per neuron (the layout of Appendix
 *   "Sparse Kernels"); idx [n_sel] neuron ids;  Y [M,Kout] double:
 *   Y[m,c] = sum_{j<n_sel} h16(H[m,j]) * W2[idx[j],c],
 * h16 = the activation as the 16-bit model stores it (rounded to the storage type, ties to even).
 * An id outside [0,N) contributes nothing; an id that appears twice contributes twice. */
int oracle_select_gemm_down(const float *H, const uint16_t *W2, const int32_t *idx, int M, int Kout,
                            int N, int n_sel, int dt, double *Y)
{
    if (!Y || M < 0 || Kout < 1 || N < 1 || n_sel < 0) return -1;
    if (n_sel > 0 && (!H || !W2 || !idx)) return -1;
    if (dt != ORACLE_F16 && dt != ORACLE_BF16) return -1;
    for (int m = 0; m < M; ++m)
        for (int c = 0; c < Kout; ++c) {
            double acc = 0.0;
            for (int j = 0; j < n_sel; ++j) {
                int n = idx[j];
                if (n < 0 || n >= N) continue;
                acc += round_to_storage((double)H[(size_t)m * n_sel + j], dt) *
                       widen(W2[(size_t)n * Kout + c], dt);
            }
            Y[(size_t)m * Kout + c] = acc;
        }
    return 0;
}

/* Tile-by-tile attention for ONE already-gathered head, as a fold of "softmax states".
 *
 * A state summarises attention over a set of cache rows: `top`, the largest scaled score in the
 * set; `mass`, the sum of exp(score - top) over the set; `mean`, the attention output over the
 * set, i.e. the exp-weighted mean of its V rows (already divided by mass).  Two states over
 * disjoint sets combine into the state of the union:
 *     top = max(top_a, top_b),  w_x = mass_x * exp(top_x - top),
 *     mass = w_a + w_b,         mean = (w_a * mean_a + w_b * mean_b) / mass.
 * The empty set is the identity (top = -inf, mass = 0).  Folding this combination from the left
 * over consecutive tiles of Bc rows, each tile's own state computed by the plain two-pass
 * definition, is what Algorithm 1 (Selective Head FlashAttention, decode) does with its running
 * maximum, running sum and per-tile renormalised output; the result is the `mean` of the final
 * state.  Inputs are doubles so a test can feed any values. */
typedef struct {
    double top;
    double mass;
    double *mean; /* d values */
} soft_state;

/* state of rows [first, last) by the two-pass definition; `w` is scratch for last - first weights */
static void soft_state_of_rows(const double *q, const double *K, const double *V, int first, int last,
                               int d, double scale, double *w, soft_state *st)
{
    st->top = -INFINITY;
    for (int r = first; r < last; ++r) {
        double dot = 0.0;
        for (int e = 0; e < d; ++e) dot += q[e] * K[(size_t)r * d + e];
        w[r - first] = scale * dot;
        if (w[r - first] > st->top) st->top = w[r - first];
    }
    st->mass = 0.0;
    for (int r = first; r < last; ++r) {
        w[r - first] = exp(w[r - first] - st->top);
        st->mass += w[r - first];
    }
    for (int e = 0; e < d; ++e) {
        double sum = 0.0;
        for (int r = first; r < last; ++r) sum += w[r - first] * V[(size_t)r * d + e];
        st->mean[e] = sum / st->mass;
    }
}

/* acc <- acc combined with t (t is not empty) */
static void soft_state_absorb(soft_state *acc, const soft_state *t, int d)
{
    const double top = acc->top > t->top ? acc->top : t->top;
    const double wa = acc->mass > 0.0 ? acc->mass * exp(acc->top - top) : 0.0; /* empty: no exp(-inf + inf) */
    const double wt = t->mass * exp(t->top - top);
    const double mass = wa + wt;
    for (int e = 0; e < d; ++e) acc->mean[e] = (wa * acc->mean[e] + wt * t->mean[e]) / mass;
    acc->top = top;
    acc->mass = mass;
}

int oracle_alg1_tiled(const double *q, const double *K, const double *V, int n, int d, int Bc,
                      double scale, double *out)
{
    if (!q || !K || !V || !out || n < 1 || d < 1 || Bc < 1) return -1;
    double *w = malloc(sizeof *w * (size_t)Bc);
    double *tile_mean = malloc(sizeof *tile_mean * (size_t)d);
    if (!w || !tile_mean) { free(w); free(tile_mean); return -2; }
    soft_state acc = {-INFINITY, 0.0, out}, tile = {0.0, 0.0, tile_mean};
    for (int e = 0; e < d; ++e) out[e] = 0.0;
    for (int first = 0; first < n; first += Bc) {
        soft_state_of_rows(q, K, V, first, first + Bc < n ? first + Bc : n, d, scale, w, &tile);
        soft_state_absorb(&acc, &tile, d);
    }
    free(w);
    free(tile_mean);
    return 0;
}
