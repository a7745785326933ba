/*
 * curdkv.h -- C ABI of the CurDKV post-prefill KV selection library for
 * AMD MI355X (gfx950).
 *
 * The library computes Algorithm 1 of "Value-Guided KV Compression for LLMs via
 * Approximated CUR Decomposition" (CurDKV) for every layer and KV group of a
 * GQA cache: sketch, project, row-norm squared, combine, normalise, keep sinks
 * plus top-k, gather.  All arithmetic runs in HIP kernels; there is no CPU
 * fallback.  Layers are an outer batch dimension over the algorithm's group
 * loop; a batch of sequences folds into `layers`.
 *
 * Conventions
 *   - Every function returns CURDKV_OK (0) or a negative error code and never
 *     throws.  Arguments are validated on the host before anything is launched;
 *     on error nothing has been launched.
 *   - "device" pointers are HIP device memory owned by the caller; the library
 *     neither frees nor keeps them.  "host" pointers are ordinary host memory,
 *     read before the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  The
 *     compute calls only enqueue work on it and do not synchronise.
 *   - The context owns the sketches, the per-block partial sums and the device
 *     copy of the offsets, all on the device that was current at curdkv_create;
 *     that device must be current for every later call (else INVALID_ARG).
 *     Calls on one context must not overlap in time on different streams.
 *   - Capturing a compute call in a HIP graph: run the same call (same offsets,
 *     same optional buffers) once and synchronise before the capture, so that
 *     the capture neither uploads offsets nor allocates scratch; both would
 *     make the call unfit for capture.  The captured kernels read the offsets
 *     and the gather's block table from the context's single device copy: as
 *     long as the graph may be replayed, call curdkv_select / curdkv_compact /
 *     curdkv_compress on that context with these same offsets only (or give the
 *     graph a context of its own).  A graph replayed after the copy has changed
 *     would run the captured grid against the new offsets: its results would be
 *     meaningless and, where the new offsets reach further than the captured
 *     buffers, its writes out of bounds: such a graph must not be replayed.
 *     curdkv_compress_adaptive keeps offsets and table in caller buffers and has
 *     no such constraint.
 *   - K and V are row-major [layers, kv_heads, n, head_dim] in the context's
 *     storage type; token j of group (l, h) starts at element
 *     ((l*kv_heads + h)*n + j)*head_dim.  Base pointers must be 16-byte aligned.
 */
#ifndef CURDKV_H
#define CURDKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CURDKV_OK               0
#define CURDKV_ERR_INVALID_ARG -1   /* null pointer, size out of range, inconsistent offsets */
#define CURDKV_ERR_UNSUPPORTED -2   /* head_dim, sketch_dim or dtype the kernels do not cover */
#define CURDKV_ERR_HIP         -3   /* a HIP runtime call failed (no device, launch error, ...) */
#define CURDKV_ERR_OOM         -4   /* device or host allocation failed */
#define CURDKV_ERR_TOO_LARGE   -5   /* more (layer, group) pairs than a non-allocating call's fixed workspace holds */

#define CURDKV_DTYPE_F32  0
#define CURDKV_DTYPE_BF16 1

/* What the score of a token is built from.  KV is the method (the combination
 * step of Algorithm 1: product of key and value scores); KEY and VALUE are the
 * ablation of the appendix ("Ablation Study") that uses one tensor alone. */
#define CURDKV_SCORE_KV    0
#define CURDKV_SCORE_KEY   1
#define CURDKV_SCORE_VALUE 2

typedef struct curdkv_ctx curdkv_ctx;

/* Problem statement of Algorithm 1 (inputs K, V in R^{g x n x d}, projection
 * dimension r) extended over layers.  group_size (query heads per KV group)
 * is carried for curdkv_fold; the scores themselves depend on K and V only. */
typedef struct curdkv_config {
    int32_t  layers;       /* >= 1 */
    int32_t  kv_heads;     /* g, number of KV groups per layer, >= 1 */
    int32_t  group_size;   /* query heads per KV group, >= 1 */
    int32_t  head_dim;     /* d; supported: 128 */
    int32_t  sketch_dim;   /* r in [1, 128]; padded internally with zero columns */
    int32_t  dtype;        /* CURDKV_DTYPE_* : storage type of K, V and of G */
    int32_t  score_source; /* CURDKV_SCORE_* ; 0 = the method's key-value product */
    int32_t  no_projection;/* 0 = sketch with G (the method); 1 = the ablation without the Gaussian
                              projection: squared norms of the stored rows */
    int64_t  max_tokens;   /* largest n any call will pass, >= 1 */
    uint64_t seed;         /* seed of the sketch generator */
} curdkv_config;

/* Create a context on the current HIP device: generates the sketch G of every
 * (layer, group) on the host, uploads it in the kernels' operand layout and
 * allocates the reduction workspace.  Synchronous.  *out is set only on success. */
int curdkv_create(curdkv_ctx** out, const curdkv_config* cfg);

/* Free everything the context owns.  Synchronises the device first.  NULL is accepted. */
int curdkv_destroy(curdkv_ctx* ctx);

/* Host-only (no GPU needed): write G of group (layer, head) to G_host[d*r],
 * row-major [head_dim, sketch_dim], as float.
 *
 * Sampling step of Algorithm 1: a d x r matrix of independent normal entries
 * with variance 1/r; one G per (layer, group), shared by K and V.  The paper fixes no generator:
 * element (i, j) has counter c = ((layer*kv_heads + head)*d + i)*r + j and
 * takes SplitMix64 outputs number 2c+1 and 2c+2 (w1, w2) of the stream started
 * at `seed`; u1 = ((w1>>11)+1)*2^-53, u2 = (w2>>11)*2^-53,
 * G_ij = sqrt(-2 ln u1) cos(2 pi u2) / sqrt(r) in double, then rounded to the
 * storage type (nearest even).  The rounded value is what the kernels use. */
int curdkv_sketch_host(const curdkv_config* cfg, int32_t layer, int32_t head, float* G_host);

/* Replace the sketch of one group by caller-supplied values (host, row-major
 * [head_dim, sketch_dim] floats; rounded to the storage type).  Synchronous.
 * For callers that draw G themselves, as Algorithm 1 literally does. */
int curdkv_set_sketch(curdkv_ctx* ctx, int32_t layer, int32_t head, const float* G_host);

/* Algorithm 1 from the projection step to the normalisation step: for every (layer, group)
 *   lK_j = ||(K G)[j]||^2,  lV_j = ||(V G)[j]||^2,  lKV_j = lK_j * lV_j,
 *   scores_j = lKV_j / sum_j lKV_j   (sum over all n rows; 1/n if the sum is 0).
 * K, V: device, [layers, kv_heads, n, head_dim], storage type, read once.
 * scores: device float [layers, kv_heads, n], written.
 * Products accumulate in fp32; lKV must stay inside the fp32 range.
 * 1 <= n <= max_tokens. */
int curdkv_scores(curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                  float* scores, void* stream);

/* GQA score fold (Section 2, GQA-compatible eviction; Section 3.2 assumes a
 * group of query heads shares one K_i, V_i): mean over the group of per-query-
 * head scores.  scores_q: device float [layers, kv_heads, group_size, n];
 * scores: device float [layers, kv_heads, n].  CurDKV's own scores are already
 * per group, so the hot path does not need this call; it serves score sources
 * that are per query head.  Summation order is fixed (head 0 first). */
int curdkv_fold(curdkv_ctx* ctx, const float* scores_q, int64_t n, float* scores,
                void* stream);

/* Sink, top-k and union steps of Algorithm 1: S = {0..s-1} U (TopK(scores[s:], k-s) + s)
 * for every (layer, group).
 * scores: device float [layers, kv_heads, n], non-negative, no NaN.
 * budgets: host int32 [layers*kv_heads], k per group (sinks included), 0 <= k <= n.
 * offsets: host int64 [layers*kv_heads + 1], offsets[0] = 0 and
 *          offsets[i+1] = offsets[i] + budgets[i].
 * indices: device int32 [offsets[last]]; group i's tokens go to
 *          indices[offsets[i] .. offsets[i+1]) in ascending token order.
 * Ties: larger score first, then smaller token index.  k <= s keeps tokens
 * 0..k-1.  n_sink >= 0. */
int curdkv_select(curdkv_ctx* ctx, const float* scores, int64_t n,
                  const int32_t* budgets, int32_t n_sink, const int64_t* offsets,
                  int32_t* indices, void* stream);

/* Gather step of Algorithm 1: K' = K[S], V' = V[S] (rows of the original cache).
 * indices, offsets: as written by / passed to curdkv_select (offsets on host;
 * non-decreasing, offsets[0] = 0, each group's count <= n; every index must lie
 * in [0, n)).
 * K_out, V_out: device, packed [offsets[last], head_dim], storage type; equal to
 * [layers, kv_heads, k, head_dim] when all budgets are k.  Bit-exact copies. */
int curdkv_compact(curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                   const int32_t* indices, const int64_t* offsets,
                   void* K_out, void* V_out, void* stream);

/* The whole of Algorithm 1 in one call: scores, selection and gather, with the
 * results of curdkv_scores + curdkv_select + curdkv_compact (same arguments,
 * same layouts; `scores` may be NULL when the caller does not want them, the
 * library then uses a scratch buffer it allocates on first need).  Where
 * curdkv_uses_fused_kernel says so, one fused kernel does everything with one
 * workgroup per (layer, group) and the scores never pass through HBM between
 * the steps (when more than 11 % of all rows are kept, only its scoring phases
 * are used and the stand-alone selection and gather kernels follow: the gather
 * kernel moves rows faster than the fused kernel's last phase); otherwise
 * the kernels of the separate calls are launched.  The normalising sum is taken
 * in a different order in the two cases, so scores can differ in the last bits
 * between them. */
int curdkv_compress(curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                    const int32_t* budgets, int32_t n_sink, const int64_t* offsets,
                    float* scores, int32_t* indices, void* K_out, void* V_out, void* stream);

/* Which kernels curdkv_scores / curdkv_compress launch for a cache of n tokens
 * per head: 1 = the fused one-workgroup-per-head kernel, 0 = the general
 * kernels; negative = error code.  The fused kernel needs bf16, a sketch of at
 * most 64 columns (or no projection), n <= 32768, and a number of (layer,
 * group) pairs that fills whole rounds of the GPU's compute units to at least
 * 90 %.  The results are the same either way (Algorithm 1); the entry exists so
 * that tests and tuning know which path they exercise. */
int curdkv_uses_fused_kernel(const curdkv_ctx* ctx, int64_t n);

/* AdaCurDKV head-wise budgets (Section 3.2, "Adaptive budget allocation"): every
 * layer keeps kv_heads*budget tokens in all, the top normalised scores ACROSS the
 * heads of the layer, but each head is guaranteed its own best floor(alpha*budget)
 * tokens (the AdaKV safeguard; the paper uses alpha = 0.20).  Reading: the first
 * s' = min(n_sink, n) tokens of a head are sinks, always kept and counted; each
 * head is guaranteed g = max(floor(alpha*budget) - s', 0) further tokens; the
 * remaining kv_heads*(budget - s' - g) places of a layer go to its largest
 * scores outside the sinks and the guaranteed ones, equal scores in (head, token)
 * order.  budget <= s' gives `budget` to every head.
 * scores: device float [layers, kv_heads, n], normalised, non-negative.
 * budgets_out: DEVICE int32 [layers*kv_heads], tokens to keep per head (sinks
 * included); each layer's entries sum to kv_heads*budget.  Copy them to the host
 * and pass them, with their prefix sums, to curdkv_select and curdkv_compact.
 * 0 <= budget <= n, 0 <= alpha <= 1. */
int curdkv_adaptive_budgets(curdkv_ctx* ctx, const float* scores, int64_t n, int32_t budget,
                            int32_t n_sink, double alpha, int32_t* budgets_out, void* stream);

/* curdkv_adaptive_budgets for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same results, same kernels; the histograms, key lists and
 * per-layer state that curdkv_adaptive_budgets keeps in a buffer its context got
 * from hipMalloc live here in a static device array of the library (24 MiB +
 * 32 KiB per GPU, resident from the moment the library is loaded, its address
 * looked up at curdkv_create).
 * The call makes no hipMalloc, hipFree or other allocating call.
 * Limit: layers*kv_heads <= 1024, else CURDKV_ERR_TOO_LARGE and nothing is launched.
 * All calls on one GPU, from every context, share the one array: two such calls
 * that overlap in time on that GPU race; calls on one stream, or otherwise
 * ordered, are safe (nothing in the array has to survive between calls). */
int curdkv_adaptive_budgets_noalloc(curdkv_ctx* ctx, const float* scores, int64_t n, int32_t budget,
                                    int32_t n_sink, double alpha, int32_t* budgets_out, void* stream);

/* AdaCurDKV in one call with nothing passing through the host (Algorithm 1 with the
 * head-wise budgets of Section 3.2, "Adaptive budget allocation"): scores as in
 * curdkv_scores, budgets as in curdkv_adaptive_budgets, their prefix sums, then the
 * selection and the gather of curdkv_select / curdkv_compact with those budgets,
 * all enqueued on `stream` without a synchronisation or a copy to the host.
 * Every layer keeps kv_heads*budget rows, so the sizes are known beforehand:
 * scores: device float [layers, kv_heads, n], or NULL (library scratch, allocated
 *   on first need);
 * budgets_out: device int32 [layers*kv_heads]; offsets_out: device int64
 *   [layers*kv_heads + 1], offsets_out[i] = budgets_out[0] + .. + budgets_out[i-1];
 * indices: device int32 [layers*kv_heads*budget]; K_out, V_out: device
 *   [layers*kv_heads*budget, head_dim]; group i owns rows offsets_out[i] ..
 *   offsets_out[i+1]-1 of all three, tokens ascending.
 * 0 <= budget <= n, 0 <= alpha <= 1, n_sink >= 0; kv_heads <= 1024. */
int curdkv_compress_adaptive(curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                             int32_t budget, int32_t n_sink, double alpha, float* scores,
                             int32_t* budgets_out, int64_t* offsets_out, int32_t* indices,
                             void* K_out, void* V_out, void* stream);

/* Scoring during generation (Section 3.2, first paragraph: the method is meant for
 * the generation phase as well as for pre-filling).  The un-normalised scores
 * lKV_j of a token do not depend on the other tokens, so a growing cache is scored
 * chunk by chunk: this call scores the m new tokens of every (layer, group),
 * writes lKV to raw[group*stride + n_old + j] and adds their sum to sums[group]
 * (n_old == 0 starts the sums afresh).
 * K_new, V_new: device, [layers, kv_heads, m, head_dim], the new rows only.
 * raw: device float [layers*kv_heads, stride]; sums: device double [layers*kv_heads].
 * 1 <= m, 0 <= n_old, n_old + m <= stride <= max_tokens. */
int curdkv_scores_append(curdkv_ctx* ctx, const void* K_new, const void* V_new, int64_t m,
                         int64_t n_old, int64_t stride, float* raw, double* sums, void* stream);

/* Normalisation step for the first n tokens of a cache scored with curdkv_scores_append:
 * scores[group*n + j] = raw[group*stride + j] / sums[group] (1/n if the sum is 0),
 * sums being those of exactly these n tokens.  The result is what curdkv_scores
 * gives on the n-token cache (up to the order of the additions in the sum) and
 * goes to curdkv_select / curdkv_adaptive_budgets. */
int curdkv_normalise(curdkv_ctx* ctx, const float* raw, const double* sums, int64_t stride,
                     int64_t n, float* scores, void* stream);

/* Text for an error code; never NULL. */
const char* curdkv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CURDKV_H */
