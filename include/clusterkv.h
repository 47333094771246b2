/*
 * clusterkv.h -- C ABI of the MI355X (gfx950) ClusterKV hot-path library.
 *
 * The library implements the data-parallel hot path of ClusterKV: cosine
 * K-means over the keys of every KV head (paper Section III-B), and per decode
 * step the scoring of the query against the cluster centroids, the selection of
 * clusters in score order up to a token budget (Section III-C), the generation
 * of the selected token indices from the clustering metadata (Section IV-C,
 * Fig. 8) and GQA decode attention over only the recalled keys/values
 * (Section II-B).
 *
 * Conventions that hold for every call
 * ------------------------------------
 *  - Pointers marked [dev] are device (HBM) pointers, [host] are host pointers.
 *    All device buffers are allocated, owned and freed by the caller; the
 *    library allocates no device memory and keeps no state between calls, with
 *    two exceptions: the text behind ck_last_error_detail() (one buffer per host
 *    thread) and the built-in scratch buffer of ck_sparse_decode_attn_static.
 *  - A "head-problem" is one (sequence s, KV head h) pair, linear index
 *    hp = s * Hkv + h.  Query head hq belongs to KV head hq / (Hq / Hkv).
 *  - All tensors are row-major with the last dimension contiguous:
 *      K, V        [S, Hkv, N_cap, d]      storage type (bf16 or fp32)
 *      q, out      [S, Hq, d]              storage type
 *      centroids   [S, Hkv, C_cap, d]      storage type (arithmetic mean of member keys)
 *      labels      [S, Hkv, N_cap]         int32, cluster id of every clustered token
 *      sizes       [S, Hkv, C_cap]         int32
 *      offsets     [S, Hkv, C_cap + 1]     int32, positions into sorted_idx;
 *                                          cluster c owns [offsets[c], offsets[c+1])
 *      sorted_idx  [S, Hkv, N_cap]         int32, token rows ordered by cluster id,
 *                                          ascending token row inside a cluster
 *    Device pointers must be 16-byte aligned.
 *  - Every call only enqueues work on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream) and returns; nothing synchronises the device.
 *  - Return value: CK_OK (0) or a negative CK_E* code.  Arguments are validated
 *    on the host before anything is enqueued; on error nothing is enqueued and
 *    no output is touched.  ck_strerror() names a code; ck_last_error_detail()
 *    gives the text of the last failure on the calling thread.
 *  - Integer outputs are bit-reproducible from run to run.  Floating-point
 *    outputs are too (no floating-point atomics are used anywhere).
 *  - Supported: d == 128; Hq / Hkv in {1, 2, 4, 8}; cluster counts up to
 *    CK_MAX_CLUSTERS per head-problem.
 */
#ifndef CLUSTERKV_H
#define CLUSTERKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CK_VERSION 100

#define CK_OK 0
#define CK_EINVALID (-1)      /* null pointer, non-positive size, inconsistent range */
#define CK_EUNSUPPORTED (-2)  /* shape or type outside what the kernels handle */
#define CK_EWORKSPACE (-3)    /* workspace missing or too small */
#define CK_EMISALIGNED (-4)   /* a device pointer is not 16-byte aligned */
#define CK_EHIP (-5)          /* the HIP runtime reported an error at launch */

#define CK_BF16 0             /* storage type of q, K, V, centroids, out */
#define CK_F32 1              /* fp32 check mode (decode-step calls only) */

#define CK_SEL_WHOLE 0u       /* recall only whole clusters: token count <= budget */
#define CK_SEL_TRIM_LAST 1u   /* paper's rule: fill the budget, trimming the last cluster */

#define CK_MAX_CLUSTERS 2048

/* flags of ck_cluster_keys_opt */
#define CK_METRIC_COSINE 0u
#define CK_METRIC_L2 1u
#define CK_METRIC_IP 2u
#define CK_METRIC_MASK 3u
#define CK_KM_UNTIL_CONVERGED 4u

/* which = argument of ck_workspace_bytes */
#define CK_WS_CLUSTER_KEYS 0
#define CK_WS_SPARSE_ATTN 1
#define CK_WS_OBJECTIVE 2

typedef struct ck_shape {
  int32_t S;       /* sequences in the batch */
  int32_t Hq;      /* query heads */
  int32_t Hkv;     /* KV heads */
  int32_t d;       /* head dimension, must be 128 */
  int64_t N_cap;   /* token rows per head-problem in K, V, labels, sorted_idx */
  int32_t C_cap;   /* rows per head-problem in centroids and sizes (offsets has C_cap + 1) */
  int32_t dtype;   /* CK_BF16 or CK_F32 */
} ck_shape;

int ck_version(void);
const char* ck_strerror(int code);
const char* ck_last_error_detail(void);

/*
 * Bytes of device scratch a call needs.
 *   CK_WS_CLUSTER_KEYS: n = number of tokens clustered per head-problem
 *                       (tok_count), c = number of clusters (c_count).
 *   CK_WS_OBJECTIVE:    n = tok_count of ck_kmeans_objective, c ignored.
 *   CK_WS_SPARSE_ATTN:  n = upper bound of attended tokens per head-problem
 *                       (budget + n_sink + recent window), c ignored.
 * Returns 0 for an invalid request.
 */
size_t ck_workspace_bytes(const ck_shape* sh, int which, int64_t n, int32_t c);

/*
 * Semantic clustering (Section III-B): cosine K-means with a fixed iteration
 * count over tokens [tok_begin, tok_begin + tok_count) of every head-problem,
 * producing clusters [c_begin, c_begin + c_count) and their metadata
 * (Section IV-C: sizes, prefix sum, label-sorted token index).
 *
 *   prefill:      tok_begin = n_sink, tok_count = N - n_sink, c_begin = 0, c_count = C0
 *   incremental:  tok_begin = first generated token not yet clustered, tok_count = m,
 *                 c_begin = clusters present so far, c_count = C+   (Section III-B, last part)
 *
 * K          [dev] keys, CK_BF16 only.
 * init_idx   [dev] int32 [S, Hkv, c_count]: absolute token rows whose keys are the
 *            initial centroids ("randomly sample key vectors"); the caller draws them.
 * n_iter     >= 1 iterations of {assignment by largest cosine similarity; update =
 *            mean of the assigned keys}.  An empty cluster keeps its previous
 *            centroid and size 0.  Ties go to the lower cluster id.
 * centroids  [dev] out: rows [c_begin, c_begin + c_count) of every head-problem.
 * labels     [dev] out: entries [tok_begin, tok_begin + tok_count), global cluster ids.
 * sizes      [dev] out: entries [c_begin, c_begin + c_count).
 * offsets    [dev] in/out: entries (c_begin, c_begin + c_count] are written;
 *            offsets[c_begin] is written as 0 when c_begin == 0 and otherwise read
 *            (it must hold the end of the previous clusters' segment).
 * sorted_idx [dev] out: positions [offsets[c_begin], offsets[c_begin] + tok_count).
 * workspace  [dev] scratch of ck_workspace_bytes(sh, CK_WS_CLUSTER_KEYS, tok_count, c_count).
 * Errors: CK_EINVALID (null, tok range outside [0, N_cap], c range outside [0, C_cap],
 *   c_count > tok_count, n_iter < 1), CK_EUNSUPPORTED (dtype != CK_BF16, d != 128,
 *   c_count > CK_MAX_CLUSTERS), CK_EWORKSPACE, CK_EMISALIGNED, CK_EHIP.
 */
int ck_cluster_keys(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                    int32_t c_begin, int32_t c_count, int32_t n_iter, const int32_t* init_idx,
                    void* centroids, int32_t* labels, int32_t* sizes, int32_t* offsets,
                    int32_t* sorted_idx, void* workspace, size_t workspace_bytes, void* stream);

/*
 * ck_cluster_keys with the options the paper discusses beside its default:
 *   flags & CK_METRIC_MASK   distance of the assignment step (Section V-B compares the
 *       three): CK_METRIC_COSINE (largest cosine similarity, the default),
 *       CK_METRIC_L2 (smallest Euclidean distance to the stored centroid) or
 *       CK_METRIC_IP (largest inner product with the stored centroid).  The update
 *       step is the mean of the assigned keys under every metric.
 *   flags & CK_KM_UNTIL_CONVERGED   stop a head-problem at the first assignment that
 *       changes no label (Section III-B: the two steps alternate until convergence);
 *       max_iter (<= 256 in this mode) bounds the iterations.  The confirming
 *       assignment counts as an iteration and is not followed by an update.  Each
 *       head-problem stops on its own; there is no host synchronisation, iterations
 *       of stopped head-problems are launches that return at once.
 * iters_done [dev] int32 [S, Hkv], nullable: iterations each head-problem ran.
 * Everything else as ck_cluster_keys (which is this call with flags = 0).
 * Errors: additionally CK_EINVALID for unknown flag bits, CK_EUNSUPPORTED for
 *   max_iter > 256 with CK_KM_UNTIL_CONVERGED.
 */
int ck_cluster_keys_opt(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                        int32_t c_begin, int32_t c_count, int32_t max_iter, uint32_t flags,
                        const int32_t* init_idx, void* centroids, int32_t* labels, int32_t* sizes,
                        int32_t* offsets, int32_t* sorted_idx, int32_t* iters_done,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * The three steps ck_cluster_keys iterates, exported so that each can be checked
 * on its own inputs (Section III-B; Section IV-C for the metadata).
 *
 * ck_kmeans_assign: labels[i] = c_begin + argmax_c <k_i, centroids_hat[c]> for the
 *   tokens of the range.  centroids_hat [dev] bf16 [S, Hkv, c_count, d] holds the
 *   unit-length copies of the centroids (dense, row stride d, head-problem stride
 *   c_count * d).  best_sim [dev] fp32 [S, Hkv, N_cap] (nullable) receives the
 *   winning similarity <k_i, centroid_hat> of every token of the range.
 */
int ck_kmeans_assign(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                     const void* centroids_hat, int32_t c_begin, int32_t c_count,
                     int32_t* labels, float* best_sim, void* stream);

/*
 * The clustering objective of a given assignment under the distance of Section
 * III-B, D(k, mu) = 1 - cos(k, mu), summed over tokens [tok_begin, tok_begin +
 * tok_count) of every head-problem:
 *   D[hp] = sum_i (1 - cos(k_i, t_i))            the paper's objective
 *   J[hp] = sum_i |k_i| (1 - cos(k_i, t_i))      the norm-weighted form, which neither
 *                                                K-means step can increase
 * with t_i = row (labels[i] - c_begin) of centroids_hat, the compact table an
 * assignment reads ([S, Hkv, c_count, d] bf16; J takes its rows as unit vectors:
 * J = sum_i (|k_i| - <k_i, t_i>)).  Calling it after each ck_kmeans_assign of a
 * step-by-step run gives the objective per iteration; ck_cluster_keys itself does
 * not report it (the value is a diagnostic and costs one more pass over the keys).
 * J, D [dev] out double [S, Hkv].  fp32 inside a row, fp64 across rows, fixed order.
 * workspace: ck_workspace_bytes(sh, CK_WS_OBJECTIVE, tok_count, 0).
 */
int ck_kmeans_objective(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                        const void* centroids_hat, int32_t c_begin, int32_t c_count,
                        const int32_t* labels, double* J, double* D, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * ck_build_metadata: from labels of the token range, sizes / offsets / sorted_idx
 *   of clusters [c_begin, c_begin + c_count) (same in/out rules as ck_cluster_keys).
 *   workspace: ck_workspace_bytes(sh, CK_WS_CLUSTER_KEYS, tok_count, c_count).
 */
int ck_build_metadata(const ck_shape* sh, const int32_t* labels, int64_t tok_begin,
                      int64_t tok_count, int32_t c_begin, int32_t c_count, int32_t* sizes,
                      int32_t* offsets, int32_t* sorted_idx, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * ck_kmeans_update: centroid = mean of its member keys, members taken from the
 *   metadata (so ck_build_metadata must have run on the labels).  Writes
 *   centroids (storage type, rows [c_begin, c_begin + c_count)), centroids_hat
 *   (bf16, dense [S, Hkv, c_count, d], unit length) and, if not NULL,
 *   centroids_f32 (fp32, dense [S, Hkv, c_count, d], the unrounded means).
 *   Rows of empty clusters are left untouched in all three.
 */
int ck_kmeans_update(const ck_shape* sh, const void* K, const int32_t* sizes,
                     const int32_t* offsets, const int32_t* sorted_idx, int32_t c_begin,
                     int32_t c_count, void* centroids, void* centroids_hat,
                     float* centroids_f32, void* stream);

/*
 * Cluster selection (Section III-C; Section IV-C up to the prefix sum): per
 * head-problem, score every cluster as sum over the query heads of the group of
 * <q_g, centroid_c> (inner product, no scaling), order the clusters by
 * descending score (ties: lower id first), and count how many leading clusters
 * are recalled under `budget`:
 *   CK_SEL_WHOLE      the longest prefix whose sizes sum to <= budget (may be 0);
 *   CK_SEL_TRIM_LAST  the shortest prefix whose sizes sum to >= budget (all
 *                     clusters if the total is smaller); the last one is cut.
 * q            [dev] [S, Hq, d].
 * n_clusters   clusters present per head-problem (<= C_cap, <= CK_MAX_CLUSTERS).
 * sel_clusters [dev] out int32 [S, Hkv, C_cap]: the recalled cluster ids in score
 *              order in the first n_sel_clusters entries; the rest is unspecified.
 * n_sel_clusters, n_sel_tokens [dev] out int32 [S, Hkv].
 * scores       [dev] out fp32 [S, Hkv, C_cap], required (the ordering step reads it).
 */
int ck_select_clusters(const ck_shape* sh, const void* q, const void* centroids,
                       const int32_t* sizes, int32_t n_clusters, int32_t budget, uint32_t flags,
                       int32_t* sel_clusters, int32_t* n_sel_clusters, int32_t* n_sel_tokens,
                       float* scores, void* stream);

/*
 * Index generation (Section IV-C, Fig. 8): concatenate, in selection order, the
 * sorted_idx segments of the recalled clusters into token_idx.
 * token_idx [dev] out int32 [S, Hkv, idx_stride], idx_stride >= budget;
 * n_tokens  [dev] out int32 [S, Hkv].  With CK_SEL_TRIM_LAST the last cluster
 * contributes only the trailing entries of its segment that still fit.
 * A cluster that would overflow idx_stride is cut the same way in either mode,
 * so the call never writes past a row.
 */
int ck_gather_indices(const ck_shape* sh, const int32_t* sel_clusters,
                      const int32_t* n_sel_clusters, const int32_t* offsets,
                      const int32_t* sorted_idx, int32_t budget, uint32_t flags,
                      int32_t* token_idx, int32_t idx_stride, int32_t* n_tokens, void* stream);

/*
 * Sparse GQA decode attention (Section II-B): for every query head,
 *   out = softmax(q K_T^T * softmax_scale) V_T
 * over T = [0, n_sink) + token_idx[0 .. n_tokens) + [recent_begin, recent_end)
 * of its KV head (the three parts are assumed disjoint; an empty T gives zeros).
 * K and V rows are read once per KV head and shared by the query heads of the
 * group.  Accumulation is fp32.
 * token_idx [dev] int32 [S, Hkv, idx_stride] (nullable if n_tokens is NULL);
 * n_tokens  [dev] int32 [S, Hkv], nullable = no recalled tokens;
 * max_tokens  host upper bound of every n_tokens entry (e.g. the budget);
 * workspace [dev] ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN,
 *           max_tokens + n_sink + recent_end - recent_begin, 0); its contents on
 *           entry do not matter (nothing has to be zero).
 * One launch: the attended positions of a head-problem are split over several
 * workgroups, and the workgroup that finishes last merges the partial results
 * (in split order, so the output does not depend on which one it is).
 */
int ck_sparse_decode_attn(const ck_shape* sh, const void* q, const void* K, const void* V,
                          const int32_t* token_idx, const int32_t* n_tokens, int32_t idx_stride,
                          int32_t max_tokens, int64_t n_sink, int64_t recent_begin,
                          int64_t recent_end, float softmax_scale, void* out, void* workspace,
                          size_t workspace_bytes, void* stream);

/*
 * The same attention with the partial results merged by a second kernel launch
 * instead of by the last workgroup: the reference form of the merge (bit-identical
 * output), kept for checking the single-launch form and for timing comparisons.
 */
int ck_sparse_decode_attn_two_pass(const ck_shape* sh, const void* q, const void* K,
                                   const void* V, const int32_t* token_idx,
                                   const int32_t* n_tokens, int32_t idx_stride,
                                   int32_t max_tokens, int64_t n_sink, int64_t recent_begin,
                                   int64_t recent_end, float softmax_scale, void* out,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * ck_sparse_decode_attn for callers that cannot allocate device memory or hand
 * over a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments, same kernels and the same result as
 * ck_sparse_decode_attn; the split partials and tickets live in a buffer of
 * CK_STATIC_SCRATCH_BYTES that is part of the library's code object (each GPU
 * the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing.
 *  - A shape whose partials exceed the buffer (ck_workspace_bytes(sh,
 *    CK_WS_SPARSE_ATTN, ...) > CK_STATIC_SCRATCH_BYTES) is rejected with
 *    CK_EWORKSPACE before anything is enqueued.
 *  - All calls on one GPU share the buffer.  It keeps the last call's contents;
 *    nothing in it has to start at zero (every partial is written before it is
 *    read).  Calls of this entry point that overlap on one GPU (different
 *    streams, no ordering between them) race on the buffer: order them.
 */
#define CK_STATIC_SCRATCH_BYTES (4u << 20)
int ck_sparse_decode_attn_static(const ck_shape* sh, const void* q, const void* K, const void* V,
                                 const int32_t* token_idx, const int32_t* n_tokens,
                                 int32_t idx_stride, int32_t max_tokens, int64_t n_sink,
                                 int64_t recent_begin, int64_t recent_end, float softmax_scale,
                                 void* out, void* stream);

/*
 * One whole decode step (Sections III-C, IV-C and II-B in one call): the same
 * results as ck_select_clusters, ck_gather_indices and ck_sparse_decode_attn in
 * sequence (scores, sel_clusters, n_sel_clusters, n_sel_tokens, token_idx,
 * n_tokens, out; all outputs bit-identical to the three calls), in ONE launch when
 * the table is bf16 with at most 512 clusters: every attention workgroup scores
 * the centroids of its head-problem, derives the recalled prefix and its own slice
 * of the index list itself instead of re-reading them from memory, and the last
 * workgroup of a head-problem merges.  Larger or fp32 tables are scored by a
 * launch of their own first.
 * Arguments as in the three calls; idx_stride >= budget and a multiple of 4;
 * workspace: ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, budget + n_sink + recent
 * window, 0).
 */
int ck_decode_step(const ck_shape* sh, const void* q, const void* K, const void* V,
                   const void* centroids, const int32_t* sizes, const int32_t* offsets,
                   const int32_t* sorted_idx, int32_t n_clusters, int32_t budget, uint32_t flags,
                   int64_t n_sink, int64_t recent_begin, int64_t recent_end, float softmax_scale,
                   float* scores, int32_t* sel_clusters, int32_t* n_sel_clusters,
                   int32_t* n_sel_tokens, int32_t* token_idx, int32_t idx_stride,
                   int32_t* n_tokens, void* out, void* workspace, size_t workspace_bytes,
                   void* stream);

/* ------------------------------------------------------------------------
 * Evaluation of a selection (paper Section V-B, "recall rate of important
 * tokens") and the full-KV / page-granular comparison points.  Not on the
 * decode path.  Same conventions as above: device pointers, caller-owned,
 * enqueue only, host-side validation.
 * ---------------------------------------------------------------------- */

/*
 * Full-KV decode attention (Section II-A): softmax(q K^T * softmax_scale) V over
 * tokens [0, n_ctx) of every head-problem, the computation the compressed path
 * approximates.  q, K, V, out as in ck_sparse_decode_attn.  workspace: at least
 * ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, n_ctx, 0) bytes.
 * Errors: CK_EINVALID for n_ctx outside [1, N_cap].
 */
int ck_full_decode_attn(const ck_shape* sh, const void* q, const void* K, const void* V,
                        int64_t n_ctx, float softmax_scale, void* out, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * Exact importance of every token of [tok_begin, tok_begin + tok_count) (Section
 * III-A: the ideal selection keeps the tokens with the largest q.k): scores[s, h, t]
 * = sum over the G query heads of the group of <q_g, K[s, h, t]>, fp32, written at
 * the token's own position in scores [S, Hkv, N_cap] (other positions untouched).
 * K may be any table of rows laid out [S, Hkv, N_cap, d] in sh->dtype, e.g. the page
 * representatives of ck_page_keys with N_cap = their row stride.
 */
int ck_token_scores(const ck_shape* sh, const void* q, const void* K, int64_t tok_begin,
                    int64_t tok_count, float* scores, void* stream);

/*
 * Exact top-k per head-problem over scores[hp * row_stride + begin + i], i < n:
 * the k largest values (equal values: lower index first; -0 == +0), their indices
 * begin + i written in ASCENDING INDEX order to out_idx [n_problems, out_stride]
 * int32; n_out [n_problems] int32 receives min(k, n).  Bit-reproducible.
 * Errors: CK_EINVALID for n < 1, k < 0, out_stride < min(k, n), n_problems outside
 * [1, 65535].
 */
int ck_topk_select(int32_t n_problems, const float* scores, int64_t row_stride, int64_t begin,
                   int32_t n, int32_t k, int32_t* out_idx, int32_t out_stride, int32_t* n_out,
                   void* stream);

/*
 * Numerator of the recall rate |I_T intersect I_true| / |I_true| (Section V-B):
 * hits [n_problems] int32 = number of the first n_tokens[p] entries of token_idx
 * [n_problems, idx_stride] that occur among the first n_ref[p] entries of ref_idx
 * [n_problems, ref_stride].  ref_idx rows must be ascending and distinct (as
 * ck_topk_select writes them); token_idx entries are expected to be distinct.
 */
int ck_recall_hits(int32_t n_problems, const int32_t* token_idx, const int32_t* n_tokens,
                   int32_t idx_stride, const int32_t* ref_idx, const int32_t* n_ref,
                   int32_t ref_stride, int32_t* hits, void* stream);

/*
 * Page-granular selector of Section II-C, step 1: representative of every page of
 * page_size consecutive tokens of [tok_begin, tok_begin + tok_count) = per-channel
 * maximum of its keys (the last page may be short).  page_keys [S, Hkv, page_stride,
 * d] in sh->dtype; rows [0, ceil(tok_count / page_size)) are written.  Scoring the
 * pages is ck_token_scores on this table, choosing them ck_topk_select with
 * k = budget / page_size.
 * Errors: CK_EINVALID for page_size < 1 or page_stride smaller than the page count.
 */
int ck_page_keys(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                 int32_t page_size, void* page_keys, int64_t page_stride, void* stream);

/*
 * Page-granular selector, last step: token ids of the selected pages.  page_idx
 * [n_problems, page_stride] int32 holds n_pages[p] distinct page numbers in ascending
 * order (page j covers tokens tok_begin + [j * page_size, (j+1) * page_size), cut
 * at tok_begin + tok_count).  token_idx [n_problems, idx_stride] receives the ids in
 * ascending order, n_tokens [n_problems] their count; pages that would not fit
 * idx_stride are dropped from the end.
 */
int ck_expand_pages(int32_t n_problems, const int32_t* page_idx, const int32_t* n_pages,
                    int32_t page_stride, int32_t page_size, int64_t tok_begin,
                    int64_t tok_count, int32_t* token_idx, int32_t idx_stride,
                    int32_t* n_tokens, void* stream);

/* ------------------------------------------------------------------------
 * Cluster-granularity cache of recalled K/V over a home copy in host memory
 * (paper Section IV-A: K/V are offloaded after prefill and only selected tokens
 * are loaded back; Section IV-D: a cache on the GPU keeps the K/V of the clusters
 * selected at the last R steps, so that only clusters not present are loaded).
 * R = 1 here, the value the paper settles on.
 * ---------------------------------------------------------------------- */

/*
 * Device buffers of the cache, all allocated by the caller.  Two generations
 * alternate: a step reads generation (step_parity ^ 1) and writes generation
 * step_parity.
 *   K[g], V[g]   [S, Hkv, cap_tokens, d] in sh->dtype: rows of the recalled list of a
 *                step, in recalled order.
 *   clusters[g]  int32 [S, Hkv, C_cap]: ids of the clusters held, in buffer order.
 *   starts[g]    int32 [S, Hkv, C_cap + 1]: first row of each held cluster; the entry
 *                after the last one is the number of rows in use.
 *   n_held[g]    int32 [S, Hkv].
 *   cap_tokens   rows per head-problem; must be >= the budget of every step.
 */
typedef struct ck_cluster_cache {
  void* K[2];
  void* V[2];
  int32_t* clusters[2];
  int32_t* starts[2];
  int32_t* n_held[2];
  int32_t cap_tokens;
  int32_t reserved;
} ck_cluster_cache;

/*
 * Device-visible address of pinned host memory (hipHostMalloc, or a torch tensor
 * created with pin_memory=True): *dev_ptr [host out].  Errors: CK_EINVALID for NULL,
 * CK_EHIP if the runtime does not know the address as mapped pinned memory.
 */
int ck_host_device_ptr(void* host_ptr, void** dev_ptr);

/* Empties both generations (n_held := 0).  Enqueues one small kernel. */
int ck_cache_reset(const ck_shape* sh, const ck_cluster_cache* cache, void* stream);

/*
 * One decode step with the cache: selection as ck_select_clusters (whole clusters
 * only: a cached cluster is always complete), then every selected cluster is copied
 * into generation step_parity of the cache, from generation step_parity ^ 1 if it is
 * held there, else row by row from the home copy through sorted_idx; then attention
 * over exactly those rows.  out equals what ck_decode_step computes on K/V resident in
 * device memory, bit for bit.
 *   K_home, V_home  device-visible pointers to K/V [S, Hkv, N_cap, d]: pinned host
 *                   memory (ck_host_device_ptr) or device memory.  Read by the GPU
 *                   itself; rows of missing clusters only.
 *   miss_tokens     [dev] int32 [S, Hkv] out: rows loaded from the home copy this step
 *                   (n_sel_tokens - miss_tokens were found in the cache).
 *   sinks and a recent window are not supported here (the step attends the recalled
 *   list only).
 *   workspace: ck_workspace_bytes(sh, CK_WS_SPARSE_ATTN, budget, 0).
 * Calls on one cache must be ordered on one stream; step_parity alternates 0, 1, 0, ...
 * Errors: CK_EINVALID (null, n_clusters / budget out of range, budget > cap_tokens,
 *   step_parity not 0 or 1), CK_EUNSUPPORTED, CK_EWORKSPACE, CK_EMISALIGNED, CK_EHIP.
 */
int ck_cached_decode_step(const ck_shape* sh, const void* q, const void* K_home,
                          const void* V_home, const void* centroids, const int32_t* sizes,
                          const int32_t* offsets, const int32_t* sorted_idx, int32_t n_clusters,
                          int32_t budget, const ck_cluster_cache* cache, int32_t step_parity,
                          float softmax_scale, float* scores, int32_t* sel_clusters,
                          int32_t* n_sel_clusters, int32_t* n_sel_tokens, int32_t* miss_tokens,
                          void* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement aid, not part of the method: a register-only loop of
 * v_mfma_f32_32x32x16_bf16 (the instruction the assignment step of Section III-B
 * runs on) over n_workgroups workgroups of 4 wavefronts, `iters` x 16 MFMAs per
 * wavefront.  *flops [host] receives the floating-point operations of the launch,
 * so that flops / elapsed time is the matrix throughput the chip sustains at its
 * real clocks.  operands [dev, 16-byte aligned] or NULL: 16384 bytes, for each of the
 * 64 lanes 8 A fragments then 8 B fragments of 8 bf16 each, used in rotation; NULL
 * uses small constants.  The clock the chip holds under matrix load depends on how many
 * operand bits toggle, so random operands give the figure that bounds a kernel
 * working on real keys, constants an upper one.  clocks [dev, 8-byte aligned] or
 * NULL: two words written by the first workgroup, the shader-clock cycles and the
 * ticks of the constant 100 MHz counter spent in its loop (their ratio x 100 MHz is
 * the clock it ran at).  sink [dev]: at least one float, never written in practice.
 * Errors: CK_EINVALID (n_workgroups outside [1, 65535], iters outside [1, 2^24],
 *   sink or flops NULL), CK_EMISALIGNED, CK_EHIP.
 */
int ck_probe_mfma_bf16(int32_t n_workgroups, int32_t iters, const void* operands,
                       uint64_t* clocks, float* sink, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CLUSTERKV_H */
