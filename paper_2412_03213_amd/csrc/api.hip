// C ABI of the ClusterKV library: argument validation (host only, before anything
// is enqueued) and the sequence of kernel launches behind every entry point.
#include <stdarg.h>
#include <stdio.h>

#include "ck_common.hpp"

namespace {

thread_local char g_detail[256] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_detail, sizeof(g_detail), fmt, ap);
  va_end(ap);
  return code;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define CK_REQUIRE_PTR(p)                                          \
  do {                                                             \
    if (!(p)) return fail(CK_EINVALID, "%s is NULL", #p);          \
    if (!aligned16(p)) return fail(CK_EMISALIGNED, "%s is not 16-byte aligned", #p); \
  } while (0)
#define CK_OPTIONAL_PTR(p)                                         \
  do {                                                             \
    if ((p) && !aligned16(p)) return fail(CK_EMISALIGNED, "%s is not 16-byte aligned", #p); \
  } while (0)

int check_shape(const ck_shape* sh, ck::Dims* dm, bool need_bf16) {
  if (!sh) return fail(CK_EINVALID, "shape is NULL");
  if (sh->S < 1 || sh->Hq < 1 || sh->Hkv < 1 || sh->N_cap < 1 || sh->C_cap < 1)
    return fail(CK_EINVALID, "S, Hq, Hkv, N_cap and C_cap must be positive");
  if (sh->d != ck::D) return fail(CK_EUNSUPPORTED, "head dimension %d (only 128)", sh->d);
  if (sh->Hq % sh->Hkv != 0)
    return fail(CK_EINVALID, "Hq=%d is not a multiple of Hkv=%d", sh->Hq, sh->Hkv);
  const int G = sh->Hq / sh->Hkv;
  if (G != 1 && G != 2 && G != 4 && G != 8)
    return fail(CK_EUNSUPPORTED, "GQA group size %d (only 1, 2, 4, 8)", G);
  if (sh->dtype != CK_BF16 && sh->dtype != CK_F32)
    return fail(CK_EINVALID, "unknown dtype %d", sh->dtype);
  if (need_bf16 && sh->dtype != CK_BF16)
    return fail(CK_EUNSUPPORTED, "clustering runs on bf16 keys only");
  if (sh->N_cap > (int64_t)0x7FFFFFFF) return fail(CK_EUNSUPPORTED, "N_cap exceeds int32 rows");
  if ((int64_t)sh->S * sh->Hkv > 65535)
    return fail(CK_EUNSUPPORTED, "more than 65535 head-problems in one call");
  dm->S = sh->S;
  dm->Hq = sh->Hq;
  dm->Hkv = sh->Hkv;
  dm->G = G;
  dm->HP = sh->S * sh->Hkv;
  dm->N_cap = sh->N_cap;
  dm->C_cap = sh->C_cap;
  dm->dtype = sh->dtype;
  return CK_OK;
}

int check_ranges(const ck_shape* sh, int64_t tok_begin, int64_t tok_count, int32_t c_begin,
                 int32_t c_count) {
  if (tok_begin < 0 || tok_count < 1 || tok_begin + tok_count > sh->N_cap)
    return fail(CK_EINVALID, "token range [%lld, +%lld) outside [0, %lld]", (long long)tok_begin,
                (long long)tok_count, (long long)sh->N_cap);
  if (c_begin < 0 || c_count < 1 || (int64_t)c_begin + c_count > sh->C_cap)
    return fail(CK_EINVALID, "cluster range [%d, +%d) outside [0, %d]", c_begin, c_count,
                sh->C_cap);
  if (c_count > CK_MAX_CLUSTERS)
    return fail(CK_EUNSUPPORTED, "%d clusters (at most %d)", c_count, CK_MAX_CLUSTERS);
  if (c_count > tok_count)
    return fail(CK_EINVALID, "more clusters (%d) than tokens (%lld)", c_count,
                (long long)tok_count);
  return CK_OK;
}

int hip_result(hipError_t e, const char* what) {
  if (e == hipSuccess) return CK_OK;
  return fail(CK_EHIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

extern "C" {

int ck_version(void) { return CK_VERSION; }

const char* ck_strerror(int code) {
  switch (code) {
    case CK_OK: return "success";
    case CK_EINVALID: return "invalid argument";
    case CK_EUNSUPPORTED: return "unsupported shape or type";
    case CK_EWORKSPACE: return "workspace missing or too small";
    case CK_EMISALIGNED: return "misaligned device pointer";
    case CK_EHIP: return "HIP runtime error";
    default: return "unknown error code";
  }
}

const char* ck_last_error_detail(void) { return g_detail; }

size_t ck_workspace_bytes(const ck_shape* sh, int which, int64_t n, int32_t c) {
  ck::Dims dm;
  if (check_shape(sh, &dm, false) != CK_OK) return 0;
  if (which == CK_WS_CLUSTER_KEYS) {
    if (n < 1 || c < 1 || c > CK_MAX_CLUSTERS) return 0;
    return ck::carve_cluster_workspace(dm, n, c, nullptr).bytes;
  }
  if (which == CK_WS_SPARSE_ATTN) {
    if (n < 0) return 0;
    return ck::attn_workspace_bytes(dm, n);
  }
  if (which == CK_WS_OBJECTIVE) {
    if (n < 1) return 0;
    return ck::objective_workspace_bytes(dm, n);
  }
  return 0;
}

int ck_kmeans_assign(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                     const void* centroids_hat, int32_t c_begin, int32_t c_count,
                     int32_t* labels, float* best_sim, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, true);
  if (rc) return rc;
  if ((rc = check_ranges(sh, tok_begin, tok_count, c_begin, c_count))) return rc;
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(centroids_hat);
  CK_REQUIRE_PTR(labels);
  CK_OPTIONAL_PTR(best_sim);
  return hip_result(ck::launch_assign(dm, (const ck::bf16*)K, tok_begin, tok_count,
                                      (const ck::bf16*)centroids_hat, c_begin, c_count, labels,
                                      best_sim, nullptr, ck::KmCtl(), (hipStream_t)stream),
                    "assignment launch");
}

int ck_kmeans_objective(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                        const void* centroids_hat, int32_t c_begin, int32_t c_count,
                        const int32_t* labels, double* J, double* D, void* workspace,
                        size_t workspace_bytes, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, true);
  if (rc) return rc;
  if ((rc = check_ranges(sh, tok_begin, tok_count, c_begin, c_count))) return rc;
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(centroids_hat);
  CK_REQUIRE_PTR(labels);
  CK_REQUIRE_PTR(J);
  CK_REQUIRE_PTR(D);
  if (!workspace) return fail(CK_EWORKSPACE, "workspace is NULL");
  if (!aligned16(workspace)) return fail(CK_EMISALIGNED, "workspace is not 16-byte aligned");
  const size_t need = ck::objective_workspace_bytes(dm, tok_count);
  if (workspace_bytes < need)
    return fail(CK_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  return hip_result(ck::launch_objective(dm, (const ck::bf16*)K, tok_begin, tok_count,
                                         (const ck::bf16*)centroids_hat, c_begin, c_count, labels,
                                         J, D, workspace, (hipStream_t)stream),
                    "objective launch");
}

int ck_build_metadata(const ck_shape* sh, const int32_t* labels, int64_t tok_begin,
                      int64_t tok_count, int32_t c_begin, int32_t c_count, int32_t* sizes,
                      int32_t* offsets, int32_t* sorted_idx, void* workspace,
                      size_t workspace_bytes, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if ((rc = check_ranges(sh, tok_begin, tok_count, c_begin, c_count))) return rc;
  CK_REQUIRE_PTR(labels);
  CK_REQUIRE_PTR(sizes);
  CK_REQUIRE_PTR(offsets);
  CK_REQUIRE_PTR(sorted_idx);
  if (!workspace) return fail(CK_EWORKSPACE, "workspace is NULL");
  if (!aligned16(workspace)) return fail(CK_EMISALIGNED, "workspace is not 16-byte aligned");
  const ck::ClusterWorkspace ws = ck::carve_cluster_workspace(dm, tok_count, c_count, workspace);
  if (workspace_bytes < ws.bytes)
    return fail(CK_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws.bytes);
  return hip_result(ck::launch_metadata(dm, labels, tok_begin, tok_count, c_begin, c_count, sizes,
                                        offsets, sorted_idx, ws.chunk_hist, false, nullptr,
                                        (hipStream_t)stream),
                    "metadata launch");
}

int ck_kmeans_update(const ck_shape* sh, const void* K, const int32_t* sizes,
                     const int32_t* offsets, const int32_t* sorted_idx, int32_t c_begin,
                     int32_t c_count, void* centroids, void* centroids_hat,
                     float* centroids_f32, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, true);
  if (rc) return rc;
  if (c_begin < 0 || c_count < 1 || (int64_t)c_begin + c_count > sh->C_cap)
    return fail(CK_EINVALID, "cluster range [%d, +%d) outside [0, %d]", c_begin, c_count,
                sh->C_cap);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(sizes);
  CK_REQUIRE_PTR(offsets);
  CK_REQUIRE_PTR(sorted_idx);
  CK_REQUIRE_PTR(centroids);
  CK_REQUIRE_PTR(centroids_hat);
  CK_OPTIONAL_PTR(centroids_f32);
  return hip_result(ck::launch_update(dm, (const ck::bf16*)K, offsets, sorted_idx, c_begin,
                                      c_count, (ck::bf16*)centroids, (ck::bf16*)centroids_hat,
                                      centroids_f32, CK_METRIC_COSINE, nullptr, 0, nullptr,
                                      (hipStream_t)stream),
                    "update launch");
}

int ck_cluster_keys_opt(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                        int32_t c_begin, int32_t c_count, int32_t max_iter, uint32_t flags,
                        const int32_t* init_idx, void* centroids, int32_t* labels, int32_t* sizes,
                        int32_t* offsets, int32_t* sorted_idx, int32_t* iters_done,
                        void* workspace, size_t workspace_bytes, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, true);
  if (rc) return rc;
  if ((rc = check_ranges(sh, tok_begin, tok_count, c_begin, c_count))) return rc;
  if (max_iter < 1) return fail(CK_EINVALID, "n_iter=%d must be at least 1", max_iter);
  const int metric = (int)(flags & CK_METRIC_MASK);
  const bool converge = (flags & CK_KM_UNTIL_CONVERGED) != 0;
  if (metric > CK_METRIC_IP || (flags & ~(CK_METRIC_MASK | CK_KM_UNTIL_CONVERGED)))
    return fail(CK_EINVALID, "unknown flags 0x%x", flags);
  if (converge && max_iter > ck::KM_MAX_ITER_CONVERGE)
    return fail(CK_EUNSUPPORTED, "at most %d iterations in run-until-convergence mode",
                ck::KM_MAX_ITER_CONVERGE);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(init_idx);
  CK_REQUIRE_PTR(centroids);
  CK_REQUIRE_PTR(labels);
  CK_REQUIRE_PTR(sizes);
  CK_REQUIRE_PTR(offsets);
  CK_REQUIRE_PTR(sorted_idx);
  CK_OPTIONAL_PTR(iters_done);
  if (!workspace) return fail(CK_EWORKSPACE, "workspace is NULL");
  if (!aligned16(workspace)) return fail(CK_EMISALIGNED, "workspace is not 16-byte aligned");
  const ck::ClusterWorkspace ws = ck::carve_cluster_workspace(dm, tok_count, c_count, workspace);
  if (workspace_bytes < ws.bytes)
    return fail(CK_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws.bytes);

  hipStream_t st = (hipStream_t)stream;
  const ck::bf16* Kb = (const ck::bf16*)K;
  if (ck::kmeans_small_fits(tok_count, c_count))        // a few hundred tokens: one launch does it all
    return hip_result(ck::launch_kmeans_small(dm, Kb, tok_begin, tok_count, c_begin, c_count,
                                              max_iter, metric, converge, init_idx,
                                              (ck::bf16*)centroids, labels, sizes, offsets,
                                              sorted_idx, iters_done, st),
                      "small K-means launch");
  float* bias = metric == CK_METRIC_L2 ? ws.bias : nullptr;
  hipError_t e = ck::launch_init_centroids(dm, Kb, init_idx, c_begin, c_count,
                                           (ck::bf16*)centroids, ws.mu_hat, metric, bias,
                                           ws.bias_stride, st);
  if (e != hipSuccess) return hip_result(e, "init launch");
  if (converge) {
    // one row of changed-label counters per iteration, all zero: a head-problem that
    // stops leaves its later rows at zero, which is what keeps it stopped
    e = ck::launch_fill_i32(ws.changed, (int64_t)max_iter * dm.HP, 0, st);
    if (e != hipSuccess) return hip_result(e, "counter fill launch");
  }
  for (int it = 0; it < max_iter; ++it) {
    ck::KmCtl ctl;
    ctl.bias = bias;
    ctl.bias_stride = ws.bias_stride;
    const int32_t* gate = nullptr;
    if (converge) {
      ctl.changed = ws.changed + (int64_t)it * dm.HP;
      ctl.first = it == 0;
      ctl.skip = it >= 2 ? ws.changed + (int64_t)(it - 1) * dm.HP : nullptr;
      gate = it >= 1 ? ctl.changed : nullptr;
    }
    e = ck::launch_assign(dm, Kb, tok_begin, tok_count, ws.mu_hat, c_begin, c_count, labels,
                          nullptr, ws.chunk_hist, ctl, st);
    if (e != hipSuccess) return hip_result(e, "assignment launch");
    e = ck::launch_metadata(dm, labels, tok_begin, tok_count, c_begin, c_count, sizes, offsets,
                            sorted_idx, ws.chunk_hist, true, gate, st);
    if (e != hipSuccess) return hip_result(e, "metadata launch");
    e = ck::launch_update(dm, Kb, offsets, sorted_idx, c_begin, c_count, (ck::bf16*)centroids,
                          ws.mu_hat, nullptr, metric, bias, ws.bias_stride, gate, st);
    if (e != hipSuccess) return hip_result(e, "update launch");
  }
  if (iters_done) {
    if (converge)
      e = ck::launch_iters_done(ws.changed, max_iter, dm.HP, iters_done, st);
    else
      e = ck::launch_fill_i32(iters_done, dm.HP, max_iter, st);
    if (e != hipSuccess) return hip_result(e, "iteration count launch");
  }
  return CK_OK;
}

int ck_cluster_keys(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                    int32_t c_begin, int32_t c_count, int32_t n_iter, const int32_t* init_idx,
                    void* centroids, int32_t* labels, int32_t* sizes, int32_t* offsets,
                    int32_t* sorted_idx, void* workspace, size_t workspace_bytes, void* stream) {
  return ck_cluster_keys_opt(sh, K, tok_begin, tok_count, c_begin, c_count, n_iter,
                             CK_METRIC_COSINE, init_idx, centroids, labels, sizes, offsets,
                             sorted_idx, nullptr, workspace, workspace_bytes, stream);
}

int ck_select_clusters(const ck_shape* sh, const void* q, const void* centroids,
                       const int32_t* sizes, int32_t n_clusters, int32_t budget, uint32_t flags,
                       int32_t* sel_clusters, int32_t* n_sel_clusters, int32_t* n_sel_tokens,
                       float* scores, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (n_clusters < 1 || n_clusters > sh->C_cap)
    return fail(CK_EINVALID, "n_clusters=%d outside [1, C_cap=%d]", n_clusters, sh->C_cap);
  if (n_clusters > CK_MAX_CLUSTERS)
    return fail(CK_EUNSUPPORTED, "%d clusters (at most %d)", n_clusters, CK_MAX_CLUSTERS);
  if (budget < 1) return fail(CK_EINVALID, "budget=%d must be positive", budget);
  if (flags > CK_SEL_TRIM_LAST) return fail(CK_EINVALID, "unknown flags 0x%x", flags);
  CK_REQUIRE_PTR(q);
  CK_REQUIRE_PTR(centroids);
  CK_REQUIRE_PTR(sizes);
  CK_REQUIRE_PTR(sel_clusters);
  CK_REQUIRE_PTR(n_sel_clusters);
  CK_REQUIRE_PTR(n_sel_tokens);
  CK_REQUIRE_PTR(scores);
  return hip_result(ck::launch_select(dm, q, centroids, sizes, n_clusters, budget, flags,
                                      sel_clusters, n_sel_clusters, n_sel_tokens, scores,
                                      (hipStream_t)stream),
                    "selection launch");
}

int ck_gather_indices(const ck_shape* sh, const int32_t* sel_clusters,
                      const int32_t* n_sel_clusters, const int32_t* offsets,
                      const int32_t* sorted_idx, int32_t budget, uint32_t flags,
                      int32_t* token_idx, int32_t idx_stride, int32_t* n_tokens, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (budget < 1) return fail(CK_EINVALID, "budget=%d must be positive", budget);
  if (idx_stride < budget)
    return fail(CK_EINVALID, "idx_stride=%d smaller than budget=%d", idx_stride, budget);
  if (idx_stride % 4 != 0) return fail(CK_EMISALIGNED, "idx_stride=%d not a multiple of 4", idx_stride);
  if (flags > CK_SEL_TRIM_LAST) return fail(CK_EINVALID, "unknown flags 0x%x", flags);
  CK_REQUIRE_PTR(sel_clusters);
  CK_REQUIRE_PTR(n_sel_clusters);
  CK_REQUIRE_PTR(offsets);
  CK_REQUIRE_PTR(sorted_idx);
  CK_REQUIRE_PTR(token_idx);
  CK_REQUIRE_PTR(n_tokens);
  return hip_result(ck::launch_gather(dm, sel_clusters, n_sel_clusters, offsets, sorted_idx,
                                      budget, flags, token_idx, idx_stride, n_tokens,
                                      (hipStream_t)stream),
                    "gather launch");
}

static int sparse_decode_attn(bool two_pass, const ck_shape* sh, const void* q, const void* K, const void* V,
                          const int32_t* token_idx, const int32_t* n_tokens, int32_t idx_stride,
                          int32_t max_tokens, int64_t n_sink, int64_t recent_begin,
                          int64_t recent_end, float softmax_scale, void* out, void* workspace,
                          size_t workspace_bytes, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (n_sink < 0 || n_sink > sh->N_cap)
    return fail(CK_EINVALID, "n_sink=%lld outside [0, N_cap]", (long long)n_sink);
  if (recent_end < recent_begin) recent_end = recent_begin;
  if (recent_begin < 0 || recent_end > sh->N_cap)
    return fail(CK_EINVALID, "recent window [%lld, %lld) outside [0, N_cap]",
                (long long)recent_begin, (long long)recent_end);
  if (max_tokens < 0) return fail(CK_EINVALID, "max_tokens=%d is negative", max_tokens);
  if (!n_tokens) max_tokens = 0;
  if (n_tokens && max_tokens > 0) {
    if (!token_idx) return fail(CK_EINVALID, "token_idx is NULL but n_tokens is given");
    if (idx_stride < max_tokens)
      return fail(CK_EINVALID, "idx_stride=%d smaller than max_tokens=%d", idx_stride, max_tokens);
  }
  if (!(softmax_scale > 0.f)) return fail(CK_EINVALID, "softmax_scale must be positive");
  CK_REQUIRE_PTR(q);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(V);
  CK_REQUIRE_PTR(out);
  CK_OPTIONAL_PTR(token_idx);
  CK_OPTIONAL_PTR(n_tokens);
  const int64_t max_total = (int64_t)max_tokens + n_sink + (recent_end - recent_begin);
  if (max_total > (int64_t)1 << 30) return fail(CK_EUNSUPPORTED, "attended set too large");
  const size_t need = ck::attn_workspace_bytes(dm, max_total);
  if (!workspace) return fail(CK_EWORKSPACE, "workspace is NULL");
  if (!aligned16(workspace)) return fail(CK_EMISALIGNED, "workspace is not 16-byte aligned");
  if (workspace_bytes < need)
    return fail(CK_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  return hip_result(ck::launch_sparse_attn(dm, q, K, V, token_idx, n_tokens, idx_stride,
                                           max_total, n_sink, recent_begin, recent_end,
                                           softmax_scale, out, workspace, two_pass,
                                           (hipStream_t)stream),
                    "attention launch");
}

int ck_sparse_decode_attn(const ck_shape* sh, const void* q, const void* K, const void* V,
                          const int32_t* token_idx, const int32_t* n_tokens, int32_t idx_stride,
                          int32_t max_tokens, int64_t n_sink, int64_t recent_begin,
                          int64_t recent_end, float softmax_scale, void* out, void* workspace,
                          size_t workspace_bytes, void* stream) {
  return sparse_decode_attn(false, sh, q, K, V, token_idx, n_tokens, idx_stride, max_tokens,
                            n_sink, recent_begin, recent_end, softmax_scale, out, workspace,
                            workspace_bytes, stream);
}

int ck_sparse_decode_attn_two_pass(const ck_shape* sh, const void* q, const void* K,
                                   const void* V, const int32_t* token_idx,
                                   const int32_t* n_tokens, int32_t idx_stride,
                                   int32_t max_tokens, int64_t n_sink, int64_t recent_begin,
                                   int64_t recent_end, float softmax_scale, void* out,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  return sparse_decode_attn(true, sh, q, K, V, token_idx, n_tokens, idx_stride, max_tokens,
                            n_sink, recent_begin, recent_end, softmax_scale, out, workspace,
                            workspace_bytes, stream);
}

int ck_sparse_decode_attn_static(const ck_shape* sh, const void* q, const void* K, const void* V,
                                 const int32_t* token_idx, const int32_t* n_tokens,
                                 int32_t idx_stride, int32_t max_tokens, int64_t n_sink,
                                 int64_t recent_begin, int64_t recent_end, float softmax_scale,
                                 void* out, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (n_sink < 0 || n_sink > sh->N_cap)
    return fail(CK_EINVALID, "n_sink=%lld outside [0, N_cap]", (long long)n_sink);
  if (recent_end < recent_begin) recent_end = recent_begin;
  if (recent_begin < 0 || recent_end > sh->N_cap)
    return fail(CK_EINVALID, "recent window [%lld, %lld) outside [0, N_cap]",
                (long long)recent_begin, (long long)recent_end);
  if (max_tokens < 0) return fail(CK_EINVALID, "max_tokens=%d is negative", max_tokens);
  if (!n_tokens) max_tokens = 0;
  if (n_tokens && max_tokens > 0) {
    if (!token_idx) return fail(CK_EINVALID, "token_idx is NULL but n_tokens is given");
    if (idx_stride < max_tokens)
      return fail(CK_EINVALID, "idx_stride=%d smaller than max_tokens=%d", idx_stride, max_tokens);
  }
  if (!(softmax_scale > 0.f)) return fail(CK_EINVALID, "softmax_scale must be positive");
  CK_REQUIRE_PTR(q);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(V);
  CK_REQUIRE_PTR(out);
  CK_OPTIONAL_PTR(token_idx);
  CK_OPTIONAL_PTR(n_tokens);
  const int64_t max_total = (int64_t)max_tokens + n_sink + (recent_end - recent_begin);
  if (max_total > (int64_t)1 << 30) return fail(CK_EUNSUPPORTED, "attended set too large");
  const size_t need = ck::attn_workspace_bytes(dm, max_total);
  if (need > (size_t)CK_STATIC_SCRATCH_BYTES)
    return fail(CK_EWORKSPACE,
                "this shape needs %zu bytes of scratch, the built-in buffer holds %zu: use "
                "ck_sparse_decode_attn with a workspace",
                need, (size_t)CK_STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  const hipError_t e = ck::attn_static_scratch(&ws);
  if (e != hipSuccess) return hip_result(e, "address of the built-in scratch buffer");
  return hip_result(ck::launch_sparse_attn(dm, q, K, V, token_idx, n_tokens, idx_stride,
                                           max_total, n_sink, recent_begin, recent_end,
                                           softmax_scale, out, ws, false, (hipStream_t)stream),
                    "attention launch");
}

int ck_decode_step(const ck_shape* sh, const void* q, const void* K, const void* V,
                   const void* centroids, const int32_t* sizes, const int32_t* offsets,
                   const int32_t* sorted_idx, int32_t n_clusters, int32_t budget, uint32_t flags,
                   int64_t n_sink, int64_t recent_begin, int64_t recent_end, float softmax_scale,
                   float* scores, int32_t* sel_clusters, int32_t* n_sel_clusters,
                   int32_t* n_sel_tokens, int32_t* token_idx, int32_t idx_stride,
                   int32_t* n_tokens, void* out, void* workspace, size_t workspace_bytes,
                   void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (n_clusters < 1 || n_clusters > sh->C_cap)
    return fail(CK_EINVALID, "n_clusters=%d outside [1, C_cap=%d]", n_clusters, sh->C_cap);
  if (n_clusters > CK_MAX_CLUSTERS)
    return fail(CK_EUNSUPPORTED, "%d clusters (at most %d)", n_clusters, CK_MAX_CLUSTERS);
  if (budget < 1) return fail(CK_EINVALID, "budget=%d must be positive", budget);
  if (flags > CK_SEL_TRIM_LAST) return fail(CK_EINVALID, "unknown flags 0x%x", flags);
  if (idx_stride < budget)
    return fail(CK_EINVALID, "idx_stride=%d smaller than budget=%d", idx_stride, budget);
  if (idx_stride % 4 != 0)
    return fail(CK_EMISALIGNED, "idx_stride=%d not a multiple of 4", idx_stride);
  if (n_sink < 0 || n_sink > sh->N_cap)
    return fail(CK_EINVALID, "n_sink=%lld outside [0, N_cap]", (long long)n_sink);
  if (recent_end < recent_begin) recent_end = recent_begin;
  if (recent_begin < 0 || recent_end > sh->N_cap)
    return fail(CK_EINVALID, "recent window [%lld, %lld) outside [0, N_cap]",
                (long long)recent_begin, (long long)recent_end);
  if (!(softmax_scale > 0.f)) return fail(CK_EINVALID, "softmax_scale must be positive");
  CK_REQUIRE_PTR(q);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(V);
  CK_REQUIRE_PTR(centroids);
  CK_REQUIRE_PTR(sizes);
  CK_REQUIRE_PTR(offsets);
  CK_REQUIRE_PTR(sorted_idx);
  CK_REQUIRE_PTR(scores);
  CK_REQUIRE_PTR(sel_clusters);
  CK_REQUIRE_PTR(n_sel_clusters);
  CK_REQUIRE_PTR(n_sel_tokens);
  CK_REQUIRE_PTR(token_idx);
  CK_REQUIRE_PTR(n_tokens);
  CK_REQUIRE_PTR(out);
  const int64_t max_total = (int64_t)budget + n_sink + (recent_end - recent_begin);
  if (max_total > (int64_t)1 << 30) return fail(CK_EUNSUPPORTED, "attended set too large");
  const size_t need = ck::attn_workspace_bytes(dm, max_total);
  if (!workspace) return fail(CK_EWORKSPACE, "workspace is NULL");
  if (!aligned16(workspace)) return fail(CK_EMISALIGNED, "workspace is not 16-byte aligned");
  if (workspace_bytes < need)
    return fail(CK_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  return hip_result(
      ck::launch_decode_fused(dm, q, K, V, centroids, sizes, offsets, sorted_idx, n_clusters,
                              budget, flags, n_sink, recent_begin, recent_end, softmax_scale,
                              scores, sel_clusters, n_sel_clusters, n_sel_tokens, token_idx,
                              idx_stride, n_tokens, out, workspace, (hipStream_t)stream),
      "fused decode launch");
}

int ck_full_decode_attn(const ck_shape* sh, const void* q, const void* K, const void* V,
                        int64_t n_ctx, float softmax_scale, void* out, void* workspace,
                        size_t workspace_bytes, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (n_ctx < 1 || n_ctx > sh->N_cap)
    return fail(CK_EINVALID, "n_ctx=%lld outside [1, N_cap]", (long long)n_ctx);
  if (n_ctx > (int64_t)1 << 30) return fail(CK_EUNSUPPORTED, "attended set too large");
  if (!(softmax_scale > 0.f)) return fail(CK_EINVALID, "softmax_scale must be positive");
  CK_REQUIRE_PTR(q);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(V);
  CK_REQUIRE_PTR(out);
  const size_t need = ck::attn_workspace_bytes(dm, n_ctx);
  if (!workspace) return fail(CK_EWORKSPACE, "workspace is NULL");
  if (!aligned16(workspace)) return fail(CK_EMISALIGNED, "workspace is not 16-byte aligned");
  if (workspace_bytes < need)
    return fail(CK_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  // the leading "sink" range of the attended set, stretched over the whole context
  return hip_result(ck::launch_sparse_attn(dm, q, K, V, nullptr, nullptr, 0, n_ctx, n_ctx, 0, 0,
                                           softmax_scale, out, workspace, false,
                                           (hipStream_t)stream),
                    "full attention launch");
}

int ck_token_scores(const ck_shape* sh, const void* q, const void* K, int64_t tok_begin,
                    int64_t tok_count, float* scores, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (tok_begin < 0 || tok_count < 1 || tok_begin + tok_count > sh->N_cap)
    return fail(CK_EINVALID, "token range [%lld, +%lld) outside [0, %lld]", (long long)tok_begin,
                (long long)tok_count, (long long)sh->N_cap);
  CK_REQUIRE_PTR(q);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(scores);
  return hip_result(ck::launch_row_scores(dm, q, K, dm.N_cap, tok_begin, (int)tok_count, scores,
                                          dm.N_cap, (hipStream_t)stream),
                    "token score launch");
}

int ck_topk_select(int32_t n_problems, const float* scores, int64_t row_stride, int64_t begin,
                   int32_t n, int32_t k, int32_t* out_idx, int32_t out_stride, int32_t* n_out,
                   void* stream) {
  if (n_problems < 1 || n_problems > 65535)
    return fail(CK_EINVALID, "n_problems=%d outside [1, 65535]", n_problems);
  if (n < 1 || k < 0) return fail(CK_EINVALID, "n=%d must be positive and k=%d non-negative", n, k);
  if (begin < 0 || row_stride < begin + n)
    return fail(CK_EINVALID, "range [%lld, +%d) outside a row of %lld", (long long)begin, n,
                (long long)row_stride);
  if (begin + n > (int64_t)0x7FFFFFFF) return fail(CK_EUNSUPPORTED, "indices exceed int32");
  if (out_stride < (k < n ? k : n))
    return fail(CK_EINVALID, "out_stride=%d smaller than min(k, n)", out_stride);
  CK_REQUIRE_PTR(scores);
  CK_REQUIRE_PTR(out_idx);
  CK_REQUIRE_PTR(n_out);
  return hip_result(ck::launch_topk(n_problems, scores, row_stride, begin, n, k, out_idx,
                                    out_stride, n_out, (hipStream_t)stream),
                    "top-k launch");
}

int ck_recall_hits(int32_t n_problems, const int32_t* token_idx, const int32_t* n_tokens,
                   int32_t idx_stride, const int32_t* ref_idx, const int32_t* n_ref,
                   int32_t ref_stride, int32_t* hits, void* stream) {
  if (n_problems < 1 || n_problems > 65535)
    return fail(CK_EINVALID, "n_problems=%d outside [1, 65535]", n_problems);
  if (idx_stride < 1 || ref_stride < 1)
    return fail(CK_EINVALID, "idx_stride=%d and ref_stride=%d must be positive", idx_stride,
                ref_stride);
  CK_REQUIRE_PTR(token_idx);
  CK_REQUIRE_PTR(n_tokens);
  CK_REQUIRE_PTR(ref_idx);
  CK_REQUIRE_PTR(n_ref);
  CK_REQUIRE_PTR(hits);
  return hip_result(ck::launch_recall_hits(n_problems, token_idx, n_tokens, idx_stride, ref_idx,
                                           n_ref, ref_stride, hits, (hipStream_t)stream),
                    "recall launch");
}

int ck_page_keys(const ck_shape* sh, const void* K, int64_t tok_begin, int64_t tok_count,
                 int32_t page_size, void* page_keys, int64_t page_stride, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (tok_begin < 0 || tok_count < 1 || tok_begin + tok_count > sh->N_cap)
    return fail(CK_EINVALID, "token range [%lld, +%lld) outside [0, %lld]", (long long)tok_begin,
                (long long)tok_count, (long long)sh->N_cap);
  if (page_size < 1) return fail(CK_EINVALID, "page_size=%d must be positive", page_size);
  const int64_t n_pages = (tok_count + page_size - 1) / page_size;
  if (page_stride < n_pages)
    return fail(CK_EINVALID, "page_stride=%lld smaller than the %lld pages", (long long)page_stride,
                (long long)n_pages);
  CK_REQUIRE_PTR(K);
  CK_REQUIRE_PTR(page_keys);
  return hip_result(ck::launch_page_keys(dm, K, tok_begin, tok_count, page_size, page_keys,
                                         page_stride, (hipStream_t)stream),
                    "page representative launch");
}

int ck_expand_pages(int32_t n_problems, const int32_t* page_idx, const int32_t* n_pages,
                    int32_t page_stride, int32_t page_size, int64_t tok_begin,
                    int64_t tok_count, int32_t* token_idx, int32_t idx_stride,
                    int32_t* n_tokens, void* stream) {
  if (n_problems < 1 || n_problems > 65535)
    return fail(CK_EINVALID, "n_problems=%d outside [1, 65535]", n_problems);
  if (page_size < 1 || page_stride < 1 || idx_stride < 1)
    return fail(CK_EINVALID, "page_size, page_stride and idx_stride must be positive");
  if (tok_begin < 0 || tok_count < 1 || tok_begin + tok_count > (int64_t)0x7FFFFFFF)
    return fail(CK_EINVALID, "token range [%lld, +%lld) invalid", (long long)tok_begin,
                (long long)tok_count);
  CK_REQUIRE_PTR(page_idx);
  CK_REQUIRE_PTR(n_pages);
  CK_REQUIRE_PTR(token_idx);
  CK_REQUIRE_PTR(n_tokens);
  return hip_result(ck::launch_expand_pages(n_problems, page_idx, n_pages, page_stride, page_size,
                                            tok_begin, tok_count, token_idx, idx_stride, n_tokens,
                                            (hipStream_t)stream),
                    "page expansion launch");
}

int ck_host_device_ptr(void* host_ptr, void** dev_ptr) {
  if (!host_ptr || !dev_ptr) return fail(CK_EINVALID, "host_ptr or dev_ptr is NULL");
  void* d = nullptr;
  const hipError_t e = hipHostGetDevicePointer(&d, host_ptr, 0);
  if (e != hipSuccess || !d) {
    (void)hipGetLastError();
    return fail(CK_EHIP, "not mapped pinned host memory: %s", hipGetErrorString(e));
  }
  *dev_ptr = d;
  return CK_OK;
}

namespace {
int check_cache(const ck_shape* sh, const ck_cluster_cache* cache) {
  if (!cache) return fail(CK_EINVALID, "cache is NULL");
  if (cache->cap_tokens < 1) return fail(CK_EINVALID, "cap_tokens=%d must be positive", cache->cap_tokens);
  for (int g = 0; g < 2; ++g) {
    CK_REQUIRE_PTR(cache->K[g]);
    CK_REQUIRE_PTR(cache->V[g]);
    CK_REQUIRE_PTR(cache->clusters[g]);
    CK_REQUIRE_PTR(cache->starts[g]);
    CK_REQUIRE_PTR(cache->n_held[g]);
  }
  (void)sh;
  return CK_OK;
}
}  // namespace

int ck_cache_reset(const ck_shape* sh, const ck_cluster_cache* cache, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if ((rc = check_cache(sh, cache))) return rc;
  for (int g = 0; g < 2; ++g) {
    const hipError_t e = ck::launch_fill_i32(cache->n_held[g], dm.HP, 0, (hipStream_t)stream);
    if (e != hipSuccess) return hip_result(e, "cache reset launch");
  }
  return CK_OK;
}

int ck_cached_decode_step(const ck_shape* sh, const void* q, const void* K_home,
                          const void* V_home, const void* centroids, const int32_t* sizes,
                          const int32_t* offsets, const int32_t* sorted_idx, int32_t n_clusters,
                          int32_t budget, const ck_cluster_cache* cache, int32_t step_parity,
                          float softmax_scale, float* scores, int32_t* sel_clusters,
                          int32_t* n_sel_clusters, int32_t* n_sel_tokens, int32_t* miss_tokens,
                          void* out, void* workspace, size_t workspace_bytes, void* stream) {
  ck::Dims dm;
  int rc = check_shape(sh, &dm, false);
  if (rc) return rc;
  if (n_clusters < 1 || n_clusters > sh->C_cap)
    return fail(CK_EINVALID, "n_clusters=%d outside [1, C_cap=%d]", n_clusters, sh->C_cap);
  if (n_clusters > CK_MAX_CLUSTERS)
    return fail(CK_EUNSUPPORTED, "%d clusters (at most %d)", n_clusters, CK_MAX_CLUSTERS);
  if (budget < 1) return fail(CK_EINVALID, "budget=%d must be positive", budget);
  if (step_parity != 0 && step_parity != 1)
    return fail(CK_EINVALID, "step_parity=%d must be 0 or 1", step_parity);
  if ((rc = check_cache(sh, cache))) return rc;
  if (budget > cache->cap_tokens)
    return fail(CK_EINVALID, "budget=%d exceeds the cache's %d rows", budget, cache->cap_tokens);
  if (!(softmax_scale > 0.f)) return fail(CK_EINVALID, "softmax_scale must be positive");
  CK_REQUIRE_PTR(q);
  CK_REQUIRE_PTR(K_home);
  CK_REQUIRE_PTR(V_home);
  CK_REQUIRE_PTR(centroids);
  CK_REQUIRE_PTR(sizes);
  CK_REQUIRE_PTR(offsets);
  CK_REQUIRE_PTR(sorted_idx);
  CK_REQUIRE_PTR(scores);
  CK_REQUIRE_PTR(sel_clusters);
  CK_REQUIRE_PTR(n_sel_clusters);
  CK_REQUIRE_PTR(n_sel_tokens);
  CK_REQUIRE_PTR(miss_tokens);
  CK_REQUIRE_PTR(out);
  ck::Dims dc = dm;                                     // the cache buffers as the K/V of attention
  dc.N_cap = cache->cap_tokens;
  const size_t need = ck::attn_workspace_bytes(dm, budget);
  if (!workspace) return fail(CK_EWORKSPACE, "workspace is NULL");
  if (!aligned16(workspace)) return fail(CK_EMISALIGNED, "workspace is not 16-byte aligned");
  if (workspace_bytes < need)
    return fail(CK_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = ck::launch_select(dm, q, centroids, sizes, n_clusters, budget, CK_SEL_WHOLE,
                                   sel_clusters, n_sel_clusters, n_sel_tokens, scores, st);
  if (e != hipSuccess) return hip_result(e, "selection launch");
  const int g = step_parity, o = step_parity ^ 1;
  ck::CacheArgs a;
  a.K_home = K_home;
  a.V_home = V_home;
  a.K_old = cache->K[o];
  a.V_old = cache->V[o];
  a.K_new = cache->K[g];
  a.V_new = cache->V[g];
  a.old_clusters = cache->clusters[o];
  a.old_starts = cache->starts[o];
  a.old_n = cache->n_held[o];
  a.new_clusters = cache->clusters[g];
  a.new_starts = cache->starts[g];
  a.new_n = cache->n_held[g];
  a.sel_clusters = sel_clusters;
  a.n_sel_clusters = n_sel_clusters;
  a.sizes = sizes;
  a.offsets = offsets;
  a.sorted_idx = sorted_idx;
  a.miss_tokens = miss_tokens;
  a.N_cap = dm.N_cap;
  a.C_cap = dm.C_cap;
  a.cap = cache->cap_tokens;
  a.row_bytes = dm.dtype == CK_BF16 ? 256 : 512;
  e = ck::launch_cache_fill(dm, a, budget, st);
  if (e != hipSuccess) return hip_result(e, "cache fill launch");
  // attention over the first n_sel_tokens rows of the new generation
  return hip_result(ck::launch_sparse_attn(dc, q, cache->K[g], cache->V[g], nullptr, n_sel_tokens,
                                           0, budget, 0, 0, 0, softmax_scale, out, workspace, false,
                                           st),
                    "attention launch");
}

int ck_probe_mfma_bf16(int32_t n_workgroups, int32_t iters, const void* operands,
                       uint64_t* clocks, float* sink, double* flops, void* stream) {
  if (n_workgroups < 1 || n_workgroups > 65535 || iters < 1 || iters > (1 << 24))
    return fail(CK_EINVALID, "n_workgroups=%d or iters=%d out of range", n_workgroups, iters);
  CK_REQUIRE_PTR(sink);
  if (!flops) return fail(CK_EINVALID, "flops is NULL");
  if (operands && ((uintptr_t)operands & 15)) return fail(CK_EMISALIGNED, "operands not 16-byte aligned");
  if (clocks && ((uintptr_t)clocks & 7)) return fail(CK_EMISALIGNED, "clocks not 8-byte aligned");
  // 4 wavefronts x 16 MFMAs per iteration x 2*32*32*16 flop
  *flops = (double)n_workgroups * 4.0 * 16.0 * iters * 32768.0;
  return hip_result(ck::launch_probe_mfma(n_workgroups, iters, operands, (unsigned long long*)clocks,
                                          sink, (hipStream_t)stream),
                    "MFMA probe launch");
}

}  // extern "C"
