// Cluster selection (paper Section III-C) and index generation (Section IV-C, Fig. 8).
#include <type_traits>

#include "decode_common.hpp"

namespace ck {

// ------------------------------------------------------------------ scoring
// s_c = sum_g <q_g, mu_c>.  The centroid table is the second largest byte stream of a
// decode step, so it is spread over many workgroups (64 or 256 rows each) instead of
// one per head-problem.  bf16 tables go through the matrix cores (score_rows16: 16 rows
// per wavefront step, all loads of a wavefront issued before the first use); fp32
// tables (check mode) keep dot products on the vector ALUs, 16 lanes per row.
constexpr int SCORE_THREADS = 256;

// SCORE_ROWS rows per workgroup: 64 when there are few head-problems (more workgroups,
// lower latency), 256 when there are many (more bytes in flight per workgroup).
template <typename T, int SCORE_ROWS>
__global__ __launch_bounds__(SCORE_THREADS) void k_score(
    const T* __restrict__ q, const T* __restrict__ table, int Hq, int Hkv, int G,
    int64_t table_stride, int64_t row_begin, int n_rows, float* __restrict__ scores,
    int64_t score_stride) {
  const int hp = blockIdx.y, tid = threadIdx.x;
  const int s = hp / Hkv, h = hp % Hkv;
  const int c0 = blockIdx.x * SCORE_ROWS;
  if constexpr (std::is_same<T, bf16>::value) {
    constexpr int U = SCORE_ROWS / 64;                      // 16-row steps per wavefront
    const int lane = tid & 63, wave = tid >> 6, col = lane & 15, kg = lane >> 4;
    bf16x8 qb[4];
    load_query_operand(q + ((int64_t)s * Hq + h * G) * D, G, lane, qb);
    const bf16* Thp = table + ((int64_t)hp * table_stride + row_begin) * D + kg * 8;
    uint4 a[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int r = c0 + (u * 4 + wave) * 16 + col;
      if (r >= n_rows) r = n_rows - 1;                      // clamp: result is discarded
#pragma unroll
      for (int sl = 0; sl < 4; ++sl)
        a[u][sl] = *reinterpret_cast<const uint4*>(Thp + (int64_t)r * D + sl * 32);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float v = score_rows16(a[u], qb, G);
      const int r = c0 + (u * 4 + wave) * 16 + lane;
      if (lane < 16 && r < n_rows) scores[(int64_t)hp * score_stride + row_begin + r] = v;
    }
  } else {
    const int l16 = tid & 15, grp = tid >> 4;               // 16 groups of 16 lanes
    const T* Chp = table + ((int64_t)hp * table_stride + row_begin) * D + l16 * 8;
    float mv[SCORE_ROWS / 16][8];
#pragma unroll
    for (int u = 0; u < SCORE_ROWS / 16; ++u) {
      int c = c0 + u * 16 + grp;
      if (c >= n_rows) c = n_rows - 1;                      // clamp: result is discarded
      load_row8<T>(Chp + (int64_t)c * D, mv[u]);
    }
    float qv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) qv[j] = 0.f;
    for (int g = 0; g < G; ++g) {
      float t[8];
      load_row8<T>(q + ((int64_t)s * Hq + h * G + g) * D + l16 * 8, t);
#pragma unroll
      for (int j = 0; j < 8; ++j) qv[j] += t[j];
    }
#pragma unroll
    for (int u = 0; u < SCORE_ROWS / 16; ++u) {
      const int c = c0 + u * 16 + grp;
      float dot = 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) dot = fmaf(qv[j], mv[u][j], dot);
      dot = row16_sum(dot);
      if (c < n_rows && l16 == 0) scores[(int64_t)hp * score_stride + row_begin + c] = dot;
    }
  }
}

// scores[hp, row_begin + r] = <sum_g q_g, table[hp, row_begin + r]> for r < n_rows: the
// centroid table of a decode step, or any other row table laid out per head-problem
// (the keys themselves for exact token importance, page representatives).
hipError_t launch_row_scores(const Dims& dm, const void* q, const void* table,
                             int64_t table_stride, int64_t row_begin, int n_rows, float* scores,
                             int64_t score_stride, hipStream_t st) {
  const bool many = (int64_t)dm.HP * ((n_rows + 63) / 64) > 2048;
  const int rows = many ? 256 : 64;
  const dim3 grid((n_rows + rows - 1) / rows, dm.HP);
#define CK_SCORE(TT, RR)                                                                    \
  hipLaunchKernelGGL((k_score<TT, RR>), grid, dim3(SCORE_THREADS), 0, st, (const TT*)q,     \
                     (const TT*)table, dm.Hq, dm.Hkv, dm.G, table_stride, row_begin, n_rows, \
                     scores, score_stride)
  if (dm.dtype == CK_BF16) {
    if (many) CK_SCORE(bf16, 256); else CK_SCORE(bf16, 64);
  } else {
    if (many) CK_SCORE(float, 256); else CK_SCORE(float, 64);
  }
#undef CK_SCORE
  return hipGetLastError();
}

hipError_t launch_score(const Dims& dm, const void* q, const void* centroids, int n_clusters,
                        float* scores, hipStream_t st) {
  return launch_row_scores(dm, q, centroids, dm.C_cap, 0, n_clusters, scores, dm.C_cap, st);
}

// ------------------------------------------------------------------ order + budget
// One workgroup per head-problem, as in the paper (its kernels use one thread block
// per KV head with the size metadata in shared memory).
template <int CMAX>
__global__ __launch_bounds__(SELP_THREADS) void k_rank(
    const float* __restrict__ scores, const int32_t* __restrict__ sizes, int C_cap,
    int n_clusters, int budget, int trim, int32_t* __restrict__ sel_clusters,
    int32_t* __restrict__ n_sel_clusters, int32_t* __restrict__ n_sel_tokens) {
  __shared__ SelectLds<CMAX> L;
  const int hp = blockIdx.x, tid = threadIdx.x;
  select_prefix<CMAX>(L, scores + (int64_t)hp * C_cap, sizes + (int64_t)hp * C_cap, nullptr,
                n_clusters, budget, trim);
  const int n_sel = L.n_sel;
  for (int j = tid; j < n_sel; j += SELP_THREADS) sel_clusters[(int64_t)hp * C_cap + j] = L.ord[j];
  if (tid == 0) {
    n_sel_clusters[hp] = n_sel;
    n_sel_tokens[hp] = L.n_tok;
  }
}

hipError_t launch_select(const Dims& dm, const void* q, const void* centroids,
                         const int32_t* sizes, int n_clusters, int budget, uint32_t flags,
                         int32_t* sel_clusters, int32_t* n_sel_clusters, int32_t* n_sel_tokens,
                         float* scores, hipStream_t st) {
  hipError_t e = launch_score(dm, q, centroids, n_clusters, scores, st);
  if (e != hipSuccess) return e;
  if (n_clusters <= SELP_SMALL)
    hipLaunchKernelGGL(k_rank<SELP_SMALL>, dim3(dm.HP), dim3(SELP_THREADS), 0, st, scores, sizes,
                       dm.C_cap, n_clusters, budget, (int)(flags & CK_SEL_TRIM_LAST),
                       sel_clusters, n_sel_clusters, n_sel_tokens);
  else
    hipLaunchKernelGGL(k_rank<CK_MAX_CLUSTERS>, dim3(dm.HP), dim3(SELP_THREADS), 0, st, scores,
                       sizes, dm.C_cap, n_clusters, budget, (int)(flags & CK_SEL_TRIM_LAST),
                       sel_clusters, n_sel_clusters, n_sel_tokens);
  return hipGetLastError();
}

// ------------------------------------------------------------------ gather
constexpr int GAT_THREADS = 256;
constexpr int GAT_ITEMS = CK_MAX_CLUSTERS / GAT_THREADS;    // 8 selected clusters per thread

__global__ __launch_bounds__(GAT_THREADS) void k_gather(
    const int32_t* __restrict__ sel_clusters, const int32_t* __restrict__ n_sel_clusters,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ sorted_idx, int64_t N_cap,
    int C_cap, int limit, int32_t* __restrict__ token_idx, int idx_stride,
    int32_t* __restrict__ n_tokens) {
  __shared__ int src_beg[CK_MAX_CLUSTERS];
  __shared__ int dst_beg[CK_MAX_CLUSTERS];
  __shared__ int cnt[CK_MAX_CLUSTERS];
  __shared__ int tmp[GAT_THREADS / WAVE + 1];
  const int hp = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int n_sel = n_sel_clusters[hp];
  n_sel = n_sel < 0 ? 0 : (n_sel > C_cap ? C_cap : n_sel);
  if (n_sel > CK_MAX_CLUSTERS) n_sel = CK_MAX_CLUSTERS;
  const int32_t* off = offsets + (int64_t)hp * (C_cap + 1);
  const int32_t* sel = sel_clusters + (int64_t)hp * C_cap;

  int v[GAT_ITEMS], beg[GAT_ITEMS];
#pragma unroll
  for (int i = 0; i < GAT_ITEMS; ++i) {
    const int j = tid * GAT_ITEMS + i;
    v[i] = 0;
    beg[i] = 0;
    if (j < n_sel) {
      int c = sel[j];
      c = c < 0 ? 0 : (c >= C_cap ? C_cap - 1 : c);
      beg[i] = off[c];
      v[i] = off[c + 1] - off[c];
      if (v[i] < 0) v[i] = 0;
    }
  }
  int size_i[GAT_ITEMS];
#pragma unroll
  for (int i = 0; i < GAT_ITEMS; ++i) size_i[i] = v[i];
  const int total = block_inclusive_scan<GAT_ITEMS>(v, tmp);
#pragma unroll
  for (int i = 0; i < GAT_ITEMS; ++i) {
    const int j = tid * GAT_ITEMS + i;
    if (j < n_sel) {
      const int d0 = v[i] - size_i[i];                      // exclusive prefix = output position
      int take = limit - d0;
      take = take < 0 ? 0 : (take > size_i[i] ? size_i[i] : take);
      dst_beg[j] = d0;
      cnt[j] = take;
      src_beg[j] = beg[i] + size_i[i] - take;               // a cut cluster keeps its trailing entries
    }
  }
  __syncthreads();
  const int32_t* src = sorted_idx + (int64_t)hp * N_cap;
  int32_t* dst = token_idx + (int64_t)hp * idx_stride;
  for (int j = wave; j < n_sel; j += GAT_THREADS / WAVE) {
    const int n = cnt[j], sb = src_beg[j], db = dst_beg[j];
    for (int t = lane; t < n; t += WAVE) {
      const int64_t sp = (int64_t)sb + t;
      if (sp >= 0 && sp < N_cap) dst[db + t] = src[sp];
    }
  }
  if (tid == 0) n_tokens[hp] = total < limit ? total : limit;
}

hipError_t launch_gather(const Dims& dm, const int32_t* sel_clusters,
                         const int32_t* n_sel_clusters, const int32_t* offsets,
                         const int32_t* sorted_idx, int budget, uint32_t flags,
                         int32_t* token_idx, int idx_stride, int32_t* n_tokens, hipStream_t st) {
  (void)flags;  // both modes copy what fits: WHOLE never overflows, TRIM_LAST cuts the last cluster
  const int limit = budget < idx_stride ? budget : idx_stride;
  hipLaunchKernelGGL(k_gather, dim3(dm.HP), dim3(GAT_THREADS), 0, st, sel_clusters,
                     n_sel_clusters, offsets, sorted_idx, dm.N_cap, dm.C_cap, limit, token_idx,
                     idx_stride, n_tokens);
  return hipGetLastError();
}

}  // namespace ck
