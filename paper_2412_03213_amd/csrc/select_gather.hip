// Cluster selection (paper Section III-C) and index generation (Section IV-C, Fig. 8).
//
// One workgroup per head-problem, as in the paper (its kernels use one thread
// block per KV head with the size metadata in shared memory); scores, order,
// sizes and their prefix sum all stay in LDS.
#include "ck_common.hpp"

namespace ck {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_ITEMS = CK_MAX_CLUSTERS / SEL_THREADS;   // 2 sorted slots per thread

// Monotone map float -> uint32 (a < b  <=>  map(a) < map(b); -0 and +0 made equal).
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  if (f == 0.f) f = 0.f;                                    // -0 -> +0
  const uint32_t u = __builtin_bit_cast(uint32_t, f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

template <typename T>
__device__ __forceinline__ void load8(const T* p, float (&v)[8]);
template <>
__device__ __forceinline__ void load8<bf16>(const bf16* p, float (&v)[8]) {
  const uint4 w = *reinterpret_cast<const uint4*>(p);
  v[0] = lo_bf16(w.x); v[1] = hi_bf16(w.x); v[2] = lo_bf16(w.y); v[3] = hi_bf16(w.y);
  v[4] = lo_bf16(w.z); v[5] = hi_bf16(w.z); v[6] = lo_bf16(w.w); v[7] = hi_bf16(w.w);
}
template <>
__device__ __forceinline__ void load8<float>(const float* p, float (&v)[8]) {
  const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

template <typename T>
__global__ __launch_bounds__(SEL_THREADS) void k_select(
    const T* __restrict__ q, const T* __restrict__ centroids, const int32_t* __restrict__ sizes,
    int Hq, int Hkv, int G, int C_cap, int n_clusters, int budget, uint32_t flags,
    int32_t* __restrict__ sel_clusters, int32_t* __restrict__ n_sel_clusters,
    int32_t* __restrict__ n_sel_tokens, float* __restrict__ scores) {
  __shared__ float qsum[D];
  __shared__ __attribute__((aligned(16))) uint32_t key[CK_MAX_CLUSTERS];  // descending-score keys
  __shared__ int ord[CK_MAX_CLUSTERS];        // cluster id at each sorted position
  __shared__ int ssz[CK_MAX_CLUSTERS];        // its size
  __shared__ int tmp[SEL_THREADS / WAVE + 1];
  __shared__ int counter;

  const int hp = blockIdx.x, tid = threadIdx.x;
  const int s = hp / Hkv, h = hp % Hkv;
  const int l16 = tid & 15, grp = tid >> 4;                 // 64 groups of 16 lanes

  // sum of the group's queries: sum_g <q_g, mu> = <sum_g q_g, mu>
  if (tid < D) {
    float a = 0.f;
    for (int g = 0; g < G; ++g) a += (float)q[((int64_t)s * Hq + h * G + g) * D + tid];
    qsum[tid] = a;
  }
  if (tid == 0) counter = 0;
  __syncthreads();

  float qv[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) qv[j] = qsum[l16 * 8 + j];
  const T* Chp = centroids + (int64_t)hp * C_cap * D;
  const int n_pad = (n_clusters + 3) & ~3;
  for (int c0 = 0; c0 < n_clusters; c0 += SEL_THREADS / 16) {
    const int c = c0 + grp;
    float dot = 0.f;
    if (c < n_clusters) {
      float mv[8];
      load8<T>(Chp + (int64_t)c * D + l16 * 8, mv);
#pragma unroll
      for (int j = 0; j < 8; ++j) dot = fmaf(qv[j], mv[j], dot);
    }
    dot = row16_sum(dot);
    if (c < n_clusters && l16 == 0) {
      key[c] = ~ordered_bits(dot);                          // ascending key = descending score
      if (scores) scores[(int64_t)hp * C_cap + c] = dot;
    }
  }
  for (int j = n_clusters + tid; j < n_pad; j += SEL_THREADS) key[j] = 0xFFFFFFFFu;  // padding ranks last
  __syncthreads();

  // rank by counting: position of cluster c = #{j : key_j < key_c or (key_j == key_c and j < c)}
  const int32_t* sz = sizes + (int64_t)hp * C_cap;
  for (int c = tid; c < n_clusters; c += SEL_THREADS) {
    const uint32_t kc = key[c];
    int rank = 0;
    for (int j = 0; j < n_pad; j += 4) {
      const uint4 k4 = *reinterpret_cast<const uint4*>(&key[j]);
      rank += (k4.x < kc || (k4.x == kc && j + 0 < c)) ? 1 : 0;
      rank += (k4.y < kc || (k4.y == kc && j + 1 < c)) ? 1 : 0;
      rank += (k4.z < kc || (k4.z == kc && j + 2 < c)) ? 1 : 0;
      rank += (k4.w < kc || (k4.w == kc && j + 3 < c)) ? 1 : 0;
    }
    ord[rank] = c;
    ssz[rank] = sz[c];
  }
  __syncthreads();

  int v[SEL_ITEMS];
#pragma unroll
  for (int i = 0; i < SEL_ITEMS; ++i) {
    const int j = tid * SEL_ITEMS + i;
    v[i] = j < n_clusters ? ssz[j] : 0;
  }
  block_inclusive_scan<SEL_ITEMS>(v, tmp);
  // the prefix sums are non-decreasing, so counting them against the budget gives
  // the length of the recalled prefix
  const bool trim = (flags & CK_SEL_TRIM_LAST) != 0;
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < SEL_ITEMS; ++i) {
    const int j = tid * SEL_ITEMS + i;
    if (j < n_clusters) cnt += trim ? (v[i] < budget) : (v[i] <= budget);
    if (j < n_clusters) ssz[j] = v[i];                      // now the inclusive prefix sum
  }
  if (cnt) atomicAdd(&counter, cnt);
  __syncthreads();
  int n_sel = counter;
  if (trim) n_sel = n_sel + 1 < n_clusters ? n_sel + 1 : n_clusters;
  for (int j = tid; j < n_clusters; j += SEL_THREADS)
    sel_clusters[(int64_t)hp * C_cap + j] = ord[j];
  if (tid == 0) {
    int n_tok = n_sel > 0 ? ssz[n_sel - 1] : 0;
    if (trim && n_tok > budget) n_tok = budget;
    n_sel_clusters[hp] = n_sel;
    n_sel_tokens[hp] = n_tok;
  }
}

hipError_t launch_select(const Dims& dm, const void* q, const void* centroids,
                         const int32_t* sizes, int n_clusters, int budget, uint32_t flags,
                         int32_t* sel_clusters, int32_t* n_sel_clusters, int32_t* n_sel_tokens,
                         float* scores, hipStream_t st) {
  if (dm.dtype == CK_BF16)
    hipLaunchKernelGGL(k_select<bf16>, dim3(dm.HP), dim3(SEL_THREADS), 0, st,
                       (const bf16*)q, (const bf16*)centroids, sizes, dm.Hq, dm.Hkv, dm.G,
                       dm.C_cap, n_clusters, budget, flags, sel_clusters, n_sel_clusters,
                       n_sel_tokens, scores);
  else
    hipLaunchKernelGGL(k_select<float>, dim3(dm.HP), dim3(SEL_THREADS), 0, st,
                       (const float*)q, (const float*)centroids, sizes, dm.Hq, dm.Hkv, dm.G,
                       dm.C_cap, n_clusters, budget, flags, sel_clusters, n_sel_clusters,
                       n_sel_tokens, scores);
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
