// Evaluation of a selection against the exact answer (paper Section V-B, "recall
// rate of important tokens"): exact per-token importance, exact top-B tokens,
// |I_T intersect I_true|, and the page-granular selector that Section II-C
// describes (a page of consecutive tokens is represented by the per-channel
// maximum of its keys).  None of this is on the decode path; the kernels are
// simple one-workgroup-per-head-problem passes over L2-resident score arrays.
#include "decode_common.hpp"

namespace ck {

// ------------------------------------------------------------------ exact top-k
// Radix selection on the order-preserving integer image of the scores: four
// 8-bit passes find the k-th largest key exactly, then one ordered pass emits
// every index whose key is larger plus the first `r` indices whose key is equal
// (lower index first), in ascending index order.
constexpr int TOPK_THREADS = 1024;
constexpr int TOPK_ITEMS = 4;

__global__ __launch_bounds__(TOPK_THREADS) void k_topk(
    const float* __restrict__ scores, int64_t row_stride, int64_t begin, int n, int k,
    int32_t* __restrict__ out_idx, int out_stride, int32_t* __restrict__ n_out) {
  __shared__ int hist[256];
  __shared__ int tmp[TOPK_THREADS / WAVE + 1];
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining;
  const int hp = blockIdx.x, tid = threadIdx.x;
  const float* sc = scores + (int64_t)hp * row_stride + begin;
  int32_t* out = out_idx + (int64_t)hp * out_stride;
  if (k > n) k = n;
  if (tid == 0) n_out[hp] = k < 0 ? 0 : k;
  if (k <= 0) return;
  if (k == n) {
    for (int i = tid; i < n; i += TOPK_THREADS) out[i] = (int32_t)(begin + i);
    return;
  }
  uint32_t prefix = 0, mask = 0;
  int remaining = k;
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) hist[tid] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += TOPK_THREADS) {
      const uint32_t key = ordered_bits(sc[i]);
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    // thread t < 256 owns bin 255 - t: the inclusive scan counts keys in bins >= its own
    int v[1] = {tid < 256 ? hist[255 - tid] : 0};
    const int own = v[0];
    block_inclusive_scan<1>(v, tmp);
    if (tid < 256 && v[0] >= remaining && v[0] - own < remaining) {
      s_prefix = prefix | ((uint32_t)(255 - tid) << shift);
      s_remaining = remaining - (v[0] - own);
    }
    __syncthreads();
    prefix = s_prefix;
    remaining = s_remaining;
    mask |= 255u << shift;
    __syncthreads();
  }
  // prefix is the k-th largest key; `remaining` of the equal keys are taken
  int base_gt = 0, base_eq = 0;
  for (int tile0 = 0; tile0 < n; tile0 += TOPK_THREADS * TOPK_ITEMS) {
    const int i0 = tile0 + tid * TOPK_ITEMS;
    int cls[TOPK_ITEMS];                                   // 2 = larger, 1 = equal, 0 = neither
    int packed[1] = {0};
#pragma unroll
    for (int j = 0; j < TOPK_ITEMS; ++j) {
      cls[j] = 0;
      if (i0 + j < n) {
        const uint32_t key = ordered_bits(sc[i0 + j]);
        cls[j] = key > prefix ? 2 : (key == prefix ? 1 : 0);
      }
      packed[0] += cls[j] == 2 ? 1 : (cls[j] == 1 ? 0x10000 : 0);
    }
    const int mine = packed[0];
    const int total = block_inclusive_scan<1>(packed, tmp);
    const int excl = packed[0] - mine;
    int gt_before = base_gt + (excl & 0xFFFF), eq_before = base_eq + (excl >> 16);
#pragma unroll
    for (int j = 0; j < TOPK_ITEMS; ++j) {
      if (cls[j] == 2) {
        out[gt_before + (eq_before < remaining ? eq_before : remaining)] = (int32_t)(begin + i0 + j);
        ++gt_before;
      } else if (cls[j] == 1) {
        if (eq_before < remaining) out[gt_before + eq_before] = (int32_t)(begin + i0 + j);
        ++eq_before;
      }
    }
    base_gt += total & 0xFFFF;
    base_eq += total >> 16;
  }
}

hipError_t launch_topk(int HP, const float* scores, int64_t row_stride, int64_t begin, int n,
                       int k, int32_t* out_idx, int out_stride, int32_t* n_out, hipStream_t st) {
  hipLaunchKernelGGL(k_topk, dim3(HP), dim3(TOPK_THREADS), 0, st, scores, row_stride, begin, n, k,
                     out_idx, out_stride, n_out);
  return hipGetLastError();
}

// ------------------------------------------------------------------ recall hits
// hits = number of entries of the selection that occur in the reference list
// (ascending, distinct): one binary search per selected token.
constexpr int HITS_THREADS = 256;

__global__ __launch_bounds__(HITS_THREADS) void k_recall_hits(
    const int32_t* __restrict__ token_idx, const int32_t* __restrict__ n_tokens, int idx_stride,
    const int32_t* __restrict__ ref_idx, const int32_t* __restrict__ n_ref, int ref_stride,
    int32_t* __restrict__ hits) {
  __shared__ int tmp[HITS_THREADS / WAVE];
  const int hp = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int ns = n_tokens[hp], nr = n_ref[hp];
  ns = ns < 0 ? 0 : (ns > idx_stride ? idx_stride : ns);
  nr = nr < 0 ? 0 : (nr > ref_stride ? ref_stride : nr);
  const int32_t* sel = token_idx + (int64_t)hp * idx_stride;
  const int32_t* ref = ref_idx + (int64_t)hp * ref_stride;
  int count = 0;
  for (int i = tid; i < ns; i += HITS_THREADS) {
    const int32_t t = sel[i];
    int lo = 0, hi = nr;                                   // first position with ref >= t
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (ref[mid] < t) lo = mid + 1; else hi = mid;
    }
    count += (lo < nr && ref[lo] == t) ? 1 : 0;
  }
  count = __builtin_amdgcn_readlane(wave_inclusive_scan(count), WAVE - 1);
  if (lane == 0) tmp[wave] = count;
  __syncthreads();
  if (tid == 0) hits[hp] = tmp[0] + tmp[1] + tmp[2] + tmp[3];
}

hipError_t launch_recall_hits(int HP, const int32_t* token_idx, const int32_t* n_tokens,
                              int idx_stride, const int32_t* ref_idx, const int32_t* n_ref,
                              int ref_stride, int32_t* hits, hipStream_t st) {
  hipLaunchKernelGGL(k_recall_hits, dim3(HP), dim3(HITS_THREADS), 0, st, token_idx, n_tokens,
                     idx_stride, ref_idx, n_ref, ref_stride, hits);
  return hipGetLastError();
}

// ------------------------------------------------------------------ page representatives
// 16 lanes per page (8 channels each), 16 pages per workgroup.
constexpr int PAGE_THREADS = 256;

__device__ __forceinline__ void store_row8(bf16* p, const float (&v)[8]) {
  uint4 w;
  w.x = float_to_bf16_bits(v[0]) | ((uint32_t)float_to_bf16_bits(v[1]) << 16);
  w.y = float_to_bf16_bits(v[2]) | ((uint32_t)float_to_bf16_bits(v[3]) << 16);
  w.z = float_to_bf16_bits(v[4]) | ((uint32_t)float_to_bf16_bits(v[5]) << 16);
  w.w = float_to_bf16_bits(v[6]) | ((uint32_t)float_to_bf16_bits(v[7]) << 16);
  *reinterpret_cast<uint4*>(p) = w;
}
__device__ __forceinline__ void store_row8(float* p, const float (&v)[8]) {
  reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
  reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
}

template <typename T>
__global__ __launch_bounds__(PAGE_THREADS) void k_page_keys(
    const T* __restrict__ K, int64_t N_cap, int64_t tok_begin, int64_t tok_count, int page_size,
    T* __restrict__ page_keys, int64_t page_stride, int n_pages) {
  const int hp = blockIdx.y, tid = threadIdx.x, l16 = tid & 15;
  const int p = blockIdx.x * 16 + (tid >> 4);
  if (p >= n_pages) return;
  const int64_t lo = (int64_t)p * page_size;
  int64_t hi = lo + page_size;
  if (hi > tok_count) hi = tok_count;
  const T* src = K + ((int64_t)hp * N_cap + tok_begin) * D + l16 * 8;
  float best[8];
  load_row8<T>(src + lo * D, best);
  for (int64_t t = lo + 1; t < hi; ++t) {
    float v[8];
    load_row8<T>(src + t * D, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) best[j] = fmaxf(best[j], v[j]);
  }
  store_row8(page_keys + ((int64_t)hp * page_stride + p) * D + l16 * 8, best);
}

hipError_t launch_page_keys(const Dims& dm, const void* K, int64_t tok_begin, int64_t tok_count,
                            int page_size, void* page_keys, int64_t page_stride, hipStream_t st) {
  const int n_pages = (int)((tok_count + page_size - 1) / page_size);
  const dim3 grid((n_pages + 15) / 16, dm.HP);
  if (dm.dtype == CK_BF16)
    hipLaunchKernelGGL(k_page_keys<bf16>, grid, dim3(PAGE_THREADS), 0, st, (const bf16*)K, dm.N_cap,
                       tok_begin, tok_count, page_size, (bf16*)page_keys, page_stride, n_pages);
  else
    hipLaunchKernelGGL(k_page_keys<float>, grid, dim3(PAGE_THREADS), 0, st, (const float*)K,
                       dm.N_cap, tok_begin, tok_count, page_size, (float*)page_keys, page_stride,
                       n_pages);
  return hipGetLastError();
}

// ------------------------------------------------------------------ pages -> tokens
// Selected pages (ascending, distinct) to their token ids; only the last page of
// the token range can be short, wherever it stands in the list.
__global__ __launch_bounds__(PAGE_THREADS) void k_expand_pages(
    const int32_t* __restrict__ page_idx, const int32_t* __restrict__ n_pages_sel, int page_stride,
    int page_size, int64_t tok_begin, int64_t tok_count, int32_t* __restrict__ token_idx,
    int idx_stride, int32_t* __restrict__ n_tokens) {
  __shared__ int short_at;
  const int hp = blockIdx.x, tid = threadIdx.x;
  int np = n_pages_sel[hp];
  np = np < 0 ? 0 : (np > page_stride ? page_stride : np);
  if ((int64_t)np * page_size > idx_stride) np = idx_stride / page_size;
  const int32_t* pages = page_idx + (int64_t)hp * page_stride;
  const int last_page = (int)((tok_count - 1) / page_size);
  const int last_len = (int)(tok_count - (int64_t)last_page * page_size);
  if (tid == 0) short_at = np;
  __syncthreads();
  if (last_len < page_size)
    for (int j = tid; j < np; j += PAGE_THREADS)
      if (pages[j] == last_page) short_at = j;             // at most one match
  __syncthreads();
  const int js = short_at, deficit = page_size - last_len;
  int32_t* out = token_idx + (int64_t)hp * idx_stride;
  for (int e = tid; e < np * page_size; e += PAGE_THREADS) {
    const int j = e / page_size, t = e % page_size;
    const int64_t tok = (int64_t)pages[j] * page_size + t;
    if (tok < tok_count) out[e - (j > js ? deficit : 0)] = (int32_t)(tok_begin + tok);
  }
  if (tid == 0) n_tokens[hp] = np * page_size - (js < np ? deficit : 0);
}

hipError_t launch_expand_pages(int HP, const int32_t* page_idx, const int32_t* n_pages_sel,
                               int page_stride, int page_size, int64_t tok_begin,
                               int64_t tok_count, int32_t* token_idx, int idx_stride,
                               int32_t* n_tokens, hipStream_t st) {
  hipLaunchKernelGGL(k_expand_pages, dim3(HP), dim3(PAGE_THREADS), 0, st, page_idx, n_pages_sel,
                     page_stride, page_size, tok_begin, tok_count, token_idx, idx_stride,
                     n_tokens);
  return hipGetLastError();
}

// ------------------------------------------------------------------ clustering objective
// Of a given assignment under the cosine distance of Section III-B, D = 1 - cos(k, mu):
//   J = sum_i |k_i| (1 - cos(k_i, t_i)) = sum_i (|k_i| - <k_i, t_i>)   for a unit-length table
//   D = sum_i (1 - <k_i, t_i> / (|k_i| |t_i|))                         (a zero vector counts 1)
// with t_i the table row of key i's label.  Products and the 128-term sums of one row in
// fp32 (bf16 products are exact there), the sum over the keys in fp64.  Two launches and
// a fixed order of additions: no floating-point atomics, bit-reproducible.
constexpr int OBJ_THREADS = 256;
constexpr int OBJ_TOKENS = 1024;                        // keys per workgroup

__global__ __launch_bounds__(OBJ_THREADS) void k_objective_partial(
    const bf16* __restrict__ K, const bf16* __restrict__ table, const int32_t* __restrict__ labels,
    int64_t N_cap, int64_t tok_begin, int64_t tok_count, int c_begin, int c_count,
    double* __restrict__ partial) {
  __shared__ double red[2][OBJ_THREADS / 16];
  const int hp = blockIdx.y, tid = threadIdx.x, l16 = tid & 15, grp = tid >> 4;
  const bf16* Khp = K + (int64_t)hp * N_cap * D + l16 * 8;
  const bf16* Thp = table + (int64_t)hp * c_count * D + l16 * 8;
  const int32_t* lab = labels + (int64_t)hp * N_cap + tok_begin;
  double j = 0.0, dsum = 0.0;
  for (int i = 0; i < OBJ_TOKENS / 16; i += 4) {
    float kv[4][8], tv[4][8];
    bool ok[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t t = (int64_t)blockIdx.x * OBJ_TOKENS + (i + u) * 16 + grp;
      ok[u] = t < tok_count;
      const int64_t tc = ok[u] ? t : tok_count - 1;
      int c = lab[tc] - c_begin;
      c = c < 0 ? 0 : (c >= c_count ? c_count - 1 : c);
      load_row8<bf16>(Khp + (tok_begin + tc) * D, kv[u]);
      load_row8<bf16>(Thp + (int64_t)c * D, tv[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      float dot = 0.f, kk = 0.f, tt = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        dot = fmaf(kv[u][e], tv[u][e], dot);
        kk = fmaf(kv[u][e], kv[u][e], kk);
        tt = fmaf(tv[u][e], tv[u][e], tt);
      }
      dot = row16_sum(dot);
      kk = row16_sum(kk);
      tt = row16_sum(tt);
      if (ok[u]) {
        const double kn = sqrt((double)kk), den = kn * sqrt((double)tt);
        j += kn - (double)dot;
        dsum += den > 0.0 ? 1.0 - (double)dot / den : 1.0;
      }
    }
  }
  if (l16 == 0) {
    red[0][grp] = j;
    red[1][grp] = dsum;
  }
  __syncthreads();
  if (tid < 2) {
    double s = 0.0;
    for (int g = 0; g < OBJ_THREADS / 16; ++g) s += red[tid][g];
    partial[((int64_t)hp * gridDim.x + blockIdx.x) * 2 + tid] = s;
  }
}

__global__ __launch_bounds__(64) void k_objective_sum(const double* __restrict__ partial, int n_wg,
                                                      double* __restrict__ J, double* __restrict__ Dsum) {
  const int hp = blockIdx.x, which = threadIdx.x;
  if (which >= 2) return;
  double s = 0.0;
  for (int w = 0; w < n_wg; ++w) s += partial[((int64_t)hp * n_wg + w) * 2 + which];
  (which == 0 ? J : Dsum)[hp] = s;
}

size_t objective_workspace_bytes(const Dims& dm, int64_t tok_count) {
  const int64_t n_wg = (tok_count + OBJ_TOKENS - 1) / OBJ_TOKENS;
  return (((size_t)dm.HP * n_wg * 2 * sizeof(double)) + 255) & ~(size_t)255;
}

hipError_t launch_objective(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                            const bf16* table, int c_begin, int c_count, const int32_t* labels,
                            double* J, double* Dsum, void* workspace, hipStream_t st) {
  const int n_wg = (int)((tok_count + OBJ_TOKENS - 1) / OBJ_TOKENS);
  hipLaunchKernelGGL(k_objective_partial, dim3(n_wg, dm.HP), dim3(OBJ_THREADS), 0, st, K, table,
                     labels, dm.N_cap, tok_begin, tok_count, c_begin, c_count, (double*)workspace);
  hipLaunchKernelGGL(k_objective_sum, dim3(dm.HP), dim3(64), 0, st, (const double*)workspace, n_wg,
                     J, Dsum);
  return hipGetLastError();
}

}  // namespace ck
