// Cluster-granularity cache of recalled K/V (paper Section IV-D) for a KV cache whose
// home is host memory (Section IV-A: keys and values are offloaded after prefill and
// only the selected ones come back).  The cache keeps the rows of the clusters
// recalled at the previous step (R = 1) in recalled order, together with their
// cluster ids; a step copies the clusters it finds there device-to-device and
// fetches only the missing clusters from the home copy.
//
// MI355X form: the home copy is pinned host memory mapped into the device address
// space, and the fetch is issued by the GPU itself (16 lanes read one 256-byte row
// over the host link), so that no miss list ever travels to the host and nothing
// synchronises: selection, cache look-up, fetch and attention stay enqueued on one
// stream.  Attention then runs over the dense cache rows of the step.
#include "decode_common.hpp"

namespace ck {

constexpr int CACHE_THREADS = 256;
constexpr int CACHE_ROWS_PER_WG = 128;                  // recalled rows one workgroup moves
constexpr int CACHE_ITEMS = CK_MAX_CLUSTERS / CACHE_THREADS;

__global__ __launch_bounds__(CACHE_THREADS) void k_cache_fill(const CacheArgs a) {
  __shared__ int old_pos[CK_MAX_CLUSTERS];              // cluster id -> first row in the old buffer, -1
  __shared__ int start[CK_MAX_CLUSTERS + 1];            // first row of the j-th selected cluster
  __shared__ int src_row[CK_MAX_CLUSTERS];              // where its rows come from: old row or ~segment begin
  __shared__ int tmp[CACHE_THREADS / WAVE + 1];
  __shared__ int s_miss;
  const int hp = blockIdx.y, tid = threadIdx.x;
  int n_sel = a.n_sel_clusters[hp];
  n_sel = n_sel < 0 ? 0 : (n_sel > a.C_cap ? a.C_cap : n_sel);
  if (n_sel > CK_MAX_CLUSTERS) n_sel = CK_MAX_CLUSTERS;
  int n_old = a.old_n[hp];
  n_old = n_old < 0 ? 0 : (n_old > a.C_cap ? a.C_cap : n_old);
  if (n_old > CK_MAX_CLUSTERS) n_old = CK_MAX_CLUSTERS;
  const int32_t* sel = a.sel_clusters + (int64_t)hp * a.C_cap;
  const int32_t* sz = a.sizes + (int64_t)hp * a.C_cap;
  const int32_t* off = a.offsets + (int64_t)hp * (a.C_cap + 1);

  for (int c = tid; c < a.C_cap && c < CK_MAX_CLUSTERS; c += CACHE_THREADS) old_pos[c] = -1;
  if (tid == 0) s_miss = 0;
  __syncthreads();
  for (int j = tid; j < n_old; j += CACHE_THREADS) {
    const int c = a.old_clusters[(int64_t)hp * a.C_cap + j];
    if (c >= 0 && c < a.C_cap && c < CK_MAX_CLUSTERS)
      old_pos[c] = a.old_starts[(int64_t)hp * (a.C_cap + 1) + j];
  }
  // rows of the selected clusters, in selection order
  int v[CACHE_ITEMS], own[CACHE_ITEMS], cid[CACHE_ITEMS];
#pragma unroll
  for (int i = 0; i < CACHE_ITEMS; ++i) {
    const int j = tid * CACHE_ITEMS + i;
    cid[i] = 0;
    own[i] = 0;
    if (j < n_sel) {
      int c = sel[j];
      c = c < 0 ? 0 : (c >= a.C_cap ? a.C_cap - 1 : c);
      cid[i] = c;
      own[i] = sz[c] < 0 ? 0 : sz[c];
    }
    v[i] = own[i];
  }
  int total = block_inclusive_scan<CACHE_ITEMS>(v, tmp);   // barriers inside: old_pos is complete
  if (total > a.cap) total = a.cap;                         // cannot happen for whole clusters <= budget <= cap
  int miss = 0;
#pragma unroll
  for (int i = 0; i < CACHE_ITEMS; ++i) {
    const int j = tid * CACHE_ITEMS + i;
    if (j < n_sel) {
      start[j] = v[i] - own[i];
      const int op = old_pos[cid[i]];
      src_row[j] = op >= 0 ? op : ~off[cid[i]];
      if (op < 0) miss += own[i];
    }
  }
  if (tid == 0) start[n_sel] = total;
  miss = __builtin_amdgcn_readlane(wave_inclusive_scan(miss), WAVE - 1);
  if ((tid & 63) == 0 && miss) atomicAdd(&s_miss, miss);
  __syncthreads();
  if (blockIdx.x == 0) {                                // the new generation's directory
    for (int j = tid; j < n_sel; j += CACHE_THREADS) {
      a.new_clusters[(int64_t)hp * a.C_cap + j] = sel[j];
      a.new_starts[(int64_t)hp * (a.C_cap + 1) + j] = start[j];
    }
    if (tid == 0) {
      a.new_starts[(int64_t)hp * (a.C_cap + 1) + n_sel] = total;
      a.new_n[hp] = n_sel;
      a.miss_tokens[hp] = s_miss;
    }
  }
  // ---- move this workgroup's rows: 16 lanes per row, 16 bytes (or 2 x 16) per lane ----
  const int l16 = tid & 15, grp = tid >> 4;
  const int p0 = blockIdx.x * CACHE_ROWS_PER_WG;
  const int64_t hp_home = (int64_t)hp * a.N_cap, hp_cache = (int64_t)hp * a.cap;
  const int32_t* sidx = a.sorted_idx + hp_home;
  const int vec = a.row_bytes / 256;                    // 16-byte pieces per lane: 1 (bf16) or 2 (fp32)
  for (int r = grp; r < CACHE_ROWS_PER_WG; r += 16) {
    const int p = p0 + r;
    if (p >= total) break;
    int lo = 0, hi = n_sel - 1;                         // last j with start[j] <= p
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (start[mid] <= p) lo = mid; else hi = mid - 1;
    }
    const int o = p - start[lo];
    const int sr = src_row[lo];
    const char *ks, *vs;
    if (sr >= 0) {
      int64_t row = (int64_t)sr + o;
      row = row >= a.cap ? a.cap - 1 : row;
      ks = static_cast<const char*>(a.K_old) + (hp_cache + row) * a.row_bytes;
      vs = static_cast<const char*>(a.V_old) + (hp_cache + row) * a.row_bytes;
    } else {
      int64_t src = (int64_t)(~sr) + o;
      src = src < 0 ? 0 : (src >= a.N_cap ? a.N_cap - 1 : src);
      int64_t row = sidx[src];
      row = row < 0 ? 0 : (row >= a.N_cap ? a.N_cap - 1 : row);
      ks = static_cast<const char*>(a.K_home) + (hp_home + row) * a.row_bytes;
      vs = static_cast<const char*>(a.V_home) + (hp_home + row) * a.row_bytes;
    }
    char* kd = static_cast<char*>(a.K_new) + (hp_cache + p) * a.row_bytes;
    char* vd = static_cast<char*>(a.V_new) + (hp_cache + p) * a.row_bytes;
    for (int e = 0; e < vec; ++e) {
      const int b = (e * 16 + l16) * 16;
      const uint4 kw = *reinterpret_cast<const uint4*>(ks + b);
      const uint4 vw = *reinterpret_cast<const uint4*>(vs + b);
      *reinterpret_cast<uint4*>(kd + b) = kw;
      *reinterpret_cast<uint4*>(vd + b) = vw;
    }
  }
}

hipError_t launch_cache_fill(const Dims& dm, const CacheArgs& a, int budget, hipStream_t st) {
  const dim3 grid((budget + CACHE_ROWS_PER_WG - 1) / CACHE_ROWS_PER_WG, dm.HP);
  hipLaunchKernelGGL(k_cache_fill, grid, dim3(CACHE_THREADS), 0, st, a);
  return hipGetLastError();
}

}  // namespace ck
