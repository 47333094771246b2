// K-means initialisation, clustering metadata and centroid update
// (paper Section III-B for init/update, Section IV-C / Fig. 8 for the metadata).
//
// The paper's update kernel accumulates keys into shared-memory sums with
// atomics, one thread block per head.  Here the update is a segmented
// reduction instead: the labels are first counting-sorted into the
// cluster-contiguous token index that the decode step needs anyway (sizes,
// prefix sum, sorted indices), then one workgroup per cluster streams its member
// rows and adds them in a fixed order.  No floating-point atomics, so the
// centroids are bit-reproducible; the sort is stable (ascending token row inside
// a cluster), so the metadata of the last iteration is the final metadata.
#include "ck_common.hpp"

namespace ck {

// ------------------------------------------------------------------ init
// centroid c of head-problem hp := key row init_idx[hp][c]; also the row of the table the
// assignment reads: its unit-length copy (cosine) or the row itself (l2, inner product),
// and for l2 the bias -|row|^2 / 2.
__global__ __launch_bounds__(64) void k_init_centroids(
    const bf16* __restrict__ K, const int32_t* __restrict__ init_idx, int64_t N_cap, int C_cap,
    int c_begin, int c_count, bf16* __restrict__ centroids, bf16* __restrict__ mu_hat, int metric,
    float* __restrict__ bias, int bias_stride) {
  const int c = blockIdx.x, hp = blockIdx.y, lane = threadIdx.x;
  int64_t row = init_idx[(int64_t)hp * c_count + c];
  row = row < 0 ? 0 : (row >= N_cap ? N_cap - 1 : row);
  const uint32_t w = reinterpret_cast<const uint32_t*>(K + ((int64_t)hp * N_cap + row) * D)[lane];
  const float a = lo_bf16(w), b = hi_bf16(w);
  const float n2 = wave_sum(a * a + b * b);
  const float inv = n2 > 0.f ? 1.0f / sqrtf(n2) : 0.f;
  reinterpret_cast<uint32_t*>(centroids + ((int64_t)hp * C_cap + c_begin + c) * D)[lane] = w;
  const uint32_t h = (uint32_t)float_to_bf16_bits(a * inv) |
                     ((uint32_t)float_to_bf16_bits(b * inv) << 16);
  reinterpret_cast<uint32_t*>(mu_hat + ((int64_t)hp * c_count + c) * D)[lane] =
      metric == CK_METRIC_COSINE ? h : w;
  if (metric == CK_METRIC_L2 && lane == 0) bias[(int64_t)hp * bias_stride + c] = -0.5f * n2;
}

__global__ void k_fill_i32(int32_t* __restrict__ p, int64_t n, int32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st) {
  hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

// iterations a head-problem ran: up to and including the first assignment that changed
// no label, or all of them
__global__ void k_iters_done(const int32_t* __restrict__ changed, int max_iter, int HP,
                             int32_t* __restrict__ iters_done) {
  const int hp = blockIdx.x * blockDim.x + threadIdx.x;
  if (hp >= HP) return;
  int n = max_iter;
  for (int t = 1; t < max_iter; ++t)
    if (changed[(int64_t)t * HP + hp] == 0) {
      n = t + 1;
      break;
    }
  iters_done[hp] = n;
}

hipError_t launch_iters_done(const int32_t* changed, int max_iter, int HP, int32_t* iters_done,
                             hipStream_t st) {
  hipLaunchKernelGGL(k_iters_done, dim3((HP + 63) / 64), dim3(64), 0, st, changed, max_iter, HP,
                     iters_done);
  return hipGetLastError();
}

hipError_t launch_init_centroids(const Dims& dm, const bf16* K, const int32_t* init_idx,
                                 int c_begin, int c_count, bf16* centroids, bf16* mu_hat,
                                 int metric, float* bias, int bias_stride, hipStream_t st) {
  hipLaunchKernelGGL(k_init_centroids, dim3(c_count, dm.HP), dim3(64), 0, st, K, init_idx,
                     dm.N_cap, dm.C_cap, c_begin, c_count, centroids, mu_hat, metric, bias,
                     bias_stride);
  return hipGetLastError();
}

// ------------------------------------------------------------------ counting sort
// Lanes of a wavefront that hold the same label, as a 64-bit mask (built from one
// ballot per label bit), restricted to `valid` lanes.
__device__ __forceinline__ uint64_t same_label_mask(int label, bool valid, int label_bits) {
  uint64_t peers = __ballot(valid);
  for (int b = 0; b < label_bits; ++b) {
    const bool bit = (label >> b) & 1;
    const uint64_t m = __ballot(bit);
    peers &= bit ? m : ~m;
  }
  return peers;
}

constexpr int SORT_THREADS = 256;                       // 4 wavefronts, one chunk each

// Pass 1 (only when the assignment kernel has not already produced it): label
// histogram of every chunk of `chunk_tokens` consecutive tokens.
__global__ __launch_bounds__(SORT_THREADS) void k_sort_hist(
    const int32_t* __restrict__ labels, int64_t N_cap, int64_t tok_begin, int64_t tok_count,
    int c_begin, int c_count, int label_bits, int n_chunks, int chunk_tokens,
    int32_t* __restrict__ chunk_hist) {
  extern __shared__ int lds_hist[];                     // [4][c_count]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hp = blockIdx.y;
  const int chunk = blockIdx.x * 4 + wave;
  if (chunk >= n_chunks) return;                        // whole wavefront leaves; no barriers below
  volatile int* hist = lds_hist + wave * c_count;
  for (int c = lane; c < c_count; c += WAVE) hist[c] = 0;
  __builtin_amdgcn_wave_barrier();
  const int32_t* lab = labels + (int64_t)hp * N_cap + tok_begin;
  const uint64_t lt = ((uint64_t)1 << lane) - 1;
  for (int r = 0; r < chunk_tokens / WAVE; ++r) {
    const int64_t t = (int64_t)chunk * chunk_tokens + r * WAVE + lane;
    const bool valid = t < tok_count;
    int l = valid ? lab[t] - c_begin : 0;
    l = l < 0 ? 0 : (l >= c_count ? c_count - 1 : l);   // never index outside the table
    const uint64_t peers = same_label_mask(l, valid, label_bits);
    if (valid && (peers & lt) == 0) hist[l] = hist[l] + __popcll(peers);
    __builtin_amdgcn_wave_barrier();
  }
  int32_t* out = chunk_hist + ((int64_t)hp * n_chunks + chunk) * c_count;
  for (int c = lane; c < c_count; c += WAVE) out[c] = hist[c];
}

// Pass 2: per cluster, exclusive scan of the chunk counts (in place) and the
// cluster size.  Workgroup = 64 clusters x 16 groups of chunks.
constexpr int SCAN_THREADS = 1024;
constexpr int SCAN_GROUPS = SCAN_THREADS / 64;
constexpr int SCAN_REG = 16;                            // chunk counts a thread keeps in registers
__global__ __launch_bounds__(SCAN_THREADS) void k_sort_scan(
    int32_t* __restrict__ chunk_hist, int n_chunks, int C_cap, int c_begin, int c_count,
    int32_t* __restrict__ sizes, const int32_t* __restrict__ gate) {
  __shared__ int part[SCAN_GROUPS][64];
  const int cl = threadIdx.x & 63, grp = threadIdx.x >> 6, hp = blockIdx.y;
  if (gate && gate[hp] == 0) return;
  const int c = blockIdx.x * 64 + cl;
  const int per = (n_chunks + SCAN_GROUPS - 1) / SCAN_GROUPS;
  const int k0 = grp * per, k1 = min(k0 + per, n_chunks);
  int32_t* H = chunk_hist + (int64_t)hp * n_chunks * c_count + c;
  int v[SCAN_REG];
  int sum = 0;
  if (c < c_count) {
#pragma unroll
    for (int i = 0; i < SCAN_REG; ++i) v[i] = (k0 + i < k1) ? H[(int64_t)(k0 + i) * c_count] : 0;
#pragma unroll
    for (int i = 0; i < SCAN_REG; ++i) sum += v[i];
    for (int k = k0 + SCAN_REG; k < k1; ++k) sum += H[(int64_t)k * c_count];
  }
  part[grp][cl] = sum;
  __syncthreads();
  int run = 0, total = 0;
#pragma unroll
  for (int g = 0; g < SCAN_GROUPS; ++g) {
    const int t = part[g][cl];
    if (g < grp) run += t;
    total += t;
  }
  if (c < c_count) {
#pragma unroll
    for (int i = 0; i < SCAN_REG; ++i)
      if (k0 + i < k1) {
        H[(int64_t)(k0 + i) * c_count] = run;
        run += v[i];
      }
    for (int k = k0 + SCAN_REG; k < k1; ++k) {
      const int t = H[(int64_t)k * c_count];
      H[(int64_t)k * c_count] = run;
      run += t;
    }
    if (grp == 0) sizes[(int64_t)hp * C_cap + c_begin + c] = total;
  }
}

// Pass 3: exclusive scan of the sizes -> offsets (every workgroup recomputes it in
// LDS, the first one of a head-problem stores it), then the stable scatter of the
// token rows of ONE chunk to their sorted positions.  The four wavefronts each rank a
// quarter of the chunk; per-wavefront label counts in LDS order the quarters.
constexpr int OFF_ITEMS = CK_MAX_CLUSTERS / SORT_THREADS;   // 8 clusters per thread
constexpr int SCAT_ROUNDS = 2;                              // chunk_tokens <= 4 * 2 * 64
__global__ __launch_bounds__(SORT_THREADS) void k_sort_scatter(
    const int32_t* __restrict__ labels, int64_t N_cap, int64_t tok_begin, int64_t tok_count,
    int C_cap, int c_begin, int c_count, int label_bits, int n_chunks, int chunk_tokens,
    const int32_t* __restrict__ chunk_hist, const int32_t* __restrict__ sizes,
    int32_t* __restrict__ offsets, int32_t* __restrict__ sorted_idx,
    const int32_t* __restrict__ gate) {
  extern __shared__ int lds_hist[];                     // [c_count] positions + [4][c_count] counts
  __shared__ int tmp[SORT_THREADS / WAVE + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hp = blockIdx.y;
  if (gate && gate[hp] == 0) return;
  const int chunk = blockIdx.x;
  // this thread's labels are requested first, unconditionally (a token beyond the range
  // re-reads token 0), so that they travel while the offsets are being prepared
  const int per_wave = chunk_tokens / 4;
  const int32_t* lab = labels + (int64_t)hp * N_cap + tok_begin;
  int lraw[SCAT_ROUNDS];
#pragma unroll
  for (int r = 0; r < SCAT_ROUNDS; ++r) {
    const int in_wave = r * WAVE + lane;
    const int64_t t = (int64_t)chunk * chunk_tokens + wave * per_wave + in_wave;
    lraw[r] = lab[(in_wave < per_wave && t < tok_count) ? t : 0];
  }
  int* offs = lds_hist;
  int* cnt = lds_hist + c_count;
  int32_t* off_g = offsets + (int64_t)hp * (C_cap + 1);
  const int base0 = c_begin == 0 ? 0 : off_g[c_begin];
  const int32_t* cbase = chunk_hist + ((int64_t)hp * n_chunks + chunk) * c_count;
  {
    const int32_t* sz = sizes + (int64_t)hp * C_cap + c_begin;
    int v[OFF_ITEMS], own[OFF_ITEMS], cb[OFF_ITEMS];
#pragma unroll
    for (int i = 0; i < OFF_ITEMS; ++i) {
      const int c = tid * OFF_ITEMS + i;
      own[i] = v[i] = c < c_count ? sz[c] : 0;
      cb[i] = c < c_count ? cbase[c] : 0;
    }
    block_inclusive_scan<OFF_ITEMS>(v, tmp);
#pragma unroll
    for (int i = 0; i < OFF_ITEMS; ++i) {
      const int c = tid * OFF_ITEMS + i;
      if (c < c_count) {
        offs[c] = base0 + v[i] - own[i] + cb[i];        // first position of this chunk's tokens
        if (chunk == 0) off_g[c_begin + c + 1] = base0 + v[i];
      }
    }
    if (chunk == 0 && tid == 0 && c_begin == 0) off_g[0] = 0;
  }
  for (int i = tid; i < 4 * c_count; i += SORT_THREADS) cnt[i] = 0;
  __syncthreads();

  const uint64_t lt = ((uint64_t)1 << lane) - 1;
  volatile int* mine = cnt + wave * c_count;
  int lbl[SCAT_ROUNDS], rank[SCAT_ROUNDS];
  int64_t tok[SCAT_ROUNDS];
#pragma unroll
  for (int r = 0; r < SCAT_ROUNDS; ++r) {
    const int in_wave = r * WAVE + lane;
    const int64_t t = (int64_t)chunk * chunk_tokens + wave * per_wave + in_wave;
    const bool valid = in_wave < per_wave && t < tok_count;
    int l = valid ? lraw[r] - c_begin : 0;
    l = l < 0 ? 0 : (l >= c_count ? c_count - 1 : l);
    const uint64_t peers = same_label_mask(l, valid, label_bits);
    const int before = mine[l];
    __builtin_amdgcn_wave_barrier();
    if (valid && (peers & lt) == 0) mine[l] = before + __popcll(peers);
    __builtin_amdgcn_wave_barrier();
    lbl[r] = l;
    rank[r] = before + __popcll(peers & lt);
    tok[r] = valid ? t : -1;
  }
  __syncthreads();
  int32_t* out = sorted_idx + (int64_t)hp * N_cap;
#pragma unroll
  for (int r = 0; r < SCAT_ROUNDS; ++r) {
    if (tok[r] >= 0) {
      int pos = offs[lbl[r]] + rank[r];
      for (int w = 0; w < wave; ++w) pos += cnt[w * c_count + lbl[r]];
      if (pos >= 0 && pos < N_cap) out[pos] = (int32_t)(tok_begin + tok[r]);
    }
  }
}

hipError_t launch_metadata(const Dims& dm, const int32_t* labels, int64_t tok_begin,
                           int64_t tok_count, int c_begin, int c_count, int32_t* sizes,
                           int32_t* offsets, int32_t* sorted_idx, int32_t* chunk_hist,
                           bool have_hist, const int32_t* gate, hipStream_t st) {
  const int chunk_tokens = assign_tile_tokens(dm, tok_count);
  const int n_chunks = (int)((tok_count + chunk_tokens - 1) / chunk_tokens);
  int label_bits = 0;
  while ((1 << label_bits) < c_count) ++label_bits;
  const dim3 grid((n_chunks + 3) / 4, dm.HP);
  if (!have_hist)
    hipLaunchKernelGGL(k_sort_hist, grid, dim3(SORT_THREADS), (size_t)4 * c_count * sizeof(int),
                       st, labels, dm.N_cap, tok_begin, tok_count, c_begin, c_count, label_bits,
                       n_chunks, chunk_tokens, chunk_hist);
  hipLaunchKernelGGL(k_sort_scan, dim3((c_count + 63) / 64, dm.HP), dim3(SCAN_THREADS), 0, st,
                     chunk_hist, n_chunks, dm.C_cap, c_begin, c_count, sizes, gate);
  hipLaunchKernelGGL(k_sort_scatter, dim3(n_chunks, dm.HP), dim3(SORT_THREADS),
                     (size_t)5 * c_count * sizeof(int), st, labels, dm.N_cap, tok_begin, tok_count,
                     dm.C_cap, c_begin, c_count, label_bits, n_chunks, chunk_tokens, chunk_hist,
                     sizes, offsets, sorted_idx, gate);
  return hipGetLastError();
}

// ------------------------------------------------------------------ update
// One workgroup per cluster.  A 16-lane group reads one member row per step
// (16 B per lane), 4 rows per wavefront step, UPD_UNR steps in flight.  Partial
// sums are combined in a fixed order: lane groups of a wavefront, then the
// wavefronts through LDS.
template <int UPD_WAVES, int UPD_UNR>
__global__ __launch_bounds__(UPD_WAVES * 64) void k_update(
    const bf16* __restrict__ K, int64_t N_cap, int C_cap, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ sorted_idx, int c_begin, int c_count,
    bf16* __restrict__ centroids, bf16* __restrict__ mu_hat, float* __restrict__ centroids_f32,
    int metric, float* __restrict__ bias, int bias_stride, const int32_t* __restrict__ gate) {
  constexpr int GROUPS = UPD_WAVES * 4;                 // 16-lane groups: member rows per step
  __shared__ float part[UPD_WAVES][D];
  const int c = blockIdx.x, hp = blockIdx.y, tid = threadIdx.x;
  if (gate && gate[hp] == 0) return;
  const int lane = tid & 63, wave = tid >> 6, l16 = tid & 15, grp = tid >> 4;
  const int32_t* off = offsets + (int64_t)hp * (C_cap + 1) + c_begin + c;
  const int beg = off[0], n = off[1] - beg;
  if (n <= 0) return;                                   // empty cluster keeps its centroid
  const int32_t* idx = sorted_idx + (int64_t)hp * N_cap + beg;
  const bf16* Khp = K + (int64_t)hp * N_cap * D + l16 * 8;

  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  for (int j0 = 0; j0 < n; j0 += GROUPS * UPD_UNR) {
    // two round trips per pass: all member ids, then all member rows.  Every load is
    // unconditional (an entry beyond the cluster re-reads its last member and is
    // replaced by zeros): a load under a branch makes the compiler wait for it, and for
    // everything requested before it, ahead of the next one.
    int64_t row[UPD_UNR];
#pragma unroll
    for (int u = 0; u < UPD_UNR; ++u) {
      const int j = j0 + u * GROUPS + grp;
      row[u] = idx[j < n ? j : n - 1];
    }
    uint4 w[UPD_UNR];
#pragma unroll
    for (int u = 0; u < UPD_UNR; ++u) {
      const int64_t r = row[u] < 0 ? 0 : (row[u] >= N_cap ? N_cap - 1 : row[u]);
      w[u] = *reinterpret_cast<const uint4*>(Khp + r * D);
    }
#pragma unroll
    for (int u = 0; u < UPD_UNR; ++u) {
      const bool real = j0 + u * GROUPS + grp < n;
      const uint32_t x = real ? w[u].x : 0u, y = real ? w[u].y : 0u;
      const uint32_t z = real ? w[u].z : 0u, q = real ? w[u].w : 0u;
      acc[0] += lo_bf16(x); acc[1] += hi_bf16(x);
      acc[2] += lo_bf16(y); acc[3] += hi_bf16(y);
      acc[4] += lo_bf16(z); acc[5] += hi_bf16(z);
      acc[6] += lo_bf16(q); acc[7] += hi_bf16(q);
    }
  }
  // groups of one wavefront
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    acc[j] += __shfl_xor(acc[j], 16, WAVE);
    acc[j] += __shfl_xor(acc[j], 32, WAVE);
  }
  if (lane < 16) {
#pragma unroll
    for (int j = 0; j < 8; ++j) part[wave][l16 * 8 + j] = acc[j];
  }
  __syncthreads();
  if (tid < 64) {
    // lane handles channels 2*lane, 2*lane+1
    const float inv_n = 1.0f / (float)n;
    float m0 = part[0][2 * lane], m1 = part[0][2 * lane + 1];
#pragma unroll
    for (int wv = 1; wv < UPD_WAVES; ++wv) {
      m0 += part[wv][2 * lane];
      m1 += part[wv][2 * lane + 1];
    }
    m0 *= inv_n;
    m1 *= inv_n;
    const float n2 = wave_sum(m0 * m0 + m1 * m1);
    const float inv = n2 > 0.f ? 1.0f / sqrtf(n2) : 0.f;
    const int64_t crow = (int64_t)hp * C_cap + c_begin + c;
    const int64_t hrow = (int64_t)hp * c_count + c;
    const uint32_t raw =
        (uint32_t)float_to_bf16_bits(m0) | ((uint32_t)float_to_bf16_bits(m1) << 16);
    reinterpret_cast<uint32_t*>(centroids + crow * D)[lane] = raw;
    // table row of the next assignment: unit length (cosine) or the stored mean itself
    reinterpret_cast<uint32_t*>(mu_hat + hrow * D)[lane] =
        metric == CK_METRIC_COSINE
            ? ((uint32_t)float_to_bf16_bits(m0 * inv) | ((uint32_t)float_to_bf16_bits(m1 * inv) << 16))
            : raw;
    if (metric == CK_METRIC_L2) {                       // wave-uniform
      const float r0 = lo_bf16(raw), r1 = hi_bf16(raw); // the rounded row is what gets compared
      const float rn2 = wave_sum(r0 * r0 + r1 * r1);
      if (lane == 0) bias[(int64_t)hp * bias_stride + c] = -0.5f * rn2;
    }
    if (centroids_f32)
      reinterpret_cast<float2*>(centroids_f32 + hrow * D)[lane] = make_float2(m0, m1);
  }
}

hipError_t launch_update(const Dims& dm, const bf16* K, const int32_t* offsets,
                         const int32_t* sorted_idx, int c_begin, int c_count, bf16* centroids,
                         bf16* mu_hat, float* centroids_f32, int metric, float* bias,
                         int bias_stride, const int32_t* gate, hipStream_t st) {
  // four wavefronts, eight rows in flight per 16-lane group: measured best of
  // {1, 2, 4 wavefronts} x {4, 8, 16 in flight} (the summation order does not depend on it)
  hipLaunchKernelGGL((k_update<4, 8>), dim3(c_count, dm.HP), dim3(4 * 64), 0, st, K, dm.N_cap,
                     dm.C_cap, offsets, sorted_idx, c_begin, c_count, centroids, mu_hat,
                     centroids_f32, metric, bias, bias_stride, gate);
  return hipGetLastError();
}

ClusterWorkspace carve_cluster_workspace(const Dims& dm, int64_t tok_count, int c_count,
                                         void* base) {
  ClusterWorkspace w;
  const int chunk_tokens = assign_tile_tokens(dm, tok_count);
  const int64_t n_chunks = (tok_count + chunk_tokens - 1) / chunk_tokens;
  size_t mu = (size_t)dm.HP * c_count * D * sizeof(bf16);
  mu = (mu + 255) & ~(size_t)255;
  size_t hist = (size_t)dm.HP * n_chunks * c_count * sizeof(int32_t);
  hist = (hist + 255) & ~(size_t)255;
  w.bias_stride = (c_count + 31) / 32 * 32;
  size_t bias = (size_t)dm.HP * w.bias_stride * sizeof(float);
  bias = (bias + 255) & ~(size_t)255;
  size_t chg = (size_t)(KM_MAX_ITER_CONVERGE + 1) * dm.HP * sizeof(int32_t);
  chg = (chg + 255) & ~(size_t)255;
  char* b = reinterpret_cast<char*>(base);
  w.mu_hat = reinterpret_cast<bf16*>(b);
  w.chunk_hist = reinterpret_cast<int32_t*>(b + mu);
  w.bias = reinterpret_cast<float*>(b + mu + hist);
  w.changed = reinterpret_cast<int32_t*>(b + mu + hist + bias);
  w.bytes = mu + hist + bias + chg;
  return w;
}

}  // namespace ck
