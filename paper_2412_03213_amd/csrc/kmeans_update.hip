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
// centroid c of head-problem hp := key row init_idx[hp][c]; also its unit-length copy.
__global__ __launch_bounds__(64) void k_init_centroids(
    const bf16* __restrict__ K, const int32_t* __restrict__ init_idx, int64_t N_cap, int C_cap,
    int c_begin, int c_count, bf16* __restrict__ centroids, bf16* __restrict__ mu_hat) {
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
  reinterpret_cast<uint32_t*>(mu_hat + ((int64_t)hp * c_count + c) * D)[lane] = h;
}

hipError_t launch_init_centroids(const Dims& dm, const bf16* K, const int32_t* init_idx,
                                 int c_begin, int c_count, bf16* centroids, bf16* mu_hat,
                                 hipStream_t st) {
  hipLaunchKernelGGL(k_init_centroids, dim3(c_count, dm.HP), dim3(64), 0, st, K, init_idx,
                     dm.N_cap, dm.C_cap, c_begin, c_count, centroids, mu_hat);
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
constexpr int SORT_ROUNDS = SORT_CHUNK / WAVE;

// Pass 1: histogram of the labels of every chunk of SORT_CHUNK tokens.
__global__ __launch_bounds__(SORT_THREADS) void k_sort_hist(
    const int32_t* __restrict__ labels, int64_t N_cap, int64_t tok_begin, int64_t tok_count,
    int c_begin, int c_count, int label_bits, int n_chunks, int32_t* __restrict__ chunk_hist) {
  extern __shared__ int lds_hist[];                     // [4][c_count]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hp = blockIdx.y;
  const int chunk = blockIdx.x * 4 + wave;
  if (chunk >= n_chunks) return;                        // whole wavefront leaves; no barriers below
  volatile int* hist = lds_hist + wave * c_count;
  for (int c = lane; c < c_count; c += WAVE) hist[c] = 0;
  __builtin_amdgcn_wave_barrier();
  const int32_t* lab = labels + (int64_t)hp * N_cap + tok_begin;
  const uint64_t lt = ((uint64_t)1 << lane) - 1;
  for (int r = 0; r < SORT_ROUNDS; ++r) {
    const int64_t t = (int64_t)chunk * SORT_CHUNK + r * WAVE + lane;
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

// Pass 2: per cluster, exclusive scan of the chunk counts (in place) -> sizes;
// then the exclusive scan over clusters -> offsets.
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = CK_MAX_CLUSTERS / SCAN_THREADS;  // 8 clusters per thread
__global__ __launch_bounds__(SCAN_THREADS) void k_sort_scan(
    int32_t* __restrict__ chunk_hist, int n_chunks, int C_cap, int c_begin, int c_count,
    int32_t* __restrict__ sizes, int32_t* __restrict__ offsets) {
  __shared__ int tmp[SCAN_THREADS / WAVE + 1];
  const int hp = blockIdx.x, tid = threadIdx.x;
  int32_t* H = chunk_hist + (int64_t)hp * n_chunks * c_count;
  int v[SCAN_ITEMS];
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    const int c = tid * SCAN_ITEMS + i;
    int run = 0;
    if (c < c_count) {
      for (int k = 0; k < n_chunks; ++k) {
        const int t = H[(int64_t)k * c_count + c];
        H[(int64_t)k * c_count + c] = run;
        run += t;
      }
      sizes[(int64_t)hp * C_cap + c_begin + c] = run;
    }
    v[i] = run;
  }
  block_inclusive_scan<SCAN_ITEMS>(v, tmp);
  int32_t* off = offsets + (int64_t)hp * (C_cap + 1);
  const int base = c_begin == 0 ? 0 : off[c_begin];
  if (c_begin == 0 && tid == 0) off[0] = 0;
#pragma unroll
  for (int i = 0; i < SCAN_ITEMS; ++i) {
    const int c = tid * SCAN_ITEMS + i;
    if (c < c_count) off[c_begin + c + 1] = base + v[i];
  }
}

// Pass 3: stable scatter of the token rows to their sorted positions.
__global__ __launch_bounds__(SORT_THREADS) void k_sort_scatter(
    const int32_t* __restrict__ labels, int64_t N_cap, int64_t tok_begin, int64_t tok_count,
    int C_cap, int c_begin, int c_count, int label_bits, int n_chunks,
    const int32_t* __restrict__ chunk_hist, const int32_t* __restrict__ offsets,
    int32_t* __restrict__ sorted_idx) {
  extern __shared__ int lds_hist[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, hp = blockIdx.y;
  const int chunk = blockIdx.x * 4 + wave;
  if (chunk >= n_chunks) return;
  volatile int* next = lds_hist + wave * c_count;       // next free position per cluster
  const int32_t* base = chunk_hist + ((int64_t)hp * n_chunks + chunk) * c_count;
  const int32_t* off = offsets + (int64_t)hp * (C_cap + 1) + c_begin;
  for (int c = lane; c < c_count; c += WAVE) next[c] = off[c] + base[c];
  __builtin_amdgcn_wave_barrier();
  const int32_t* lab = labels + (int64_t)hp * N_cap + tok_begin;
  int32_t* out = sorted_idx + (int64_t)hp * N_cap;
  const uint64_t lt = ((uint64_t)1 << lane) - 1;
  for (int r = 0; r < SORT_ROUNDS; ++r) {
    const int64_t t = (int64_t)chunk * SORT_CHUNK + r * WAVE + lane;
    const bool valid = t < tok_count;
    int l = valid ? lab[t] - c_begin : 0;
    l = l < 0 ? 0 : (l >= c_count ? c_count - 1 : l);
    const uint64_t peers = same_label_mask(l, valid, label_bits);
    const int first = next[l];
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      const int64_t pos = first + __popcll(peers & lt);
      if (pos >= 0 && pos < N_cap) out[pos] = (int32_t)(tok_begin + t);
      if ((peers & lt) == 0) next[l] = first + __popcll(peers);
    }
    __builtin_amdgcn_wave_barrier();
  }
}

hipError_t launch_metadata(const Dims& dm, const int32_t* labels, int64_t tok_begin,
                           int64_t tok_count, int c_begin, int c_count, int32_t* sizes,
                           int32_t* offsets, int32_t* sorted_idx, int32_t* chunk_hist,
                           hipStream_t st) {
  const int n_chunks = (int)((tok_count + SORT_CHUNK - 1) / SORT_CHUNK);
  int label_bits = 0;
  while ((1 << label_bits) < c_count) ++label_bits;
  const dim3 grid((n_chunks + 3) / 4, dm.HP);
  const size_t lds = (size_t)4 * c_count * sizeof(int);
  hipLaunchKernelGGL(k_sort_hist, grid, dim3(SORT_THREADS), lds, st, labels, dm.N_cap, tok_begin,
                     tok_count, c_begin, c_count, label_bits, n_chunks, chunk_hist);
  hipLaunchKernelGGL(k_sort_scan, dim3(dm.HP), dim3(SCAN_THREADS), 0, st, chunk_hist, n_chunks,
                     dm.C_cap, c_begin, c_count, sizes, offsets);
  hipLaunchKernelGGL(k_sort_scatter, grid, dim3(SORT_THREADS), lds, st, labels, dm.N_cap,
                     tok_begin, tok_count, dm.C_cap, c_begin, c_count, label_bits, n_chunks,
                     chunk_hist, offsets, sorted_idx);
  return hipGetLastError();
}

// ------------------------------------------------------------------ update
// One workgroup per cluster.  A 16-lane group reads one member row per step
// (16 B per lane), 16 rows per workgroup step, four steps in flight.  Partial
// sums are combined in a fixed order: lane groups of a wavefront, then the four
// wavefronts through LDS.
constexpr int UPD_THREADS = 256;
__global__ __launch_bounds__(UPD_THREADS) void k_update(
    const bf16* __restrict__ K, int64_t N_cap, int C_cap, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ sorted_idx, int c_begin, int c_count,
    bf16* __restrict__ centroids, bf16* __restrict__ mu_hat, float* __restrict__ centroids_f32) {
  __shared__ float part[4][D];
  const int c = blockIdx.x, hp = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l16 = tid & 15, grp = tid >> 4;  // 16 groups
  const int32_t* off = offsets + (int64_t)hp * (C_cap + 1) + c_begin + c;
  const int beg = off[0], n = off[1] - beg;
  if (n <= 0) return;                                   // empty cluster keeps its centroid
  const int32_t* idx = sorted_idx + (int64_t)hp * N_cap + beg;
  const bf16* Khp = K + (int64_t)hp * N_cap * D + l16 * 8;

  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  for (int j0 = 0; j0 < n; j0 += 64) {
    uint4 w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int j = j0 + u * 16 + grp;
      if (j < n) {
        int64_t row = idx[j];
        row = row < 0 ? 0 : (row >= N_cap ? N_cap - 1 : row);
        w[u] = *reinterpret_cast<const uint4*>(Khp + row * D);
      } else {
        w[u] = make_uint4(0, 0, 0, 0);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      acc[0] += lo_bf16(w[u].x); acc[1] += hi_bf16(w[u].x);
      acc[2] += lo_bf16(w[u].y); acc[3] += hi_bf16(w[u].y);
      acc[4] += lo_bf16(w[u].z); acc[5] += hi_bf16(w[u].z);
      acc[6] += lo_bf16(w[u].w); acc[7] += hi_bf16(w[u].w);
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
    float m0 = ((part[0][2 * lane] + part[1][2 * lane]) + part[2][2 * lane]) + part[3][2 * lane];
    float m1 = ((part[0][2 * lane + 1] + part[1][2 * lane + 1]) + part[2][2 * lane + 1]) +
               part[3][2 * lane + 1];
    m0 *= inv_n;
    m1 *= inv_n;
    const float n2 = wave_sum(m0 * m0 + m1 * m1);
    const float inv = n2 > 0.f ? 1.0f / sqrtf(n2) : 0.f;
    const int64_t crow = (int64_t)hp * C_cap + c_begin + c;
    const int64_t hrow = (int64_t)hp * c_count + c;
    reinterpret_cast<uint32_t*>(centroids + crow * D)[lane] =
        (uint32_t)float_to_bf16_bits(m0) | ((uint32_t)float_to_bf16_bits(m1) << 16);
    reinterpret_cast<uint32_t*>(mu_hat + hrow * D)[lane] =
        (uint32_t)float_to_bf16_bits(m0 * inv) | ((uint32_t)float_to_bf16_bits(m1 * inv) << 16);
    if (centroids_f32)
      reinterpret_cast<float2*>(centroids_f32 + hrow * D)[lane] = make_float2(m0, m1);
  }
}

hipError_t launch_update(const Dims& dm, const bf16* K, const int32_t* offsets,
                         const int32_t* sorted_idx, int c_begin, int c_count, bf16* centroids,
                         bf16* mu_hat, float* centroids_f32, hipStream_t st) {
  hipLaunchKernelGGL(k_update, dim3(c_count, dm.HP), dim3(UPD_THREADS), 0, st, K, dm.N_cap,
                     dm.C_cap, offsets, sorted_idx, c_begin, c_count, centroids, mu_hat,
                     centroids_f32);
  return hipGetLastError();
}

ClusterWorkspace carve_cluster_workspace(const Dims& dm, int64_t tok_count, int c_count,
                                         void* base) {
  ClusterWorkspace w;
  const int64_t n_chunks = (tok_count + SORT_CHUNK - 1) / SORT_CHUNK;
  size_t mu = (size_t)dm.HP * c_count * D * sizeof(bf16);
  mu = (mu + 255) & ~(size_t)255;
  size_t hist = (size_t)dm.HP * n_chunks * c_count * sizeof(int32_t);
  hist = (hist + 255) & ~(size_t)255;
  w.mu_hat = reinterpret_cast<bf16*>(base);
  w.chunk_hist = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(base) + mu);
  w.bytes = mu + hist;
  return w;
}

}  // namespace ck
