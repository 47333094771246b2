// Whole K-means of a small token range in ONE kernel (paper Section III-B, decode
// stage: every m generated tokens are clustered among themselves into a handful of
// new clusters).  At m = 320 tokens and 4 clusters an iteration is ~0.3 MFLOP per
// head-problem, so the four-kernels-per-iteration pipeline of the prefill path spends
// its time on launches; here one workgroup per head-problem keeps the keys in LDS and
// runs init, all iterations (assignment, update), the metadata and the stores itself.
// Same arithmetic rules as the large path: bf16-rounded table rows compared in fp32,
// ties to the lower id, fp32 sums in a fixed order, means of raw keys, an empty cluster
// keeps its centroid.
#include "ck_common.hpp"

namespace ck {


struct SmallArgs {
  const bf16* K;
  const int32_t* init_idx;
  bf16* centroids;
  int32_t *labels, *sizes, *offsets, *sorted_idx, *iters_done;
  int64_t N_cap, tok_begin;
  int tok_count, C_cap, c_begin, c_count, max_iter, metric, converge;
};

// MAXC: compile-time bound of the cluster count (register arrays); SM_THREADS: workgroup size
// (more wavefronts hide the LDS and cross-lane latencies of the 16-lane dot products).
template <int MAXC, int SM_THREADS>
__global__ __launch_bounds__(SM_THREADS) void k_kmeans_small(const SmallArgs a) {
  constexpr int SM_SLICES = SM_THREADS / WAVE;           // partial sums of the update: one per wavefront
  __shared__ __attribute__((aligned(16))) bf16 keys[KM_SMALL_MAX_TOKENS * D];
  __shared__ __attribute__((aligned(16))) float table[MAXC][D];
  __shared__ float mu[MAXC][D];
  __shared__ float part[SM_SLICES][MAXC][D];
  __shared__ int cnt[SM_SLICES][MAXC];
  __shared__ int wave_cnt[SM_THREADS / WAVE][MAXC];
  __shared__ float bias[MAXC];
  __shared__ int lab[KM_SMALL_MAX_TOKENS];
  __shared__ int s_changed;

  const int hp = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_tok = a.tok_count, C = a.c_count;
  const bf16* Khp = a.K + (int64_t)hp * a.N_cap * D;

  // ---- keys of the range into LDS (16-byte pieces), initial centroids ----
  for (int i = tid; i < n_tok * 16; i += SM_THREADS)
    reinterpret_cast<uint4*>(keys)[i] =
        reinterpret_cast<const uint4*>(Khp + a.tok_begin * D)[i];
  for (int e = tid; e < C * D; e += SM_THREADS) {
    const int c = e / D, ch = e % D;
    int64_t row = a.init_idx[(int64_t)hp * C + c];
    row = row < 0 ? 0 : (row >= a.N_cap ? a.N_cap - 1 : row);
    mu[c][ch] = bf16_bits_to_float(reinterpret_cast<const uint16_t*>(Khp + row * D)[ch]);
  }
  for (int t = tid; t < n_tok; t += SM_THREADS) lab[t] = -1;
  for (int e = tid; e < SM_SLICES * MAXC; e += SM_THREADS)
    cnt[e / MAXC][e % MAXC] = 0;
  __syncthreads();

  const int l16 = tid & 15, grp = tid >> 4;             // 32 groups of 16 lanes
  int n_done = 0;
  for (int it = 0; it < a.max_iter; ++it) {
    // ---- table row (and l2 bias) of cluster `wave`: lane holds channels 2*lane, 2*lane+1 ----
    if (wave < C) {
      const float m0 = mu[wave][2 * lane], m1 = mu[wave][2 * lane + 1];
      float r0, r1;
      if (a.metric == CK_METRIC_COSINE) {
        const float n2 = wave_sum(m0 * m0 + m1 * m1);
        const float inv = n2 > 0.f ? 1.0f / sqrtf(n2) : 0.f;
        r0 = bf16_bits_to_float(float_to_bf16_bits(m0 * inv));
        r1 = bf16_bits_to_float(float_to_bf16_bits(m1 * inv));
      } else {
        r0 = bf16_bits_to_float(float_to_bf16_bits(m0));
        r1 = bf16_bits_to_float(float_to_bf16_bits(m1));
      }
      table[wave][2 * lane] = r0;
      table[wave][2 * lane + 1] = r1;
      if (a.metric == CK_METRIC_L2) {
        const float rn2 = wave_sum(r0 * r0 + r1 * r1);
        if (lane == 0) bias[wave] = -0.5f * rn2;
      } else if (lane == 0) {
        bias[wave] = 0.f;
      }
    }
    if (tid == 0) s_changed = 0;
    __syncthreads();

    // ---- assignment, and the sums of the update in the same pass: 16 lanes per key, 8
    // channels per lane; every lane of the group learns the label and adds its channels of
    // the key to the sums of that cluster.  A stopped run discards the sums. ----
    float tb[MAXC][8], acc[MAXC][8];
    int n[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      n[c] = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        tb[c][j] = c < C ? table[c][l16 * 8 + j] : 0.f;
        acc[c][j] = 0.f;
      }
    }
    int diff = 0;
    for (int t = grp; t < n_tok; t += SM_THREADS / 16) {
      const uint4 w = *reinterpret_cast<const uint4*>(keys + t * D + l16 * 8);
      float kv[8];
      kv[0] = lo_bf16(w.x); kv[1] = hi_bf16(w.x); kv[2] = lo_bf16(w.y); kv[3] = hi_bf16(w.y);
      kv[4] = lo_bf16(w.z); kv[5] = hi_bf16(w.z); kv[6] = lo_bf16(w.w); kv[7] = hi_bf16(w.w);
      float best = 0.f;
      int bc = 0;
#pragma unroll
      for (int c = 0; c < MAXC; ++c) {
        if (c < C) {                                    // uniform
          float d = 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) d = fmaf(kv[j], tb[c][j], d);
          d = row16_sum(d) + bias[c];
          if (c == 0 || d > best) {
            best = d;
            bc = c;
          }
        }
      }
#pragma unroll
      for (int c = 0; c < MAXC; ++c) {
        if (c < C) {
          const float on = bc == c ? 1.f : 0.f;
          n[c] += bc == c ? 1 : 0;
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[c][j] = fmaf(on, kv[j], acc[c][j]);
        }
      }
      if (l16 == 0) {
        diff += lab[t] != bc ? 1 : 0;
        lab[t] = bc;
      }
    }
    diff = __builtin_amdgcn_readlane(wave_inclusive_scan(diff), WAVE - 1);
    if (lane == 0 && diff) atomicAdd(&s_changed, diff);
    // the four groups of a wavefront, then (below) the wavefronts in order
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
      if (c < C) {
        n[c] += __shfl_xor(n[c], 16, WAVE);
        n[c] += __shfl_xor(n[c], 32, WAVE);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[c][j] = xor32(xor16(acc[c][j], OpSum()), OpSum());
        if (lane < 16) {
#pragma unroll
          for (int j = 0; j < 8; ++j) part[wave][c][l16 * 8 + j] = acc[c][j];
          if (lane == 0) cnt[wave][c] = n[c];
        }
      }
    }
    __syncthreads();
    ++n_done;
    if (a.converge && it > 0 && s_changed == 0) break;  // uniform: the previous update stands

    // ---- update: mean of the assigned keys; an empty cluster keeps its centroid ----
    for (int e = tid; e < C * D; e += SM_THREADS) {
      const int c = e / D, ch = e % D;
      int nn = 0;
      float sum = 0.f;
#pragma unroll
      for (int wv = 0; wv < SM_THREADS / WAVE; ++wv) {
        nn += cnt[wv][c];
        sum += part[wv][c][ch];
      }
      if (nn > 0) mu[c][ch] = sum * (1.0f / (float)nn);
    }
    __syncthreads();
  }

  // ---- stores: centroids, labels, sizes, offsets, stable label-sorted index ----
  for (int e = tid; e < C * D; e += SM_THREADS) {
    const int c = e / D, ch = e % D;
    reinterpret_cast<uint16_t*>(a.centroids + ((int64_t)hp * a.C_cap + a.c_begin + c) * D)[ch] =
        float_to_bf16_bits(mu[c][ch]);
  }
  int32_t* off_g = a.offsets + (int64_t)hp * (a.C_cap + 1);
  const int base0 = a.c_begin == 0 ? 0 : off_g[a.c_begin];
  const bool valid = tid < n_tok;
  const int l = valid ? lab[tid] : -1;
  const uint64_t lt = ((uint64_t)1 << lane) - 1;
  int rank = 0;
  for (int c = 0; c < C; ++c) {
    const uint64_t m = __ballot(l == c);
    if (l == c) rank = __popcll(m & lt);
    if (lane == 0) wave_cnt[wave][c] = __popcll(m);
  }
  __syncthreads();
  if (valid) {
    int pos = base0 + rank;
    for (int c = 0; c < l; ++c)
      for (int w = 0; w < SM_THREADS / WAVE; ++w) pos += wave_cnt[w][c];
    for (int w = 0; w < wave; ++w) pos += wave_cnt[w][l];
    if (pos >= 0 && pos < a.N_cap) a.sorted_idx[(int64_t)hp * a.N_cap + pos] = (int32_t)(a.tok_begin + tid);
    a.labels[(int64_t)hp * a.N_cap + a.tok_begin + tid] = a.c_begin + l;
  }
  if (tid == 0) {
    int run = base0;
    if (a.c_begin == 0) off_g[0] = 0;
    for (int c = 0; c < C; ++c) {
      int n = 0;
      for (int w = 0; w < SM_THREADS / WAVE; ++w) n += wave_cnt[w][c];
      a.sizes[(int64_t)hp * a.C_cap + a.c_begin + c] = n;
      run += n;
      off_g[a.c_begin + c + 1] = run;
    }
    if (a.iters_done) a.iters_done[hp] = n_done;
  }
}

bool kmeans_small_fits(int64_t tok_count, int c_count) {
  return tok_count <= KM_SMALL_MAX_TOKENS && c_count <= KM_SMALL_MAX_CLUSTERS;
}

hipError_t launch_kmeans_small(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                               int c_begin, int c_count, int max_iter, int metric, bool converge,
                               const int32_t* init_idx, bf16* centroids, int32_t* labels,
                               int32_t* sizes, int32_t* offsets, int32_t* sorted_idx,
                               int32_t* iters_done, hipStream_t st) {
  SmallArgs a;
  a.K = K;
  a.init_idx = init_idx;
  a.centroids = centroids;
  a.labels = labels;
  a.sizes = sizes;
  a.offsets = offsets;
  a.sorted_idx = sorted_idx;
  a.iters_done = iters_done;
  a.N_cap = dm.N_cap;
  a.tok_begin = tok_begin;
  a.tok_count = (int)tok_count;
  a.C_cap = dm.C_cap;
  a.c_begin = c_begin;
  a.c_count = c_count;
  a.max_iter = max_iter;
  a.metric = metric;
  a.converge = converge ? 1 : 0;
  if (c_count <= 4)
    hipLaunchKernelGGL((k_kmeans_small<4, 1024>), dim3(dm.HP), dim3(1024), 0, st, a);
  else
    hipLaunchKernelGGL((k_kmeans_small<KM_SMALL_MAX_CLUSTERS, 512>), dim3(dm.HP), dim3(512), 0, st, a);
  return hipGetLastError();
}

}  // namespace ck
