// Device code shared by the decode-step kernels: loading rows of the storage type
// and the selection of the recalled cluster prefix (paper Section III-C and the
// size gather / prefix sum of Section IV-C, Fig. 8).
#pragma once
#include "ck_common.hpp"

namespace ck {

template <typename T>
__device__ __forceinline__ void load_row8(const T* p, float (&v)[8]);
template <>
__device__ __forceinline__ void load_row8<bf16>(const bf16* p, float (&v)[8]) {
  const uint4 w = *reinterpret_cast<const uint4*>(p);
  v[0] = lo_bf16(w.x); v[1] = hi_bf16(w.x); v[2] = lo_bf16(w.y); v[3] = hi_bf16(w.y);
  v[4] = lo_bf16(w.z); v[5] = hi_bf16(w.z); v[6] = lo_bf16(w.w); v[7] = hi_bf16(w.w);
}
template <>
__device__ __forceinline__ void load_row8<float>(const float* p, float (&v)[8]) {
  const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

// Monotone map float -> uint32 (a < b  <=>  map(a) < map(b); -0 and +0 made equal).
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  if (f == 0.f) f = 0.f;                                    // -0 -> +0
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int SELP_THREADS = 256;          // every kernel that selects runs 256 threads
constexpr int SELP_BINS = 256;
constexpr int SELP_MAX_CAND = 512;         // more candidates than this: rank all clusters
constexpr int SELP_ITEMS = CK_MAX_CLUSTERS / SELP_THREADS;

// LDS of one selection.  After select_prefix(): ord[j], cbeg[j], csz[j], cum[j] for
// j < n_sel describe the recalled clusters in score order (cum = inclusive prefix
// sum of their sizes).
struct alignas(16) SelectLds {
  uint32_t key[CK_MAX_CLUSTERS];   // ~ordered(score): ascending key = descending score
  int ssz[CK_MAX_CLUSTERS];        // size per cluster id
  int soff[CK_MAX_CLUSTERS];       // offsets[cluster] per cluster id (when offsets are given)
  int ord[CK_MAX_CLUSTERS];        // cluster id per sorted position
  int cum[CK_MAX_CLUSTERS];        // inclusive prefix sum of sizes per sorted position
  int cbeg[SELP_MAX_CAND];         // offsets[cluster] per sorted position (candidate path only)
  int cand[SELP_MAX_CAND];         // candidate cluster ids (compacted, any order)
  uint32_t ckey[SELP_MAX_CAND];    // their keys, dense, so that the ranking loop streams
  int bin_size[SELP_BINS];
  int bin_cnt[SELP_BINS];
  float red_f[2 * (SELP_THREADS / WAVE)];
  int tmp[SELP_THREADS / WAVE + 1];
  int n_cand, n_sel, n_tok, counter, full_rank, last_bin, n_app;
};

// Orders the clusters of one head-problem by descending score (ties: lower id
// first) as far as needed and counts the recalled prefix under `budget`:
//   trim == 0: longest prefix whose sizes sum to <= budget;
//   trim == 1: shortest prefix whose sizes sum to >= budget (all if the total is smaller).
// A histogram of the scores (sizes accumulated per bin) bounds the prefix first, so
// that only a few dozen candidates are ranked; degenerate score distributions fall
// back to ranking every cluster.  Must be called by all SELP_THREADS threads.
__device__ __forceinline__ void select_prefix(SelectLds& L, const float* __restrict__ scores,
                                              const int32_t* __restrict__ sizes,
                                              const int32_t* __restrict__ offsets, int C,
                                              int budget, int trim) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float sc[SELP_ITEMS];
  int sz[SELP_ITEMS];
  float smax = -INFINITY, smin = INFINITY;
#pragma unroll
  for (int i = 0; i < SELP_ITEMS; ++i) {
    const int c = tid + i * SELP_THREADS;
    sc[i] = c < C ? scores[c] : 0.f;
    sz[i] = c < C ? sizes[c] : 0;
  }
  if (offsets) {                       // same round trip as the scores: no dependent load later
    int of[SELP_ITEMS];
#pragma unroll
    for (int i = 0; i < SELP_ITEMS; ++i) {
      const int c = tid + i * SELP_THREADS;
      of[i] = c < C ? offsets[c] : 0;
    }
#pragma unroll
    for (int i = 0; i < SELP_ITEMS; ++i) {
      const int c = tid + i * SELP_THREADS;
      if (c < C) L.soff[c] = of[i];
    }
  }
#pragma unroll
  for (int i = 0; i < SELP_ITEMS; ++i) {
    const int c = tid + i * SELP_THREADS;
    if (c < C) {
      L.key[c] = ~ordered_bits(sc[i]);
      L.ssz[c] = sz[i];
      smax = fmaxf(smax, sc[i]);
      smin = fminf(smin, sc[i]);
    }
  }
  for (int b = tid; b < SELP_BINS; b += SELP_THREADS) {
    L.bin_size[b] = 0;
    L.bin_cnt[b] = 0;
  }
  for (int i = tid; i < SELP_MAX_CAND; i += SELP_THREADS) {
    L.ckey[i] = 0xFFFFFFFFu;                     // padding that never ranks before anything
    L.cand[i] = 0x7FFFFFFF;
  }
  if (tid == 0) {
    L.n_app = 0;
    L.counter = 0;
  }
  smax = wave_max(smax);
  smin = wave_min(smin);
  if (lane == 0) {
    L.red_f[wave] = smax;
    L.red_f[SELP_THREADS / WAVE + wave] = smin;
  }
  __syncthreads();
#pragma unroll
  for (int w = 0; w < SELP_THREADS / WAVE; ++w) {
    smax = fmaxf(smax, L.red_f[w]);
    smin = fminf(smin, L.red_f[SELP_THREADS / WAVE + w]);
  }
  const float span = smax - smin;
  const float inv = span > 0.f ? (float)(SELP_BINS - 1) / span : 0.f;
  int bin[SELP_ITEMS];
#pragma unroll
  for (int i = 0; i < SELP_ITEMS; ++i) {
    const int c = tid + i * SELP_THREADS;
    // monotone: a larger score never lands in a later bin
    int b = (int)((smax - sc[i]) * inv);
    b = b < 0 ? 0 : (b > SELP_BINS - 1 ? SELP_BINS - 1 : b);
    bin[i] = b;
    if (c < C) {
      atomicAdd(&L.bin_size[b], sz[i]);
      atomicAdd(&L.bin_cnt[b], 1);
    }
  }
  __syncthreads();
  // first bin at which the running size crosses the budget; everything up to and
  // including it is a candidate
  if (wave == 0) {
    constexpr int PER = SELP_BINS / WAVE;
    int s[PER], n[PER];
    int ssum = 0, nsum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      ssum += L.bin_size[lane * PER + i];
      nsum += L.bin_cnt[lane * PER + i];
      s[i] = ssum;
      n[i] = nsum;
    }
    const int sp = wave_inclusive_scan(ssum), np = wave_inclusive_scan(nsum);
    const int sbase = sp - ssum, nbase = np - nsum;
    int first = SELP_BINS, ncand = 0;
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
      const int cs = sbase + s[i];
      if (trim ? cs >= budget : cs > budget) {
        first = lane * PER + i;
        ncand = nbase + n[i];
      }
    }
    // lowest crossing bin over the wavefront (bin numbers are exact in fp32)
    const int best = (int)wave_min((float)first);
    if (best == SELP_BINS) {                 // no crossing: every cluster is recalled
      if (lane == 0) {
        L.last_bin = SELP_BINS - 1;
        L.n_cand = C;
      }
    } else if (first == best) {
      L.last_bin = best;
      L.n_cand = ncand;
    }
  }
  __syncthreads();
  const int last_bin = L.last_bin, m = L.n_cand;
  if (m <= SELP_MAX_CAND) {
    // ---- compact the candidates (id and key side by side), then rank them among
    // themselves ----
#pragma unroll
    for (int i = 0; i < SELP_ITEMS; ++i) {
      const int c = tid + i * SELP_THREADS;
      if (c < C && bin[i] <= last_bin) {
        const int pos = atomicAdd(&L.n_app, 1);
        L.cand[pos] = c;
        L.ckey[pos] = ~ordered_bits(sc[i]);
      }
    }
    __syncthreads();
    const int m_pad = (m + 3) & ~3;
    for (int i = tid; i < m; i += SELP_THREADS) {
      const int c = L.cand[i];
      const uint32_t kc = L.ckey[i];
      const int ob = offsets ? L.soff[c] : 0;
      int rank = 0;
      for (int j = 0; j < m_pad; j += 4) {
        const uint4 k4 = *reinterpret_cast<const uint4*>(&L.ckey[j]);
        const int4 c4 = *reinterpret_cast<const int4*>(&L.cand[j]);
        rank += (k4.x < kc || (k4.x == kc && c4.x < c)) ? 1 : 0;
        rank += (k4.y < kc || (k4.y == kc && c4.y < c)) ? 1 : 0;
        rank += (k4.z < kc || (k4.z == kc && c4.z < c)) ? 1 : 0;
        rank += (k4.w < kc || (k4.w == kc && c4.w < c)) ? 1 : 0;
      }
      L.ord[rank] = c;
      L.cum[rank] = L.ssz[c];
      L.cbeg[rank] = ob;
    }
  } else {
    // ---- rank every cluster (all scores equal, budget beyond the total, ...) ----
    const int n_pad = (C + 3) & ~3;
    for (int j = C + tid; j < n_pad; j += SELP_THREADS) L.key[j] = 0xFFFFFFFFu;
    __syncthreads();
    for (int c = tid; c < C; c += SELP_THREADS) {
      const uint32_t kc = L.key[c];
      int rank = 0;
      for (int j = 0; j < n_pad; j += 4) {
        const uint4 k4 = *reinterpret_cast<const uint4*>(&L.key[j]);
        rank += (k4.x < kc || (k4.x == kc && j + 0 < c)) ? 1 : 0;
        rank += (k4.y < kc || (k4.y == kc && j + 1 < c)) ? 1 : 0;
        rank += (k4.z < kc || (k4.z == kc && j + 2 < c)) ? 1 : 0;
        rank += (k4.w < kc || (k4.w == kc && j + 3 < c)) ? 1 : 0;
      }
      L.ord[rank] = c;
      L.cum[rank] = L.ssz[c];
    }
  }
  __syncthreads();
  // ---- inclusive prefix sum of the sizes in score order, and the recalled count ----
  if (m <= WAVE) {
    // the usual case (a few dozen candidates): one wavefront, no further barriers inside
    if (wave == 0) {
      const int own = lane < m ? L.cum[lane] : 0;
      const int v = wave_inclusive_scan(own);
      if (lane < m) L.cum[lane] = v;
      const bool in = lane < m && (trim ? (v < budget) : (v <= budget));
      int n_sel = __popcll(__ballot(in));
      if (trim) n_sel = n_sel + 1 < m ? n_sel + 1 : m;
      // prefix sum at position n_sel - 1, taken from the lane that holds it
      int n_tok = n_sel > 0 ? __shfl(v, n_sel - 1, WAVE) : 0;
      if (trim && n_tok > budget) n_tok = budget;
      if (lane == 0) {
        L.n_sel = n_sel;
        L.n_tok = n_tok;
        L.full_rank = 0;
      }
    }
    __syncthreads();
    return;
  }
  int v[SELP_ITEMS];
#pragma unroll
  for (int i = 0; i < SELP_ITEMS; ++i) {
    const int j = tid * SELP_ITEMS + i;
    v[i] = j < m ? L.cum[j] : 0;
  }
  block_inclusive_scan<SELP_ITEMS>(v, L.tmp);
  int cnt = 0;
#pragma unroll
  for (int i = 0; i < SELP_ITEMS; ++i) {
    const int j = tid * SELP_ITEMS + i;
    if (j < m) {
      cnt += trim ? (v[i] < budget) : (v[i] <= budget);
      L.cum[j] = v[i];
    }
  }
  if (cnt) atomicAdd(&L.counter, cnt);
  __syncthreads();
  if (tid == 0) {
    int n_sel = L.counter;
    if (trim) n_sel = n_sel + 1 < m ? n_sel + 1 : m;
    int n_tok = n_sel > 0 ? L.cum[n_sel - 1] : 0;
    if (trim && n_tok > budget) n_tok = budget;
    L.n_sel = n_sel;
    L.n_tok = n_tok;
    L.full_rank = m > SELP_MAX_CAND;
  }
  __syncthreads();
}

}  // namespace ck
