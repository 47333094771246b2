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

// ---- cluster / row scores of a bf16 table on the matrix cores ----
// s_r = sum_g <q_g, row_r> for 16 consecutive table rows per wavefront step:
// v_mfma_f32_16x16x32_bf16 with the query heads of the group as the rows of A (row >= G
// is zero) and the 16 table rows as the columns of B.  Lane l < 16 then holds, for table
// row l of the step, the four heads 0..3 in its four accumulators (lanes 16..31: heads
// 4..7), so the sum over the heads is three in-lane additions (one lane exchange more for
// G = 8) and the 16 scores leave the wavefront as one 64-byte store.  Every caller that
// scores a bf16 table goes through these two functions, so that the separate scoring
// kernel and the fused decode kernel produce bit-identical scores.
// The query heads as a 16 x 32 MFMA operand per slab: lane l holds head l%16, channels
// 32*sl + 8*(l/16) .. +8.  Heads >= G do not exist: their lanes re-read head 0 (always a
// valid address) and whatever the matrix cores compute for them is never looked at --
// rows (or columns) of an MFMA result do not mix.
__device__ __forceinline__ void load_query_operand(const bf16* __restrict__ q_group, int G,
                                                   int lane, bf16x8 (&qb)[4]) {
  const int col = lane & 15, kg = lane >> 4;
  const bf16* p = q_group + (int64_t)(col < G ? col : 0) * D + kg * 8;
#pragma unroll
  for (int sl = 0; sl < 4; ++sl)
    qb[sl] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p + sl * 32));
}
// t[sl]: this lane's 16 bytes of table row lane%16 (channels 32*sl + 8*(lane/16) ..).
// Returns in lanes 0..15 the score of table row `lane` of the step.
__device__ __forceinline__ float score_rows16(const uint4 (&t)[4], const bf16x8 (&qb)[4], int G) {
  floatx4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int sl = 0; sl < 4; ++sl)
    d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qb[sl], __builtin_bit_cast(bf16x8, t[sl]), d, 0, 0, 0);
  // accumulator i of lanes 0..15 is head i, of lanes 16..31 head 4 + i
  float v = d[0];
  if (G >= 2) v += d[1];
  if (G >= 4) v = v + (d[2] + d[3]);
  if (G == 8) v = xor16(v, OpSum());
  return v;
}

// Makes the compiler fetch a kernel argument where this stands.  Kernel arguments are
// read with scalar loads that the compiler otherwise issues piecemeal, each where it is
// first needed and each a full (cold) memory round trip; a kernel that starts with a
// chain of dependent steps pins one argument per 64-byte line of its argument block at
// its top, so that the lines arrive together.
#define CK_FETCH_ARG(x) asm volatile("" ::"s"(x))

// Monotone map float -> uint32 (a < b  <=>  map(a) < map(b); -0 and +0 made equal).
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  if (f == 0.f) f = 0.f;                                    // -0 -> +0
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int SELP_THREADS = 256;          // every kernel that selects runs 256 threads
constexpr int SELP_BINS = 256;
constexpr int SELP_MAX_CAND = 512;         // more candidates than this: rank all clusters
constexpr int SELP_SMALL = 512;            // cluster bound of the small instantiation

// LDS of one selection, sized for at most CMAX clusters (512 or CK_MAX_CLUSTERS: the
// launcher picks the smallest that holds the table, so that a few hundred clusters do
// not reserve the LDS of two thousand and more workgroups fit a CU).  After
// select_prefix(): ord[j], cbeg[j], cum[j] for j < n_sel describe the recalled clusters
// in score order (cum = inclusive prefix sum of their sizes).
template <int CMAX>
struct alignas(16) SelectLds {
  static_assert(CMAX % SELP_THREADS == 0 && CMAX >= SELP_MAX_CAND, "cluster bound");
  uint32_t key[CMAX];              // ~ordered(score): ascending key = descending score
  int ssz[CMAX];                   // size per cluster id
  int soff[CMAX];                  // offsets[cluster] per cluster id (when offsets are given)
  int ord[CMAX];                   // cluster id per sorted position
  int cum[CMAX];                   // inclusive prefix sum of sizes per sorted position
  int cbeg[SELP_MAX_CAND];         // offsets[cluster] per sorted position (candidate path only)
  int cand[SELP_MAX_CAND];         // candidate cluster ids (compacted, any order)
  uint32_t ckey[SELP_MAX_CAND];    // their keys, dense, so that the ranking loop streams
  int bin_size[SELP_BINS];
  int bin_cnt[SELP_BINS];
  float red_f[2 * (SELP_THREADS / WAVE)];
  int tmp[SELP_THREADS / WAVE + 1];
  int n_cand, n_sel, n_tok, counter, full_rank, last_bin, n_app, fast_ok;
};

// Orders the clusters of one head-problem by descending score (ties: lower id
// first) as far as needed and counts the recalled prefix under `budget`:
//   trim == 0: longest prefix whose sizes sum to <= budget;
//   trim == 1: shortest prefix whose sizes sum to >= budget (all if the total is smaller).
// A histogram of the scores (sizes accumulated per bin) bounds the prefix first, so
// that only a few dozen candidates are ranked; degenerate score distributions fall
// back to ranking every cluster.  Must be called by all SELP_THREADS threads.
// This form takes the values a thread owns in registers (cluster tid + i * SELP_THREADS;
// entries beyond C are ignored), so that a caller can have fetched them long before.
template <int CMAX>
__device__ __forceinline__ void select_prefix_regs(SelectLds<CMAX>& L,
                                                   const float (&sc)[CMAX / SELP_THREADS],
                                                   const int (&sz)[CMAX / SELP_THREADS],
                                                   const int (&of)[CMAX / SELP_THREADS],
                                                   bool offsets, int C, int budget, int trim) {
  constexpr int SELP_ITEMS = CMAX / SELP_THREADS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float smax = -INFINITY, smin = INFINITY;
  if (offsets) {
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

// LDS operations of ONE wavefront are served in order; this only keeps the compiler
// from moving them across the point.
__device__ __forceinline__ void wave_lds_order() {
  __builtin_amdgcn_wave_barrier();
  asm volatile("" ::: "memory");
}

// The selection by ONE wavefront, without workgroup barriers, for tables of at most
// SELP_SMALL clusters whose recalled prefix is bounded by at most 64 candidates (the usual
// case: a few dozen).  Same result as select_prefix_regs.  Before the call: sc[c] (LDS),
// L.ssz[c] and L.soff[c] hold score, size and offset of every cluster c < C, and a
// workgroup barrier has been passed.  All threads call it; it ends with a barrier and
// returns false (for every thread) when the candidate bound does not hold, in which case
// nothing has been selected and the general form has to run.
__device__ __forceinline__ bool select_prefix_wave(SelectLds<SELP_SMALL>& L, const float* sc,
                                                   int C, int budget, int trim) {
  constexpr int PER_LANE = SELP_SMALL / WAVE;           // 8 clusters per lane: 8*lane + i
  const int tid = threadIdx.x, lane = tid & 63;
  if (tid < WAVE) {
    float s[PER_LANE];
    int z[PER_LANE];
    {
      const floatx4* sp = reinterpret_cast<const floatx4*>(sc + lane * PER_LANE);
      const int4* zp = reinterpret_cast<const int4*>(&L.ssz[lane * PER_LANE]);
#pragma unroll
      for (int h = 0; h < PER_LANE / 4; ++h) {
        const floatx4 a = sp[h];
        const int4 b = zp[h];
        s[4 * h] = a[0]; s[4 * h + 1] = a[1]; s[4 * h + 2] = a[2]; s[4 * h + 3] = a[3];
        z[4 * h] = b.x; z[4 * h + 1] = b.y; z[4 * h + 2] = b.z; z[4 * h + 3] = b.w;
      }
    }
    float smax = -INFINITY, smin = INFINITY;
#pragma unroll
    for (int i = 0; i < PER_LANE; ++i) {
      const bool ok = lane * PER_LANE + i < C;
      smax = fmaxf(smax, ok ? s[i] : -INFINITY);
      smin = fminf(smin, ok ? s[i] : INFINITY);
    }
    smax = wave_max(smax);
    smin = wave_min(smin);
    const float span = smax - smin;
    const float inv = span > 0.f ? (float)(SELP_BINS - 1) / span : 0.f;
    // histogram of the scores, sizes accumulated per bin
    {
      int4* bs = reinterpret_cast<int4*>(&L.bin_size[lane * 4]);
      int4* bc = reinterpret_cast<int4*>(&L.bin_cnt[lane * 4]);
      *bs = make_int4(0, 0, 0, 0);
      *bc = make_int4(0, 0, 0, 0);
    }
    wave_lds_order();
    int bin[PER_LANE];
#pragma unroll
    for (int i = 0; i < PER_LANE; ++i) {
      int b = (int)((smax - s[i]) * inv);               // monotone: a larger score, no later bin
      b = b < 0 ? 0 : (b > SELP_BINS - 1 ? SELP_BINS - 1 : b);
      const bool ok = lane * PER_LANE + i < C;
      bin[i] = ok ? b : SELP_BINS;                      // never a candidate
      if (ok) {
        atomicAdd(&L.bin_size[b], z[i]);
        atomicAdd(&L.bin_cnt[b], 1);
      }
    }
    wave_lds_order();
    // first bin at which the running size crosses the budget
    constexpr int PER = SELP_BINS / WAVE;
    int ss[PER], nn[PER];
    int ssum = 0, nsum = 0;
    {
      const int4 a = *reinterpret_cast<const int4*>(&L.bin_size[lane * PER]);
      const int4 b = *reinterpret_cast<const int4*>(&L.bin_cnt[lane * PER]);
      ss[0] = a.x; ss[1] = ss[0] + a.y; ss[2] = ss[1] + a.z; ss[3] = ss[2] + a.w;
      nn[0] = b.x; nn[1] = nn[0] + b.y; nn[2] = nn[1] + b.z; nn[3] = nn[2] + b.w;
      ssum = ss[3];
      nsum = nn[3];
    }
    const int sbase = wave_inclusive_scan(ssum) - ssum, nbase = wave_inclusive_scan(nsum) - nsum;
    int first = SELP_BINS, ncand = 0;
#pragma unroll
    for (int i = PER - 1; i >= 0; --i) {
      const int cs = sbase + ss[i];
      if (trim ? cs >= budget : cs > budget) {
        first = lane * PER + i;
        ncand = nbase + nn[i];
      }
    }
    const uint64_t crossing = __ballot(first < SELP_BINS);
    int last_bin = SELP_BINS - 1, m = C;                // no crossing: every cluster is recalled
    if (crossing) {
      const int src = __builtin_ctzll(crossing);        // lowest lane = lowest bin
      last_bin = __builtin_amdgcn_readlane(first, src);
      m = __builtin_amdgcn_readlane(ncand, src);
    }
    if (m > WAVE) {                                     // wave-uniform
      if (lane == 0) L.fast_ok = 0;
    } else {
      // compact the candidates (any order), one per lane afterwards
      const uint64_t lt = ((uint64_t)1 << lane) - 1;
      int base = 0;
#pragma unroll
      for (int i = 0; i < PER_LANE; ++i) {
        const bool is_c = bin[i] <= last_bin;
        const uint64_t mask = __ballot(is_c);
        if (is_c) {
          const int pos = base + __popcll(mask & lt);
          L.cand[pos] = lane * PER_LANE + i;
          L.ckey[pos] = ~ordered_bits(s[i]);
        }
        base += __popcll(mask);
      }
      wave_lds_order();
      const int c = lane < m ? L.cand[lane] : 0x7FFFFFFF;
      const uint32_t kc = lane < m ? L.ckey[lane] : 0xFFFFFFFFu;
      // rank among the candidates: ascending key = descending score, ties to the lower id
      int rank = 0;
      for (int j = 0; j < m; ++j) {
        const uint32_t kj = (uint32_t)__builtin_amdgcn_readlane((int)kc, j);
        const int cj = __builtin_amdgcn_readlane(c, j);
        rank += (kj < kc || (kj == kc && cj < c)) ? 1 : 0;
      }
      if (lane < m) {
        L.ord[rank] = c;
        L.cum[rank] = L.ssz[c];
        L.cbeg[rank] = L.soff[c];
      }
      wave_lds_order();
      const int own = lane < m ? L.cum[lane] : 0;
      const int v = wave_inclusive_scan(own);
      if (lane < m) L.cum[lane] = v;
      const bool in = lane < m && (trim ? (v < budget) : (v <= budget));
      int n_sel = __popcll(__ballot(in));
      if (trim) n_sel = n_sel + 1 < m ? n_sel + 1 : m;
      int n_tok = n_sel > 0 ? __shfl(v, n_sel - 1, WAVE) : 0;
      if (trim && n_tok > budget) n_tok = budget;
      if (lane == 0) {
        L.n_sel = n_sel;
        L.n_tok = n_tok;
        L.full_rank = 0;
        L.fast_ok = 1;
      }
    }
  }
  __syncthreads();
  return L.fast_ok != 0;
}

// The same, loading scores (global memory or LDS), sizes and offsets (nullable) here.
template <int CMAX>
__device__ __forceinline__ void select_prefix(SelectLds<CMAX>& L, const float* scores,
                                              const int32_t* __restrict__ sizes,
                                              const int32_t* __restrict__ offsets, int C,
                                              int budget, int trim) {
  constexpr int SELP_ITEMS = CMAX / SELP_THREADS;
  const int tid = threadIdx.x;
  float sc[SELP_ITEMS];
  int sz[SELP_ITEMS], of[SELP_ITEMS];
#pragma unroll
  for (int i = 0; i < SELP_ITEMS; ++i) {
    const int c = tid + i * SELP_THREADS;
    sc[i] = c < C ? scores[c] : 0.f;
    sz[i] = c < C ? sizes[c] : 0;
    of[i] = (offsets && c < C) ? offsets[c] : 0;      // same round trip as the scores
  }
  select_prefix_regs<CMAX>(L, sc, sz, of, offsets != nullptr, C, budget, trim);
}

}  // namespace ck
