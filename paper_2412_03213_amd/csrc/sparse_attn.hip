// Sparse GQA decode attention over the recalled tokens (paper Section II-B:
// softmax(q K_S^T / sqrt(d)) V_S with K_S, V_S the selected rows), alone or fused
// with the centroid scoring and cluster selection of Section III-C and the index
// generation of Section IV-C: a whole decode step is then ONE kernel launch.
//
// HBM-bound: every recalled K and V row (256 B in bf16) is read exactly once per
// KV head and shared by the G query heads of the group.  A wavefront takes 16
// tokens per step.  V rows are owned by 16-lane groups (16 B of the row per lane)
// and accumulated on the vector ALUs; in bf16 the K rows go straight into
// v_mfma_f32_16x16x32_bf16 as the A operand with the query heads as B columns,
// which removes the unpacking, the dot products and their cross-lane reductions
// from the vector ALUs (fp32 check mode keeps the all-VALU form).  The attended
// positions of a head-problem are split over several workgroups (split-KV) so that
// a batch of a few sequences still fills 256 CUs.  Inside a workgroup the token rows
// of its positions are resolved into LDS first, and the K/V loads of the next TWO
// steps are in flight while the current one is reduced.
//
// Merging the splits without a second launch: every workgroup publishes its partial
// (max, sum, accumulator) with agent-scope stores, takes a ticket from a counter of
// its head-problem, and the workgroup that draws the last ticket reads all partials
// back with agent-scope loads and writes the output.  Nobody waits for anybody, so
// nothing can hang; agent-scope accesses are performed past the XCD-private L2
// caches, so no cache write-back or invalidate is needed.  The merge adds the
// partials in split order, whoever runs it: results are bit-reproducible.
//
// Fused modes: every workgroup of a head-problem repeats the (cheap, LDS-only)
// selection of the recalled cluster prefix and maps its own positions through the
// cluster-contiguous index directly; the index list is still written out (each
// workgroup its own part) but never re-read.  With at most 512 clusters in bf16 the
// centroid scores are computed by every workgroup as well (the workgroups of one
// head-problem are placed on one XCD, so the table comes from HBM once and out of
// that XCD's L2 otherwise); larger or fp32 tables are scored by a launch of their own.
#include <mutex>
#include <type_traits>

#include "decode_common.hpp"

namespace ck {

constexpr int ATT_THREADS = SELP_THREADS;  // 4 wavefronts = 16 token slots per workgroup step
constexpr int ATT_UNROLL = 4;              // token slots in flight per 16-lane group
constexpr int ATT_STEP_TOKENS = 16 * ATT_UNROLL;   // 64 tokens per workgroup iteration
constexpr int ATT_MAX_CHUNK = 2048;        // positions one workgroup may own (rows held in LDS)
constexpr int ATT_MAX_SPLITS = 1024;       // workgroups per head-problem
constexpr float NEG_BIG = -1.0e30f;        // "no token yet": finite so that differences stay finite
constexpr int ATT_TARGET_WGS = 256;        // one per CU on 256 CUs
constexpr int PEX_WAVE = 16 * 8 + 8;       // floats of probability exchange per wavefront (G <= 8)
constexpr int PART_STRIDE = D + 2;         // floats per (split, query head): max, sum, acc[128]
constexpr int N_XCD = 8;                   // workgroup i of a launch runs on XCD i % 8
constexpr unsigned long long TICKET_MAGIC = 0x434B7469636Bull;   // marks a ticket word as ours

enum { ATT_PLAIN = 0, ATT_FUSED = 1, ATT_FUSED_SCORE = 2 };

template <typename T> struct RawRow;
template <> struct RawRow<bf16> {
  uint4 w;
  __device__ __forceinline__ void load(const bf16* p) { w = *reinterpret_cast<const uint4*>(p); }
  __device__ __forceinline__ void unpack(float (&v)[8]) const {
    v[0] = lo_bf16(w.x); v[1] = hi_bf16(w.x); v[2] = lo_bf16(w.y); v[3] = hi_bf16(w.y);
    v[4] = lo_bf16(w.z); v[5] = hi_bf16(w.z); v[6] = lo_bf16(w.w); v[7] = hi_bf16(w.w);
  }
};
template <> struct RawRow<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = reinterpret_cast<const float4*>(p)[0];
    b = reinterpret_cast<const float4*>(p)[1];
  }
  __device__ __forceinline__ void unpack(float (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};

__device__ __forceinline__ void store_out(bf16* p, float v) {
  *reinterpret_cast<uint16_t*>(p) = float_to_bf16_bits(v);
}
__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }

// ---- partials in memory: pairs of floats, moved as one 64-bit word ----
// Agent scope: the access is performed past the XCD-private L2, so a workgroup on
// another XCD sees the value without any cache maintenance.
__device__ __forceinline__ void put_pair_agent(float* p, float x, float y) {
  const unsigned long long w =
      (unsigned long long)__float_as_uint(x) | ((unsigned long long)__float_as_uint(y) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), w, __ATOMIC_RELAXED,
                     __HIP_MEMORY_SCOPE_AGENT);
}
struct PairAgent {
  __device__ __forceinline__ float2 operator()(const float* p) const {
    const unsigned long long w =
        __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                          __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((uint32_t)w), __uint_as_float((uint32_t)(w >> 32)));
  }
};
struct PairPlain {
  __device__ __forceinline__ float2 operator()(const float* p) const {
    return *reinterpret_cast<const float2*>(p);
  }
};

// out channels (c2, c2 + 1) of one query head from its n_split partials:
//   sum_i acc_i 2^(m_i - M) / sum_i l_i 2^(m_i - M), splits added in index order,
// MERGE_BATCH partials loaded together so that their latencies overlap.
// base = partial of split 0 for this head, stride = floats between splits.
constexpr int MERGE_BATCH = 16;
template <typename Load>
__device__ __forceinline__ float2 merge_splits(const float* base, int64_t stride, int n_split,
                                               int c2, Load load) {
  float M = NEG_BIG, ls = 0.f, a0 = 0.f, a1 = 0.f;
  for (int i0 = 0; i0 < n_split; i0 += MERGE_BATCH) {
    float2 ml[MERGE_BATCH], av[MERGE_BATCH];
#pragma unroll
    for (int i = 0; i < MERGE_BATCH; ++i) {
      const bool ok = i0 + i < n_split;
      const float* p = base + (int64_t)(ok ? i0 + i : 0) * stride;
      ml[i] = load(p);
      av[i] = load(p + 2 + c2);
      if (!ok) {
        ml[i] = make_float2(NEG_BIG, 0.f);
        av[i] = make_float2(0.f, 0.f);
      }
    }
    float mx = M;
#pragma unroll
    for (int i = 0; i < MERGE_BATCH; ++i) mx = fmaxf(mx, ml[i].x);
    const float corr = __builtin_amdgcn_exp2f(M - mx);
    ls *= corr;
    a0 *= corr;
    a1 *= corr;
    M = mx;
#pragma unroll
    for (int i = 0; i < MERGE_BATCH; ++i) {
      const float f = __builtin_amdgcn_exp2f(ml[i].x - mx);
      ls += ml[i].y * f;
      a0 += av[i].x * f;
      a1 += av[i].y * f;
    }
  }
  const float inv = ls > 0.f ? 1.0f / ls : 0.f;
  return make_float2(a0 * inv, a1 * inv);
}

struct AttnArgs {
  const void *q, *K, *V;
  void* out;
  float* part;                  // [HP, n_split, G, PART_STRIDE]
  unsigned long long* tickets;  // [HP]: (TICKET_MAGIC << 16) | workgroups arrived so far
  // given index list
  const int32_t* token_idx;
  const int32_t* n_tokens;
  // fused selection
  const void* centroids;        // ATT_FUSED_SCORE: the table to score
  float* scores;                // ATT_FUSED: read; ATT_FUSED_SCORE: written
  const int32_t *sizes, *offsets, *sorted_idx;
  int32_t *sel_clusters, *n_sel_clusters, *n_sel_tokens, *token_idx_out, *n_tokens_out;
  int n_clusters, budget, trim, C_cap;
  // common
  int HP, idx_stride, max_tokens, Hq, Hkv, n_sink, n_recent, chunk, n_split, two_pass;
  int64_t N_cap, recent_begin;
  float scale_log2e;
};

template <int G> struct PlainLds { float red[4 * G * PART_STRIDE]; };

// Attended position p of a head-problem -> token row:
//   [0, n_sink) sinks, then the recalled list, then [recent_begin, recent_end).
// One-dimensional grid: workgroup i runs on XCD i % 8 (round-robin dispatch), so the
// n_split workgroups of a head-problem are given ids of one residue class and share
// that XCD's L2 (sizes, offsets, scores or the centroid table).  Placement only affects
// speed, never results.
template <typename T, int G, int MODE, int CMAX>
__global__ __launch_bounds__(ATT_THREADS) void k_attn(const AttnArgs a) {
  constexpr bool FUSED = MODE != ATT_PLAIN;
  using Big = typename std::conditional<FUSED, SelectLds<CMAX>, PlainLds<G>>::type;
  static_assert(sizeof(Big) >= sizeof(PlainLds<G>), "the wavefront partials reuse the selection's LDS");
  __shared__ Big big;                                   // selection, later the wavefront partials
  __shared__ int rows[ATT_MAX_CHUNK];
  __shared__ __attribute__((aligned(16))) float pex[4 * PEX_WAVE];
  __shared__ __attribute__((aligned(16))) float sc_lds[MODE == ATT_FUSED_SCORE ? CMAX : 4];
  __shared__ int s_last;
  float* red = reinterpret_cast<float*>(&big);

  // one argument per 64-byte line of the argument block: all lines are requested now
  CK_FETCH_ARG(a.q);
  CK_FETCH_ARG(a.n_tokens);
  CK_FETCH_ARG(a.sorted_idx);
  CK_FETCH_ARG(a.n_tokens_out);
  CK_FETCH_ARG(a.n_clusters);
  CK_FETCH_ARG(a.C_cap);
  CK_FETCH_ARG(a.n_sink);
  CK_FETCH_ARG(a.scale_log2e);
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l16 = tid & 15, slot = tid >> 4;  // 16 slots
  const int wg = blockIdx.x, xcd = wg % N_XCD, seq = wg / N_XCD;
  const int hp = (seq / a.n_split) * N_XCD + xcd, split = seq % a.n_split;
  if (hp >= a.HP) return;                               // the grid is padded to whole groups of 8
  const int s = hp / a.Hkv, h = hp % a.Hkv;
  const T* q = static_cast<const T*>(a.q);

  // the query heads of the group as an MFMA operand (bf16): for the scores and for q K^T
  bf16x8 qb[4];
  if constexpr (std::is_same<T, bf16>::value)
    load_query_operand(reinterpret_cast<const bf16*>(q) + ((int64_t)s * a.Hq + h * G) * D, G, lane, qb);

  int n_idx;
  if constexpr (FUSED) {
    SelectLds<CMAX>& L = big;
    if constexpr (MODE == ATT_FUSED_SCORE) {
      // ---- scores of all clusters of this head-problem (bf16 table, matrix cores) ----
      // Every load of the prologue is issued before the first use: the table rows of
      // this wavefront (16 rows per step, steps wave, wave + 4, ...), the query heads,
      // the sizes and offsets this thread will bring to the selection: one round trip.
      constexpr int ITEMS = CMAX / SELP_THREADS;
      constexpr int SB = CMAX / 64;                     // 16-row steps per wavefront
      const int col = lane & 15, kg = lane >> 4;
      int sz[ITEMS], of[ITEMS];
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        const int c = tid + i * SELP_THREADS;
        sz[i] = c < a.n_clusters ? a.sizes[(int64_t)hp * a.C_cap + c] : 0;
        of[i] = c < a.n_clusters ? a.offsets[(int64_t)hp * (a.C_cap + 1) + c] : 0;
      }
      const bf16* Thp = static_cast<const bf16*>(a.centroids) + (int64_t)hp * a.C_cap * D + kg * 8;
      const int n_steps = (a.n_clusters + 15) >> 4;
      uint4 ar[SB][4];
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        if (wave + 4 * u < n_steps) {                   // wave-uniform
          int r = (wave + 4 * u) * 16 + col;
          if (r >= a.n_clusters) r = a.n_clusters - 1;  // clamp: result is discarded
#pragma unroll
          for (int sl = 0; sl < 4; ++sl)
            ar[u][sl] = *reinterpret_cast<const uint4*>(Thp + (int64_t)r * D + sl * 32);
        }
      }
#pragma unroll
      for (int u = 0; u < SB; ++u) {
        if (wave + 4 * u < n_steps) {
          const float v = score_rows16(ar[u], qb, G);
          const int r = (wave + 4 * u) * 16 + lane;
          if (lane < 16 && r < a.n_clusters) {
            sc_lds[r] = v;
            if (split == 0) a.scores[(int64_t)hp * a.C_cap + r] = v;
          }
        }
      }
#pragma unroll
      for (int i = 0; i < ITEMS; ++i) {
        const int c = tid + i * SELP_THREADS;
        if (c < a.n_clusters) {
          L.ssz[c] = sz[i];
          L.soff[c] = of[i];
        }
      }
      __syncthreads();
      // one wavefront selects when a few dozen candidates bound the prefix (the usual
      // case); otherwise all four do, the general way
      if (!select_prefix_wave(L, sc_lds, a.n_clusters, a.budget, a.trim)) {
        float sc[ITEMS];
#pragma unroll
        for (int i = 0; i < ITEMS; ++i) {
          const int c = tid + i * SELP_THREADS;
          sc[i] = c < a.n_clusters ? sc_lds[c] : 0.f;
        }
        select_prefix_regs<CMAX>(L, sc, sz, of, true, a.n_clusters, a.budget, a.trim);
      }
    } else {
      select_prefix<CMAX>(L, a.scores + (int64_t)hp * a.C_cap, a.sizes + (int64_t)hp * a.C_cap,
                          a.offsets + (int64_t)hp * (a.C_cap + 1), a.n_clusters, a.budget, a.trim);
    }
    n_idx = L.n_tok;
    if (split == 0) {
      for (int j = tid; j < L.n_sel; j += ATT_THREADS)
        a.sel_clusters[(int64_t)hp * a.C_cap + j] = L.ord[j];
      if (tid == 0) {
        a.n_sel_clusters[hp] = L.n_sel;
        a.n_sel_tokens[hp] = n_idx;
        a.n_tokens_out[hp] = n_idx;
      }
    }
  } else {
    n_idx = a.n_tokens ? a.n_tokens[hp] : 0;
    n_idx = n_idx < 0 ? 0 : (n_idx > a.max_tokens ? a.max_tokens : n_idx);
  }
  const int n_total = a.n_sink + n_idx + a.n_recent;
  const int p_begin = split * a.chunk;
  int p_end = p_begin + a.chunk;
  if (p_end > n_total) p_end = n_total;
  const int n_pos = p_end > p_begin ? p_end - p_begin : 0;

  // ---- token row of every position this workgroup owns ----
  for (int i = tid; i < n_pos; i += ATT_THREADS) {
    const int p = p_begin + i;
    int64_t row;
    if (p < a.n_sink) {
      row = p;
    } else if (p < a.n_sink + n_idx) {
      const int qpos = p - a.n_sink;
      if constexpr (FUSED) {
        SelectLds<CMAX>& L = big;
        // smallest j with cum[j] > qpos (empty clusters in the prefix are skipped)
        int lo = 0, hi = L.n_sel - 1;
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (L.cum[mid] > qpos) hi = mid; else lo = mid + 1;
        }
        const int c = L.ord[lo];
        const int prev = lo ? L.cum[lo - 1] : 0;
        const int size = L.cum[lo] - prev;
        int take = a.budget - prev;                     // a cut cluster keeps its trailing entries
        take = take > size ? size : take;
        const int beg = L.full_rank ? L.soff[c] : L.cbeg[lo];
        int64_t src = (int64_t)beg + (size - take) + (qpos - prev);
        src = src < 0 ? 0 : (src >= a.N_cap ? a.N_cap - 1 : src);
        row = a.sorted_idx[(int64_t)hp * a.N_cap + src];
        a.token_idx_out[(int64_t)hp * a.idx_stride + qpos] = (int32_t)row;
      } else {
        // no list: the first n_tokens rows of K/V themselves (a dense per-head-problem prefix)
        row = a.token_idx ? a.token_idx[(int64_t)hp * a.idx_stride + qpos] : qpos;
      }
    } else {
      row = a.recent_begin + (p - a.n_sink - n_idx);
    }
    row = row < 0 ? 0 : (row >= a.N_cap ? a.N_cap - 1 : row);
    rows[i] = (int)row;
  }
  __syncthreads();                                      // rows complete; the selection's LDS is free

  float acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[g][j] = 0.f;
  const T* Vhp = static_cast<const T*>(a.V) + (int64_t)hp * a.N_cap * D + l16 * 8;

  if constexpr (std::is_same<T, bf16>::value) {
    // ---- bf16: q K^T on the matrix cores ----
    // One v_mfma_f32_16x16x32_bf16 per 32-channel slab: A = 16 token rows of the
    // step (lane: token lane%16, channels 8*(lane/16)..+8 of the slab), B = the
    // query heads as columns (column >= G is zero).  The result leaves lane
    // (g + 16u) with the scores of tokens (u, 0..3) for head g, so the running
    // max / sum of a head live in the four lanes of its column and the
    // probabilities reach the lanes that own the V rows through a few hundred
    // bytes of wavefront-private LDS.  All four token slots of a wavefront share
    // one running max per head.
    const int col = lane & 15, kg = lane >> 4;          // kg is also this lane's slot in the wavefront
    float m_run = NEG_BIG, l_run = 0.f;                 // of head `col`, identical in its four lanes
    float* px = pex + wave * PEX_WAVE;                  // [slot][u][g] probabilities, then [g] rescale factors
    const bf16* Khp = static_cast<const bf16*>(a.K) + (int64_t)hp * a.N_cap * D + kg * 8;
    const int tpos = (col >> 2) * 16 + wave * 4 + (col & 3);   // A row `col` = token (u = col/4, slot = col%4)
    struct Regs { uint4 k[4], v[ATT_UNROLL]; };
    auto fetch = [&](int i0, Regs& r) {
      const int ik = i0 + tpos;
      const bf16* kp = Khp + (int64_t)(ik < n_pos ? rows[ik] : 0) * D;
#pragma unroll
      for (int sl = 0; sl < 4; ++sl) r.k[sl] = *reinterpret_cast<const uint4*>(kp + sl * 32);
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        const int i = i0 + u * 16 + slot;
        r.v[u] = *reinterpret_cast<const uint4*>(Vhp + (int64_t)(i < n_pos ? rows[i] : 0) * D);
      }
    };
    auto reduce = [&](int i0, const Regs& r) {
      floatx4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int sl = 0; sl < 4; ++sl)
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, r.k[sl]), qb[sl], d, 0, 0, 0);
      // d[i]: token (u = kg, slot i) against head `col`
      float sc[4];
      const int ibase = i0 + kg * 16 + wave * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) sc[i] = (ibase + i < n_pos) ? d[i] * a.scale_log2e : -INFINITY;
      float mx = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
      mx = xor32(xor16(mx, OpMax()), OpMax());
      mx = fmaxf(mx, m_run);
      const float corr = __builtin_amdgcn_exp2f(m_run - mx);
      m_run = mx;
      float pw[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) pw[i] = __builtin_amdgcn_exp2f(sc[i] - mx);
      float ps = (pw[0] + pw[1]) + (pw[2] + pw[3]);
      ps = xor32(xor16(ps, OpSum()), OpSum());
      l_run = l_run * corr + ps;
      if (col < G) {
#pragma unroll
        for (int i = 0; i < 4; ++i) px[(i * 4 + kg) * G + col] = pw[i];
        if (kg == 0) px[16 * G + col] = corr;
      }
      // LDS serves one wavefront's requests in order: the reads below see the writes above
      __builtin_amdgcn_wave_barrier();
      asm volatile("" ::: "memory");
      float pr[ATT_UNROLL][G], cr[G];
      {
        const floatx4* src = reinterpret_cast<const floatx4*>(px + kg * 4 * G);
        floatx4 tmp[G];
#pragma unroll
        for (int k = 0; k < G; ++k) tmp[k] = src[k];
#pragma unroll
        for (int k = 0; k < G; ++k)
#pragma unroll
          for (int e = 0; e < 4; ++e) pr[(k * 4 + e) / G][(k * 4 + e) % G] = tmp[k][e];
#pragma unroll
        for (int g = 0; g < G; ++g) cr[g] = px[16 * G + g];
      }
      asm volatile("" ::: "memory");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[g][j] *= cr[g];
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        float vv[8];
        vv[0] = lo_bf16(r.v[u].x); vv[1] = hi_bf16(r.v[u].x); vv[2] = lo_bf16(r.v[u].y); vv[3] = hi_bf16(r.v[u].y);
        vv[4] = lo_bf16(r.v[u].z); vv[5] = hi_bf16(r.v[u].z); vv[6] = lo_bf16(r.v[u].w); vv[7] = hi_bf16(r.v[u].w);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[g][j] = fmaf(pr[u][g], vv[j], acc[g][j]);
      }
    };
    // NS register sets in rotation: the loads of steps t + 1 .. t + NS - 1 are in flight
    // while step t is reduced (4 and 6 sets were measured: no faster, the row stream is
    // bound by memory bandwidth, not by the depth of the prefetch)
    constexpr int NS = 3;
    Regs rs[NS];
    constexpr int ST = ATT_STEP_TOKENS;
#pragma unroll
    for (int j = 0; j < NS - 1; ++j)
      if (j * ST < n_pos) fetch(j * ST, rs[j]);
    for (int i0 = 0; i0 < n_pos; i0 += NS * ST) {
#pragma unroll
      for (int j = 0; j < NS; ++j) {
        if (i0 + j * ST < n_pos) {
          if (i0 + (j + NS - 1) * ST < n_pos) fetch(i0 + (j + NS - 1) * ST, rs[(j + NS - 1) % NS]);
          reduce(i0 + j * ST, rs[j]);
        }
      }
    }
    // ---- combine the 4 slots of a wavefront: they share the running max ----
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[g][j] = xor32(xor16(acc[g][j], OpSum()), OpSum());
    if (lane < 16) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float* r = red + (wave * G + g) * PART_STRIDE;
#pragma unroll
        for (int j = 0; j < 8; ++j) r[2 + l16 * 8 + j] = acc[g][j];
      }
      if (lane < G) {
        float* r = red + (wave * G + lane) * PART_STRIDE;
        r[0] = m_run;
        r[1] = l_run;
      }
    }
  } else {
    // ---- fp32 check mode: dot products on the vector ALUs ----
    // this lane's 8 channels of every query head of the group, pre-scaled
    float qv[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      load_row8<T>(q + ((int64_t)s * a.Hq + h * G + g) * D + l16 * 8, qv[g]);
#pragma unroll
      for (int j = 0; j < 8; ++j) qv[g][j] *= a.scale_log2e;
    }

    float m[G], l[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m[g] = NEG_BIG;
      l[g] = 0.f;
    }

    const T* Khp = static_cast<const T*>(a.K) + (int64_t)hp * a.N_cap * D + l16 * 8;
    RawRow<T> kc[ATT_UNROLL], vc[ATT_UNROLL], kn[ATT_UNROLL], vn[ATT_UNROLL];
    auto fetch = [&](int i0, RawRow<T>(&kr)[ATT_UNROLL], RawRow<T>(&vr)[ATT_UNROLL]) {
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        const int i = i0 + u * 16 + slot;
        const int64_t row = i < n_pos ? rows[i] : 0;
        kr[u].load(Khp + row * D);
        vr[u].load(Vhp + row * D);
      }
    };
    if (n_pos > 0) fetch(0, kc, vc);
    for (int i0 = 0; i0 < n_pos; i0 += ATT_STEP_TOKENS) {
      if (i0 + ATT_STEP_TOKENS < n_pos) fetch(i0 + ATT_STEP_TOKENS, kn, vn);
      float kv[ATT_UNROLL][8];
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) kc[u].unpack(kv[u]);
      float sc[G][ATT_UNROLL];
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int u = 0; u < ATT_UNROLL; ++u) {
          float d = 0.f;
#pragma unroll
          for (int j = 0; j < 8; ++j) d = fmaf(qv[g][j], kv[u][j], d);
          d = row16_sum(d);
          sc[g][u] = (i0 + u * 16 + slot < n_pos) ? d : -INFINITY;
        }
      float pw[G][ATT_UNROLL];
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float mx = m[g];
#pragma unroll
        for (int u = 0; u < ATT_UNROLL; ++u) mx = fmaxf(mx, sc[g][u]);
        const float corr = __builtin_amdgcn_exp2f(m[g] - mx);
        m[g] = mx;
        float ls = l[g] * corr;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[g][j] *= corr;
#pragma unroll
        for (int u = 0; u < ATT_UNROLL; ++u) {
          pw[g][u] = __builtin_amdgcn_exp2f(sc[g][u] - mx);
          ls += pw[g][u];
        }
        l[g] = ls;
      }
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        float vv[8];
        vc[u].unpack(vv);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[g][j] = fmaf(pw[g][u], vv[j], acc[g][j]);
      }
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        kc[u] = kn[u];
        vc[u] = vn[u];
      }
    }

    // ---- combine the 4 slots of a wavefront (lanes l16 + 16*k) ----
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mx = xor32(xor16(m[g], OpMax()), OpMax());
      const float w = __builtin_amdgcn_exp2f(m[g] - mx);
      const float ls = xor32(xor16(l[g] * w, OpSum()), OpSum());
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[g][j] = xor32(xor16(acc[g][j] * w, OpSum()), OpSum());
      if (lane < 16) {
        float* r = red + (wave * G + g) * PART_STRIDE;
        r[0] = mx;
        r[1] = ls;
#pragma unroll
        for (int j = 0; j < 8; ++j) r[2 + l16 * 8 + j] = acc[g][j];
      }
    }
  }
  __syncthreads();
  // ---- combine the 4 wavefronts: thread = (query head g, channel pair) ----
  T* out = static_cast<T*>(a.out);
  float* part_hp = a.part + (int64_t)hp * a.n_split * G * PART_STRIDE;
  for (int e = tid; e < G * (D / 2); e += ATT_THREADS) {
    const int g = e / (D / 2), c2 = (e % (D / 2)) * 2;
    const float* r0 = red + (0 * G + g) * PART_STRIDE;
    const float* r1 = red + (1 * G + g) * PART_STRIDE;
    const float* r2 = red + (2 * G + g) * PART_STRIDE;
    const float* r3 = red + (3 * G + g) * PART_STRIDE;
    const float mx = fmaxf(fmaxf(r0[0], r1[0]), fmaxf(r2[0], r3[0]));
    const float f0 = __builtin_amdgcn_exp2f(r0[0] - mx), f1 = __builtin_amdgcn_exp2f(r1[0] - mx);
    const float f2 = __builtin_amdgcn_exp2f(r2[0] - mx), f3 = __builtin_amdgcn_exp2f(r3[0] - mx);
    const float ls = ((r0[1] * f0 + r1[1] * f1) + r2[1] * f2) + r3[1] * f3;
    const float a0 = ((r0[2 + c2] * f0 + r1[2 + c2] * f1) + r2[2 + c2] * f2) + r3[2 + c2] * f3;
    const float a1 = ((r0[3 + c2] * f0 + r1[3 + c2] * f1) + r2[3 + c2] * f2) + r3[3 + c2] * f3;
    if (a.n_split == 1) {
      const float inv = ls > 0.f ? 1.0f / ls : 0.f;
      T* o = out + ((int64_t)s * a.Hq + h * G + g) * D + c2;
      store_out(o, a0 * inv);
      store_out(o + 1, a1 * inv);
    } else {
      float* pr = part_hp + ((int64_t)split * G + g) * PART_STRIDE;
      if (a.two_pass) {
        if (c2 == 0) *reinterpret_cast<float2*>(pr) = make_float2(mx, ls);
        *reinterpret_cast<float2*>(pr + 2 + c2) = make_float2(a0, a1);
      } else {
        if (c2 == 0) put_pair_agent(pr, mx, ls);
        put_pair_agent(pr + 2 + c2, a0, a1);
      }
    }
  }
  if (a.n_split == 1 || a.two_pass) return;

  // ---- ticket: the last workgroup of the head-problem to get here merges ----
  // Every thread waits until its stores above have been acknowledged (they are
  // agent-scope stores: performed where every XCD looks) before it passes the barrier;
  // only then is the ticket drawn.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();
  if (tid == 0) {
    // Idle state of a ticket word: TICKET_MAGIC in the upper 48 bits, count 0.  One
    // fetch-add draws the ticket.  A word that does not carry the mark (memory this
    // library has never used: the first launch on a fresh workspace) is taken over with
    // a compare-and-swap loop instead; whoever added to it before the take-over adds
    // itself again through the same loop, so every workgroup is counted exactly once.
    unsigned long long* tk = a.tickets + hp;
    unsigned long long old =
        __hip_atomic_fetch_add(tk, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long now = old + 1;
    if ((old >> 16) != TICKET_MAGIC) {
      unsigned long long seen = now;
      do {
        now = (seen >> 16) == TICKET_MAGIC ? seen + 1 : ((TICKET_MAGIC << 16) | 1ull);
      } while (!__hip_atomic_compare_exchange_strong(tk, &seen, now, __ATOMIC_RELAXED,
                                                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    const int last = (int)(now & 0xFFFFull) == a.n_split;
    // back to idle: ready for the next launch (or a replay of this one from a graph)
    if (last) __hip_atomic_store(tk, TICKET_MAGIC << 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = last;
  }
  __syncthreads();
  if (!s_last) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  for (int e = tid; e < G * (D / 2); e += ATT_THREADS) {
    const int g = e / (D / 2), c2 = (e % (D / 2)) * 2;
    const float2 o2 = merge_splits(part_hp + (int64_t)g * PART_STRIDE, (int64_t)G * PART_STRIDE,
                                   a.n_split, c2, PairAgent());
    T* o = out + ((int64_t)s * a.Hq + h * G + g) * D + c2;
    store_out(o, o2.x);
    store_out(o + 1, o2.y);
  }
}

// Second pass of the two-pass form: the same merge, by a kernel of its own.
template <typename T>
__global__ __launch_bounds__(D / 2) void k_attn_merge(const float* __restrict__ part, int n_split,
                                                      int G, int Hq, int Hkv, T* __restrict__ out) {
  const int hq_lin = blockIdx.x;                        // s * Hq + hq
  const int s = hq_lin / Hq, hq = hq_lin % Hq;
  const int hp = s * Hkv + hq / G, g = hq % G, c2 = threadIdx.x * 2;
  const float* base = part + (((int64_t)hp * n_split) * G + g) * PART_STRIDE;
  const float2 o2 = merge_splits(base, (int64_t)G * PART_STRIDE, n_split, c2, PairPlain());
  store_out(out + (int64_t)hq_lin * D + c2, o2.x);
  store_out(out + (int64_t)hq_lin * D + c2 + 1, o2.y);
}

int attn_num_splits(const Dims& dm, int64_t max_total) {
  // Aim for one workgroup per CU (measured best of 64..1024 workgroups per launch at 8 to
  // 128 head-problems for the one-launch decode step: every split repeats the scoring and
  // the selection, which costs more than the shorter token run saves; the attention over
  // a given list would like twice as many at 64 head-problems, 17.1 against 18.5 us, but
  // takes the same rule: the split boundaries fix the order of the fp32 sums, and all
  // forms of the step must give the same bits).  Keep at least one full step of tokens
  // per workgroup and never more positions than its LDS row table holds.
  const int64_t by_work = (max_total + ATT_STEP_TOKENS - 1) / ATT_STEP_TOKENS;
  const int64_t by_fill = (ATT_TARGET_WGS + dm.HP - 1) / dm.HP;
  int64_t n = by_work < by_fill ? by_work : by_fill;
  if (n > 64) n = 64;
  const int64_t need = (max_total + ATT_MAX_CHUNK - 1) / ATT_MAX_CHUNK;
  if (n < need) n = need;
  if (n < 1) n = 1;
  return (int)n;
}

static size_t partial_bytes(const Dims& dm, int n_split) {
  const size_t b = (size_t)dm.HP * n_split * dm.G * PART_STRIDE * sizeof(float);
  return (b + 255) & ~(size_t)255;
}

size_t attn_workspace_bytes(const Dims& dm, int64_t max_total) {
  // split partials, then one 64-bit ticket word per head-problem
  const size_t t = ((size_t)dm.HP * sizeof(unsigned long long) + 255) & ~(size_t)255;
  return partial_bytes(dm, attn_num_splits(dm, max_total)) + t;
}

template <typename T, int MODE, int CMAX>
static hipError_t launch_attn_t(const Dims& dm, AttnArgs a, int64_t max_total, bool two_pass,
                                hipStream_t st) {
  const int n_split = attn_num_splits(dm, max_total);
  if (n_split > ATT_MAX_SPLITS) return hipErrorInvalidValue;
  int chunk = (int)((max_total + n_split - 1) / n_split);
  chunk = (chunk + ATT_STEP_TOKENS - 1) / ATT_STEP_TOKENS * ATT_STEP_TOKENS;
  if (chunk < ATT_STEP_TOKENS) chunk = ATT_STEP_TOKENS;
  if (chunk > ATT_MAX_CHUNK) return hipErrorInvalidValue;
  a.chunk = chunk;
  a.n_split = n_split;
  a.two_pass = two_pass ? 1 : 0;
  a.HP = dm.HP;
  a.tickets = reinterpret_cast<unsigned long long*>(reinterpret_cast<char*>(a.part) +
                                                    partial_bytes(dm, n_split));
  const int hp_groups = (dm.HP + N_XCD - 1) / N_XCD;
  const dim3 grid((unsigned)hp_groups * N_XCD * n_split), block(ATT_THREADS);
  switch (dm.G) {
    case 1: hipLaunchKernelGGL((k_attn<T, 1, MODE, CMAX>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((k_attn<T, 2, MODE, CMAX>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((k_attn<T, 4, MODE, CMAX>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((k_attn<T, 8, MODE, CMAX>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  if (n_split > 1 && two_pass)
    hipLaunchKernelGGL(k_attn_merge<T>, dim3(dm.S * dm.Hq), dim3(D / 2), 0, st, a.part, n_split,
                       dm.G, dm.Hq, dm.Hkv, (T*)a.out);
  return hipGetLastError();
}

static AttnArgs common_args(const Dims& dm, const void* q, const void* K, const void* V,
                            int idx_stride, int max_tokens, int64_t n_sink, int64_t recent_begin,
                            int64_t recent_end, float softmax_scale, void* out, void* workspace) {
  AttnArgs a = {};
  a.q = q;
  a.K = K;
  a.V = V;
  a.out = out;
  a.part = reinterpret_cast<float*>(workspace);
  a.idx_stride = idx_stride;
  a.max_tokens = max_tokens;
  a.Hq = dm.Hq;
  a.Hkv = dm.Hkv;
  a.C_cap = dm.C_cap;
  a.N_cap = dm.N_cap;
  a.n_sink = (int)n_sink;
  a.recent_begin = recent_begin;
  a.n_recent = (int)(recent_end > recent_begin ? recent_end - recent_begin : 0);
  a.scale_log2e = softmax_scale * 1.4426950408889634f;
  return a;
}

hipError_t launch_sparse_attn(const Dims& dm, const void* q, const void* K, const void* V,
                              const int32_t* token_idx, const int32_t* n_tokens, int idx_stride,
                              int64_t max_total, int64_t n_sink, int64_t recent_begin,
                              int64_t recent_end, float softmax_scale, void* out, void* workspace,
                              bool two_pass, hipStream_t st) {
  const int n_recent = (int)(recent_end > recent_begin ? recent_end - recent_begin : 0);
  AttnArgs a = common_args(dm, q, K, V, idx_stride, (int)(max_total - n_sink - n_recent), n_sink,
                           recent_begin, recent_end, softmax_scale, out, workspace);
  a.token_idx = token_idx;
  a.n_tokens = n_tokens;
  if (dm.dtype == CK_BF16)
    return launch_attn_t<bf16, ATT_PLAIN, SELP_SMALL>(dm, a, max_total, two_pass, st);
  return launch_attn_t<float, ATT_PLAIN, SELP_SMALL>(dm, a, max_total, two_pass, st);
}

hipError_t launch_decode_fused(const Dims& dm, const void* q, const void* K, const void* V,
                               const void* centroids, const int32_t* sizes,
                               const int32_t* offsets, const int32_t* sorted_idx, int n_clusters,
                               int budget, uint32_t flags, int64_t n_sink, int64_t recent_begin,
                               int64_t recent_end, float softmax_scale, float* scores,
                               int32_t* sel_clusters, int32_t* n_sel_clusters,
                               int32_t* n_sel_tokens, int32_t* token_idx, int idx_stride,
                               int32_t* n_tokens, void* out, void* workspace, hipStream_t st) {
  AttnArgs a = common_args(dm, q, K, V, idx_stride, budget, n_sink, recent_begin, recent_end,
                           softmax_scale, out, workspace);
  a.centroids = centroids;
  a.scores = scores;
  a.sizes = sizes;
  a.offsets = offsets;
  a.sorted_idx = sorted_idx;
  a.sel_clusters = sel_clusters;
  a.n_sel_clusters = n_sel_clusters;
  a.n_sel_tokens = n_sel_tokens;
  a.token_idx_out = token_idx;
  a.n_tokens_out = n_tokens;
  a.n_clusters = n_clusters;
  a.budget = budget;
  a.trim = (int)(flags & CK_SEL_TRIM_LAST);
  const int64_t max_total = (int64_t)budget + n_sink + a.n_recent;
  if (dm.dtype == CK_BF16 && n_clusters <= SELP_SMALL)  // one launch for the whole step
    return launch_attn_t<bf16, ATT_FUSED_SCORE, SELP_SMALL>(dm, a, max_total, false, st);
  const hipError_t e = launch_score(dm, q, centroids, n_clusters, scores, st);
  if (e != hipSuccess) return e;
  if (dm.dtype == CK_BF16)
    return launch_attn_t<bf16, ATT_FUSED, CK_MAX_CLUSTERS>(dm, a, max_total, false, st);
  if (n_clusters <= SELP_SMALL)
    return launch_attn_t<float, ATT_FUSED, SELP_SMALL>(dm, a, max_total, false, st);
  return launch_attn_t<float, ATT_FUSED, CK_MAX_CLUSTERS>(dm, a, max_total, false, st);
}

// ---- library-owned scratch for callers that cannot allocate ----
// The split partials and tickets of one attention call, in device memory that exists
// from the moment the code object is loaded: every GPU the library runs on holds its
// own copy of the array until the process ends.  Host code never passes the array's
// name anywhere; it asks the runtime once per device for the array's address on
// that device and uses that pointer from then on.
static __device__ __align__(256) unsigned char scratch[CK_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[MAX_DEVICES];                // address of `scratch` per device

hipError_t attn_static_scratch(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace ck
