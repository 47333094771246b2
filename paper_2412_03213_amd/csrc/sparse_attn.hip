// Sparse GQA decode attention over the recalled tokens (paper Section II-B:
// softmax(q K_S^T / sqrt(d)) V_S with K_S, V_S the selected rows), alone or fused
// with the cluster selection and index generation of Sections III-C / IV-C.
//
// HBM-bound: every recalled K and V row (256 B in bf16) is read exactly once per
// KV head and shared by the G query heads of the group.  A wavefront takes 16
// tokens per step.  V rows are owned by 16-lane groups (16 B of the row per lane)
// and accumulated on the vector ALUs; in bf16 the K rows go straight into
// v_mfma_f32_16x16x32_bf16 as the A operand with the query heads as B columns,
// which removes the unpacking, the dot products and their cross-lane reductions
// from the vector ALUs (fp32 check mode keeps the all-VALU form).  The attended
// positions of a head-problem are split over several workgroups (split-KV) so that
// a batch of a few sequences still fills 256 CUs, and a small second kernel merges
// the partial (max, sum, accumulator) triples.  Inside a workgroup the token rows
// of its positions are resolved into LDS first, so the K/V loads of the next step
// are always in flight while the current one is reduced.
//
// Fused mode: every workgroup of a head-problem repeats the (cheap, LDS-only)
// selection of the recalled cluster prefix from the precomputed scores and maps
// its own positions through the cluster-contiguous index directly; the index
// list is still written out (each workgroup its own part) but never re-read.
#include <mutex>
#include <type_traits>

#include "decode_common.hpp"

namespace ck {

constexpr int ATT_THREADS = SELP_THREADS;  // 4 wavefronts = 16 token slots per workgroup step
constexpr int ATT_UNROLL = 4;              // token slots in flight per 16-lane group
constexpr int ATT_STEP_TOKENS = 16 * ATT_UNROLL;   // 64 tokens per workgroup iteration
constexpr int ATT_MAX_CHUNK = 4096;        // positions one workgroup may own (rows held in LDS)
constexpr float NEG_BIG = -1.0e30f;        // "no token yet": finite so that differences stay finite
constexpr int ATT_TARGET_WGS = 512;        // 2 per CU on 256 CUs
constexpr int PEX_WAVE = 16 * 8 + 8;             // floats of probability exchange per wavefront (G <= 8)
constexpr int PART_STRIDE = D + 2;         // floats per (split, query head): max, sum, acc[128]

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

struct AttnArgs {
  const void *q, *K, *V;
  void* out;
  float* part;
  // given index list
  const int32_t* token_idx;
  const int32_t* n_tokens;
  // fused selection
  const float* scores;
  const int32_t *sizes, *offsets, *sorted_idx;
  int32_t *sel_clusters, *n_sel_clusters, *n_sel_tokens, *token_idx_out, *n_tokens_out;
  int n_clusters, budget, trim, C_cap;
  // common
  int idx_stride, max_tokens, Hq, Hkv, n_sink, n_recent, chunk, n_split;
  int64_t N_cap, recent_begin;
  float scale_log2e;
};

template <int G>
struct AttnPlainLds {
  int rows[ATT_MAX_CHUNK];
  float red[4 * G * PART_STRIDE];
};

// Attended position p of a head-problem -> token row:
//   [0, n_sink) sinks, then the recalled list, then [recent_begin, recent_end).
template <typename T, int G, bool FUSED>
__global__ __launch_bounds__(ATT_THREADS) void k_attn_partial(const AttnArgs a) {
  using Lds = typename std::conditional<FUSED, SelectLds, AttnPlainLds<G>>::type;
  __shared__ Lds lds;
  __shared__ __attribute__((aligned(16))) float pex[4 * PEX_WAVE];
  int* rows;
  float* red;
  const int split = blockIdx.x, hp = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l16 = tid & 15, slot = tid >> 4;  // 16 slots
  const int s = hp / a.Hkv, h = hp % a.Hkv;
  const T* q = static_cast<const T*>(a.q);

  int n_idx;
  if constexpr (FUSED) {
    SelectLds& L = lds;
    select_prefix(L, a.scores + (int64_t)hp * a.C_cap, a.sizes + (int64_t)hp * a.C_cap,
                  a.offsets + (int64_t)hp * (a.C_cap + 1), a.n_clusters, a.budget, a.trim);
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
    rows = reinterpret_cast<int*>(L.key);               // key + ssz: free after the ranking
    red = reinterpret_cast<float*>(L.ord);              // ord, cum, cbeg, cand: free once the rows are known
  } else {
    rows = lds.rows;
    red = lds.red;
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
        SelectLds& L = lds;
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
  __syncthreads();

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
    bf16x8 qb[4];
#pragma unroll
    for (int sl = 0; sl < 4; ++sl) {
      uint4 w = make_uint4(0, 0, 0, 0);
      if (col < G)
        w = *reinterpret_cast<const uint4*>(q + ((int64_t)s * a.Hq + h * G + col) * D + sl * 32 + kg * 8);
      qb[sl] = __builtin_bit_cast(bf16x8, w);
    }
    float m_run = NEG_BIG, l_run = 0.f;                 // of head `col`, identical in its four lanes
    float* px = pex + wave * PEX_WAVE;                  // [slot][u][g] probabilities, then [g] rescale factors
    const bf16* Khp = static_cast<const bf16*>(a.K) + (int64_t)hp * a.N_cap * D + kg * 8;
    const int tpos = (col >> 2) * 16 + wave * 4 + (col & 3);   // A row `col` = token (u = col/4, slot = col%4)
    uint4 kc[4], kn[4], vc[ATT_UNROLL], vn[ATT_UNROLL];
    auto fetch = [&](int i0, uint4(&kr)[4], uint4(&vr)[ATT_UNROLL]) {
      const int ik = i0 + tpos;
      const bf16* kp = Khp + (int64_t)(ik < n_pos ? rows[ik] : 0) * D;
#pragma unroll
      for (int sl = 0; sl < 4; ++sl) kr[sl] = *reinterpret_cast<const uint4*>(kp + sl * 32);
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        const int i = i0 + u * 16 + slot;
        vr[u] = *reinterpret_cast<const uint4*>(Vhp + (int64_t)(i < n_pos ? rows[i] : 0) * D);
      }
    };
    if (n_pos > 0) fetch(0, kc, vc);
    for (int i0 = 0; i0 < n_pos; i0 += ATT_STEP_TOKENS) {
      if (i0 + ATT_STEP_TOKENS < n_pos) fetch(i0 + ATT_STEP_TOKENS, kn, vn);
      floatx4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int sl = 0; sl < 4; ++sl)
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kc[sl]), qb[sl], d, 0, 0, 0);
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
        vv[0] = lo_bf16(vc[u].x); vv[1] = hi_bf16(vc[u].x); vv[2] = lo_bf16(vc[u].y); vv[3] = hi_bf16(vc[u].y);
        vv[4] = lo_bf16(vc[u].z); vv[5] = hi_bf16(vc[u].z); vv[6] = lo_bf16(vc[u].w); vv[7] = hi_bf16(vc[u].w);
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int j = 0; j < 8; ++j) acc[g][j] = fmaf(pr[u][g], vv[j], acc[g][j]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        kc[u] = kn[u];
        vc[u] = vn[u];
      }
    }
    // ---- combine the 4 slots of a wavefront: they share the running max ----
    if constexpr (FUSED) __syncthreads();   // red aliases arrays the row resolution read
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
    if constexpr (FUSED) __syncthreads();   // red aliases arrays the row resolution read
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
      float* pr = a.part + (((int64_t)hp * a.n_split + split) * G + g) * PART_STRIDE;
      if (c2 == 0) {
        pr[0] = mx;
        pr[1] = ls;
      }
      pr[2 + c2] = a0;
      pr[3 + c2] = a1;
    }
  }
}

// out[hq] = sum_i acc_i 2^(m_i - M) / sum_i l_i 2^(m_i - M); the partials of up to
// MERGE_BATCH splits are loaded together so that their latencies overlap.
constexpr int MERGE_BATCH = 16;
template <typename T>
__global__ __launch_bounds__(D) void k_attn_merge(const float* __restrict__ part, int n_split,
                                                  int G, int Hq, int Hkv, T* __restrict__ out) {
  const int hq_lin = blockIdx.x;                        // s * Hq + hq
  const int s = hq_lin / Hq, hq = hq_lin % Hq;
  const int hp = s * Hkv + hq / G, g = hq % G, t = threadIdx.x;
  const float* base = part + (((int64_t)hp * n_split) * G + g) * PART_STRIDE;
  const int64_t stride = (int64_t)G * PART_STRIDE;
  float M = NEG_BIG, ls = 0.f, acc = 0.f;
  for (int i0 = 0; i0 < n_split; i0 += MERGE_BATCH) {
    float mi[MERGE_BATCH], li[MERGE_BATCH], ai[MERGE_BATCH];
#pragma unroll
    for (int i = 0; i < MERGE_BATCH; ++i) {
      const bool ok = i0 + i < n_split;
      const float* p = base + (int64_t)(ok ? i0 + i : 0) * stride;
      mi[i] = ok ? p[0] : NEG_BIG;
      li[i] = ok ? p[1] : 0.f;
      ai[i] = ok ? p[2 + t] : 0.f;
    }
    float mx = M;
#pragma unroll
    for (int i = 0; i < MERGE_BATCH; ++i) mx = fmaxf(mx, mi[i]);
    const float corr = __builtin_amdgcn_exp2f(M - mx);
    ls *= corr;
    acc *= corr;
    M = mx;
#pragma unroll
    for (int i = 0; i < MERGE_BATCH; ++i) {
      const float f = __builtin_amdgcn_exp2f(mi[i] - mx);
      ls += li[i] * f;
      acc += ai[i] * f;
    }
  }
  store_out(out + (int64_t)hq_lin * D + t, ls > 0.f ? acc / ls : 0.f);
}

int attn_num_splits(const Dims& dm, int64_t max_total) {
  // aim for two workgroups per CU (measured best: longer token runs per workgroup keep
  // the prefetch pipeline full and the merge small), but keep at least one full step
  // of tokens per workgroup and never more positions than its LDS row table holds
  const int64_t by_work = (max_total + ATT_STEP_TOKENS - 1) / ATT_STEP_TOKENS;
  const int64_t by_fill = (ATT_TARGET_WGS + dm.HP - 1) / dm.HP;
  int64_t n = by_work < by_fill ? by_work : by_fill;
  if (n > 64) n = 64;
  const int64_t need = (max_total + ATT_MAX_CHUNK - 1) / ATT_MAX_CHUNK;
  if (n < need) n = need;
  if (n < 1) n = 1;
  return (int)n;
}

size_t attn_workspace_bytes(const Dims& dm, int64_t max_total) {
  const int n_split = attn_num_splits(dm, max_total);
  size_t b = (size_t)dm.HP * n_split * dm.G * PART_STRIDE * sizeof(float);
  return (b + 255) & ~(size_t)255;
}

template <typename T, bool FUSED>
static hipError_t launch_attn_t(const Dims& dm, AttnArgs a, int64_t max_total, hipStream_t st) {
  const int n_split = attn_num_splits(dm, max_total);
  int chunk = (int)((max_total + n_split - 1) / n_split);
  chunk = (chunk + ATT_STEP_TOKENS - 1) / ATT_STEP_TOKENS * ATT_STEP_TOKENS;
  if (chunk < ATT_STEP_TOKENS) chunk = ATT_STEP_TOKENS;
  if (chunk > ATT_MAX_CHUNK) return hipErrorInvalidValue;
  a.chunk = chunk;
  a.n_split = n_split;
  const dim3 grid(n_split, dm.HP), block(ATT_THREADS);
  switch (dm.G) {
    case 1: hipLaunchKernelGGL((k_attn_partial<T, 1, FUSED>), grid, block, 0, st, a); break;
    case 2: hipLaunchKernelGGL((k_attn_partial<T, 2, FUSED>), grid, block, 0, st, a); break;
    case 4: hipLaunchKernelGGL((k_attn_partial<T, 4, FUSED>), grid, block, 0, st, a); break;
    case 8: hipLaunchKernelGGL((k_attn_partial<T, 8, FUSED>), grid, block, 0, st, a); break;
    default: return hipErrorInvalidValue;
  }
  if (n_split > 1)
    hipLaunchKernelGGL(k_attn_merge<T>, dim3(dm.S * dm.Hq), dim3(D), 0, st, a.part, n_split, dm.G,
                       dm.Hq, dm.Hkv, (T*)a.out);
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
                              hipStream_t st) {
  const int n_recent = (int)(recent_end > recent_begin ? recent_end - recent_begin : 0);
  AttnArgs a = common_args(dm, q, K, V, idx_stride, (int)(max_total - n_sink - n_recent), n_sink,
                           recent_begin, recent_end, softmax_scale, out, workspace);
  a.token_idx = token_idx;
  a.n_tokens = n_tokens;
  if (dm.dtype == CK_BF16) return launch_attn_t<bf16, false>(dm, a, max_total, st);
  return launch_attn_t<float, false>(dm, a, max_total, st);
}

// ---- library-owned scratch for callers that cannot allocate ----
// The split partials of one attention call, in device memory that exists from the
// moment the code object is loaded: every GPU the library runs on holds its own
// copy of the array until the process ends.  Host code never passes the array's
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

hipError_t launch_decode_fused(const Dims& dm, const void* q, const void* K, const void* V,
                               const void* centroids, const int32_t* sizes,
                               const int32_t* offsets, const int32_t* sorted_idx, int n_clusters,
                               int budget, uint32_t flags, int64_t n_sink, int64_t recent_begin,
                               int64_t recent_end, float softmax_scale, float* scores,
                               int32_t* sel_clusters, int32_t* n_sel_clusters,
                               int32_t* n_sel_tokens, int32_t* token_idx, int idx_stride,
                               int32_t* n_tokens, void* out, void* workspace, hipStream_t st) {
  hipError_t e = launch_score(dm, q, centroids, n_clusters, scores, st);
  if (e != hipSuccess) return e;
  AttnArgs a = common_args(dm, q, K, V, idx_stride, budget, n_sink, recent_begin, recent_end,
                           softmax_scale, out, workspace);
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
  if (dm.dtype == CK_BF16) return launch_attn_t<bf16, true>(dm, a, max_total, st);
  return launch_attn_t<float, true>(dm, a, max_total, st);
}

}  // namespace ck
