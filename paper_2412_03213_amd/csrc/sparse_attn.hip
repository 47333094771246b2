// Sparse GQA decode attention over the recalled tokens (paper Section II-B:
// softmax(q K_S^T / sqrt(d)) V_S with K_S, V_S the selected rows).
//
// HBM-bound: every recalled K and V row (256 B in bf16) is read exactly once per
// KV head and shared by the G query heads of the group.  A 16-lane group owns one
// token at a time (16 B of the row per lane, so a wavefront load instruction
// covers four whole rows = eight 128-byte lines); the token list of a
// head-problem is split over several workgroups (split-KV) so that a batch of a
// few sequences still fills 256 CUs, and a small second kernel merges the
// partial (max, sum, accumulator) triples.
#include "ck_common.hpp"

namespace ck {

constexpr int ATT_THREADS = 256;           // 4 wavefronts = 16 token slots per workgroup step
constexpr int ATT_UNROLL = 4;              // steps in flight per wavefront
constexpr int ATT_STEP_TOKENS = 16 * ATT_UNROLL;   // 64 tokens per workgroup iteration
constexpr float NEG_BIG = -1.0e30f;        // "no token yet": finite so that differences stay finite
constexpr int PART_STRIDE = D + 2;         // floats per (split, query head): max, sum, acc[128]

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
__device__ __forceinline__ void store_out(bf16* p, float v) {
  *reinterpret_cast<uint16_t*>(p) = float_to_bf16_bits(v);
}
__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }

// Attended position p of a head-problem -> token row:
//   [0, n_sink) sinks, then the recalled list, then [recent_begin, recent_end).
template <typename T, int G>
__global__ __launch_bounds__(ATT_THREADS) void k_attn_partial(
    const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V,
    const int32_t* __restrict__ token_idx, const int32_t* __restrict__ n_tokens, int idx_stride,
    int max_tokens, int Hq, int Hkv, int64_t N_cap, int n_sink, int64_t recent_begin,
    int n_recent, float scale_log2e, int chunk, int n_split, float* __restrict__ part,
    T* __restrict__ out) {
  __shared__ float red[4][G][PART_STRIDE];
  const int split = blockIdx.x, hp = blockIdx.y, tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6, l16 = tid & 15, slot = tid >> 4;  // 16 slots
  const int s = hp / Hkv, h = hp % Hkv;

  int n_idx = n_tokens ? n_tokens[hp] : 0;
  n_idx = n_idx < 0 ? 0 : (n_idx > max_tokens ? max_tokens : n_idx);
  const int n_total = n_sink + n_idx + n_recent;
  const int p_begin = split * chunk;
  int p_end = p_begin + chunk;
  if (p_end > n_total) p_end = n_total;

  // this lane's 8 channels of every query head of the group, pre-scaled
  float qv[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    load_row8<T>(q + ((int64_t)s * Hq + h * G + g) * D + l16 * 8, qv[g]);
#pragma unroll
    for (int j = 0; j < 8; ++j) qv[g][j] *= scale_log2e;
  }
  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = NEG_BIG;
    l[g] = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[g][j] = 0.f;
  }

  const T* Khp = K + (int64_t)hp * N_cap * D + l16 * 8;
  const T* Vhp = V + (int64_t)hp * N_cap * D + l16 * 8;
  const int32_t* idx = token_idx ? token_idx + (int64_t)hp * idx_stride : nullptr;

  for (int p0 = p_begin; p0 < p_end; p0 += ATT_STEP_TOKENS) {
    float kv[ATT_UNROLL][8], vv[ATT_UNROLL][8];
    bool ok[ATT_UNROLL];
#pragma unroll
    for (int u = 0; u < ATT_UNROLL; ++u) {
      const int p = p0 + u * 16 + slot;
      ok[u] = p < p_end;
      int64_t row = 0;
      if (ok[u]) {
        if (p < n_sink) row = p;
        else if (p < n_sink + n_idx) row = idx[p - n_sink];
        else row = recent_begin + (p - n_sink - n_idx);
        row = row < 0 ? 0 : (row >= N_cap ? N_cap - 1 : row);
      }
      load_row8<T>(Khp + row * D, kv[u]);
      load_row8<T>(Vhp + row * D, vv[u]);
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float sc[ATT_UNROLL];
      float mx = m[g];
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        float d = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) d = fmaf(qv[g][j], kv[u][j], d);
        d = row16_sum(d);
        sc[u] = ok[u] ? d : -INFINITY;
        mx = fmaxf(mx, sc[u]);
      }
      const float corr = __builtin_amdgcn_exp2f(m[g] - mx);
      m[g] = mx;
      float ls = l[g] * corr;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[g][j] *= corr;
#pragma unroll
      for (int u = 0; u < ATT_UNROLL; ++u) {
        const float pw = __builtin_amdgcn_exp2f(sc[u] - mx);
        ls += pw;
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[g][j] = fmaf(pw, vv[u][j], acc[g][j]);
      }
      l[g] = ls;
    }
  }

  // ---- combine the 4 slots of a wavefront (lanes l16 + 16*k) ----
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float mx = fmaxf(m[g], __shfl_xor(m[g], 16, WAVE));
    mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
    const float w = __builtin_amdgcn_exp2f(m[g] - mx);
    float ls = l[g] * w;
    ls += __shfl_xor(ls, 16, WAVE);
    ls += __shfl_xor(ls, 32, WAVE);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float a = acc[g][j] * w;
      a += __shfl_xor(a, 16, WAVE);
      a += __shfl_xor(a, 32, WAVE);
      acc[g][j] = a;
    }
    if (lane < 16) {
      red[wave][g][0] = mx;
      red[wave][g][1] = ls;
#pragma unroll
      for (int j = 0; j < 8; ++j) red[wave][g][2 + l16 * 8 + j] = acc[g][j];
    }
  }
  __syncthreads();
  // ---- combine the 4 wavefronts: thread = (query head g, channel pair) ----
  for (int e = tid; e < G * (D / 2); e += ATT_THREADS) {
    const int g = e / (D / 2), c2 = (e % (D / 2)) * 2;
    float mx = fmaxf(fmaxf(red[0][g][0], red[1][g][0]), fmaxf(red[2][g][0], red[3][g][0]));
    float ls = 0.f, a0 = 0.f, a1 = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float f = __builtin_amdgcn_exp2f(red[w][g][0] - mx);
      ls += red[w][g][1] * f;
      a0 += red[w][g][2 + c2] * f;
      a1 += red[w][g][3 + c2] * f;
    }
    if (n_split == 1) {
      const float inv = ls > 0.f ? 1.0f / ls : 0.f;
      T* o = out + ((int64_t)s * Hq + h * G + g) * D + c2;
      store_out(o, a0 * inv);
      store_out(o + 1, a1 * inv);
    } else {
      float* pr = part + (((int64_t)hp * n_split + split) * G + g) * PART_STRIDE;
      if (c2 == 0) {
        pr[0] = mx;
        pr[1] = ls;
      }
      pr[2 + c2] = a0;
      pr[3 + c2] = a1;
    }
  }
}

// out[hq] = sum_i acc_i 2^(m_i - M) / sum_i l_i 2^(m_i - M)
template <typename T>
__global__ __launch_bounds__(D) void k_attn_merge(const float* __restrict__ part, int n_split,
                                                  int G, int Hq, int Hkv, T* __restrict__ out) {
  const int hq_lin = blockIdx.x;                        // s * Hq + hq
  const int s = hq_lin / Hq, hq = hq_lin % Hq;
  const int hp = s * Hkv + hq / G, g = hq % G, t = threadIdx.x;
  const float* base = part + (((int64_t)hp * n_split) * G + g) * PART_STRIDE;
  const int64_t stride = (int64_t)G * PART_STRIDE;
  float mx = NEG_BIG;
  for (int i = 0; i < n_split; ++i) mx = fmaxf(mx, base[i * stride]);
  float ls = 0.f, a = 0.f;
  for (int i = 0; i < n_split; ++i) {
    const float f = __builtin_amdgcn_exp2f(base[i * stride] - mx);
    ls += base[i * stride + 1] * f;
    a += base[i * stride + 2 + t] * f;
  }
  store_out(out + (int64_t)hq_lin * D + t, ls > 0.f ? a / ls : 0.f);
}

int attn_num_splits(const Dims& dm, int64_t max_total) {
  // aim for ~4 workgroups per CU, but keep at least one full step of tokens per workgroup
  int64_t by_work = (max_total + ATT_STEP_TOKENS - 1) / ATT_STEP_TOKENS;
  int64_t by_fill = (1024 + dm.HP - 1) / dm.HP;
  int64_t n = by_work < by_fill ? by_work : by_fill;
  if (n < 1) n = 1;
  if (n > 64) n = 64;
  return (int)n;
}

size_t attn_workspace_bytes(const Dims& dm, int64_t max_total) {
  const int n_split = attn_num_splits(dm, max_total);
  size_t b = (size_t)dm.HP * n_split * dm.G * PART_STRIDE * sizeof(float);
  return (b + 255) & ~(size_t)255;
}

template <typename T, int G>
static void launch_partial(const Dims& dm, const void* q, const void* K, const void* V,
                           const int32_t* token_idx, const int32_t* n_tokens, int idx_stride,
                           int max_tokens, int n_sink, int64_t recent_begin, int n_recent,
                           float scale_log2e, int chunk, int n_split, float* part, void* out,
                           hipStream_t st) {
  hipLaunchKernelGGL((k_attn_partial<T, G>), dim3(n_split, dm.HP), dim3(ATT_THREADS), 0, st,
                     (const T*)q, (const T*)K, (const T*)V, token_idx, n_tokens, idx_stride,
                     max_tokens, dm.Hq, dm.Hkv, dm.N_cap, n_sink, recent_begin, n_recent,
                     scale_log2e, chunk, n_split, part, (T*)out);
}

template <typename T>
static hipError_t launch_attn_t(const Dims& dm, const void* q, const void* K, const void* V,
                                const int32_t* token_idx, const int32_t* n_tokens, int idx_stride,
                                int64_t max_total, int64_t n_sink, int64_t recent_begin,
                                int64_t recent_end, float softmax_scale, void* out,
                                void* workspace, hipStream_t st) {
  const int n_recent = (int)(recent_end > recent_begin ? recent_end - recent_begin : 0);
  const int max_tokens = (int)(max_total - n_sink - n_recent);
  const int n_split = attn_num_splits(dm, max_total);
  int chunk = (int)((max_total + n_split - 1) / n_split);
  chunk = (chunk + 15) & ~15;
  if (chunk < 16) chunk = 16;
  const float scale_log2e = softmax_scale * 1.4426950408889634f;
  float* part = reinterpret_cast<float*>(workspace);
#define CK_ATT(GG)                                                                              \
  launch_partial<T, GG>(dm, q, K, V, token_idx, n_tokens, idx_stride, max_tokens, (int)n_sink, \
                        recent_begin, n_recent, scale_log2e, chunk, n_split, part, out, st)
  switch (dm.G) {
    case 1: CK_ATT(1); break;
    case 2: CK_ATT(2); break;
    case 4: CK_ATT(4); break;
    case 8: CK_ATT(8); break;
    default: return hipErrorInvalidValue;
  }
#undef CK_ATT
  if (n_split > 1)
    hipLaunchKernelGGL(k_attn_merge<T>, dim3(dm.S * dm.Hq), dim3(D), 0, st, part, n_split, dm.G,
                       dm.Hq, dm.Hkv, (T*)out);
  return hipGetLastError();
}

hipError_t launch_sparse_attn(const Dims& dm, const void* q, const void* K, const void* V,
                              const int32_t* token_idx, const int32_t* n_tokens, int idx_stride,
                              int64_t max_total, int64_t n_sink, int64_t recent_begin,
                              int64_t recent_end, float softmax_scale, void* out, void* workspace,
                              hipStream_t st) {
  if (dm.dtype == CK_BF16)
    return launch_attn_t<bf16>(dm, q, K, V, token_idx, n_tokens, idx_stride, max_total, n_sink,
                               recent_begin, recent_end, softmax_scale, out, workspace, st);
  return launch_attn_t<float>(dm, q, K, V, token_idx, n_tokens, idx_stride, max_total, n_sink,
                              recent_begin, recent_end, softmax_scale, out, workspace, st);
}

}  // namespace ck
