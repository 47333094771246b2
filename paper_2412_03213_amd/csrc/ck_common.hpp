// Shared device helpers and internal launcher declarations of the ClusterKV library.
// gfx950 (CDNA4) only: 64-wide wavefronts, 160 KB LDS per CU, bf16 MFMA.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "clusterkv.h"

namespace ck {

constexpr int D = 128;           // head dimension every kernel is written for
constexpr int WAVE = 64;

typedef __bf16 bf16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

// ---- bf16 <-> fp32 (round to nearest even; inputs are finite) ----
__device__ __forceinline__ float bf16_bits_to_float(uint32_t hi16) {
  return __builtin_bit_cast(float, hi16 << 16);
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// the two bf16 halves of a 32-bit word (element 2j in the low half)
__device__ __forceinline__ float lo_bf16(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t w) {
  return __builtin_bit_cast(float, w & 0xFFFF0000u);
}

// ---- cross-lane helpers ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, WAVE));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fminf(v, __shfl_xor(v, m, WAVE));
  return v;
}
// sum over the 16 lanes of a DPP row; every lane of the row gets the total
template <int CTRL>
__device__ __forceinline__ float dpp_row_ror(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_row_ror<0x128>(v);  // row_ror:8
  v += dpp_row_ror<0x124>(v);  // row_ror:4
  v += dpp_row_ror<0x122>(v);  // row_ror:2
  v += dpp_row_ror<0x121>(v);  // row_ror:1
  return v;
}

// Inclusive prefix sum over blockDim.x * ITEMS ints held ITEMS per thread in
// consecutive order; `tmp` is LDS of at least blockDim.x / 64 + 1 ints.
// Returns the grand total to every thread.
template <int ITEMS>
__device__ __forceinline__ int block_inclusive_scan(int (&v)[ITEMS], int* tmp) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
#pragma unroll
  for (int i = 1; i < ITEMS; ++i) v[i] += v[i - 1];
  int run = v[ITEMS - 1];
#pragma unroll
  for (int o = 1; o < WAVE; o <<= 1) {
    int t = __shfl_up(run, o, WAVE);
    if (lane >= o) run += t;
  }
  __syncthreads();  // tmp may still be in use by a previous call
  if (lane == WAVE - 1) tmp[wave] = run;
  __syncthreads();
  int wave_base = 0, total = 0;
  for (int w = 0; w < nwaves; ++w) {
    int t = tmp[w];
    if (w < wave) wave_base += t;
    total += t;
  }
  const int excl = wave_base + run - v[ITEMS - 1];
#pragma unroll
  for (int i = 0; i < ITEMS; ++i) v[i] += excl;
  return total;
}

// ---- internal launchers (host side, defined next to their kernels) ----
struct Dims {
  int S, Hq, Hkv, G, HP;   // HP = S * Hkv head-problems
  int64_t N_cap;
  int C_cap;
  int dtype;
};


struct ClusterWorkspace {
  bf16* mu_hat;       // [HP, c_count, D] unit-length centroids the assignment reads
  int32_t* chunk_hist;  // [HP, n_chunks, c_count] per-chunk histogram / base positions
  size_t bytes;
};
ClusterWorkspace carve_cluster_workspace(const Dims& dm, int64_t tok_count, int c_count,
                                         void* base);

hipError_t launch_init_centroids(const Dims& dm, const bf16* K, const int32_t* init_idx,
                                 int c_begin, int c_count, bf16* centroids, bf16* mu_hat,
                                 hipStream_t st);
int assign_tile_tokens(const Dims& dm, int64_t tok_count);
// chunk_hist (nullable): [HP, n_chunks, c_count] label histogram per workgroup tile
hipError_t launch_assign(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                         const bf16* mu_hat, int c_begin, int c_count, int32_t* labels,
                         float* best_sim, int32_t* chunk_hist, hipStream_t st);
// have_hist: chunk_hist already holds the histograms (written by launch_assign)
hipError_t launch_metadata(const Dims& dm, const int32_t* labels, int64_t tok_begin,
                           int64_t tok_count, int c_begin, int c_count, int32_t* sizes,
                           int32_t* offsets, int32_t* sorted_idx, int32_t* chunk_hist,
                           bool have_hist, hipStream_t st);
hipError_t launch_update(const Dims& dm, const bf16* K, const int32_t* offsets,
                         const int32_t* sorted_idx, int c_begin, int c_count, bf16* centroids,
                         bf16* mu_hat, float* centroids_f32, hipStream_t st);
hipError_t launch_select(const Dims& dm, const void* q, const void* centroids,
                         const int32_t* sizes, int n_clusters, int budget, uint32_t flags,
                         int32_t* sel_clusters, int32_t* n_sel_clusters, int32_t* n_sel_tokens,
                         float* scores, hipStream_t st);
hipError_t launch_score(const Dims& dm, const void* q, const void* centroids, int n_clusters,
                        float* scores, hipStream_t st);
hipError_t launch_decode_fused(const Dims& dm, const void* q, const void* K, const void* V,
                               const void* centroids, const int32_t* sizes,
                               const int32_t* offsets, const int32_t* sorted_idx, int n_clusters,
                               int budget, uint32_t flags, int64_t n_sink, int64_t recent_begin,
                               int64_t recent_end, float softmax_scale, float* scores,
                               int32_t* sel_clusters, int32_t* n_sel_clusters,
                               int32_t* n_sel_tokens, int32_t* token_idx, int idx_stride,
                               int32_t* n_tokens, void* out, void* workspace, hipStream_t st);
hipError_t launch_gather(const Dims& dm, const int32_t* sel_clusters,
                         const int32_t* n_sel_clusters, const int32_t* offsets,
                         const int32_t* sorted_idx, int budget, uint32_t flags,
                         int32_t* token_idx, int idx_stride, int32_t* n_tokens, hipStream_t st);
hipError_t launch_probe_mfma(int n_workgroups, int iters, float* sink, hipStream_t st);
int attn_num_splits(const Dims& dm, int64_t max_total);
size_t attn_workspace_bytes(const Dims& dm, int64_t max_total);
hipError_t launch_sparse_attn(const Dims& dm, const void* q, const void* K, const void* V,
                              const int32_t* token_idx, const int32_t* n_tokens, int idx_stride,
                              int64_t max_total, int64_t n_sink, int64_t recent_begin,
                              int64_t recent_end, float softmax_scale, void* out, void* workspace,
                              hipStream_t st);

}  // namespace ck
