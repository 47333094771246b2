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
// All built on DPP and the gfx950 lane-swap instructions (a few cycles each) instead
// of ds_bpermute round trips through the LDS crossbar.  The butterflies combine the
// same two partial results in every lane, so all lanes end with bit-identical values.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i0(int v) {      // lanes without a source read 0
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
constexpr int DPP_XOR1 = 0xB1;          // quad_perm:[1,0,3,2]
constexpr int DPP_XOR2 = 0x4E;          // quad_perm:[2,3,0,1]
constexpr int DPP_HALF_MIRROR = 0x141;  // lane i <-> 7 - i inside each 8
constexpr int DPP_MIRROR = 0x140;       // lane i <-> 15 - i inside each row of 16

struct OpSum { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };
struct OpMin { __device__ __forceinline__ float operator()(float a, float b) const { return fminf(a, b); } };

// v[i] (op) v[i ^ 16] and v[i] (op) v[i ^ 32]: v_permlane16_swap / v_permlane32_swap
// applied to two copies of v leave "my half" in one result and "the other half" in the other.
template <typename Op>
__device__ __forceinline__ float xor16(float v, Op op) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return op(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
template <typename Op>
__device__ __forceinline__ float xor32(float v, Op op) {
  const unsigned u = __float_as_uint(v);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return op(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// over the 16 lanes of a DPP row; every lane of the row gets the result
template <typename Op>
__device__ __forceinline__ float row16_reduce(float v, Op op) {
  v = op(v, dpp_f<DPP_XOR1>(v));
  v = op(v, dpp_f<DPP_XOR2>(v));
  v = op(v, dpp_f<DPP_HALF_MIRROR>(v));
  v = op(v, dpp_f<DPP_MIRROR>(v));
  return v;
}
template <typename Op>
__device__ __forceinline__ float wave_reduce(float v, Op op) {
  v = row16_reduce(v, op);
  v = xor16(v, op);
  return xor32(v, op);
}
__device__ __forceinline__ float row16_sum(float v) { return row16_reduce(v, OpSum()); }
__device__ __forceinline__ float wave_sum(float v) { return wave_reduce(v, OpSum()); }
__device__ __forceinline__ float wave_max(float v) { return wave_reduce(v, OpMax()); }
__device__ __forceinline__ float wave_min(float v) { return wave_reduce(v, OpMin()); }

// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  v += dpp_i0<0x111>(v);   // row_shr:1
  v += dpp_i0<0x112>(v);   // row_shr:2
  v += dpp_i0<0x114>(v);   // row_shr:4
  v += dpp_i0<0x118>(v);   // row_shr:8
  const int t0 = __builtin_amdgcn_readlane(v, 15);
  const int t1 = __builtin_amdgcn_readlane(v, 31);
  const int t2 = __builtin_amdgcn_readlane(v, 47);
  const int row = (threadIdx.x & 63) >> 4;
  return v + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}

// Inclusive prefix sum over blockDim.x * ITEMS ints held ITEMS per thread in
// consecutive order; `tmp` is LDS of at least blockDim.x / 64 + 1 ints.
// Returns the grand total to every thread.
template <int ITEMS>
__device__ __forceinline__ int block_inclusive_scan(int (&v)[ITEMS], int* tmp) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
#pragma unroll
  for (int i = 1; i < ITEMS; ++i) v[i] += v[i - 1];
  const int run = wave_inclusive_scan(v[ITEMS - 1]);
  __syncthreads();  // tmp may still be in use by a previous call
  if (lane == WAVE - 1) tmp[wave] = run;
  __syncthreads();
  int wave_base = 0, total = 0;
  for (int w = 0; w < nwaves; ++w) {
    const int t = tmp[w];
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


constexpr int KM_SMALL_MAX_TOKENS = 384;    // token ranges up to this size (and up to
constexpr int KM_SMALL_MAX_CLUSTERS = 8;    // this many clusters) are clustered by one kernel
constexpr int KM_MAX_ITER_CONVERGE = 256;   // iteration cap of the run-until-convergence mode

struct ClusterWorkspace {
  bf16* mu_hat;         // [HP, c_count, D] table the assignment reads (unit-length or raw means)
  int32_t* chunk_hist;  // [HP, n_chunks, c_count] per-chunk histogram / base positions
  float* bias;          // [HP, bias_stride] -|mu_c|^2 / 2 of the table rows (l2 metric)
  int bias_stride;      // c_count rounded up to whole 32-row tiles
  int32_t* changed;     // [KM_MAX_ITER_CONVERGE + 1, HP] labels changed per iteration
  size_t bytes;
};

// What an assignment launch needs beyond the contraction itself.
struct KmCtl {
  const float* bias = nullptr;     // l2 metric: added to <k, mu_c> before the argmax
  int bias_stride = 0;
  const int32_t* skip = nullptr;   // [HP] changed-label counts of the previous iteration:
                                   // 0 = that head-problem has converged, leave it alone
  int32_t* changed = nullptr;      // [HP] receives the number of labels this launch changed
  int first = 0;                   // no previous labels exist: count every token as changed
};
ClusterWorkspace carve_cluster_workspace(const Dims& dm, int64_t tok_count, int c_count,
                                         void* base);

// metric: CK_METRIC_* of the table the assignment will read
hipError_t launch_init_centroids(const Dims& dm, const bf16* K, const int32_t* init_idx,
                                 int c_begin, int c_count, bf16* centroids, bf16* mu_hat,
                                 int metric, float* bias, int bias_stride, hipStream_t st);
hipError_t launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st);
bool kmeans_small_fits(int64_t tok_count, int c_count);
hipError_t launch_kmeans_small(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                               int c_begin, int c_count, int max_iter, int metric, bool converge,
                               const int32_t* init_idx, bf16* centroids, int32_t* labels,
                               int32_t* sizes, int32_t* offsets, int32_t* sorted_idx,
                               int32_t* iters_done, hipStream_t st);
hipError_t launch_iters_done(const int32_t* changed, int max_iter, int HP, int32_t* iters_done,
                             hipStream_t st);
int assign_tile_tokens(const Dims& dm, int64_t tok_count);
// chunk_hist (nullable): [HP, n_chunks, c_count] label histogram per workgroup tile
hipError_t launch_assign(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                         const bf16* mu_hat, int c_begin, int c_count, int32_t* labels,
                         float* best_sim, int32_t* chunk_hist, const KmCtl& ctl, hipStream_t st);
// streaming form for small tables (whole table in LDS); chunk size 512 tokens as above
bool assign_stream_fits(int c_count);
hipError_t launch_assign_stream(const Dims& dm, const bf16* K, int64_t tok_begin,
                                int64_t tok_count, const bf16* mu_hat, int c_begin, int c_count,
                                int32_t* labels, float* best_sim, int32_t* chunk_hist,
                                const KmCtl& ctl, int n_cu, hipStream_t st);
// have_hist: chunk_hist already holds the histograms (written by launch_assign)
hipError_t launch_metadata(const Dims& dm, const int32_t* labels, int64_t tok_begin,
                           int64_t tok_count, int c_begin, int c_count, int32_t* sizes,
                           int32_t* offsets, int32_t* sorted_idx, int32_t* chunk_hist,
                           bool have_hist, const int32_t* gate, hipStream_t st);
// gate (nullable, [HP]): head-problems whose entry is 0 are left untouched
hipError_t launch_update(const Dims& dm, const bf16* K, const int32_t* offsets,
                         const int32_t* sorted_idx, int c_begin, int c_count, bf16* centroids,
                         bf16* mu_hat, float* centroids_f32, int metric, float* bias,
                         int bias_stride, const int32_t* gate, hipStream_t st);
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
hipError_t launch_probe_mfma(int n_workgroups, int iters, const void* operands,
                             unsigned long long* clocks, float* sink, hipStream_t st);
// cluster cache
struct CacheArgs {
  const void *K_home, *V_home;                          // [HP, N_cap, D]
  const void *K_old, *V_old;                            // [HP, cap, D] rows of the previous step
  void *K_new, *V_new;
  const int32_t *old_clusters, *old_starts, *old_n;     // [HP, C_cap], [HP, C_cap + 1], [HP]
  int32_t *new_clusters, *new_starts, *new_n;
  const int32_t *sel_clusters, *n_sel_clusters;         // this step's selection (score order)
  const int32_t *sizes, *offsets, *sorted_idx;
  int32_t* miss_tokens;                                 // [HP] rows fetched from the home copy
  int64_t N_cap;
  int C_cap, cap, row_bytes;
};
hipError_t launch_cache_fill(const Dims& dm, const CacheArgs& a, int budget, hipStream_t st);
// evaluation helpers
hipError_t launch_row_scores(const Dims& dm, const void* q, const void* table,
                             int64_t table_stride, int64_t row_begin, int n_rows, float* scores,
                             int64_t score_stride, hipStream_t st);
hipError_t launch_topk(int HP, const float* scores, int64_t row_stride, int64_t begin, int n,
                       int k, int32_t* out_idx, int out_stride, int32_t* n_out, hipStream_t st);
hipError_t launch_recall_hits(int HP, const int32_t* token_idx, const int32_t* n_tokens,
                              int idx_stride, const int32_t* ref_idx, const int32_t* n_ref,
                              int ref_stride, int32_t* hits, hipStream_t st);
hipError_t launch_page_keys(const Dims& dm, const void* K, int64_t tok_begin, int64_t tok_count,
                            int page_size, void* page_keys, int64_t page_stride, hipStream_t st);
hipError_t launch_expand_pages(int HP, const int32_t* page_idx, const int32_t* n_pages_sel,
                               int page_stride, int page_size, int64_t tok_begin,
                               int64_t tok_count, int32_t* token_idx, int idx_stride,
                               int32_t* n_tokens, hipStream_t st);
size_t objective_workspace_bytes(const Dims& dm, int64_t tok_count);
hipError_t launch_objective(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                            const bf16* table, int c_begin, int c_count, const int32_t* labels,
                            double* J, double* Dsum, void* workspace, hipStream_t st);
int attn_num_splits(const Dims& dm, int64_t max_total);
size_t attn_workspace_bytes(const Dims& dm, int64_t max_total);
// address, on the current device, of the library-owned scratch array
// (CK_STATIC_SCRATCH_BYTES bytes); looked up once per device
hipError_t attn_static_scratch(void** ptr);
hipError_t launch_sparse_attn(const Dims& dm, const void* q, const void* K, const void* V,
                              const int32_t* token_idx, const int32_t* n_tokens, int idx_stride,
                              int64_t max_total, int64_t n_sink, int64_t recent_begin,
                              int64_t recent_end, float softmax_scale, void* out, void* workspace,
                              bool two_pass, hipStream_t st);

}  // namespace ck
