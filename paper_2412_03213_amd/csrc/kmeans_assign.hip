// K-means assignment step (paper Section III-B): every key gets the label of the
// centroid with the largest cosine similarity.  Since the key's own length does
// not change the argmax, this is argmax_c <k_i, mu_hat_c> with unit-length
// centroids: a dense [tokens x d] . [d x C] contraction, run on bf16 MFMA with
// the argmax folded into the accumulator read-out, so the similarity matrix
// never exists in memory.
//
// Mapping (gfx950, v_mfma_f32_32x32x16_bf16): the CENTROIDS are the A operand
// (rows of the 32x32 result) and the KEYS the B operand (columns).  A lane then
// owns one key column and 16 centroid rows of every tile, so the running
// (max, argmax) lives in plain registers and only one exchange between lanes
// l and l+32 is needed at the very end.  Keys stay in registers for the whole
// kernel (NKB blocks of 32 keys per wavefront); centroid tiles stream through
// LDS in double-buffered chunks of 64 rows shared by the four wavefronts.
#include "ck_common.hpp"

namespace ck {

constexpr int CHUNK_ROWS = 64;             // centroid rows per LDS chunk (two MFMA tiles)
constexpr int LDS_ROW = D + 8;             // bf16 elements per LDS row: 272 B, rows shift 4 banks
constexpr int ASSIGN_THREADS = 256;

template <int NKB>
__global__ __launch_bounds__(ASSIGN_THREADS) void k_assign(
    const bf16* __restrict__ K, const bf16* __restrict__ mu_hat, int32_t* __restrict__ labels,
    float* __restrict__ best_sim, int64_t N_cap, int64_t tok_begin, int64_t tok_count,
    int c_begin, int c_count) {
  __shared__ __attribute__((aligned(16))) bf16 lds[2][CHUNK_ROWS * LDS_ROW];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int hp = blockIdx.y;
  const bf16* Khp = K + (int64_t)hp * N_cap * D;
  const bf16* Mhp = mu_hat + (int64_t)hp * c_count * D;

  // ---- keys of this wavefront into registers, in B-operand layout ----
  const int64_t wave_tok0 = ((int64_t)blockIdx.x * 4 + wave) * (NKB * 32);
  bf16x8 bk[NKB][8];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    int64_t t = wave_tok0 + kb * 32 + col;
    if (t >= tok_count) t = tok_count - 1;            // clamp: result is discarded
    const bf16* row = Khp + (tok_begin + t) * D + half * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) bk[kb][kk] = *reinterpret_cast<const bf16x8*>(row + kk * 16);
  }

  float best[NKB];
  int bidx[NKB];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    best[kb] = -INFINITY;
    bidx[kb] = 0;
  }

  const int n_chunks = (c_count + CHUNK_ROWS - 1) / CHUNK_ROWS;
  uint4 stage[4];
  // chunk = 64 rows x 256 B = 1024 segments of 16 B; thread handles 4 of them
  auto fetch = [&](int ch) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int seg = tid + i * ASSIGN_THREADS;
      const int r = ch * CHUNK_ROWS + (seg >> 4);
      if (r < c_count)
        stage[i] = *reinterpret_cast<const uint4*>(Mhp + (int64_t)r * D + (seg & 15) * 8);
      else
        stage[i] = make_uint4(0, 0, 0, 0);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int seg = tid + i * ASSIGN_THREADS;
      *reinterpret_cast<uint4*>(&lds[buf][(seg >> 4) * LDS_ROW + (seg & 15) * 8]) = stage[i];
    }
  };

  fetch(0);
  stash(0);
  __syncthreads();

  for (int ch = 0; ch < n_chunks; ++ch) {
    if (ch + 1 < n_chunks) fetch(ch + 1);
    const bf16* buf = lds[ch & 1];
#pragma unroll
    for (int tile = 0; tile < 2; ++tile) {
      const int row0 = ch * CHUNK_ROWS + tile * 32;
      if (row0 < c_count) {                            // wave-uniform
        floatx16 acc[NKB];
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[kb][i] = 0.f;
        const bf16* arow = buf + (tile * 32 + col) * LDS_ROW + half * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(arow + kk * 16);
#pragma unroll
          for (int kb = 0; kb < NKB; ++kb)
            acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bk[kb][kk], acc[kb], 0, 0, 0);
        }
        // accumulator i of a lane is centroid row 8*(i/4) + 4*half + i%4 of the tile
        const bool partial = row0 + 32 > c_count;      // wave-uniform
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int c = row0 + 8 * (i >> 2) + 4 * half + (i & 3);
#pragma unroll
          for (int kb = 0; kb < NKB; ++kb) {
            float v = acc[kb][i];
            if (partial && c >= c_count) v = -INFINITY;
            if (v > best[kb]) {                        // strict: the lower id keeps a tie
              best[kb] = v;
              bidx[kb] = c;
            }
          }
        }
      }
    }
    if (ch + 1 < n_chunks) stash((ch + 1) & 1);
    __syncthreads();
  }

  // ---- lanes l and l+32 hold the two halves of each key's candidates ----
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    const float ob = __shfl_xor(best[kb], 32, WAVE);
    const int oi = __shfl_xor(bidx[kb], 32, WAVE);
    if (ob > best[kb] || (ob == best[kb] && oi < bidx[kb])) {
      best[kb] = ob;
      bidx[kb] = oi;
    }
    const int64_t t = wave_tok0 + kb * 32 + col;
    if (half == 0 && t < tok_count) {
      const int64_t o = (int64_t)hp * N_cap + tok_begin + t;
      labels[o] = c_begin + bidx[kb];
      if (best_sim) best_sim[o] = best[kb];
    }
  }
}

hipError_t launch_assign(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                         const bf16* mu_hat, int c_begin, int c_count, int32_t* labels,
                         float* best_sim, hipStream_t st) {
  // Large problems: 128 keys per wavefront (4 MFMAs per centroid fragment read).
  // Small ones (incremental clustering of a few hundred tokens): 32 keys per
  // wavefront so that more workgroups exist.
  if (tok_count * dm.HP >= 64 * 1024) {
    constexpr int NKB = 4;
    dim3 grid((unsigned)((tok_count + 4 * NKB * 32 - 1) / (4 * NKB * 32)), dm.HP);
    hipLaunchKernelGGL(k_assign<NKB>, grid, dim3(ASSIGN_THREADS), 0, st, K, mu_hat, labels,
                       best_sim, dm.N_cap, tok_begin, tok_count, c_begin, c_count);
  } else {
    constexpr int NKB = 1;
    dim3 grid((unsigned)((tok_count + 4 * NKB * 32 - 1) / (4 * NKB * 32)), dm.HP);
    hipLaunchKernelGGL(k_assign<NKB>, grid, dim3(ASSIGN_THREADS), 0, st, K, mu_hat, labels,
                       best_sim, dm.N_cap, tok_begin, tok_count, c_begin, c_count);
  }
  return hipGetLastError();
}

}  // namespace ck
