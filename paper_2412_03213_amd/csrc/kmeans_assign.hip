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
// LDS in double-buffered chunks of 64 rows shared by all wavefronts of the workgroup.
#include <atomic>

#include "ck_common.hpp"

namespace ck {

constexpr int CHUNK_ROWS = 64;             // centroid rows per LDS chunk (two MFMA tiles)
constexpr int LDS_ROW = D + 8;             // bf16 elements per LDS row: 272 B, rows shift 4 banks

// WAVES wavefronts per workgroup, each with NKB blocks of 32 keys.  With PHASED the
// odd wavefronts of a SIMD pair (waves >= WAVES/2 share SIMDs with waves < WAVES/2)
// delay the accumulator read-out of a tile until after the next barrier, so that on
// every SIMD one wavefront is in its MFMA phase while the other reduces on the
// vector ALUs.
// HAS_BIAS (l2 metric): a per-centroid bias, held in LDS, is added to every
// similarity before the argmax.
template <int NKB, int WAVES, int WAVES_PER_SIMD, bool PHASED, bool HAS_BIAS>
__global__ __launch_bounds__(WAVES * 64, WAVES_PER_SIMD) void k_assign(
    const bf16* __restrict__ K, const bf16* __restrict__ mu_hat, int32_t* __restrict__ labels,
    float* __restrict__ best_sim, int32_t* __restrict__ chunk_hist, int n_hist_chunks,
    int64_t N_cap, int64_t tok_begin, int64_t tok_count, int c_begin, int c_count,
    const KmCtl ctl) {
  constexpr int THREADS = WAVES * 64;
  constexpr int SEGS = CHUNK_ROWS * 16 / THREADS;      // 16-byte segments of a chunk per thread
  __shared__ __attribute__((aligned(16))) bf16 lds[2][CHUNK_ROWS * LDS_ROW];
  __shared__ __attribute__((aligned(16))) float lds_bias[HAS_BIAS ? CK_MAX_CLUSTERS + 32 : 4];
  __shared__ int s_changed;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int hp = blockIdx.y;
  if (ctl.skip && ctl.skip[hp] == 0) return;            // converged: whole workgroup leaves
  const bf16* Khp = K + (int64_t)hp * N_cap * D;
  const bf16* Mhp = mu_hat + (int64_t)hp * c_count * D;

  const int n_chunks = (c_count + CHUNK_ROWS - 1) / CHUNK_ROWS;
  const int n_tiles = (c_count + 31) / 32;
  uint4 stage[SEGS];
  auto fetch = [&](int ch) {
#pragma unroll
    for (int i = 0; i < SEGS; ++i) {
      const int seg = tid + i * THREADS;
      const int r = ch * CHUNK_ROWS + (seg >> 4);
      if (r < c_count)
        stage[i] = *reinterpret_cast<const uint4*>(Mhp + (int64_t)r * D + (seg & 15) * 8);
      else
        stage[i] = make_uint4(0, 0, 0, 0);
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int i = 0; i < SEGS; ++i) {
      const int seg = tid + i * THREADS;
      *reinterpret_cast<uint4*>(&lds[buf][(seg >> 4) * LDS_ROW + (seg & 15) * 8]) = stage[i];
    }
  };
  // first centroid chunk ahead of the keys, so that it does not queue behind them
  fetch(0);
  if (tid == 0) s_changed = 0;
  if constexpr (HAS_BIAS) {
    for (int c = tid; c < n_tiles * 32; c += THREADS)
      lds_bias[c] = c < c_count ? ctl.bias[(int64_t)hp * ctl.bias_stride + c] : 0.f;
  }

  // ---- keys of this wavefront into registers, in B-operand layout ----
  // Issued fragment-major (all key blocks' fragment 0, then fragment 1, ...): the first
  // tile's MFMAs then start as soon as the first few loads have landed and follow the
  // arriving data instead of waiting for all of it.
  const int64_t wave_tok0 = ((int64_t)blockIdx.x * WAVES + wave) * (NKB * 32);
  bf16x8 bk[NKB][8];
  {
    const bf16* rows[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      int64_t t = wave_tok0 + kb * 32 + col;
      if (t >= tok_count) t = tok_count - 1;            // clamp: result is discarded
      rows[kb] = Khp + (tok_begin + t) * D + half * 8;
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
#pragma unroll
      for (int kb = 0; kb < NKB; ++kb)
        bk[kb][kk] = *reinterpret_cast<const bf16x8*>(rows[kb] + kk * 16);
  }

  // Running maximum per key block as a "packed" float: the low 4 mantissa bits of
  // every similarity are replaced by 15 - (accumulator slot), so one v_max3 chain
  // finds value and slot together and equal values resolve to the lower centroid.
  // The truncation moves a similarity by < 2^-19 relative, far inside the 1e-4
  // cosine near-tie band in which labels may legitimately differ.  (Exception to
  // "lower id wins": when a key's best similarity is NEGATIVE and bit-equal for two
  // of the 16 rows one lane holds of a tile, the slot bits order the other way and
  // the higher of the two rows is taken -- an exact tie, so inside that band too.)
  float bestp[NKB];
  int btile[NKB];
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    bestp[kb] = -INFINITY;
    btile[kb] = 0;
  }
  floatx16 acc[NKB];

  // similarities of centroid tile `t` (rows of chunk buffer `buf`) against the keys
  auto contract = [&](const bf16* buf, int tile) {
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
  };
  // folds the accumulators of tile `tile_id` into the running maxima
  auto reduce = [&](int tile_id) {
    const int row0 = tile_id * 32;
    // accumulator i of a lane is centroid row 8*(i/4) + 4*half + i%4 of the tile
    if constexpr (HAS_BIAS) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const floatx4 b = *reinterpret_cast<const floatx4*>(&lds_bias[row0 + 8 * j + 4 * half]);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[kb][4 * j + e] += b[e];
      }
    }
    if (row0 + 32 > c_count) {                         // wave-uniform: zero-padded rows lose
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int c = row0 + 8 * (i >> 2) + 4 * half + (i & 3);
#pragma unroll
        for (int kb = 0; kb < NKB; ++kb)
          if (c >= c_count) acc[kb][i] = -3.0e38f;     // finite: the slot bits must not make a NaN
      }
    }
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      float p[16];
#pragma unroll
      for (int i = 0; i < 16; ++i)
        p[i] = __uint_as_float((__float_as_uint(acc[kb][i]) & 0xFFFFFFF0u) | (uint32_t)(15 - i));
      float m = bestp[kb];
      m = fmaxf(fmaxf(m, p[0]), p[1]);
#pragma unroll
      for (int i = 2; i < 16; i += 2) m = fmaxf(fmaxf(m, p[i]), p[i + 1]);
      // a later tile takes over only with a strictly larger (truncated) value: an equal
      // one would be a higher centroid id, whatever its slot bits say
      const bool up = __uint_as_float(__float_as_uint(m) & 0xFFFFFFF0u) >
                      __uint_as_float(__float_as_uint(bestp[kb]) & 0xFFFFFFF0u);
      btile[kb] = up ? tile_id : btile[kb];
      bestp[kb] = up ? m : bestp[kb];
    }
  };

  stash(0);
  __syncthreads();

  const bool late = PHASED && wave >= WAVES / 2;        // wave-uniform
  for (int ch = 0; ch < n_chunks; ++ch) {
    if (ch + 1 < n_chunks) fetch(ch + 1);
    const bf16* buf = lds[ch & 1];
    if (!late) {
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) {
        const int t = ch * 2 + tile;
        if (t < n_tiles) {                               // wave-uniform
          contract(buf, tile);
          reduce(t);
        }
      }
    } else {
#pragma unroll
      for (int tile = 0; tile < 2; ++tile) {
        const int t = ch * 2 + tile;
        if (t < n_tiles) {
          if (t > 0) reduce(t - 1);
          contract(buf, tile);
        }
      }
    }
    if (ch + 1 < n_chunks) stash((ch + 1) & 1);
    __syncthreads();
  }
  if (late) reduce(n_tiles - 1);

  // ---- lanes l and l+32 hold the two halves of each key's candidates ----
  // (the centroid buffers are free now: the loop ended with a barrier)
  // One label histogram per 4 wavefronts = per chunk of the counting sort.
  constexpr int HISTS = WAVES / 4;
  int* hist = reinterpret_cast<int*>(&lds[0][0]) + (wave >> 2) * c_count;
  if (chunk_hist) {
    for (int c = tid; c < HISTS * c_count; c += THREADS) reinterpret_cast<int*>(&lds[0][0])[c] = 0;
    __syncthreads();
  }
  int diff = 0;
#pragma unroll
  for (int kb = 0; kb < NKB; ++kb) {
    const int slot = 15 - (int)(__float_as_uint(bestp[kb]) & 15u);
    float best = bestp[kb];
    int bidx = btile[kb] * 32 + 8 * (slot >> 2) + 4 * half + (slot & 3);
    const float ob = __shfl_xor(best, 32, WAVE);
    const int oi = __shfl_xor(bidx, 32, WAVE);
    // compare without the slot bits so that an exact tie goes to the lower id
    const float bt = __uint_as_float(__float_as_uint(best) & 0xFFFFFFF0u);
    const float ot = __uint_as_float(__float_as_uint(ob) & 0xFFFFFFF0u);
    if (ot > bt || (ot == bt && oi < bidx)) {
      best = ob;
      bidx = oi;
    }
    const int64_t t = wave_tok0 + kb * 32 + col;
    if (half == 0 && t < tok_count) {
      const int64_t o = (int64_t)hp * N_cap + tok_begin + t;
      if (ctl.changed) diff += (ctl.first || labels[o] != c_begin + bidx) ? 1 : 0;
      labels[o] = c_begin + bidx;
      if (best_sim) best_sim[o] = __uint_as_float(__float_as_uint(best) & 0xFFFFFFF0u);
      if (chunk_hist) atomicAdd(&hist[bidx], 1);       // integer counts: order does not matter
    }
  }
  if (ctl.changed) {
    const int wsum = __builtin_amdgcn_readlane(wave_inclusive_scan(diff), WAVE - 1);
    if (lane == 0 && wsum) atomicAdd(&s_changed, wsum);
  }
  if (chunk_hist || ctl.changed) __syncthreads();
  if (ctl.changed && tid == 0 && s_changed) atomicAdd(&ctl.changed[hp], s_changed);
  // label histograms of this workgroup's tokens = chunks of the counting sort
  if (chunk_hist) {
    for (int e = tid; e < HISTS * c_count; e += THREADS) {
      const int hc = (int)blockIdx.x * HISTS + e / c_count;
      if (hc < n_hist_chunks)
        chunk_hist[((int64_t)hp * n_hist_chunks + hc) * c_count + e % c_count] =
            reinterpret_cast<int*>(&lds[0][0])[e];
    }
  }
}

template <int NKB, int WAVES, int WPS, bool PHASED>
static void launch_assign_variant(const Dims& dm, const bf16* K, int64_t tok_begin,
                                  int64_t tok_count, const bf16* mu_hat, int c_begin, int c_count,
                                  int32_t* labels, float* best_sim, int32_t* chunk_hist,
                                  const KmCtl& ctl, hipStream_t st) {
  constexpr int TOK = WAVES * NKB * 32;
  const int sort_chunk = 4 * NKB * 32;
  const int n_hist_chunks = (int)((tok_count + sort_chunk - 1) / sort_chunk);
  dim3 grid((unsigned)((tok_count + TOK - 1) / TOK), dm.HP);
  if (ctl.bias)
    // the bias table takes 8 KB more LDS: at most three of the small workgroups fit a CU
    hipLaunchKernelGGL((k_assign<NKB, WAVES, (WPS > 3 ? 3 : WPS), PHASED, true>), grid, dim3(WAVES * 64), 0, st, K,
                       mu_hat, labels, best_sim, chunk_hist, n_hist_chunks, dm.N_cap, tok_begin,
                       tok_count, c_begin, c_count, ctl);
  else
    hipLaunchKernelGGL((k_assign<NKB, WAVES, WPS, PHASED, false>), grid, dim3(WAVES * 64), 0, st, K,
                       mu_hat, labels, best_sim, chunk_hist, n_hist_chunks, dm.N_cap, tok_begin,
                       tok_count, c_begin, c_count, ctl);
}

// Chunk size of the counting sort = the tokens of four assignment wavefronts (every
// group of four emits the label histogram of exactly its own tokens).
// Large problems: 128 keys per wavefront (4 MFMAs per centroid fragment read), eight
// wavefronts per workgroup.  Small ones (incremental clustering of a few hundred
// tokens): 32 keys per wavefront, four per workgroup, so that more workgroups exist.
int assign_tile_tokens(const Dims& dm, int64_t tok_count) {
  return tok_count * dm.HP >= 64 * 1024 ? 512 : 128;
}

// Compute units of the current device, asked once per device (the query costs a few
// microseconds of host time and a clustering call launches the kernel many times).
static int compute_units() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
      n = 256;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

hipError_t launch_assign(const Dims& dm, const bf16* K, int64_t tok_begin, int64_t tok_count,
                         const bf16* mu_hat, int c_begin, int c_count, int32_t* labels,
                         float* best_sim, int32_t* chunk_hist, const KmCtl& ctl, hipStream_t st) {
  if (assign_tile_tokens(dm, tok_count) == 512) {
    // Eight-wavefront workgroups (one per CU, each centroid chunk staged once for all
    // eight, the two wavefronts of a SIMD half a tile apart) win when the whole grid is
    // resident in one round or the tile loop is long; with several rounds of short loops,
    // two independent four-wavefront workgroups per CU overlap one's key load and
    // epilogue with the other's tile loop (measured: +8 % at 64 head-problems, C = 400).
    const int n_cu = compute_units();
    if (assign_stream_fits(c_count))
      return launch_assign_stream(dm, K, tok_begin, tok_count, mu_hat, c_begin, c_count, labels,
                                  best_sim, chunk_hist, ctl, n_cu, st);
    const int64_t wg8 = (tok_count + 1023) / 1024 * dm.HP;
    if (wg8 > n_cu && c_count < 1024) {
      launch_assign_variant<4, 4, 2, false>(dm, K, tok_begin, tok_count, mu_hat, c_begin, c_count,
                                            labels, best_sim, chunk_hist, ctl, st);
      return hipGetLastError();
    }
    launch_assign_variant<4, 8, 2, true>(dm, K, tok_begin, tok_count, mu_hat, c_begin, c_count,
                                         labels, best_sim, chunk_hist, ctl, st);
  } else {
    launch_assign_variant<1, 4, 4, false>(dm, K, tok_begin, tok_count, mu_hat, c_begin, c_count,
                                          labels, best_sim, chunk_hist, ctl, st);
  }
  return hipGetLastError();
}

}  // namespace ck
