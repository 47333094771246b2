// K-means assignment step (paper Section III-B), streaming form: see k_assign in
// kmeans_assign.hip for the mapping onto v_mfma_f32_32x32x16_bf16 and the packed
// running maximum.  This file is compiled with the MFMA results kept in vector
// registers (the read-out works on them directly) and the operands that only the
// matrix cores touch in the accumulator half of the register file.
#include <type_traits>

#include "ck_common.hpp"

namespace ck {

constexpr int LDS_ROW = D + 8;             // bf16 elements per LDS row: 272 B, rows shift 4 banks

// ---------------------------------------------------------------- streaming form
// For tables of at most 512 centroids (the paper's C0 = L/80 at 32k tokens is 400): the
// WHOLE unit-centroid table of the head-problem stays in LDS for the life of the
// workgroup (one workgroup of eight wavefronts per CU, two per SIMD), so the tile loop
// has no barriers, and every wavefront walks through several blocks of 64 keys with the
// NEXT block's loads in flight while the current block is contracted against all tiles:
// the key stream (the only HBM traffic that matters) runs under the matrix work instead
// of before it.
// The loop is software-pipelined by hand inside each wavefront: the 8 MFMAs of one key
// block (a dependent chain on one accumulator: chains cost nothing) are issued with the
// read-out (packed running maximum) of the OTHER key block's accumulator cut into 8
// slices between them, about 3.5 vector instructions per MFMA, which is what issues for
// free while an MFMA executes; an A fragment is replaced by the next tile's as soon as
// its last MFMA has been issued.  Two such wavefronts per SIMD cover each other's
// remaining stalls.  Measured on a stand-alone replica of this loop (no memory traffic):
// 76 % of the 2.5 PFLOP/s peak on all-zero operands at a 2.05 GHz shader clock, 54 % on
// random operands, where the chip drops to 1.4 GHz under the load -- 93 % of what that
// clock allows.  The loop is bound by the clock the chip holds, not by its schedule.
// Eight consecutive tasks of 64 tokens are one 512-token chunk of the counting sort.
constexpr int ST_WAVES = 8;
constexpr int ST_NKB = 2;                               // 64 keys per wavefront and block
constexpr int ST_CHUNK = ST_WAVES * ST_NKB * 32;        // 512 tokens per block of a workgroup
constexpr int ST_MAX_TILES = 16;                        // 512 centroids
constexpr int ST_MAX_BLOCKS = 8;
constexpr int ST_HIST_INTS = 5600;                      // LDS left for the label histograms

template <bool HAS_BIAS>
__global__ __launch_bounds__(ST_WAVES * 64, 2) void k_assign_stream(
    const bf16* __restrict__ K, const bf16* __restrict__ mu_hat, int32_t* __restrict__ labels,
    float* __restrict__ best_sim, int32_t* __restrict__ chunk_hist, int n_hist_chunks,
    int64_t N_cap, int64_t tok_begin, int64_t tok_count, int c_begin, int c_count, int blocks,
    const KmCtl ctl) {
  constexpr int NKB = ST_NKB, THREADS = ST_WAVES * 64;
  __shared__ __attribute__((aligned(16))) bf16 table[ST_MAX_TILES * 32 * LDS_ROW];
  __shared__ __attribute__((aligned(16))) float lds_bias[HAS_BIAS ? ST_MAX_TILES * 32 : 4];
  __shared__ int hist[ST_HIST_INTS];
  __shared__ int s_changed, s_next_task;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int hp = blockIdx.y;
  if (ctl.skip && ctl.skip[hp] == 0) return;            // converged: whole workgroup leaves
  const bf16* Khp = K + (int64_t)hp * N_cap * D;
  const bf16* Mhp = mu_hat + (int64_t)hp * c_count * D;
  const int n_tiles = (c_count + 31) / 32;
  const int64_t wg_tok0 = (int64_t)blockIdx.x * blocks * ST_CHUNK;

  // keys of task b (64 consecutive tokens of this workgroup's range), in B-operand layout
  auto load_keys = [&](int b, bf16x8 (&bk)[NKB][8]) {
    const bf16* rows[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      int64_t t = wg_tok0 + (int64_t)b * (NKB * 32) + kb * 32 + col;
      if (t >= tok_count) t = tok_count - 1;            // clamp: result is discarded
      rows[kb] = Khp + (tok_begin + t) * D + half * 8;
    }
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb)
#pragma unroll
      for (int kk = 0; kk < 8; ++kk)
        bk[kb][kk] = *reinterpret_cast<const bf16x8*>(rows[kb] + kk * 16);
  };
  bf16x8 ka[NKB][8], kb2[NKB][8];

  // ---- the table into LDS (rows beyond c_count are zero), bias, histograms ----
  {
    const int n_seg = n_tiles * 32 * 16;                // 16-byte segments
    constexpr int PER = ST_MAX_TILES * 32 * 16 / THREADS;   // 16 per thread, all in flight at once
    uint4 stage[PER];
    // every load is unconditional (rows beyond the table re-read its last row and are
    // replaced by zeros when they are written to LDS): a load under a branch makes the
    // compiler wait for it before it issues the next one
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int seg = tid + i * THREADS;
      int r = seg >> 4;
      r = r < c_count ? r : c_count - 1;
      stage[i] = *reinterpret_cast<const uint4*>(Mhp + (int64_t)r * D + (seg & 15) * 8);
    }
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int seg = tid + i * THREADS;
      const bool real = (seg >> 4) < c_count;
      uint4 v = stage[i];
      v.x = real ? v.x : 0u; v.y = real ? v.y : 0u; v.z = real ? v.z : 0u; v.w = real ? v.w : 0u;
      if (seg < n_seg)
        *reinterpret_cast<uint4*>(&table[(seg >> 4) * LDS_ROW + (seg & 15) * 8]) = v;
    }
  }
  // the first keys are requested after the table has arrived: loads come back in the
  // order they were issued and share the memory system's bandwidth, and every earlier
  // placement of this request that was tried (before the table, between its loads and
  // its LDS writes, for half of the wavefronts only) delayed the table by more than it
  // advanced the keys
  load_keys(wave, ka);
  if constexpr (HAS_BIAS) {
    for (int c = tid; c < n_tiles * 32; c += THREADS)
      lds_bias[c] = c < c_count ? ctl.bias[(int64_t)hp * ctl.bias_stride + c] : 0.f;
  }
  if (chunk_hist)
    for (int c = tid; c < blocks * c_count; c += THREADS) hist[c] = 0;
  if (tid == 0) {
    s_changed = 0;
    s_next_task = ST_WAVES;                             // tasks 0..7 are the wavefronts' first ones
  }
  __syncthreads();

  int diff = 0;
  const bf16* arow0 = table + col * LDS_ROW + half * 8; // this lane's A fragments of tile 0

  // One block of 128 keys against every centroid tile, then its labels.
  auto process = [&](int b, const bf16x8 (&bk)[NKB][8]) {
    const int64_t wave_tok0 = wg_tok0 + (int64_t)b * (NKB * 32);
    if (wave_tok0 >= tok_count) return;                 // wave-uniform: nothing of this block exists
    float bestp[NKB];
    int btile[NKB];
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      bestp[kb] = -INFINITY;
      btile[kb] = 0;
    }
    floatx16 acc[NKB];
    bf16x8 a[8];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) a[kk] = *reinterpret_cast<const bf16x8*>(arow0 + kk * 16);

    // Slice r (0..7) of the read-out of one accumulator: two of its 16 similarities
    // join the packed running maximum; the last slice settles tile and value.
    // accumulator i of a lane is centroid row 8*(i/4) + 4*half + i%4 of the tile
    float mrun = 0.f;
    auto readout = [&](int kb, int tile_id, int r, bool last_tile) {
      float v0 = acc[kb][2 * r], v1 = acc[kb][2 * r + 1];
      const int row = tile_id * 32 + 8 * (r >> 1) + 4 * half + 2 * (r & 1);
      if constexpr (HAS_BIAS) {
        v0 += lds_bias[row];
        v1 += lds_bias[row + 1];
      }
      if (last_tile) {                                  // zero-padded rows lose (finite: no NaN)
        v0 = row >= c_count ? -3.0e38f : v0;
        v1 = row + 1 >= c_count ? -3.0e38f : v1;
      }
      const float p0 = __uint_as_float((__float_as_uint(v0) & 0xFFFFFFF0u) | (uint32_t)(15 - 2 * r));
      const float p1 = __uint_as_float((__float_as_uint(v1) & 0xFFFFFFF0u) | (uint32_t)(14 - 2 * r));
      if (r == 0) mrun = bestp[kb];
      mrun = fmaxf(fmaxf(mrun, p0), p1);
      if (r == 7) {
        const bool up = __uint_as_float(__float_as_uint(mrun) & 0xFFFFFFF0u) >
                        __uint_as_float(__float_as_uint(bestp[kb]) & 0xFFFFFFF0u);
        btile[kb] = up ? tile_id : btile[kb];
        bestp[kb] = up ? mrun : bestp[kb];
      }
    };
    // The 8 MFMAs of key block KB against the tile whose A fragments are in a[], with the
    // read-out of the other key block's accumulator (tile `ro_tile`) between them.  While
    // key block 1 runs, every A fragment is replaced by the next tile's.
    auto step = [&](auto KBT, auto READOUT, int ro_tile, bool ro_last, const bf16* next_arow) {
      constexpr int kb = decltype(KBT)::value;
      constexpr bool RO = decltype(READOUT)::value;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        if (kk == 0) {
          floatx16 z;
#pragma unroll
          for (int i = 0; i < 16; ++i) z[i] = 0.f;
          acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], bk[kb][kk], z, 0, 0, 0);
        } else {
          acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], bk[kb][kk], acc[kb], 0, 0, 0);
        }
        if (RO) readout(1 - kb, ro_tile, kk, ro_last);
        if (kb == 1 && next_arow) a[kk] = *reinterpret_cast<const bf16x8*>(next_arow + kk * 16);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    using T0 = std::integral_constant<int, 0>;
    using T1 = std::integral_constant<int, 1>;
    using Yes = std::true_type;
    using No = std::false_type;
    const int last = n_tiles - 1;
    step(T0(), No(), 0, false, nullptr);                // tile 0, key block 0: nothing to read out yet
    for (int tile = 0; tile < last; ++tile) {
      step(T1(), Yes(), tile, false, arow0 + (tile + 1) * 32 * LDS_ROW);   // reads out block 0 of `tile`
      step(T0(), Yes(), tile, false, nullptr);          // block 0 of tile + 1; reads out block 1 of `tile`
    }
    step(T1(), Yes(), last, true, nullptr);             // last tile, key block 1; reads out its block 0
#pragma unroll
    for (int r = 0; r < 8; ++r) readout(1, last, r, true);

    // lanes l and l+32 hold the two halves of each key's candidates
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
      const int slot = 15 - (int)(__float_as_uint(bestp[kb]) & 15u);
      float best = bestp[kb];
      int bidx = btile[kb] * 32 + 8 * (slot >> 2) + 4 * half + (slot & 3);
      const float ob = __shfl_xor(best, 32, WAVE);
      const int oi = __shfl_xor(bidx, 32, WAVE);
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
        if (chunk_hist) atomicAdd(&hist[(b / ST_WAVES) * c_count + bidx], 1);   // integer counts: any order
      }
    }
  };

  // A workgroup's range is cut into tasks of 64 tokens (8 per 512-token chunk).  Every
  // wavefront starts with the task of its own number and then takes the next free one
  // from a shared counter, always one task ahead so that the keys can be requested a
  // whole task early.  Two wavefronts share a SIMD and the hardware does not split it
  // evenly between them; with a fixed share the slower one would finish alone, at the
  // speed of one wavefront.
  const int n_tasks = blocks * ST_WAVES;
  auto grab = [&]() {
    int t = 0;
    if (lane == 0) t = atomicAdd(&s_next_task, 1);
    return __builtin_amdgcn_readfirstlane(t);
  };
  int cur = wave;
  while (cur < n_tasks) {
    int nxt = grab();
    if (nxt < n_tasks) load_keys(nxt, kb2);
    process(cur, ka);
    cur = nxt;
    if (cur >= n_tasks) break;
    nxt = grab();
    if (nxt < n_tasks) load_keys(nxt, ka);
    process(cur, kb2);
    cur = nxt;
  }

  if (ctl.changed) {
    const int wsum = __builtin_amdgcn_readlane(wave_inclusive_scan(diff), WAVE - 1);
    if (lane == 0 && wsum) atomicAdd(&s_changed, wsum);
  }
  if (chunk_hist || ctl.changed) __syncthreads();
  if (ctl.changed && tid == 0 && s_changed) atomicAdd(&ctl.changed[hp], s_changed);
  if (chunk_hist) {
    for (int e = tid; e < blocks * c_count; e += THREADS) {
      const int hc = (int)blockIdx.x * blocks + e / c_count;
      if (hc < n_hist_chunks)
        chunk_hist[((int64_t)hp * n_hist_chunks + hc) * c_count + e % c_count] = hist[e];
    }
  }
}

bool assign_stream_fits(int c_count) { return c_count <= ST_MAX_TILES * 32; }

hipError_t launch_assign_stream(const Dims& dm, const bf16* K, int64_t tok_begin,
                                int64_t tok_count, const bf16* mu_hat, int c_begin, int c_count,
                                int32_t* labels, float* best_sim, int32_t* chunk_hist,
                                const KmCtl& ctl, int n_cu, hipStream_t st) {
  // blocks of 512 tokens per workgroup: as many as keep every CU busy (at most 8, and
  // what the label histograms leave room for)
  const int64_t chunks_hp = (tok_count + ST_CHUNK - 1) / ST_CHUNK;
  int64_t blocks = chunks_hp * dm.HP / n_cu;
  if (blocks > ST_MAX_BLOCKS) blocks = ST_MAX_BLOCKS;
  if (blocks > ST_HIST_INTS / c_count) blocks = ST_HIST_INTS / c_count;
  if (blocks > chunks_hp) blocks = chunks_hp;
  if (blocks < 1) blocks = 1;
  const dim3 grid((unsigned)((chunks_hp + blocks - 1) / blocks), dm.HP);
  if (ctl.bias)
    hipLaunchKernelGGL(k_assign_stream<true>, grid, dim3(ST_WAVES * 64), 0, st, K, mu_hat, labels,
                       best_sim, chunk_hist, (int)chunks_hp, dm.N_cap, tok_begin, tok_count,
                       c_begin, c_count, (int)blocks, ctl);
  else
    hipLaunchKernelGGL(k_assign_stream<false>, grid, dim3(ST_WAVES * 64), 0, st, K, mu_hat, labels,
                       best_sim, chunk_hist, (int)chunks_hp, dm.N_cap, tok_begin, tok_count,
                       c_begin, c_count, (int)blocks, ctl);
  return hipGetLastError();
}

}  // namespace ck
