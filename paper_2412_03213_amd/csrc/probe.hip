// Measurement aid: a register-only bf16 MFMA loop, to find the matrix throughput the
// chip sustains at its real clocks (the denominator next to the published peak when
// the assignment kernel's MFMA fraction is judged).  The operands can be supplied by
// the caller: the clock the chip holds under matrix load depends on how many operand
// bits toggle, so constant operands and random ones give different answers, and the
// second is the one that bounds a kernel working on real keys.
#include "ck_common.hpp"

namespace ck {

__global__ __launch_bounds__(256, 2) void k_probe_mfma(int iters, const uint4* __restrict__ operands,
                                                       unsigned long long* __restrict__ clocks,
                                                       float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  // 8 A fragments and 8 B fragments per lane, used in rotation, so that consecutive
  // MFMAs see different operand bits as they do in a real tile loop
  bf16x8 a[8], b[8];
  if (operands) {
    // 64 lanes x (8 A fragments, 8 B fragments), 16 bytes each
#pragma unroll
    for (int f = 0; f < 8; ++f) {
      const uint4 ua = operands[16 * lane + f], ub = operands[16 * lane + 8 + f];
      a[f] = *reinterpret_cast<const bf16x8*>(&ua);
      b[f] = *reinterpret_cast<const bf16x8*>(&ub);
    }
  } else {
#pragma unroll
    for (int f = 0; f < 8; ++f)
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        a[f][i] = (bf16)(float)((lane + i) & 3);
        b[f][i] = (bf16)(float)((lane * 3 + i) & 1);
      }
  }
  floatx16 c0, c1, c2, c3;
#pragma unroll
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
  // shader-clock cycles and ticks of the constant 100 MHz counter over the same loop:
  // their ratio is the clock this compute unit actually ran at
  const unsigned long long cyc0 = clock64(), tick0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * u], b[u], c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[2 * u + 1], b[u + 4], c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[7 - 2 * u], b[7 - u], c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[6 - 2 * u], b[3 - u], c3, 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  const unsigned long long cyc1 = clock64(), tick1 = wall_clock64();
  if (clocks && blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = cyc1 - cyc0;
    clocks[1] = tick1 - tick0;
  }
  if (s == -1.2345e-30f) sink[0] = s;                    // never true: keeps the loop alive
}

hipError_t launch_probe_mfma(int n_workgroups, int iters, const void* operands,
                             unsigned long long* clocks, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(k_probe_mfma, dim3(n_workgroups), dim3(256), 0, st, iters,
                     (const uint4*)operands, clocks, sink);
  return hipGetLastError();
}

}  // namespace ck
