// Measurement aid: a register-only bf16 MFMA loop, to find the matrix throughput the
// chip sustains at its real clocks (the denominator next to the published peak when
// the assignment kernel's MFMA fraction is judged).
#include "ck_common.hpp"

namespace ck {

__global__ __launch_bounds__(256, 2) void k_probe_mfma(int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (bf16)(float)((lane + i) & 3);
    b[i] = (bf16)(float)((lane * 3 + i) & 1);
  }
  floatx16 c0, c1, c2, c3;
#pragma unroll
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  if (s == -1.f) sink[0] = s;                            // never true: keeps the loop alive
}

hipError_t launch_probe_mfma(int n_workgroups, int iters, float* sink, hipStream_t st) {
  hipLaunchKernelGGL(k_probe_mfma, dim3(n_workgroups), dim3(256), 0, st, iters, sink);
  return hipGetLastError();
}

}  // namespace ck
