// Measurement aid, not part of the attention path: what the matrix cores of THIS chip sustain.
// Every wave runs a loop of independent v_mfma_f32_32x32x16_bf16 instructions on register
// operands (no memory traffic at all); wave 0 of work-group 0 reads the shader-clock counter and
// the constant-rate (100 MHz) counter around its loop.  Their ratio is the shader clock the chip
// settles at under sustained matrix load; (instructions issued) x 32768 FLOP / elapsed time is the
// matrix-instruction ceiling at that clock, against which a kernel's rate can be put next to the
// nominal peak.
#include "common.hpp"

namespace {

__global__ __launch_bounds__(256, 2) void mfma_probe_kernel(long long* __restrict__ out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    a[i] = (bf16_t)(float)((threadIdx.x + i) & 7);
    b[i] = (bf16_t)(float)((threadIdx.x * 3 + i) & 3);
  }
  f32x16 acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] = mfma32(a, b, acc[j]);
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  if (s == 12345.678f) out[2] = 1;                 // keeps the loop alive; never true
  if (blockIdx.x == 0 && threadIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; }
}

}  // namespace

hipError_t attn_probe_dispatch(long long* out, int workgroups, int iters, hipStream_t st) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, st, out, iters);
  return hipGetLastError();
}
