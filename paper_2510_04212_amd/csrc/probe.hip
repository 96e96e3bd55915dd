// Measurement aids for the benchmark, built into a library of their own (libattn_probe_gfx950.so,
// declared in probe.h): no attention arithmetic, nothing from the paper.
//
// Matrix cores: every wave runs a loop of independent v_mfma_f32_32x32x16_bf16 instructions on
// register operands (no memory traffic at all); the first wave of EVERY work-group reads the
// shader-clock counter and the constant-rate (100 MHz) counter around its loop and records both.
// Their ratio is the shader clock that work-group's CU ran at under sustained matrix load; the
// longest loop in constant-rate ticks is the kernel's duration as the device saw it; (instructions
// issued) x 32768 FLOP / elapsed time is the matrix-instruction ceiling, against which a kernel's
// rate can be put next to the nominal peak.
#include "common.hpp"
#include "probe.h"

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
  if (threadIdx.x == 0) {
    out[4 + 2 * blockIdx.x] = c1 - c0; out[5 + 2 * blockIdx.x] = w1 - w0;
    if (blockIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; }
  }
}

// The same for the LDS: four waves per work-group, each issuing 16 * iters conflict-free LDS
// reads from a 16 KB window and nothing else.  KIND 0: ds_read_b128 (64 lanes x 16 bytes = 1 KB
// per instruction, one matrix-instruction operand fragment); KIND 1: ds_read_b64_tr_b16 (the
// transposing read, 512 bytes per instruction, two per fragment).  Bytes read / elapsed shader
// cycles is the LDS read bandwidth per CU the kernels' fragment traffic has to fit into.
template <int KIND>
__global__ __launch_bounds__(256, 1) void lds_probe_kernel(long long* __restrict__ out, int iters) {
  __shared__ __attribute__((aligned(16))) char lds[16384];
  for (int i = threadIdx.x; i < 4096; i += 256) reinterpret_cast<float*>(lds)[i] = (float)i;
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const long long c0 = clock64(), w0 = wall_clock64();
  if (KIND == 0) {
    const char* base = lds + lane * 16;
    for (int it = 0; it < iters; ++it) {
      u32x4 t[16];
#pragma unroll
      for (int j = 0; j < 16; ++j) t[j] = *reinterpret_cast<const u32x4*>(base + j * 1024);
      // all 16 bytes of every read are "used" by an empty asm statement: no vector instruction
      // competes with the reads, and the compiler cannot narrow them
#pragma unroll
      for (int j = 0; j < 16; ++j) asm volatile("" : : "v"(t[j]));
    }
  } else {
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    // the access pattern of the kernels' transposing reads on a 128-column tile: 16 lanes cover
    // 4 rows x 32 bytes, the four 16-lane groups of a wave four different 4-row bands
    // (16 different addresses per pass: identical ones would be merged by the compiler)
    const int i = lane & 15;
    const char* base[4];
#pragma unroll
    for (int c = 0; c < 4; ++c)
      base[c] = lds + tile_off<128>(4 * (lane >> 4) + (i >> 2), 32 * c + ((i & 3) << 2));
    for (int it = 0; it < iters; ++it) {
      s16x4 t[16];
#pragma unroll
      for (int j = 0; j < 16; ++j)
        t[j] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(base[j >> 2] + (j & 3) * 4096));
#pragma unroll
      for (int j = 0; j < 16; ++j) asm volatile("" : : "v"(t[j]));
    }
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  if (blockIdx.x == 0 && threadIdx.x == 0) { out[0] = c1 - c0; out[1] = w1 - w0; }
}

}  // namespace

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" int attn_probe_lds_clock(long long* out, int kind, int workgroups, int iters, void* stream) {
  if (kind < 0 || kind > 1) return 2;
  if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 22)) return 2;
  if (!out) return 1;
  if (!aligned16(out)) return 2;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (kind == 0) hipLaunchKernelGGL(lds_probe_kernel<0>, dim3(workgroups), dim3(256), 0, st, out, iters);
  else hipLaunchKernelGGL(lds_probe_kernel<1>, dim3(workgroups), dim3(256), 0, st, out, iters);
  return hipGetLastError() == hipSuccess ? 0 : 5;
}

extern "C" int attn_probe_matrix_clock(long long* out, int workgroups, int iters, void* stream) {
  if (workgroups < 1 || workgroups > 65536 || iters < 1 || iters > (1 << 22)) return 2;
  if (!out) return 1;
  if (!aligned16(out)) return 2;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), out, iters);
  return hipGetLastError() == hipSuccess ? 0 : 5;
}
