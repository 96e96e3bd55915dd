// delta = rowsum(dO o O)  (Alg. 2 step 4 of arXiv 2510.04212): one float32 per row from the
// bf16 O and dO.  Pure streaming: 4d bytes read and 4 bytes written per row, HBM-bound.
// With OHP the first operand is the float32 O_hp the forward can emit (delta_hp of Sec. 3.2;
// 6d bytes read per row).
// D/8 lanes cooperate on one row (16 bytes each of O and of dO); the partial sums are combined
// with lane shuffles inside the group.
#include "common.hpp"

namespace {

template <int D, int UNROLL, bool OHP>
__global__ __launch_bounds__(256) void attn_delta_kernel(const void* __restrict__ Ov,
                                                         const bf16_t* __restrict__ dO,
                                                         float* __restrict__ delta, long rows,
                                                         int N, Layout lay) {
  const bf16_t* O = static_cast<const bf16_t*>(Ov);
  const float* Of = static_cast<const float*>(Ov);
  constexpr int LPR = kLdsD<D> / 8;      // lanes per row (a power of two; D = 96: lanes 12..15 of a row idle)
  constexpr int RPB = 256 / LPR;         // rows per block per step
  const int sub = threadIdx.x % LPR;
  const int rib = threadIdx.x / LPR;
  long row = (long)blockIdx.x * (RPB * UNROLL) + rib;
  u32x4 a[UNROLL], b[UNROLL];
  f32x4 f0[UNROLL], f1[UNROLL];          // OHP: the 8 float32 values of O_hp
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    long rr = row + (long)u * RPB;
    if (rr < rows && sub < D / 8) {
      // row rr of the [B,H,N] order -> its place in the (possibly strided) bf16 tensors
      const size_t at = head_base(lay, (int)(rr / N)) + (size_t)(rr % N) * lay.sn + sub * 8;
      if (OHP) {
        f0[u] = *reinterpret_cast<const f32x4*>(Of + rr * D + sub * 8);
        f1[u] = *reinterpret_cast<const f32x4*>(Of + rr * D + sub * 8 + 4);
      } else {
        a[u] = *reinterpret_cast<const u32x4*>(O + at);
      }
      b[u] = *reinterpret_cast<const u32x4*>(dO + at);
    } else {
      a[u] = u32x4{0, 0, 0, 0};
      b[u] = u32x4{0, 0, 0, 0};
      f0[u] = f32x4{0.f, 0.f, 0.f, 0.f};
      f1[u] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      float alo, ahi;
      if (OHP) {
        alo = (w < 2) ? f0[u][2 * w] : f1[u][2 * w - 4];
        ahi = (w < 2) ? f0[u][2 * w + 1] : f1[u][2 * w - 3];
      } else {
        alo = __uint_as_float(a[u][w] << 16); ahi = __uint_as_float(a[u][w] & 0xFFFF0000u);
      }
      float blo = __uint_as_float(b[u][w] << 16), bhi = __uint_as_float(b[u][w] & 0xFFFF0000u);
      s = __builtin_fmaf(alo, blo, s);
      s = __builtin_fmaf(ahi, bhi, s);
    }
#pragma unroll
    for (int off = LPR / 2; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    long rr = row + (long)u * RPB;
    if (sub == 0 && rr < rows) delta[rr] = s;
  }
}

}  // namespace

// o_is_f32: O points to float32 values (O_hp) instead of bf16.
hipError_t attn_delta_dispatch(const void* O, const void* dO, float* delta, long rows, int N, int d,
                               int o_is_f32, Layout lay, hipStream_t st) {
  constexpr int UNROLL = 4;
  if (rows == 0) return hipSuccess;
  if (d != 32 && d != 64 && d != 96 && d != 128 && d != 256) return hipErrorInvalidValue;
  const int rpb = 256 / ((d == 96 ? 128 : d) / 8) * UNROLL;
  dim3 grid((unsigned)((rows + rpb - 1) / rpb));
#define LAUNCH(DD, HP)                                                                          \
  hipLaunchKernelGGL((attn_delta_kernel<DD, UNROLL, HP>), grid, dim3(256), 0, st, O,           \
                     (const bf16_t*)dO, delta, rows, N, lay)
  if (d == 256) { if (o_is_f32) LAUNCH(256, true); else LAUNCH(256, false); }
  else if (d == 128) { if (o_is_f32) LAUNCH(128, true); else LAUNCH(128, false); }
  else if (d == 96) { if (o_is_f32) LAUNCH(96, true); else LAUNCH(96, false); }
  else if (d == 64) { if (o_is_f32) LAUNCH(64, true); else LAUNCH(64, false); }
  else              { if (o_is_f32) LAUNCH(32, true); else LAUNCH(32, false); }
#undef LAUNCH
  return hipGetLastError();
}
