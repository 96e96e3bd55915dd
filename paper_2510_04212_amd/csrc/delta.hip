// delta = rowsum(dO o O)  (Alg. 2 step 4 of arXiv 2510.04212): one float32 per row from the
// bf16 O and dO.  Pure streaming: 4d bytes read and 4 bytes written per row, HBM-bound.
// D/8 lanes cooperate on one row (16 bytes each of O and of dO); the partial sums are combined
// with lane shuffles inside the group.
#include "common.hpp"

namespace {

template <int D, int UNROLL>
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16_t* __restrict__ O,
                                                         const bf16_t* __restrict__ dO,
                                                         float* __restrict__ delta, long rows) {
  constexpr int LPR = D / 8;             // lanes per row
  constexpr int RPB = 256 / LPR;         // rows per block per step
  const int sub = threadIdx.x % LPR;
  const int rib = threadIdx.x / LPR;
  long row = (long)blockIdx.x * (RPB * UNROLL) + rib;
  u32x4 a[UNROLL], b[UNROLL];
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    long rr = row + (long)u * RPB;
    if (rr < rows) {
      a[u] = *reinterpret_cast<const u32x4*>(O + rr * D + sub * 8);
      b[u] = *reinterpret_cast<const u32x4*>(dO + rr * D + sub * 8);
    } else {
      a[u] = u32x4{0, 0, 0, 0};
      b[u] = u32x4{0, 0, 0, 0};
    }
  }
#pragma unroll
  for (int u = 0; u < UNROLL; ++u) {
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      float alo = __uint_as_float(a[u][w] << 16), ahi = __uint_as_float(a[u][w] & 0xFFFF0000u);
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

hipError_t attn_delta_dispatch(const void* O, const void* dO, float* delta, long rows, int d,
                               hipStream_t st) {
  constexpr int UNROLL = 4;
  if (rows == 0) return hipSuccess;
  if (d == 128) {
    constexpr int RPB = 256 / 16 * UNROLL;
    dim3 grid((unsigned)((rows + RPB - 1) / RPB));
    hipLaunchKernelGGL((attn_delta_kernel<128, UNROLL>), grid, dim3(256), 0, st,
                       (const bf16_t*)O, (const bf16_t*)dO, delta, rows);
  } else if (d == 64) {
    constexpr int RPB = 256 / 8 * UNROLL;
    dim3 grid((unsigned)((rows + RPB - 1) / RPB));
    hipLaunchKernelGGL((attn_delta_kernel<64, UNROLL>), grid, dim3(256), 0, st,
                       (const bf16_t*)O, (const bf16_t*)dO, delta, rows);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
