// C ABI of the attention library (see include/attn.h): argument validation and dispatch only.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <cmath>
#include "../../include/attn.h"

// Mirrors the device-side struct of the same name (common.hpp): element (b,h,n,k) of a bf16
// tensor lives at b*sb + h*sh + n*sn + k.
struct Layout {
  long long sb, sh;
  int sn;
  int H;
  long long sb_kv, sh_kv;   // batch / head strides of K, V, dK, dV
  int group;                // query heads per key/value head
  int Nk;                   // rows of K, V, dK, dV per head (N counts the queries)
};

hipError_t attn_fwd_dispatch(const void*, const void*, const void*, void*, float*, int, int, int,
                             int, float, int, float, float, float*, int*, int*, int, Layout,
                             hipStream_t);
hipError_t attn_delta_dispatch(const void*, const void*, float*, long, int, int, int, Layout,
                               hipStream_t);
hipError_t attn_bwd_dkdv_dispatch(const void*, const void*, const void*, const void*, const float*,
                                  const float*, void*, void*, int, int, int, int, float, Layout,
                                  hipStream_t);
hipError_t attn_bwd_dq_dispatch(const void*, const void*, const void*, const void*, const float*,
                                const float*, const void*, void*, float*, int, int, int, int,
                                float, Layout, hipStream_t);
hipError_t attn_delta_recompute_dispatch(const void*, const void*, const void*, const void*,
                                         const float*, float*, int, int, int, int, float, Layout,
                                         hipStream_t);

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

Layout contiguous(int H, int N, int d, int H_kv = 0, int Nk = 0) {
  if (H_kv <= 0) H_kv = H;
  if (Nk <= 0) Nk = N;
  return Layout{(long long)H * N * d, (long long)N * d, d, H,
                (long long)H_kv * Nk * d, (long long)Nk * d, H / H_kv, Nk};
}

// Strides of the strided entry points: positive multiples of 8 elements (rows start on 16-byte
// boundaries), rows at least d apart, and small enough for the 32-bit per-lane offsets the tile
// loader uses inside a 64-row tile.
bool strides_ok(long long sb, long long sh, long long sn, int d) {
  if (sb <= 0 || sh <= 0 || sn <= 0) return false;
  if ((sb & 7) || (sh & 7) || (sn & 7)) return false;
  return sn >= d && sn < (1ll << 24);
}

// Shape check shared by all entry points.  Returns ATTN_OK with *empty = true for B*H == 0.
int check_shape(int B, int H, int N, int d, bool* empty) {
  *empty = false;
  if (B < 0 || H < 0 || N < 0 || d < 0) return ATTN_ERR_BAD_ARG;
  if (B == 0 || H == 0) { *empty = true; return ATTN_OK; }
  if (d != 32 && d != 64 && d != 96 && d != 128 && d != 256) return ATTN_ERR_UNSUPPORTED;
  if (N == 0) return ATTN_ERR_UNSUPPORTED;
  const double elems = (double)B * H * (double)N * d;
  if (elems >= 1099511627776.0) return ATTN_ERR_UNSUPPORTED;      // 2^40
  if ((double)B * H * ((N + 127) / 128) >= 2147483648.0) return ATTN_ERR_UNSUPPORTED;
  return ATTN_OK;
}

}  // namespace

extern "C" const char* attn_status_string(int status) {
  switch (status) {
    case ATTN_OK: return "ATTN_OK";
    case ATTN_ERR_NULL: return "ATTN_ERR_NULL: a required pointer is NULL";
    case ATTN_ERR_BAD_ARG: return "ATTN_ERR_BAD_ARG: invalid argument value or misaligned pointer";
    case ATTN_ERR_UNSUPPORTED: return "ATTN_ERR_UNSUPPORTED: d must be 32, 64, 96, 128 or 256 and N positive";
    case ATTN_ERR_WORKSPACE: return "ATTN_ERR_WORKSPACE: workspace too small or misaligned (attn_bwd_noalloc: B*H*N above attn_bwd_noalloc_max_rows())";
    case ATTN_ERR_LAUNCH: return "ATTN_ERR_LAUNCH: HIP launch failed";
    default: return "unknown attn_status";
  }
}

static int fwd_entry(const void* Q, const void* K, const void* V, void* O, float* LSE,
                     float* O_hp, int* ones_count, int* fired_count,
                     int B, int H, int N, int d, int causal, float softmax_scale,
                     int variant, float beta, float eps, unsigned flags, const Layout* user_lay,
                     void* stream) {
  bool empty;
  if (flags & ~(unsigned)(ATTN_FWD_SINGLE_ROUNDING | ATTN_FWD_PV_E4M3 | ATTN_FWD_GUARD_UNDERFLOW)) return ATTN_ERR_BAD_ARG;
  int st = check_shape(B, H, N, d, &empty);
  if (st != ATTN_OK) return st;
  if (variant < ATTN_VARIANT_STANDARD || variant > ATTN_VARIANT_MITIGATED_ROW) return ATTN_ERR_BAD_ARG;
  if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale)) return ATTN_ERR_BAD_ARG;
  if (variant != ATTN_VARIANT_STANDARD) {
    if (!(beta > 1.f) || !std::isfinite(beta)) return ATTN_ERR_BAD_ARG;
    if (!(eps >= 0.f) || !std::isfinite(eps)) return ATTN_ERR_BAD_ARG;
  }
  if (empty) return ATTN_OK;
  if (!Q || !K || !V || !O || !LSE) return ATTN_ERR_NULL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE))
    return ATTN_ERR_BAD_ARG;
  if (O == Q || O == K || O == V) return ATTN_ERR_BAD_ARG;
  if (!aligned16(O_hp) || !aligned16(ones_count) || !aligned16(fired_count)) return ATTN_ERR_BAD_ARG;
  if (O_hp && (O_hp == Q || O_hp == K || O_hp == V || O_hp == O)) return ATTN_ERR_BAD_ARG;
  if (ones_count && ones_count == fired_count) return ATTN_ERR_BAD_ARG;
  const Layout lay = user_lay ? *user_lay : contiguous(H, N, d);
  hipError_t e = attn_fwd_dispatch(Q, K, V, O, LSE, B * H, N, d, causal, softmax_scale, variant,
                                   beta, eps, O_hp, ones_count, fired_count,
                                   ((flags & ATTN_FWD_SINGLE_ROUNDING) ? 1 : 0) | ((flags & ATTN_FWD_PV_E4M3) ? 2 : 0) |
                                       ((flags & ATTN_FWD_GUARD_UNDERFLOW) ? 4 : 0), lay,
                                   static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" int attn_fwd_opt(const void* Q, const void* K, const void* V, void* O, float* LSE,
                            float* O_hp, int* ones_count, int* fired_count,
                            int B, int H, int N, int d, int causal, float softmax_scale,
                            int variant, float beta, float eps, unsigned flags, void* stream) {
  return fwd_entry(Q, K, V, O, LSE, O_hp, ones_count, fired_count, B, H, N, d, causal,
                   softmax_scale, variant, beta, eps, flags, nullptr, stream);
}

extern "C" int attn_fwd_strided(const void* Q, const void* K, const void* V, void* O, float* LSE,
                                long long stride_b, long long stride_h, long long stride_n,
                                int B, int H, int N, int d, int causal, float softmax_scale,
                                int variant, float beta, float eps, void* stream) {
  if (B < 0 || H < 0 || N < 0 || d < 0) return ATTN_ERR_BAD_ARG;
  if (!strides_ok(stride_b, stride_h, stride_n, d)) return ATTN_ERR_BAD_ARG;
  const Layout lay{stride_b, stride_h, (int)stride_n, H, stride_b, stride_h, 1, N};
  return fwd_entry(Q, K, V, O, LSE, nullptr, nullptr, nullptr, B, H, N, d, causal, softmax_scale,
                   variant, beta, eps, 0u, &lay, stream);
}

extern "C" int attn_fwd_ex(const void* Q, const void* K, const void* V, void* O, float* LSE,
                           int B, int H, int N, int d, int causal, float softmax_scale,
                           int variant, float beta, float eps, void* stream) {
  return attn_fwd_opt(Q, K, V, O, LSE, nullptr, nullptr, nullptr, B, H, N, d, causal,
                      softmax_scale, variant, beta, eps, 0u, stream);
}

extern "C" int attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B,
                        int H, int N, int d, int causal, float softmax_scale, int variant,
                        void* stream) {
  return attn_fwd_ex(Q, K, V, O, LSE, B, H, N, d, causal, softmax_scale, variant,
                     ATTN_DEFAULT_BETA, ATTN_DEFAULT_EPS, stream);
}

static int delta_entry(const void* O, const void* dO, float* delta, int B, int H, int N, int d,
                       int o_is_f32, void* stream) {
  bool empty;
  int st = check_shape(B, H, N, d, &empty);
  if (st != ATTN_OK) return st;
  if (empty) return ATTN_OK;
  if (!O || !dO || !delta) return ATTN_ERR_NULL;
  if (!aligned16(O) || !aligned16(dO) || !aligned16(delta)) return ATTN_ERR_BAD_ARG;
  if (static_cast<const void*>(delta) == O || static_cast<const void*>(delta) == dO) return ATTN_ERR_BAD_ARG;
  hipError_t e = attn_delta_dispatch(O, dO, delta, (long)B * H * N, N, d, o_is_f32,
                                     contiguous(H, N, d), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" int attn_delta(const void* O, const void* dO, float* delta, int B, int H, int N, int d,
                          void* stream) {
  return delta_entry(O, dO, delta, B, H, N, d, 0, stream);
}

extern "C" int attn_delta_hp(const float* O_hp, const void* dO, float* delta, int B, int H, int N,
                             int d, void* stream) {
  return delta_entry(O_hp, dO, delta, B, H, N, d, 1, stream);
}

extern "C" size_t attn_bwd_workspace_bytes(int B, int H, int N, int d) {
  bool empty;
  if (check_shape(B, H, N, d, &empty) != ATTN_OK || empty) return 0;
  size_t bytes = (size_t)B * H * N * sizeof(float);   // delta
  return (bytes + 255) & ~(size_t)255;
}

// Checks shared by attn_bwd and its two stage entry points.
static int check_bwd_common(int B, int H, int N, int d, float softmax_scale, bool* empty) {
  int st = check_shape(B, H, N, d, empty);
  if (st != ATTN_OK) return st;
  if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale)) return ATTN_ERR_BAD_ARG;
  return ATTN_OK;
}

extern "C" int attn_bwd_dkdv(const void* Q, const void* K, const void* V, const void* dO,
                             const float* LSE, const float* delta, void* dK, void* dV, int B,
                             int H, int N, int d, int causal, float softmax_scale, void* stream) {
  bool empty;
  int st = check_bwd_common(B, H, N, d, softmax_scale, &empty);
  if (st != ATTN_OK) return st;
  if (empty) return ATTN_OK;
  if (!Q || !K || !V || !dO || !LSE || !delta || !dK || !dV) return ATTN_ERR_NULL;
  const void* ptrs[] = {Q, K, V, dO, LSE, delta, dK, dV};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ATTN_ERR_BAD_ARG;
  const void* ins[] = {Q, K, V, dO};
  for (const void* p : ins)
    if (p == dK || p == dV) return ATTN_ERR_BAD_ARG;
  if (dK == dV) return ATTN_ERR_BAD_ARG;
  hipError_t e = attn_bwd_dkdv_dispatch(Q, K, V, dO, LSE, delta, dK, dV, B * H, N, d, causal,
                                        softmax_scale, contiguous(H, N, d),
                                        static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" int attn_bwd_dq(const void* Q, const void* K, const void* V, const void* dO,
                           const float* LSE, const float* delta, void* dQ, int B, int H, int N,
                           int d, int causal, float softmax_scale, void* stream) {
  bool empty;
  int st = check_bwd_common(B, H, N, d, softmax_scale, &empty);
  if (st != ATTN_OK) return st;
  if (empty) return ATTN_OK;
  if (!Q || !K || !V || !dO || !LSE || !delta || !dQ) return ATTN_ERR_NULL;
  const void* ptrs[] = {Q, K, V, dO, LSE, delta, dQ};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ATTN_ERR_BAD_ARG;
  const void* ins[] = {Q, K, V, dO};
  for (const void* p : ins)
    if (p == dQ) return ATTN_ERR_BAD_ARG;
  hipError_t e = attn_bwd_dq_dispatch(Q, K, V, dO, LSE, delta, nullptr, dQ, nullptr, B * H, N, d,
                                      causal, softmax_scale, contiguous(H, N, d),
                                      static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" int attn_bwd_dq_delta(const void* Q, const void* K, const void* V, const void* O,
                                 const void* dO, const float* LSE, void* dQ, float* delta, int B,
                                 int H, int N, int d, int causal, float softmax_scale,
                                 void* stream) {
  bool empty;
  int st = check_bwd_common(B, H, N, d, softmax_scale, &empty);
  if (st != ATTN_OK) return st;
  if (empty) return ATTN_OK;
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !delta) return ATTN_ERR_NULL;
  const void* ptrs[] = {Q, K, V, O, dO, LSE, dQ, delta};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ATTN_ERR_BAD_ARG;
  const void* ins[] = {Q, K, V, O, dO, LSE};
  for (const void* p : ins)
    if (p == dQ || p == static_cast<const void*>(delta)) return ATTN_ERR_BAD_ARG;
  if (dQ == static_cast<void*>(delta)) return ATTN_ERR_BAD_ARG;
  hipError_t e = attn_bwd_dq_dispatch(Q, K, V, dO, LSE, nullptr, O, dQ, delta, B * H, N, d, causal,
                                      softmax_scale, contiguous(H, N, d),
                                      static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

static int bwd_entry(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                     const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                     size_t workspace_bytes, int B, int H, int N, int d, int causal,
                     float softmax_scale, int variant, const Layout* user_lay, void* stream) {
  bool empty;
  int st = check_shape(B, H, N, d, &empty);
  if (st != ATTN_OK) return st;
  if (variant < ATTN_VARIANT_STANDARD || variant > ATTN_VARIANT_MITIGATED_ROW) return ATTN_ERR_BAD_ARG;
  if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale)) return ATTN_ERR_BAD_ARG;
  if (empty) return ATTN_OK;
  if (!Q || !K || !V || !O || !dO || !LSE || !dQ || !dK || !dV) return ATTN_ERR_NULL;
  const void* ptrs[] = {Q, K, V, O, dO, LSE, dQ, dK, dV};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ATTN_ERR_BAD_ARG;
  const void* ins[] = {Q, K, V, O, dO};
  for (const void* p : ins)
    if (p == dQ || p == dK || p == dV) return ATTN_ERR_BAD_ARG;
  if (dQ == dK || dQ == dV || dK == dV) return ATTN_ERR_BAD_ARG;
  if (!workspace) return ATTN_ERR_NULL;
  if (workspace_bytes < attn_bwd_workspace_bytes(B, H, N, d) ||
      (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return ATTN_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* delta = static_cast<float*>(workspace);
  const Layout lay = user_lay ? *user_lay : contiguous(H, N, d);
  // the dQ kernel forms delta = rowsum(dO o O) for its own rows (Alg. 2 step 4) and leaves it in
  // the workspace for the dK/dV kernel: no separate pass over O and dO
  hipError_t e = attn_bwd_dq_dispatch(Q, K, V, dO, LSE, nullptr, O, dQ, delta, B * H, N, d, causal,
                                      softmax_scale, lay, s);
  if (e != hipSuccess) return ATTN_ERR_LAUNCH;
  e = attn_bwd_dkdv_dispatch(Q, K, V, dO, LSE, delta, dK, dV, B * H, N, d, causal, softmax_scale, lay, s);
  return e == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

extern "C" int attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                        const float* LSE, void* dQ, void* dK, void* dV, void* workspace,
                        size_t workspace_bytes, int B, int H, int N, int d, int causal,
                        float softmax_scale, int variant, void* stream) {
  return bwd_entry(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, H, N, d, causal,
                   softmax_scale, variant, nullptr, stream);
}

// ---- attn_bwd for callers that cannot allocate.  delta, the one buffer attn_bwd takes through its
// workspace argument, lives in a device array of this library instead: one copy per GPU, at an
// address of its own on each, held until the process ends.
constexpr size_t kScratchRows = (size_t)1 << 20;                  // B*H*N at most; 4 MiB of float32
static __device__ __align__(256) float scratch[kScratchRows];
constexpr int kMaxDevices = 64;
static std::atomic<float*> scratch_ptr[kMaxDevices];             // device address of `scratch`, per GPU

// Device address of this GPU's copy of `scratch` (looked up once per device, with that device
// current; in host code the array's name is only a handle for this lookup).
static int scratch_address(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ATTN_ERR_LAUNCH;
  float* p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    void* sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || sym == nullptr) return ATTN_ERR_LAUNCH;
    p = static_cast<float*>(sym);
    scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return ATTN_OK;
}

extern "C" size_t attn_bwd_noalloc_max_rows(void) { return kScratchRows; }

extern "C" int attn_bwd_noalloc(const void* Q, const void* K, const void* V, const void* O,
                                const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                                int B, int H, int N, int d, int causal, float softmax_scale,
                                int variant, void* stream) {
  bool empty;
  int st = check_shape(B, H, N, d, &empty);
  if (st != ATTN_OK) return st;
  if (!empty && (size_t)B * H * (size_t)N > kScratchRows) return ATTN_ERR_WORKSPACE;
  float* delta = nullptr;
  if (!empty && (st = scratch_address(&delta)) != ATTN_OK) return st;
  // every row of delta that the dK/dV kernel reads is written by the dQ kernel first: nothing
  // needs clearing between calls
  return bwd_entry(Q, K, V, O, dO, LSE, dQ, dK, dV, empty ? nullptr : delta,
                   kScratchRows * sizeof(float), B, H, N, d, causal, softmax_scale, variant, nullptr,
                   stream);
}

extern "C" int attn_bwd_strided(const void* Q, const void* K, const void* V, const void* O,
                                const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                                void* workspace, size_t workspace_bytes,
                                long long stride_b, long long stride_h, long long stride_n,
                                int B, int H, int N, int d, int causal, float softmax_scale,
                                int variant, void* stream) {
  if (B < 0 || H < 0 || N < 0 || d < 0) return ATTN_ERR_BAD_ARG;
  if (!strides_ok(stride_b, stride_h, stride_n, d)) return ATTN_ERR_BAD_ARG;
  const Layout lay{stride_b, stride_h, (int)stride_n, H, stride_b, stride_h, 1, N};
  return bwd_entry(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, H, N, d, causal,
                   softmax_scale, variant, &lay, stream);
}

extern "C" int attn_delta_recompute(const void* Q, const void* K, const void* V, const void* dO,
                                    const float* LSE, float* delta, int B, int H, int N, int d,
                                    int causal, float softmax_scale, void* stream) {
  bool empty;
  int st = check_bwd_common(B, H, N, d, softmax_scale, &empty);
  if (st != ATTN_OK) return st;
  if (empty) return ATTN_OK;
  if (!Q || !K || !V || !dO || !LSE || !delta) return ATTN_ERR_NULL;
  const void* ptrs[] = {Q, K, V, dO, LSE, delta};
  for (const void* p : ptrs)
    if (!aligned16(p)) return ATTN_ERR_BAD_ARG;
  for (int i = 0; i < 5; ++i)
    if (ptrs[i] == static_cast<const void*>(delta)) return ATTN_ERR_BAD_ARG;
  hipError_t e = attn_delta_recompute_dispatch(Q, K, V, dO, LSE, delta, B * H, N, d, causal,
                                               softmax_scale, contiguous(H, N, d),
                                               static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ATTN_OK : ATTN_ERR_LAUNCH;
}

// Grouped-query attention: H query heads, H_kv key/value heads.
static bool gqa_heads_ok(int H, int H_kv) { return H_kv >= 1 && H >= H_kv && H % H_kv == 0; }

extern "C" int attn_fwd_gqa(const void* Q, const void* K, const void* V, void* O, float* LSE,
                            int B, int H, int H_kv, int N, int d, int causal, float softmax_scale,
                            int variant, float beta, float eps, void* stream) {
  if (B < 0 || H < 0 || H_kv < 0 || N < 0 || d < 0) return ATTN_ERR_BAD_ARG;
  if (B > 0 && H > 0 && !gqa_heads_ok(H, H_kv)) return ATTN_ERR_BAD_ARG;
  const Layout lay = (B > 0 && H > 0) ? contiguous(H, N, d, H_kv) : contiguous(1, N, d);
  return fwd_entry(Q, K, V, O, LSE, nullptr, nullptr, nullptr, B, H, N, d, causal, softmax_scale,
                   variant, beta, eps, 0u, &lay, stream);
}

extern "C" int attn_bwd_gqa(const void* Q, const void* K, const void* V, const void* O,
                            const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                            void* workspace, size_t workspace_bytes, int B, int H, int H_kv, int N,
                            int d, int causal, float softmax_scale, int variant, void* stream) {
  if (B < 0 || H < 0 || H_kv < 0 || N < 0 || d < 0) return ATTN_ERR_BAD_ARG;
  if (B > 0 && H > 0 && !gqa_heads_ok(H, H_kv)) return ATTN_ERR_BAD_ARG;
  const Layout lay = (B > 0 && H > 0) ? contiguous(H, N, d, H_kv) : contiguous(1, N, d);
  return bwd_entry(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, H, N, d, causal,
                   softmax_scale, variant, &lay, stream);
}

// Different numbers of queries and keys.
static int check_rect(int B, int H, int Nq, int Nk, int d) {
  if (B < 0 || H < 0 || Nq < 0 || Nk < 0 || d < 0) return ATTN_ERR_BAD_ARG;
  bool empty;
  int st = check_shape(B, H, Nk, d, &empty);      // size limits also for the key side
  if (st != ATTN_OK) return st;
  return ATTN_OK;
}

extern "C" int attn_fwd_rect(const void* Q, const void* K, const void* V, void* O, float* LSE,
                             int B, int H, int Nq, int Nk, int d, int causal, float softmax_scale,
                             int variant, float beta, float eps, void* stream) {
  int st = check_rect(B, H, Nq, Nk, d);
  if (st != ATTN_OK) return st;
  const Layout lay = (B > 0 && H > 0) ? contiguous(H, Nq, d, 0, Nk) : contiguous(1, 1, d);
  return fwd_entry(Q, K, V, O, LSE, nullptr, nullptr, nullptr, B, H, Nq, d, causal, softmax_scale,
                   variant, beta, eps, 0u, &lay, stream);
}

extern "C" int attn_bwd_rect(const void* Q, const void* K, const void* V, const void* O,
                             const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                             void* workspace, size_t workspace_bytes, int B, int H, int Nq, int Nk,
                             int d, int causal, float softmax_scale, int variant, void* stream) {
  int st = check_rect(B, H, Nq, Nk, d);
  if (st != ATTN_OK) return st;
  const Layout lay = (B > 0 && H > 0) ? contiguous(H, Nq, d, 0, Nk) : contiguous(1, 1, d);
  return bwd_entry(Q, K, V, O, dO, LSE, dQ, dK, dV, workspace, workspace_bytes, B, H, Nq, d, causal,
                   softmax_scale, variant, &lay, stream);
}
