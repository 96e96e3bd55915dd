/*
 * attn.h -- C ABI of the MI355X (gfx950) bf16 flash-attention library.
 *
 * What is computed (paper = "Why Low-Precision Transformer Training Fails: An Analysis on
 * Flash Attention", arXiv 2510.04212):
 *   forward   O = softmax(alpha Q K^T) V  and  L = rowwise logsumexp(alpha Q K^T)
 *             by the tiled online-softmax algorithm (Alg. 1), or by its stabilised form
 *             (Alg. 3, Sec. 4) which moves the softmax normaliser away from a repeated
 *             row maximum so that no unnormalised probability is exactly 1;
 *   backward  delta = rowsum(dO o O), P = exp(S - L), dV = P^T dO, dP = dO V^T,
 *             dS = P o (dP - delta), dQ = alpha dS K, dK = alpha dS^T Q   (Alg. 2, Eq. 2).
 *
 * Conventions shared by every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller.  The library never allocates,
 *     frees, copies to the host or synchronises; all work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and the call returns at once.
 *   - Layout: contiguous [B][H][N][d], d fastest.  Q, K, V, O, dO, dQ, dK, dV are bfloat16;
 *     LSE and delta are float32 [B][H][N].  Pointers must be 16-byte aligned.  Outputs must not
 *     alias inputs.
 *   - Self-attention: N queries and N keys.  causal != 0: query r attends to keys c <= r.
 *   - Supported shapes: d in {32, 64, 96, 128, 256}; any N >= 1 (N need not be a multiple of a tile: the
 *     kernels clamp their reads to row N-1 and store nothing past it); B*H*N*d < 2^40.
 *     B == 0 or H == 0 is a no-op that returns ATTN_OK.  Anything else: ATTN_ERR_UNSUPPORTED.
 *   - Return value: an attn_status.  No exceptions, aborts or global mutable state.
 *   - Arithmetic: bf16 matrix-core products with float32 accumulation; scores, softmax
 *     statistics and LSE in float32; the rounding points follow Sec. 3.3.2 of the paper:
 *     the unnormalised probabilities P-bar are rounded to bf16 before use (and their rounded
 *     values are what the row sum l adds up), the unnormalised output P-bar V is accumulated
 *     in float32 over all key tiles, rounded to bf16 ONCE, then divided by l and rounded to
 *     bf16 again.
 */
#ifndef PAPER_2510_04212_ATTN_H
#define PAPER_2510_04212_ATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ATTN_OK = 0,
  ATTN_ERR_NULL = 1,         /* a required pointer is NULL */
  ATTN_ERR_BAD_ARG = 2,      /* negative size, misaligned pointer, bad variant/beta/eps/scale */
  ATTN_ERR_UNSUPPORTED = 3,  /* shape outside the supported set (see above) */
  ATTN_ERR_WORKSPACE = 4,    /* workspace smaller than attn_bwd_workspace_bytes() */
  ATTN_ERR_LAUNCH = 5        /* the HIP runtime refused a launch (hipGetLastError) */
} attn_status;

enum {
  ATTN_VARIANT_STANDARD = 0,  /* Alg. 1: safe softmax, normaliser = running row maximum */
  ATTN_VARIANT_MITIGATED = 1, /* Alg. 3: normaliser beta*r_m (r_m > 0) or 0 (r_m < 0) whenever a
                                 key tile's row maximum r_m is attained (within eps) more than once */
  ATTN_VARIANT_MITIGATED_ROW = 2 /* the same rule applied to the WHOLE row (the paper's untiled
                                 form, Sec. 4: r_m and the count are taken over all keys), so the
                                 result does not depend on the key-tile size.  Two passes: the two
                                 largest scores of every row are found first (a repeated maximum
                                 <=> the second largest lies within eps of the largest), then the
                                 forward runs with that fixed normaliser.  Costs one extra
                                 Q K^T product; LSE[] is used as scratch between the passes. */
};

/* Default parameters of the stabilised forward (Sec. 4: beta in [2,8], beta = 2 in the paper's
 * training runs; eps "e.g. 1e-3"). */
#define ATTN_DEFAULT_BETA 2.0f
#define ATTN_DEFAULT_EPS 1e-3f

/* Key-tile size B_c used by the forward kernel for head dimension d (0 if d is unsupported).
 * Alg. 3 looks for a repeated maximum inside one key tile of one row, so its result depends on
 * B_c; tiles start at multiples of B_c. */
int attn_fwd_key_tile(int d);

/*
 * Forward pass (Alg. 1 / Alg. 3).
 *   in : Q, K, V   bf16 [B,H,N,d]
 *   out: O         bf16 [B,H,N,d];  LSE float32 [B,H,N] = m + log(l) in natural-log units of
 *                  the alpha-scaled scores
 *   softmax_scale  alpha > 0, multiplies the float32 Q K^T (Q is never pre-scaled in bf16)
 *   variant        ATTN_VARIANT_*; attn_fwd uses ATTN_DEFAULT_BETA / ATTN_DEFAULT_EPS
 * attn_fwd_ex additionally takes beta > 1 and eps >= 0 (both ignored by the standard variant).
 * eps and the sign tests of Alg. 3 apply to the alpha-scaled scores.
 * Note (Sec. 4, "larger values risk underflow"): when a repeated maximum satisfies
 * (beta-1)*r_m > ~87.3, every exp underflows (the hardware exponential returns 0 below 2^-126),
 * l = 0, that row of O is NaN and its LSE is -inf -- which is how a caller can detect it: with
 * N queries and N keys no other row has LSE = -inf.  This is the algorithm's own limit and is
 * not masked here; attn_fwd_opt has an opt-in guard (ATTN_FWD_GUARD_UNDERFLOW).
 */
int attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
             int B, int H, int N, int d, int causal, float softmax_scale, int variant,
             void* stream);
int attn_fwd_ex(const void* Q, const void* K, const void* V, void* O, float* LSE,
                int B, int H, int N, int d, int causal, float softmax_scale, int variant,
                float beta, float eps, void* stream);

/*
 * Forward pass with the switches and side outputs of the paper's isolation experiments
 * (Sec. 3.2, Sec. 3.3.2) and its tie statistics (Sec. 3.3.2, Sec. 4).  Same arithmetic, layouts,
 * checks and error codes as attn_fwd_ex; in addition
 *   O_hp         optional (NULL = off) float32 [B,H,N,d]: accumulator / l with NO bf16 rounding,
 *                i.e. the "O computed in high precision" from which delta_hp is formed
 *                (attn_delta_hp); O and LSE are written as usual.
 *   ones_count   optional int32 [B,H,N]: per query row, the number of keys whose P-bar, after
 *                rounding to bf16, was exactly 1 when it was produced (the precondition of the
 *                biased rounding, Claim 3).
 *   fired_count  optional int32 [B,H,N]: per query row, the number of key tiles in which the
 *                rule of Alg. 3 replaced the row maximum as normaliser (always 0 for the
 *                standard variant).
 *   flags        ATTN_FWD_SINGLE_ROUNDING: the unnormalised output is NOT rounded to bf16 before
 *                the division by l ("computing only O-bar = P-bar V in FP32", Sec. 3.3.2); O is
 *                still stored as bf16.
 *                ATTN_FWD_PV_E4M3: an exploration beyond the paper (its closing remark on FP8):
 *                the P-bar V product takes both operands in the 8-bit format E4M3 -- P-bar is
 *                rounded to E4M3 instead of bf16, V is quantised to E4M3 without a scale
 *                factor -- on the FP8 matrix instruction, sums in float32; the row sum l is of
 *                the rounded P-bar, ones_count counts its unit entries, everything else is
 *                unchanged.  The backward pass has no such mode.
 *                ATTN_FWD_GUARD_UNDERFLOW: a labelled deviation from Alg. 3, NOT part of the paper
 *                (which only warns, Sec. 4, that a larger beta risks underflow): the rule is
 *                skipped -- the tile row keeps its maximum r_m as normaliser, as in Alg. 1 -- where
 *                it would move the normaliser by more than 60 ((beta-1) r_m > 60 for a positive
 *                repeated maximum, r_m < -60 for a negative one).  Without the flag such a row
 *                loses every probability once the move exceeds ~87.3 (the hardware exponential
 *                returns 0 below 2^-126): l = 0, the row of O is NaN, its LSE is -inf, and a
 *                backward pass fed with them returns NaN in dQ of that row and in dK / dV of
 *                every key the row attends to.  fired_count does not count skipped tiles.
 *                Other bits: ATTN_ERR_BAD_ARG.
 * Optional pointers must be 16-byte aligned and must not alias any other argument.
 */
#define ATTN_FWD_SINGLE_ROUNDING 1u
#define ATTN_FWD_PV_E4M3 2u
#define ATTN_FWD_GUARD_UNDERFLOW 4u
int attn_fwd_opt(const void* Q, const void* K, const void* V, void* O, float* LSE,
                 float* O_hp, int* ones_count, int* fired_count,
                 int B, int H, int N, int d, int causal, float softmax_scale, int variant,
                 float beta, float eps, unsigned flags, void* stream);

/*
 * delta = rowsum(dO o O)  (Alg. 2, step 4), float32 [B,H,N], from the bf16 O the forward pass
 * stored (the low-precision delta of Claim 1).  Products and the row sum are float32.
 * A pure streaming pass, bound by HBM bandwidth.
 */
int attn_delta(const void* O, const void* dO, float* delta, int B, int H, int N, int d,
               void* stream);

/*
 * delta_hp = rowsum(dO o O_hp) from the float32 O_hp of attn_fwd_opt (Sec. 3.2: using the
 * high-precision output in delta, everything else unchanged, restores stability).  Feed the
 * result to attn_bwd_dkdv / attn_bwd_dq in place of attn_delta's.
 */
int attn_delta_hp(const float* O_hp, const void* dO, float* delta, int B, int H, int N, int d,
                  void* stream);

/*
 * delta = rowsum(P o dP) with P = exp(alpha Q K^T - LSE) and dP = dO V^T recomputed in float32
 * (Sec. 3.2: recomputing the output inside the backward pass instead of reading the forward's
 * bf16 O stabilises training; rowsum(P o dP) = rowsum(dO o (P V)) is that quantity without ever
 * forming O).  Costs two of the backward's matrix products again.  Inputs as for attn_bwd_dq;
 * delta float32 [B,H,N] is written.  Feed it to attn_bwd_dkdv / attn_bwd_dq.
 */
int attn_delta_recompute(const void* Q, const void* K, const void* V, const void* dO,
                         const float* LSE, float* delta, int B, int H, int N, int d, int causal,
                         float softmax_scale, void* stream);

/*
 * Backward pass (Alg. 2).
 *   in : Q, K, V, O, dO  bf16 [B,H,N,d];  LSE float32 [B,H,N] from attn_fwd
 *   out: dQ, dK, dV      bf16 [B,H,N,d]
 *   workspace            device scratch of at least attn_bwd_workspace_bytes(B,H,N,d) bytes,
 *                        256-byte aligned; holds delta [B,H,N] float32 (readable by the caller
 *                        after the call: it starts at offset 0).  Contents on entry are ignored.
 *   variant              accepted for symmetry and validated, but has no effect: Alg. 3 leaves the
 *                        backward pass unchanged (Sec. 4).
 * P = exp(S - L) is rounded to bf16 as the operand of P^T dO; dS = P o (dP - delta) uses the
 * float32 P and is rounded to bf16 as the operand of dS K and dS^T Q; alpha multiplies the
 * float32 dQ / dK accumulators once; results are rounded to bf16 when stored.
 * Deterministic: no atomics, results are bit-identical from run to run.
 */
int attn_bwd(const void* Q, const void* K, const void* V, const void* O, const void* dO,
             const float* LSE, void* dQ, void* dK, void* dV,
             void* workspace, size_t workspace_bytes,
             int B, int H, int N, int d, int causal, float softmax_scale, int variant,
             void* stream);
size_t attn_bwd_workspace_bytes(int B, int H, int N, int d);

/*
 * attn_bwd for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * arithmetic, kernels, checks and error codes as attn_bwd, minus the workspace: delta lives in a
 * 4 MiB device array inside the library (one copy per GPU, held until the process ends).
 *   - B*H*N must not exceed attn_bwd_noalloc_max_rows() (2^20 rows): ATTN_ERR_WORKSPACE otherwise.
 *   - The call allocates nothing, frees nothing and does not synchronise.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time on the same GPU
 *     (different streams, or graphs replayed concurrently) race on it and must be serialised by
 *     the caller.  Nothing needs to be cleared between calls: every value read is written by the
 *     same call first.
 */
int attn_bwd_noalloc(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                     const float* LSE, void* dQ, void* dK, void* dV,
                     int B, int H, int N, int d, int causal, float softmax_scale, int variant,
                     void* stream);
size_t attn_bwd_noalloc_max_rows(void);

/*
 * The stages of attn_bwd, exposed separately so that a caller can time them or feed them
 * another delta.  attn_bwd == attn_bwd_dq_delta (delta into the workspace), then attn_bwd_dkdv;
 * attn_delta, then attn_bwd_dkdv and attn_bwd_dq in either order, gives the same bits.
 * `delta` is float32 [B,H,N].  Same layouts, checks and error codes as attn_bwd.
 *   attn_bwd_dkdv      Alg. 2 steps 8-12 and 10/14 for one key block per work-group:
 *                      S = Q K^T, P = exp(S - L), dP = dO V^T, dS = P o (dP - delta),
 *                      dV = P^T dO, dK = alpha dS^T Q.  `delta` is an input.
 *   attn_bwd_dq        Alg. 2 steps 8-13 for one query block per work-group (S and dP recomputed):
 *                      dQ = alpha dS K.  `delta` is an input.
 *   attn_bwd_dq_delta  the same, and Alg. 2 step 4 on the way: each work-group first forms
 *                      delta = rowsum(dO o O) for its own query rows (it holds their dO already),
 *                      writes it to `delta` (an OUTPUT here) and uses it.  The sum is taken in
 *                      attn_delta's order: identical bits, one pass over O and dO saved.
 */
int attn_bwd_dkdv(const void* Q, const void* K, const void* V, const void* dO, const float* LSE,
                  const float* delta, void* dK, void* dV,
                  int B, int H, int N, int d, int causal, float softmax_scale, void* stream);
int attn_bwd_dq(const void* Q, const void* K, const void* V, const void* dO, const float* LSE,
                const float* delta, void* dQ,
                int B, int H, int N, int d, int causal, float softmax_scale, void* stream);
int attn_bwd_dq_delta(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                      const float* LSE, void* dQ, float* delta,
                      int B, int H, int N, int d, int causal, float softmax_scale, void* stream);

/*
 * Strided forms of attn_fwd_ex and attn_bwd: element (b, h, n, k) of every bf16 tensor of the
 * call (Q, K, V, O, dO, dQ, dK, dV) lives at  base + b*stride_b + h*stride_h + n*stride_n + k
 * (strides in elements, the last dimension contiguous, the same three strides for all tensors
 * of the call).  [B,H,N,d] contiguous is (H*N*d, N*d, d) and is what the other entry points use;
 * [B,N,H,d] contiguous is (N*H*d, d, H*d); views into a fused projection buffer work as well.
 * LSE and the workspace's delta stay float32 [B,H,N] contiguous.
 * Strides must be positive multiples of 8 (every row starts on a 16-byte boundary) with
 * d <= stride_n < 2^24, otherwise ATTN_ERR_BAD_ARG; that the strides describe non-overlapping
 * memory inside the caller's allocations is the caller's responsibility.  Same arithmetic as
 * the contiguous entry points: for equal values the results are bit-identical.
 */
int attn_fwd_strided(const void* Q, const void* K, const void* V, void* O, float* LSE,
                     long long stride_b, long long stride_h, long long stride_n,
                     int B, int H, int N, int d, int causal, float softmax_scale, int variant,
                     float beta, float eps, void* stream);
int attn_bwd_strided(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                     const float* LSE, void* dQ, void* dK, void* dV,
                     void* workspace, size_t workspace_bytes,
                     long long stride_b, long long stride_h, long long stride_n,
                     int B, int H, int N, int d, int causal, float softmax_scale, int variant,
                     void* stream);

/*
 * Grouped-query attention (multi-query when H_kv == 1): Q, O, dO, dQ have H heads, K, V, dK, dV
 * have H_kv heads, H a multiple of H_kv; query head h attends to key/value head h / (H / H_kv).
 * Contiguous layouts [B,H,N,d] and [B,H_kv,N,d]; LSE and the workspace's delta are [B,H,N].
 * Forward and dQ are the ordinary kernels reading the shared head; dK and dV are accumulated in
 * float32 over the query heads of a group inside one work-group and rounded to bf16 once.
 * H_kv == H is exactly attn_fwd_ex / attn_bwd.  ATTN_ERR_BAD_ARG if H is not a multiple of H_kv.
 */
int attn_fwd_gqa(const void* Q, const void* K, const void* V, void* O, float* LSE,
                 int B, int H, int H_kv, int N, int d, int causal, float softmax_scale, int variant,
                 float beta, float eps, void* stream);
int attn_bwd_gqa(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                 const float* LSE, void* dQ, void* dK, void* dV,
                 void* workspace, size_t workspace_bytes,
                 int B, int H, int H_kv, int N, int d, int causal, float softmax_scale, int variant,
                 void* stream);

/*
 * Different numbers of queries and keys: Q, O, dO, dQ are [B,H,Nq,d], K, V, dK, dV are
 * [B,H,Nk,d] (contiguous), LSE and the workspace's delta are [B,H,Nq]; the workspace size is
 * attn_bwd_workspace_bytes(B, H, Nq, d).  The algorithms are those of attn_fwd_ex / attn_bwd
 * (Alg. 1 / 3 and Alg. 2 are written for any pair of lengths).  The paper does not say how a
 * causal mask is placed on a rectangular score matrix; it is aligned at the bottom right here:
 * query r sees keys c <= r + (Nk - Nq), so that the last query sees every key (Nq < Nk is a
 * chunk of queries at the end of a longer sequence).  With Nq > Nk the first Nq - Nk queries see
 * no key at all: their rows of O and dQ are 0, their LSE is -infinity, and they add nothing to
 * dK, dV.  Nq == Nk is exactly attn_fwd_ex / attn_bwd.  Nq, Nk >= 1; same checks and error codes
 * otherwise.
 */
int attn_fwd_rect(const void* Q, const void* K, const void* V, void* O, float* LSE,
                  int B, int H, int Nq, int Nk, int d, int causal, float softmax_scale, int variant,
                  float beta, float eps, void* stream);
int attn_bwd_rect(const void* Q, const void* K, const void* V, const void* O, const void* dO,
                  const float* LSE, void* dQ, void* dK, void* dV,
                  void* workspace, size_t workspace_bytes,
                  int B, int H, int Nq, int Nk, int d, int causal, float softmax_scale, int variant,
                  void* stream);

/* Human-readable name of an attn_status (static storage, never NULL). */
const char* attn_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif
