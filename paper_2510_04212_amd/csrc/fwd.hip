// Flash-attention forward for gfx950: Alg. 1 (standard safe softmax) and Alg. 3 (stabilised
// normaliser, Sec. 4) of arXiv 2510.04212, one work-group per (batch, head, 128-query block).
//
// Work split: 4 waves, each owning 32 query rows; key tiles of B_c = 64 rows of K and V are
// staged in LDS (double buffered) and shared by the 4 waves.  Per tile a wave computes
//     S^T[key][query] = K_j Q_i^T           (A = K_j from LDS, B = Q_i^T held in registers)
// so that one query row lives in lane r and lane r+32; row max / row sum / near-max count are
// in-register reductions plus one exchange with the partner lane.  P-bar^T in the accumulator
// layout is directly the B operand of
//     O^T[d][query] += V_j^T P-bar^T          (A = V_j^T via transposing LDS reads)
// which keeps the per-query rescale factor uniform over a lane's accumulator registers.
#include "common.hpp"

#include <atomic>
#include <type_traits>

namespace {

constexpr int kBr = 128;   // query rows per work-group
constexpr int kBc = 64;    // key rows per tile

// Optional outputs and switches of the forward (the experiments of Sec. 3.2 / 3.3.2 and the
// tie statistics of Sec. 3.3.2 / 4).  Only kernels instantiated with EXTRAS look at them.
struct FwdExtras {
  float* O_hp;          // [B,H,N,d] float32: accumulator / l with no bf16 rounding, or null
  int* ones;            // [B,H,N]: number of keys whose rounded P-bar was exactly 1, or null
  int* fired;           // [B,H,N]: number of key tiles in which Alg. 3 moved the normaliser, or null
  int single_rounding;  // nonzero: O-bar is NOT rounded to bf16 before the division by l
  int pv_e4m3;          // nonzero: the P-bar V product takes both operands in 8-bit E4M3
  int guard;            // nonzero: Alg. 3's rule is not applied where it would move the normaliser
                        // by more than kGuardLimit (a labelled deviation from Sec. 4, see attn.h)
};

// Largest move of the normaliser the guarded form of Alg. 3 makes, in natural-log units of the
// alpha-scaled scores: the row maximum then still maps to exp(-60) ~ 9e-27, far above the point
// where the hardware exponential returns 0 (2^-126).
constexpr float kGuardLimit = 60.0f;
DEVI bool guard_allows(float r_m, float beta) {
  const float shift_by = r_m > 0.f ? (beta - 1.0f) * r_m : -r_m;
  return shift_by <= kGuardLimit;
}

// Eight float32 values -> eight E4M3 bytes (hardware conversion: round to nearest even).
DEVI long pack_e4m3(const float (&v)[8]) {
  int w0 = 0, w1 = 0;
  w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[0], v[1], w0, false);
  w0 = __builtin_amdgcn_cvt_pk_fp8_f32(v[2], v[3], w0, true);
  w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[4], v[5], w1, false);
  w1 = __builtin_amdgcn_cvt_pk_fp8_f32(v[6], v[7], w1, true);
  return (long)(((unsigned long long)(unsigned)w1 << 32) | (unsigned)w0);
}

// VARIANT: 0 = Alg. 1, 1 = Alg. 3 (repeated maximum looked for inside each key tile, as the
// algorithm is written), and the two passes of the tile-size-independent form of Alg. 3
// (the rule of Sec. 4 applied to the whole row, as in the paper's untiled analysis):
//   kRowStats   scores only; per row the two largest scores over ALL keys decide the normaliser
//               (a repeated maximum <=> the second largest is within eps of the largest), which
//               is written to LSE[] as a scratch value;
//   kFixedNorm  the forward with that fixed per-row normaliser read back from LSE[] (no running
//               maximum, no accumulator rescale), LSE[] then receives m + log l as usual.
constexpr int kRowStats = 3, kFixedNorm = 2;

// Waves per SIMD are stated as a range, not only as a minimum: at D = 128 two work-groups fit a
// CU (LDS), and told so the compiler spends the registers of the third wave it would otherwise
// keep room for on issuing LDS fragment reads ahead of their matrix instructions.
template <int D, bool CAUSAL, int VARIANT, bool RAGGED, bool EXTRAS>
__global__ __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu(D <= 128 ? 2 : 1, kLdsD<D> == 128 ? 2 : (D > 128 ? 1 : 8)))) void attn_fwd_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    bf16_t* __restrict__ O, float* __restrict__ LSE, int N, float alpha, float beta, float eps,
    FwdExtras ex, Layout lay, int pairs, BlockOrder ord) {
  constexpr int TILE_BYTES = kBc * kLdsD<D> * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // layout: K buffers [2][TILE_BYTES], then V buffers [2][TILE_BYTES]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;

  // RAGGED: the bounds-checking instantiation.  N (queries) need not be a multiple of the block:
  // the last block's missing rows are computed on clamped data and not stored; NK keys, those
  // past the end are masked like future keys; the causal mask is  key <= query + shift.
  const int NK = RAGGED ? lay.Nk : N;
  const int shift = RAGGED ? NK - N : 0;
  const int nqt = (N + kBr - 1) / kBr;
  // pairs != 0 (causal problems with enough work-groups): a work-group takes query block
  // nqt-1-idx and then its mirror image idx, which together always meet the same number of key
  // tiles, so every work-group carries the same load, there is no tail of heavy blocks at the
  // end of the grid, and half as many work-groups have to start and drain.  pairs == 0: one
  // block per work-group, for causal grids in the order the table `ord` gives (or, where the
  // table does not apply, heavy blocks first with a per-lap rotation on small grids).
  const int wg = logical_wg(ord, blockIdx.x, gridDim.x);
  const int npw = pairs ? (nqt + 1) / 2 : nqt;          // work-groups per head
  const int bh = wg / npw;
  const int idx = wg % npw;
  const size_t head_off = head_base(lay, bh);
  const int sn = lay.sn;
  const bf16_t* Qh = Q + head_off;
  const bf16_t* Kh = K + head_base_kv(lay, bh);
  const bf16_t* Vh = V + head_base_kv(lay, bh);

  TileLoader<D> loader;
  loader.init(tid, sn);
  FragOffsets<D> fo;
  init_frag_offsets<D>(fo, lane);
  frag_offsets_add_base<D>(fo, lds_address(smem));
  const float c2 = alpha * kLog2e;
  // Alg. 3's test  r_m - alpha*s <= eps  in terms of the raw score s:  s >= (r_m - eps) / alpha
  const float inv_alpha = 1.0f / alpha;

  for (int part = 0; part < (pairs ? 2 : 1); ++part) {
  if (part > 0) __syncthreads();                      // the first block's output staging is done with the tile buffers
  // heavy (late) query blocks first under the causal mask
  const int qt = pairs ? (part == 0 ? nqt - 1 - idx : idx)
                       : nqt - 1 - (idx + (CAUSAL && ord.n == 0 ? small_grid_rotation(bh, nqt, gridDim.x, D == 128 ? 768 : 1536) : 0)) % nqt;
  if (part == 1 && qt == nqt - 1 - idx) break;        // odd number of blocks: the middle one has no partner
  const int q0 = qt * kBr;
  const int qw = q0 + 32 * wave;                 // first query row of this wave
  const int q = qw + r;
  const int qc = (RAGGED && q >= N) ? N - 1 : q;   // row actually read for this lane

  // keys [0, kend) can matter to this block
  const int kend = !CAUSAL ? NK : !RAGGED ? q0 + kBr : max(0, min(NK, q0 + kBr + shift));
  const int ntiles = RAGGED ? (kend + kBc - 1) / kBc : kend / kBc;
  loader.template load_rows<RAGGED>(smem, Kh, 0, NK, tid);
  if (VARIANT != kRowStats) loader.template load_rows<RAGGED>(smem + 2 * TILE_BYTES, Vh, 0, NK, tid);

  // Q_i^T fragments: lane (r,h) holds Q[qw + r][16kc + 8h .. +7] for every kc.
  bf16x8 qf[D / 16];
#pragma unroll
  for (int kc = 0; kc < D / 16; ++kc)
    qf[kc] = *reinterpret_cast<const bf16x8*>(Qh + (size_t)qc * sn + 16 * kc + 8 * h);

  f32x16 acc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[db][i] = 0.f;

  int ones_cnt = 0, fired_cnt = 0;   // EXTRAS only
  float top1 = -INFINITY, top2 = -INFINITY;   // kRowStats: the lane's two largest raw scores so far
  // running normaliser, natural-log units of the alpha-scaled scores (kFixedNorm: the row's
  // normaliser chosen by the kRowStats pass)
  float m = (VARIANT == kFixedNorm) ? LSE[(size_t)bh * N + qc] : -INFINITY;
  float lsum = 0.f;         // this lane's share of the running row sum (its 32 of the 64 keys per tile)

  wait_vmem();
#pragma unroll
  for (int kc = 0; kc < D / 16; ++kc) settle(qf[kc]);
  if (VARIANT == kFixedNorm) settle(m);
  __syncthreads();

  // One key tile; BUF (which LDS buffer holds it) is a compile-time constant so that every LDS
  // address is a precomputed per-lane offset plus an immediate.
  auto tile_step = [&](auto buf_c, int j) {
    constexpr int BUF = decltype(buf_c)::value;
    constexpr int tK = BUF * TILE_BYTES;          // byte offsets of this tile's K and V in smem
    constexpr int tV = (2 + BUF) * TILE_BYTES;
    // The next tile lands in the other buffer while this one is being processed.  Its transfer
    // instructions are not issued in one burst (all eight waves of a CU would queue 64 KB of
    // requests right behind the barrier and sit at the head of the tile until the queue takes
    // them) but one per step of the score product.  After the last tile the current one is
    // fetched once more into the idle buffer: harmless, and the instruction stream stays free of
    // branches.
    const int jn = (j + 1 < ntiles) ? j + 1 : j;
    constexpr int NLD = TileLoader<D>::NI;
    const auto pendK = loader.template prepare<RAGGED>(smem + (BUF ^ 1) * TILE_BYTES, Kh, jn * kBc, NK);
    const auto pendV = loader.template prepare<RAGGED>(smem + (2 + (BUF ^ 1)) * TILE_BYTES, Vh, jn * kBc, NK);
    auto issue_part = [&](int i) {
      if (i < NLD) loader.template issue<RAGGED>(pendK, tid, i);
      else if (i < 2 * NLD && VARIANT != kRowStats) loader.template issue<RAGGED>(pendV, tid, i - NLD);
    };
    bool issued = false;
    const int k0 = j * kBc;
    // A wave whose 32 rows all lie above this key tile has nothing to do in it (causal).
    if (!CAUSAL || (k0 <= qw + shift + 31)) {
      // ---- S^T = K_j Q_i^T (Alg. 1 step 6); raw scores, alpha not yet applied
      f32x16 s[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kb][i] = 0.f;
#pragma unroll
      for (int kc = 0; kc < D / 16; ++kc) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) s[kb] = mfma32(lds_row8<D>(tK, fo, 32 * kb, kc), qf[kc], s[kb]);
        issue_part(kc);
      }
#pragma unroll
      for (int i = D / 16; i < 2 * NLD; ++i) issue_part(i);
      issued = true;
      sched_reads_ahead_of_mfma<D / 8, 1, 4>();
      // ---- mask: causal (key > query) in the tile that crosses the diagonal, and keys beyond
      // the sequence end in the last, partial tile -> -inf
      if ((CAUSAL && (k0 + kBc - 1 > qw + shift)) || (RAGGED && k0 + kBc > NK)) {
        // element (kb, i) of this lane is key k0 + 4h + c with c = 32 kb + 8 (i / 4) + i % 4 a
        // compile-time constant: masked <=> c > lim, one per-lane limit for both conditions
        int lim = CAUSAL ? q + shift - k0 - 4 * h : 0x7fffffff;
        if (RAGGED) lim = min(lim, NK - 1 - k0 - 4 * h);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (32 * kb + 8 * (i >> 2) + (i & 3) > lim) s[kb][i] = -INFINITY;
      }
      if (VARIANT == kRowStats) {
        // two largest values seen by this lane (duplicates count: a value met twice is both)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            top2 = __builtin_amdgcn_fmed3f(top1, top2, s[kb][i]);
            top1 = fmaxf(top1, s[kb][i]);
          }
      } else {
        float corr = 1.f;    // factor the accumulated output and row sum are multiplied by
        float mneg;          // -m log2(e) of the normaliser used for this tile
        if (VARIANT == kFixedNorm) {
          mneg = (RAGGED && m == -INFINITY) ? 0.f : -m * kLog2e;   // a query that sees no key at all
        } else {
          // ---- tile row maximum r_m (of the alpha-scaled scores)
          float mx;
          bool repeated = false;
          if (VARIANT == 1) {
            // Alg. 3: r_s = #{ r_m - S <= eps } over the tile row; a repeated maximum moves the
            // normaliser to beta*r_m (r_m > 0) or to 0 (r_m < 0).  The count only matters through
            // "more than one", i.e. through whether the SECOND largest score of the row passes the
            // test: the lane keeps the two largest of its 32 scores (two chains of 16; a value met
            // twice is both), then the two lanes that share a query row are merged.  Three vector
            // instructions per two scores and no mask bookkeeping.
            float a1[2], a2[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
              a1[kb] = fmaxf(s[kb][0], s[kb][1]);
              a2[kb] = fminf(s[kb][0], s[kb][1]);
#pragma unroll
              for (int i = 2; i < 16; i += 2) {
                // two more scores x, y: the largest of {a1, x, y} is the new a1; the second largest
                // of {a1, a2, x, y} is the median of {a1, x, y} or the old a2 (a2 <= a1)
                const float x = s[kb][i], y = s[kb][i + 1];
                const float mid = __builtin_amdgcn_fmed3f(a1[kb], x, y);
                a1[kb] = fmaxf(fmaxf(a1[kb], x), y);
                a2[kb] = fmaxf(mid, a2[kb]);
              }
            }
            const float t1 = fmaxf(a1[0], a1[1]);
            const float t2 = fmaxf(fminf(a1[0], a1[1]), fmaxf(a2[0], a2[1]));
            const float o1 = partner32(t1), o2 = partner32(t2);
            mx = fmaxf(t1, o1);
            const float second = fmaxf(fminf(t1, o1), fmaxf(t2, o2));
            // the test  r_m - alpha*s <= eps  in terms of the raw score:  s >= (r_m - eps) / alpha
            // (a row with nothing visible in this tile has r_m = -inf: no rule, no update)
            repeated = second >= (mx * alpha - eps) * inv_alpha && (!RAGGED || mx > -INFINITY);
            if (EXTRAS && ex.guard != 0) repeated = repeated && guard_allows(mx * alpha, beta);
          } else {
            mx = s[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
              for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[kb][i]);
            mx = max_with_partner32(mx);
          }
          const float r_m = mx * alpha;
          float m_prime = r_m;
          if (VARIANT == 1) {
            m_prime = (repeated && r_m > 0.f) ? beta * r_m : r_m;
            m_prime = (repeated && r_m < 0.f) ? 0.f : m_prime;
            if (EXTRAS) fired_cnt += (m_prime != r_m) ? 1 : 0;
          }
          const float m_new = fmaxf(m, m_prime);         // Alg. 1 step 7 / Alg. 3
          const bool unseen = RAGGED && m_new == -INFINITY;   // nothing visible so far: P-bar = 0, nothing to rescale
          corr = unseen ? 1.f : __builtin_amdgcn_exp2f((m - m_new) * kLog2e);
          m = m_new;
          mneg = unseen ? 0.f : -m_new * kLog2e;
        }
        if (EXTRAS && ex.pv_e4m3 != 0) {
          // ---- exploration beyond the paper (its future-work remark on FP8): the same step with
          // P-bar and V_j rounded to E4M3 and multiplied by the FP8 matrix instruction; the row sum
          // is of the rounded P-bar, everything downstream is unchanged.  Same k-slot order in
          // both operands as in the bf16 path.
          long pf8[2][2];
          float psum8 = 0.f;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
              float pv[8];
#pragma unroll
              for (int jj = 0; jj < 8; ++jj)
                pv[jj] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][8 * cc + jj], c2, mneg));
              const long pk = pack_e4m3(pv);
              pf8[kb][cc] = pk;
              const int w0 = (int)(unsigned)pk, w1 = (int)(unsigned)((unsigned long long)pk >> 32);
              const float back[8] = {__builtin_amdgcn_cvt_f32_fp8(w0, 0), __builtin_amdgcn_cvt_f32_fp8(w0, 1),
                                     __builtin_amdgcn_cvt_f32_fp8(w0, 2), __builtin_amdgcn_cvt_f32_fp8(w0, 3),
                                     __builtin_amdgcn_cvt_f32_fp8(w1, 0), __builtin_amdgcn_cvt_f32_fp8(w1, 1),
                                     __builtin_amdgcn_cvt_f32_fp8(w1, 2), __builtin_amdgcn_cvt_f32_fp8(w1, 3)};
#pragma unroll
              for (int jj = 0; jj < 8; ++jj) {
                psum8 += back[jj];
                ones_cnt += back[jj] == 1.0f ? 1 : 0;
              }
            }
          lsum = lsum * corr + psum8;
          if (VARIANT != kFixedNorm && j > 0 && __builtin_amdgcn_ballot_w64(corr != 1.f) != 0) {
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
              for (int i = 0; i < 16; ++i) acc[db][i] *= corr;
          }
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc)
#pragma unroll
              for (int db = 0; db < D / 32; ++db) {
                const bf16x8 v8 = lds_col8<D>(tV, fo, 32 * kb + 16 * cc, db);
                float vv[8];
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) vv[jj] = (float)v8[jj];
                acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_fp8_fp8(pack_e4m3(vv), pf8[kb][cc], acc[db], 0, 0, 0);
              }
        } else {
        // ---- P-bar = exp(S - m), rounded to bf16; row sum of the ROUNDED values
        bf16x8 pf[2][2];
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int cc = 0; cc < 2; ++cc)
#pragma unroll
            for (int jj = 0; jj < 8; jj += 2) {
              bf16x2 pp;
#pragma unroll
              for (int e = 0; e < 2; ++e)
                pp[e] = (bf16_t)__builtin_amdgcn_exp2f(__builtin_fmaf(s[kb][8 * cc + jj + e], c2, mneg));
              pf[kb][cc][jj] = pp[0];
              pf[kb][cc][jj + 1] = pp[1];
              psum = add_pair_bf16(pp, psum);
              if (EXTRAS) ones_cnt += ((float)pp[0] == 1.0f ? 1 : 0) + ((float)pp[1] == 1.0f ? 1 : 0);
            }
        lsum = lsum * corr + psum;
        // ---- O^T <- diag(corr) O^T + V_j^T P-bar^T (Alg. 1 step 8); in the first tile the
        // accumulator is still zero (corr = exp(-inf) = 0 there), nothing to rescale
        if (VARIANT != kFixedNorm && j > 0 && __builtin_amdgcn_ballot_w64(corr != 1.f) != 0) {
#pragma unroll
          for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][i] *= corr;
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int cc = 0; cc < 2; ++cc)
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
              acc[db] = mfma32(lds_col8<D>(tV, fo, 32 * kb + 16 * cc, db), pf[kb][cc], acc[db]);
        }
      }
    }
    if (!issued) {      // a wave that skipped the tile still has its share of the transfer to issue
#pragma unroll
      for (int i = 0; i < 2 * NLD; ++i) issue_part(i);
    }
    wait_vmem();
    __syncthreads();
  };

  for (int j = 0; j < ntiles; j += 2) {
    tile_step(std::integral_constant<int, 0>{}, j);
    if (j + 1 < ntiles) tile_step(std::integral_constant<int, 1>{}, j + 1);
  }

  if (VARIANT == kRowStats) {
    // merge the two lanes of a row, then the rule of Sec. 4 on the whole row
    const float o1 = partner32(top1), o2 = partner32(top2);
    const float M1 = fmaxf(top1, o1);
    const float M2 = fmaxf(fminf(top1, o1), fmaxf(top2, o2));
    const float r_m = M1 * alpha;
    bool repeated = (r_m - M2 * alpha) <= eps;            // r_s > 1
    if (EXTRAS && ex.guard != 0) repeated = repeated && guard_allows(r_m, beta);
    float m_row = (repeated && r_m > 0.f) ? beta * r_m : r_m;
    m_row = (repeated && r_m < 0.f) ? 0.f : m_row;
    if (h == 0 && (!RAGGED || q < N)) {
      LSE[(size_t)bh * N + q] = m_row;
      if (EXTRAS && ex.fired != nullptr) ex.fired[(size_t)bh * N + q] = (m_row != r_m) ? 1 : 0;
    }
    continue;
  }
  // ---- epilogue (Alg. 1 steps 10-13).  Rounding points of Sec. 3.3.2: the unnormalised
  // output is rounded to bf16 first, then divided by l, then rounded again.
  const float l = sum_with_partner32(lsum);
  int ones_row = 0;
  if (EXTRAS) {   // the partner lane counted the other 32 keys of every tile
    auto sw = __builtin_amdgcn_permlane32_swap((unsigned)ones_cnt, (unsigned)ones_cnt, false, false);
    ones_row = (int)(sw[0] + sw[1]);
  }
  const bool keep_obar_f32 = EXTRAS && ex.single_rounding != 0;
  const bool unseen_row = RAGGED && m == -INFINITY;        // no visible key (more queries than keys): O = 0, LSE = -inf
  const Divisor by_l = make_divisor(l);
  auto o_piece = [&](int db, int g) {
    bf16x4 o4;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = acc[db][4 * g + e];
      const float obar = keep_obar_f32 ? a : (float)(bf16_t)a;
      o4[e] = (bf16_t)(unseen_row ? 0.f : divide(obar, by_l));
    }
    return o4;
  };
  if constexpr (kCanStage<D / 32>) {
    // the tile buffers are free now (every wave is past the last tile's barrier) and serve as the
    // staging areas of store_rows_staged; the barrier at the top of the part loop keeps the next
    // block's tile transfers from overwriting an area a slower wave is still reading
    store_rows_staged<D / 32>(smem, o_piece, O + head_off + (size_t)qw * sn, sn, RAGGED ? N - qw : 32, tid);
  }
  if (!RAGGED || q < N) {                                  // rows past the sequence end exist only as padding
  if constexpr (!kCanStage<D / 32>) {
    bf16_t* Oq = O + head_off + (size_t)q * sn;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) *reinterpret_cast<bf16x4*>(Oq + 32 * db + 8 * g + 4 * h) = o_piece(db, g);
  }
  if (EXTRAS && ex.O_hp != nullptr) {
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 hp;
#pragma unroll
        for (int e = 0; e < 4; ++e) hp[e] = unseen_row ? 0.f : divide(acc[db][4 * g + e], by_l);
        *reinterpret_cast<f32x4*>(ex.O_hp + ((size_t)bh * N + q) * D + 32 * db + 8 * g + 4 * h) = hp;
      }
  }
  if (h == 0) {
    LSE[(size_t)bh * N + q] = m + __logf(l);
    if (EXTRAS && ex.ones != nullptr) ex.ones[(size_t)bh * N + q] = ones_row;
    if (EXTRAS && VARIANT != kFixedNorm && ex.fired != nullptr) ex.fired[(size_t)bh * N + q] = fired_cnt;
  }
  }
  }   // part
}

}  // namespace

extern "C" int attn_fwd_key_tile(int d) { return (d == 32 || d == 64 || d == 96 || d == 128 || d == 256) ? kBc : 0; }

template <int D, bool CAUSAL, int VARIANT, bool RAGGED, bool EXTRAS>
static hipError_t launch_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                             int BH, int N, float alpha, float beta, float eps, FwdExtras ex,
                             Layout lay, hipStream_t st) {
  constexpr int smem = 4 * kBc * kLdsD<D> * 2;
  static std::atomic<bool> attr_set{false};   // (calls from several host threads may race to set it: harmless, the call is idempotent)
  auto kern = attn_fwd_kernel<D, CAUSAL, VARIANT, RAGGED, EXTRAS>;
  if (!attr_set.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set.store(true, std::memory_order_release);
  }
  // Under the causal mask a work-group takes a query block and its mirror image (equal work for
  // all) when that still leaves at least two full rounds of work-groups (two fit a CU, 256 CUs);
  // smaller grids keep one block per work-group, in a balanced order (below).
  const int nqt = (N + kBr - 1) / kBr;
  const int pairs = (CAUSAL && (long long)BH * ((nqt + 1) / 2) >= 1024) ? 1 : 0;
  dim3 grid(BH * (pairs ? (nqt + 1) / 2 : nqt));
  // one block per work-group: in the order that balances the compute units (block_order.hpp)
  // whenever the table can express the grid (measured: -12..-21 % at one to three rounds of
  // work-groups against heavy-first order)
  static std::atomic<int> resident{0};
  static thread_local OrderCache cache;
  const BlockOrder& ord = (CAUSAL && !pairs)
      ? small_grid_order(cache, (int)grid.x, nqt, resident_per_cu(kern, smem, resident), 8 * kMaxOrder) : kNoOrder;
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, st, (const bf16_t*)Q, (const bf16_t*)K,
                     (const bf16_t*)V, (bf16_t*)O, LSE, N, alpha, beta, eps, ex, lay, pairs, ord);
  return hipGetLastError();
}

// Host-side dispatch used by the C ABI (api.hip).  Shapes are validated by the caller.
// The optional outputs / switches select a second set of kernels (always the bounds-checking
// instantiation), so that the plain forward carries none of their instructions.
hipError_t attn_fwd_dispatch(const void* Q, const void* K, const void* V, void* O, float* LSE,
                             int BH, int N, int d, int causal, float alpha, int variant,
                             float beta, float eps, float* O_hp, int* ones, int* fired,
                             int flags, Layout lay, hipStream_t st) {
  // flags: bit 0 = single rounding of the output, bit 1 = P-bar V in E4M3, bit 2 = guarded Alg. 3
  const bool extras = O_hp != nullptr || ones != nullptr || fired != nullptr || flags != 0;
  const FwdExtras ex{O_hp, ones, fired, flags & 1, (flags >> 1) & 1, (flags >> 2) & 1};
  if (variant == 2) {   // whole-row detection: statistics pass, then the fixed-normaliser pass
#define CASE2(DD, CC)                                                                           \
  if (d == DD && (causal != 0) == CC) {                                                          \
    hipError_t e = launch_fwd<DD, CC, kRowStats, true, true>(Q, K, V, O, LSE, BH, N, alpha, beta, eps, ex, lay, st); \
    if (e != hipSuccess) return e;                                                               \
    return launch_fwd<DD, CC, kFixedNorm, true, true>(Q, K, V, O, LSE, BH, N, alpha, beta, eps, ex, lay, st); \
  }
    CASE2(32, false) CASE2(32, true) CASE2(64, false) CASE2(64, true) CASE2(128, false) CASE2(128, true)
    CASE2(256, false) CASE2(256, true) CASE2(96, false) CASE2(96, true)
#undef CASE2
    return hipErrorInvalidValue;
  }
#define CASE(DD, CC, VV)                                                                      \
  if (d == DD && (causal != 0) == CC && variant == VV) {                                       \
    if (extras) return launch_fwd<DD, CC, VV, true, true>(Q, K, V, O, LSE, BH, N, alpha, beta, eps, ex, lay, st); \
    return (N % kBr || lay.Nk != N) ? launch_fwd<DD, CC, VV, true, false>(Q, K, V, O, LSE, BH, N, alpha, beta, eps, ex, lay, st) \
                     : launch_fwd<DD, CC, VV, false, false>(Q, K, V, O, LSE, BH, N, alpha, beta, eps, ex, lay, st); \
  }
  CASE(32, false, 0) CASE(32, false, 1) CASE(32, true, 0) CASE(32, true, 1)
  CASE(64, false, 0) CASE(64, false, 1) CASE(64, true, 0) CASE(64, true, 1)
  CASE(128, false, 0) CASE(128, false, 1) CASE(128, true, 0) CASE(128, true, 1)
  CASE(256, false, 0) CASE(256, false, 1) CASE(256, true, 0) CASE(256, true, 1)
  CASE(96, false, 0) CASE(96, false, 1) CASE(96, true, 0) CASE(96, true, 1)
#undef CASE
  return hipErrorInvalidValue;
}
