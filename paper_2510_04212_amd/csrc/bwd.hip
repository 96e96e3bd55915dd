// Flash-attention backward for gfx950 (Alg. 2 of arXiv 2510.04212), as two kernels so that no
// gradient needs a cross-work-group reduction (no atomics, deterministic):
//
//   attn_bwd_dkdv_kernel  one work-group per (batch, head, 128-key block) -- under the causal mask
//                         per pair of mirrored blocks, one after the other, unless the grid is
//                         small (then one block each, in a balanced order); K_j / V_j fragments
//                         stay in registers, query tiles (Q_i, dO_i, L_i, delta_i; 64 rows) stream
//                         through LDS.  Per tile:  S = Q_i K_j^T,  P = exp(S - L),  dP = dO_i V_j^T,
//                         dS = P o (dP - delta),  dV_j^T += dO_i^T P,  dK_j^T += Q_i^T dS.
//   attn_bwd_dq_kernel    one work-group per (batch, head, 128-query block); Q_i / dO_i fragments,
//                         L_i and delta_i stay in registers, key tiles (K_j, V_j; 64 rows) stream
//                         through LDS.  Per tile:  S^T = K_j Q_i^T,  dP^T = V_j dO_i^T,
//                         dS^T = P^T o (dP^T - delta),  dQ_i^T += K_j^T dS^T.
//
// S and dP are recomputed in the second kernel (7 matrix products per tile pair instead of
// Alg. 2's 5); in exchange every contraction finds its operands already in fragment layout:
// the accumulator-layout P / dS tiles are fed back as B operands unchanged, and the operands
// whose contraction index runs along tile rows come from transposing LDS reads.
//
// Rounding points: P (float32) -> bf16 as the operand of dO^T P; dS = P o (dP - delta) is formed
// from the float32 P and rounded to bf16 as an operand; accumulators are float32; alpha
// multiplies the float32 dQ / dK accumulators once; outputs are rounded to bf16 when stored.
#include "common.hpp"

#include <atomic>
#include <type_traits>

namespace {

constexpr int kKeysPerWG = 128;   // dK/dV kernel: keys per work-group (32 per wave)
constexpr int kQTile = 64;        // dK/dV kernel: query rows per streamed tile
constexpr int kQPerWG = 128;      // dQ kernel: queries per work-group (32 per wave)
constexpr int kKTile = 64;        // dQ kernel: key rows per streamed tile

template <int NDB>
DEVI void store_acc_T(bf16_t* dst_row, const f32x16 (&acc)[NDB], float scale, int h) {
  // acc[db][i] = X^T[d = 32db + 8(i/4) + 4h + (i%4)][row of this lane]; 4 consecutive d -> 8 bytes
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = (bf16_t)(acc[db][4 * g + e] * scale);
      *reinterpret_cast<bf16x4*>(dst_row + 32 * db + 8 * g + 4 * h) = o4;
    }
}

// GROUPED: grouped-query attention (lay.group > 1): the work-group serves several query heads.
// Kept out of the ordinary kernel so that its tile loop has a fixed head and no bookkeeping.
// At D = 256 the two accumulator sets of a full key block would not fit the register file next
// to the K / V fragments: a work-group then owns 128 of the 256 columns of dK and dV (kDSplit
// work-groups per key block, each recomputing S and dP), and the four-phase pipeline, whose
// phases assume as many update as score instructions, is not used.
template <int D> constexpr int kDSplit = D > 128 ? 2 : 1;
// dK / dV rows leave through a per-wave LDS staging area (store_rows_staged) where the row width
// allows it and LDS has room for it next to the tiles (not at D = 256).
template <int D> constexpr bool kStagedDkDv = kCanStage<D / 32 / kDSplit<D>> && D <= 128;

template <int D, bool CAUSAL, bool RAGGED, bool GROUPED>
__global__ __launch_bounds__(256, D <= 64 ? 2 : 1) void attn_bwd_dkdv_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    bf16_t* __restrict__ dK, bf16_t* __restrict__ dV, int N, float alpha, Layout lay, int pairs,
    BlockOrder ord) {
  constexpr int TILE_BYTES = kQTile * kLdsD<D> * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  // layout: Q buffers [2][TILE_BYTES], dO buffers [2][TILE_BYTES], L2 [2][64] float, delta [2][64] float
  char* ldsQ = smem;
  char* ldsdO = smem + 2 * TILE_BYTES;
  float* ldsL = reinterpret_cast<float*>(smem + 4 * TILE_BYTES);
  float* ldsD = ldsL + 2 * kQTile;
  // behind them: one staging area per wave for the output rows (store_rows_staged)

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;

  // RAGGED: the bounds-checking instantiation: N queries and NK keys, neither need be a multiple
  // of the block; causal mask  key <= query + shift.
  const int NK = RAGGED ? lay.Nk : N;
  const int shift = RAGGED ? NK - N : 0;
  const int nkt = (NK + kKeysPerWG - 1) / kKeysPerWG;
  // Under the causal mask key block kt meets nkt - kt query blocks' worth of tiles.  pairs != 0: a
  // work-group takes block kt and then its mirror image nkt - 1 - kt, so that all work-groups
  // carry the same load (and there are half as many to start and drain).  pairs == 0 (grids so
  // small that equal but few work-groups would leave compute units idle): one block per
  // work-group, in the order the table `ord` gives.
  const int npw = pairs ? (nkt + 1) / 2 : nkt;         // work-groups per key/value head and column part
  constexpr int DS = kDSplit<D>;
  constexpr int NDB = D / 32 / DS;                     // 32-column blocks of dK / dV this work-group owns
  const int wg_all = logical_wg(ord, blockIdx.x, gridDim.x);
  const int db0 = (DS > 1) ? (wg_all % DS) * NDB : 0;  // first of them
  const int wg = wg_all / DS;
  // with grouped queries a work-group serves the `group` query heads that share its key/value
  // head, one after the other
  const int bhk = wg / npw;
  const int group = GROUPED ? lay.group : 1;
  const int Hkv = lay.H / group;
  const int bq0 = (bhk / Hkv) * lay.H + (bhk % Hkv) * group;   // first of those query heads
  const int kt_first = wg % npw;
  const int sn = lay.sn;
  const size_t head_off = head_base_kv(lay, bq0);              // K, V, dK, dV
  const float c2 = alpha * kLog2e;
  FragOffsets<D> fo;
  init_frag_offsets<D>(fo, lane);
  // Transposing reads of the update products address column block db0 + db: a column block only
  // enters the offset through chunk bits the swizzle leaves alone, so shifting by db0 blocks is one
  // XOR per offset (32 columns = 4 chunks = 64 bytes).
  FragOffsets<D> fo_upd = fo;
  if (DS > 1) {
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int db = 0; db < D / 32; ++db) fo_upd.col[half][db] ^= 64 * db0;
  }
  frag_offsets_add_base<D>(fo, lds_address(smem));
  frag_offsets_add_base<D>(fo_upd, lds_address(smem));
  TileLoader<D> loader;
  loader.init(tid, sn);

  for (int part = 0; part < (CAUSAL ? 2 : 1); ++part) {
    const int kt = (part == 0) ? kt_first : nkt - 1 - kt_first;
    if (part == 1 && (!pairs || kt == kt_first)) break;   // no partner: one block per work-group, or the middle one of an odd number
    const int k0 = kt * kKeysPerWG;
    const int kw = k0 + 32 * wave;

    // K_j^T / V_j^T fragments (B operands): lane (r,h) holds K[kw + r][16kc + 8h .. +7]
    // (keys past the sequence end read the last row; their gradients are not stored)
    const int keyc = (RAGGED && kw + r >= NK) ? NK - 1 : kw + r;
    bf16x8 kf[D / 16], vf[D / 16];
#pragma unroll
    for (int kc = 0; kc < D / 16; ++kc) {
      kf[kc] = *reinterpret_cast<const bf16x8*>(K + head_off + (size_t)keyc * sn + 16 * kc + 8 * h);
      vf[kc] = *reinterpret_cast<const bf16x8*>(V + head_off + (size_t)keyc * sn + 16 * kc + 8 * h);
    }
    f32x16 dVt[NDB], dKt[NDB];
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) { dVt[db][i] = 0.f; dKt[db][i] = 0.f; }

    // first query tile that sees any key of this block
    const int t0 = !CAUSAL ? 0 : !RAGGED ? k0 / kQTile : max(0, k0 - shift) / kQTile;
    const int nt = RAGGED ? (N + kQTile - 1) / kQTile : N / kQTile;
    if (RAGGED && t0 >= nt) {                        // no query sees these keys (more keys than queries reach): zero gradients
      if (kw + r < NK) {
        store_acc_T<NDB>(dV + 32 * db0 + head_off + (size_t)(kw + r) * sn, dVt, 1.0f, h);
        store_acc_T<NDB>(dK + 32 * db0 + head_off + (size_t)(kw + r) * sn, dKt, alpha, h);
      }
      continue;
    }

    // Q_i / dO_i tiles go global -> LDS asynchronously; L_i (pre-multiplied by log2 e) and -delta_i
    // (64 floats each) pass through one register of threads 0..127.  The dP accumulator starts
    // from -delta, so that the matrix instructions deliver dP - delta directly (Alg. 2 step 12).
    float sreg = 0.f;
    // Current query head: its first element in Q / dO and in LSE / delta.  With GROUPED the
    // work-group moves on to the next head of its group (at distance lay.sh and N) after tile
    // nt - 1, without breaking the double buffering: `step` counts tiles over all heads.
    const bf16_t* Qh = Q + head_base(lay, bq0);
    const bf16_t* dOh = dO + head_base(lay, bq0);
    const float* Lh = LSE + (size_t)bq0 * N;
    const float* Dh = delta + (size_t)bq0 * N;
    const int total = group * (nt - t0);
    auto load_stats = [&](const float* Lp, const float* Dp, int t) {
      const int row = t * kQTile + (tid & (kQTile - 1));
      const int rowc = (RAGGED && row >= N) ? N - 1 : row;
      if (tid < kQTile) {
        sreg = Lp[rowc];
      } else if (tid < 2 * kQTile) sreg = Dp[rowc];
      // (The loaded values are not touched before store_stats: any arithmetic on them here would
      // make the wave wait, at the start of the tile, for these loads and for the tile transfer
      // issued just before them.)
    };
    auto store_stats = [&](int buf) {
      if (tid < kQTile) {
        float l = sreg * kLog2e;
        if (RAGGED && l == -INFINITY) l = 0.f;         // a query that sees no key: all its scores are masked below
        ldsL[buf * kQTile + tid] = l;
      } else if (tid < 2 * kQTile) ldsD[buf * kQTile + tid - kQTile] = -sreg;   // LDS holds -delta
    };
    loader.template load_rows<RAGGED>(ldsQ, Qh, t0 * kQTile, N, tid);
    loader.template load_rows<RAGGED>(ldsdO, dOh, t0 * kQTile, N, tid);
    load_stats(Lh, Dh, t0);
    store_stats(0);
    wait_vmem();
    __syncthreads();

    // One query tile; BUF (which LDS buffer holds it) is a compile-time constant so that every LDS
    // address is a precomputed per-lane offset plus an immediate.
    auto tile_step = [&](auto buf_c, int t, int step) {
      constexpr int buf = decltype(buf_c)::value;
      const bool has_next = (step + 1 < total);
      // The next tile (after the last one: this tile once more, harmlessly) goes into the other
      // buffer.  On the pipelined path its transfer instructions are issued one per two slots of
      // the first phase instead of in one burst behind the barrier.
      int tn = has_next ? t + 1 : t;
      if (GROUPED && has_next && t + 1 == nt) {   // on to the next query head of the group
        Qh += lay.sh; dOh += lay.sh; Lh += N; Dh += N;
        tn = t0;
      }
      constexpr int NLD = TileLoader<D>::NI;
      const auto pendQ = loader.template prepare<RAGGED>(ldsQ + (buf ^ 1) * TILE_BYTES, Qh, tn * kQTile, N);
      const auto pendD = loader.template prepare<RAGGED>(ldsdO + (buf ^ 1) * TILE_BYTES, dOh, tn * kQTile, N);
      auto issue_part = [&](int i) {
        if (i < NLD) loader.template issue<RAGGED>(pendQ, tid, i);
        else if (i < 2 * NLD) loader.template issue<RAGGED>(pendD, tid, i - NLD);
      };
      if (has_next) load_stats(Lh, Dh, tn);
      constexpr int tQ = buf * TILE_BYTES;          // byte offsets of this tile's Q and dO in smem
      constexpr int tdO = (2 + buf) * TILE_BYTES;
      const float* tL = reinterpret_cast<const float*>(smem + 4 * TILE_BYTES) + buf * kQTile;
      const float* tD = reinterpret_cast<const float*>(smem + 4 * TILE_BYTES) + 2 * kQTile + buf * kQTile;
      const int qt0 = t * kQTile;
      // one 32-query block against this wave's 32 keys; DIAG: the block crosses the diagonal
      auto qblock = [&](auto diag_c, int qb) {
        constexpr bool DIAG = decltype(diag_c)::value;
        const int qb0 = qt0 + 32 * qb;
        const bool tail = RAGGED && qb0 + 32 > N;              // some query rows lie past the sequence end
        // ---- S = Q_i K_j^T and dP = dO_i V_j^T (Alg. 2 steps 8, 11); rows = queries, lane = key
        f32x16 s, dp;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(tD + 32 * qb + 8 * g + 4 * h);
#pragma unroll
          for (int e = 0; e < 4; ++e) { s[4 * g + e] = 0.f; dp[4 * g + e] = d4[e]; }
        }
#pragma unroll
        for (int kc = 0; kc < D / 16; ++kc) {
          s = mfma32(lds_row8<D>(tQ, fo, 32 * qb, kc), kf[kc], s);
          dp = mfma32(lds_row8<D>(tdO, fo, 32 * qb, kc), vf[kc], dp);
        }
        sched_reads_ahead_of_mfma<D / 8, 1, 4>();
        // element i of this lane is query qb0 + 4h + c with c = 8 (i / 4) + i % 4 a compile-time constant
        if (tail) {   // rows past the sequence end: P = exp(-inf) = 0, so they add nothing to dK, dV
          const int lim = N - qb0 - 4 * h;
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (8 * (i >> 2) + (i & 3) >= lim) s[i] = -INFINITY;
        }
        // ---- P = exp(S - L) (step 9), dS = P o (dP - delta) (step 12)
        bf16x8 pf[2], dsf[2];
        const int first_seen = kw + r - shift - qb0 - 4 * h;   // DIAG: queries with c below it do not see this lane's key
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(tL + 32 * qb + 8 * g + 4 * h);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * g + e;
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], c2, -l4[e]));
            float ds = p * dp[i];                     // dp already holds dP - delta
            if (DIAG) {   // a masked entry contributes exactly nothing, whatever its row holds
              if (8 * g + e < first_seen) { p = 0.f; ds = 0.f; }
            }
            pf[i >> 3][i & 7] = (bf16_t)p;
            dsf[i >> 3][i & 7] = (bf16_t)ds;
          }
        }
        // ---- dV_j^T += dO_i^T P ,  dK_j^T += Q_i^T dS  (steps 10, 14)
#pragma unroll
        for (int cc = 0; cc < 2; ++cc)
#pragma unroll
          for (int db = 0; db < NDB; ++db) {
            dVt[db] = mfma32(lds_col8<D>(tdO, fo_upd, 32 * qb + 16 * cc, db), pf[cc], dVt[db]);
            dKt[db] = mfma32(lds_col8<D>(tQ, fo_upd, 32 * qb + 16 * cc, db), dsf[cc], dKt[db]);
          }
        sched_reads_ahead_of_mfma<4 * NDB, 2, 4>();
      };
      // Both 32-query blocks of a tile that lies entirely below the diagonal for this wave, as one
      // software-pipelined sequence of 4 x NS "slots" (one matrix instruction each).  The phase
      // order is fixed by hand (scheduling fences between the phases and between the slots of the
      // two pure matrix phases; inside the mixed phases the compiler interleaves):
      //   phase 1  S,dP of block 0
      //   phase 2  S,dP of block 1        | vector work of block 0 (P, dS), one element per slot
      //   phase 3  dV,dK += block 0       | vector work of block 1
      //   phase 4  dV,dK += block 1
      // and every LDS fragment read is issued AH slots before the matrix instruction that uses it.
      auto tile_pipelined = [&]() {
        constexpr int NS = D / 8;            // slots per phase
        constexpr int AH = (D >= 128) ? 8 : 4;  // LDS read-ahead, in slots
        constexpr int R = 2 * AH;            // fragment ring size (> AH)
        constexpr int EPS = 16 / NS;         // score elements handled per slot
        bf16x8 ring[R];
        // slot s of an S/dP phase: kc = s/2, even -> S (Q_i, K_j), odd -> dP (dO_i, V_j)
        auto rd_sdp = [&](int qb, int sl) -> bf16x8 {
          return lds_row8<D>((sl & 1) ? tdO : tQ, fo, 32 * qb, sl >> 1);
        };
        // slot s of a dV/dK phase: cc = s / (2 NDB), db = (s/2) % NDB, even -> dV (dO_i^T), odd -> dK (Q_i^T)
        // (this path is only taken when the work-group owns all columns, NDB = D/32)
        auto rd_dvdk = [&](int qb, int sl) -> bf16x8 {
          return lds_col8<D>((sl & 1) ? tQ : tdO, fo_upd, 32 * qb + 16 * ((sl / (2 * NDB)) & 1),
                             (sl >> 1) % NDB);
        };
        f32x16 s0, dp0, s1, dp1;
        bf16x8 pf0[2], dsf0[2], pf1[2], dsf1[2];
        f32x4 lq0[4], lq1[4];                        // L_i log2e of the 16 rows a lane sees
#pragma unroll
        for (int g = 0; g < 4; ++g) {                // the dP accumulators start from -delta_i
          lq0[g] = *reinterpret_cast<const f32x4*>(tL + 8 * g + 4 * h);
          const f32x4 d0 = *reinterpret_cast<const f32x4*>(tD + 8 * g + 4 * h);
          const f32x4 d1 = *reinterpret_cast<const f32x4*>(tD + 32 + 8 * g + 4 * h);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            s0[4 * g + e] = 0.f; s1[4 * g + e] = 0.f;
            dp0[4 * g + e] = d0[e]; dp1[4 * g + e] = d1[e];
          }
        }
#pragma unroll
        for (int a = 0; a < AH; ++a) ring[a] = rd_sdp(0, a);
        __builtin_amdgcn_sched_barrier(0);
        // ---- phase 1
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
          ring[(sl + AH) % R] = (sl + AH < NS) ? rd_sdp(0, sl + AH) : rd_sdp(1, sl + AH - NS);
          if (sl & 1) dp0 = mfma32(ring[sl % R], vf[sl >> 1], dp0);
          else s0 = mfma32(ring[sl % R], kf[sl >> 1], s0);
          if (sl & 1) issue_part(sl >> 1);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = NS / 2; i < 2 * NLD; ++i) issue_part(i);
#pragma unroll
        for (int g = 0; g < 4; ++g) lq1[g] = *reinterpret_cast<const f32x4*>(tL + 32 + 8 * g + 4 * h);
        // ---- phase 2
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
          ring[(NS + sl + AH) % R] = (sl + AH < NS) ? rd_sdp(1, sl + AH) : rd_dvdk(0, sl + AH - NS);
          if (sl & 1) dp1 = mfma32(ring[(NS + sl) % R], vf[sl >> 1], dp1);
          else s1 = mfma32(ring[(NS + sl) % R], kf[sl >> 1], s1);
#pragma unroll
          for (int e = 0; e < EPS; ++e) {
            const int i = sl * EPS + e;
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[i], c2, -lq0[i >> 2][i & 3]));
            float ds = p * dp0[i];
            pf0[i >> 3][i & 7] = (bf16_t)p;
            dsf0[i >> 3][i & 7] = (bf16_t)ds;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- phase 3
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
          ring[(2 * NS + sl + AH) % R] = (sl + AH < NS) ? rd_dvdk(0, sl + AH) : rd_dvdk(1, sl + AH - NS);
          const int cc = (sl / (2 * NDB)) & 1, db = (sl >> 1) % NDB;
          if (sl & 1) dKt[db] = mfma32(ring[(2 * NS + sl) % R], dsf0[cc], dKt[db]);
          else dVt[db] = mfma32(ring[(2 * NS + sl) % R], pf0[cc], dVt[db]);
#pragma unroll
          for (int e = 0; e < EPS; ++e) {
            const int i = sl * EPS + e;
            float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[i], c2, -lq1[i >> 2][i & 3]));
            float ds = p * dp1[i];
            pf1[i >> 3][i & 7] = (bf16_t)p;
            dsf1[i >> 3][i & 7] = (bf16_t)ds;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- phase 4
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
          if (sl + AH < NS) ring[(3 * NS + sl + AH) % R] = rd_dvdk(1, sl + AH);
          const int cc = (sl / (2 * NDB)) & 1, db = (sl >> 1) % NDB;
          if (sl & 1) dKt[db] = mfma32(ring[(3 * NS + sl) % R], dsf1[cc], dKt[db]);
          else dVt[db] = mfma32(ring[(3 * NS + sl) % R], pf1[cc], dVt[db]);
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      if (DS == 1 && D != 96 && (!CAUSAL || qt0 + shift >= kw + 31) && (!RAGGED || qt0 + kQTile <= N)) {
        tile_pipelined();
      } else {
#pragma unroll
        for (int i = 0; i < 2 * NLD; ++i) issue_part(i);
#pragma unroll
        for (int qb = 0; qb < kQTile / 32; ++qb) {
          const int qb0 = qt0 + 32 * qb;
          if (CAUSAL && qb0 + shift + 31 < kw) continue;   // no query of the block sees a key of the wave
          if (RAGGED && qb0 >= N) continue;                    // nothing but padding
          if (CAUSAL && qb0 + shift < kw + 31) qblock(std::true_type{}, qb);
          else qblock(std::false_type{}, qb);
        }
      }
      if (has_next) store_stats(buf ^ 1);
      wait_vmem();
      __syncthreads();
    };
    if (!GROUPED) {
      for (int t = t0; t < nt; t += 2) {
        tile_step(std::integral_constant<int, 0>{}, t, t - t0);
        if (t + 1 < nt) tile_step(std::integral_constant<int, 1>{}, t + 1, t + 1 - t0);
      }
    } else {
      int t = t0;
      for (int step = 0; step < total; step += 2) {
        tile_step(std::integral_constant<int, 0>{}, t, step);
        t = (t + 1 == nt) ? t0 : t + 1;
        if (step + 1 < total) {
          tile_step(std::integral_constant<int, 1>{}, t, step + 1);
          t = (t + 1 == nt) ? t0 : t + 1;
        }
      }
    }
    if constexpr (kStagedDkDv<D>) {
      char* stage = smem + 4 * TILE_BYTES + 4 * kQTile * (int)sizeof(float);
      const int rows_valid = RAGGED ? NK - kw : 32;
      auto rounded = [&](const f32x16 (&acc)[NDB], float scale) {
        return [&acc, scale](int db, int g) {
          bf16x4 o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) o4[e] = (bf16_t)(acc[db][4 * g + e] * scale);
          return o4;
        };
      };
      store_rows_staged<NDB>(stage, rounded(dVt, 1.0f), dV + 32 * db0 + head_off + (size_t)kw * sn, sn, rows_valid, tid);
      store_rows_staged<NDB>(stage, rounded(dKt, alpha), dK + 32 * db0 + head_off + (size_t)kw * sn, sn, rows_valid, tid);
    } else if (!RAGGED || kw + r < NK) {
      store_acc_T<NDB>(dV + 32 * db0 + head_off + (size_t)(kw + r) * sn, dVt, 1.0f, h);
      store_acc_T<NDB>(dK + 32 * db0 + head_off + (size_t)(kw + r) * sn, dKt, alpha, h);
    }
  }
}

// MODE of the dQ kernel:
//   kGivenDelta     delta is read from `delta` (Alg. 2 with delta computed by attn_delta);
//   kRecomputeDelta instead of dQ the kernel forms delta = rowsum(P o dP) (the recomputed,
//                   float32 form of delta of Sec. 3.2: mathematically rowsum(dO o O), but free of the
//                   forward's bf16 roundings of O); `delta` is not read, `delta_out` receives the
//                   result, dQ is not touched;
//   kOwnDelta       the kernel forms delta = rowsum(dO o O) (Alg. 2 step 4) itself, for the rows it
//                   holds anyway, from `O`, writes it to `delta_out` for the dK/dV kernel that
//                   follows, and goes on as kGivenDelta.  The sum is taken in the order of the
//                   stand-alone delta kernel (8-element chains per 16-byte chunk, then a binary tree
//                   over chunks at distances D/16 ... 1), so both give the same bits.
constexpr int kGivenDelta = 0, kRecomputeDelta = 1, kOwnDelta = 2;

template <int D, bool CAUSAL, bool RAGGED, int MODE>
__global__ __launch_bounds__(256, D <= 128 ? 2 : 1) void attn_bwd_dq_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const bf16_t* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    const bf16_t* __restrict__ O, bf16_t* __restrict__ dQ, float* __restrict__ delta_out, int N,
    float alpha, Layout lay, int pairs, BlockOrder ord) {
  constexpr bool DELTA_MODE = MODE == kRecomputeDelta;
  constexpr int TILE_BYTES = kKTile * kLdsD<D> * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* ldsK = smem;
  char* ldsV = smem + 2 * TILE_BYTES;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int r = lane & 31, h = lane >> 5;

  const int NK = RAGGED ? lay.Nk : N;                 // bounds-checking instantiation: N queries, NK keys,
  const int shift = RAGGED ? NK - N : 0;              // causal mask  key <= query + shift
  const int nqt = (N + kQPerWG - 1) / kQPerWG;
  // pairs != 0 (causal problems with enough work-groups): a work-group takes query block
  // nqt-1-idx and then its mirror image idx; together they always meet the same number of key
  // tiles, so every work-group carries the same load and the grid has no tail of heavy blocks.
  // pairs == 0: one block per work-group, for causal grids in the order the table `ord` gives.
  const int wg = logical_wg(ord, blockIdx.x, gridDim.x);
  const int npw = pairs ? (nqt + 1) / 2 : nqt;          // work-groups per head
  const int bh = wg / npw;
  const int idx = wg % npw;
  const size_t head_off = head_base(lay, bh);
  const int sn = lay.sn;
  const bf16_t* Kh = K + head_base_kv(lay, bh);
  const bf16_t* Vh = V + head_base_kv(lay, bh);
  const float c2 = alpha * kLog2e;
  TileLoader<D> loader;
  loader.init(tid, sn);
  FragOffsets<D> fo;
  init_frag_offsets<D>(fo, lane);
  frag_offsets_add_base<D>(fo, lds_address(smem));

  for (int part = 0; part < (pairs ? 2 : 1); ++part) {
  if (part > 0) __syncthreads();                      // the first block's output staging is done with the tile buffers
  const int qt = pairs ? (part == 0 ? nqt - 1 - idx : idx)
                       : nqt - 1 - (idx + (CAUSAL && ord.n == 0 ? small_grid_rotation(bh, nqt, gridDim.x, D == 128 ? 768 : 1152) : 0)) % nqt;
  if (part == 1 && qt == nqt - 1 - idx) break;        // odd number of blocks: the middle one has no partner
  const int q0 = qt * kQPerWG;
  const int qw = q0 + 32 * wave;

  // Q_i^T / dO_i^T fragments (B operands): lane (r,h) holds Q[qw + r][16kc + 8h .. +7]
  // (rows past the sequence end read the last row; their dQ is not stored)
  const int qc = (RAGGED && qw + r >= N) ? N - 1 : qw + r;
  bf16x8 qf[D / 16], dof[D / 16];
#pragma unroll
  for (int kc = 0; kc < D / 16; ++kc) {
    qf[kc] = *reinterpret_cast<const bf16x8*>(Q + head_off + (size_t)qc * sn + 16 * kc + 8 * h);
    dof[kc] = *reinterpret_cast<const bf16x8*>(dO + head_off + (size_t)qc * sn + 16 * kc + 8 * h);
  }
  float l2 = LSE[(size_t)bh * N + qc] * kLog2e;
  if (RAGGED && l2 == -INFINITY) l2 = 0.f;             // a query that sees no key: all its scores are masked below
  float dl = 0.f;
  if (MODE == kGivenDelta) dl = delta[(size_t)bh * N + qc];
  if (MODE == kOwnDelta) {
    // this lane holds chunks 2kc + h of its row: the chains of its chunks, the tree levels that
    // stay inside one parity class, and the last level (chunk 0 + chunk 1 classes) across the
    // two lanes of the row
    constexpr int NCS = kLdsD<D> / 16;     // D = 96: the tree of a 128-wide row whose last chunks are zero
    float cs[NCS];
#pragma unroll
    for (int kc = 0; kc < NCS; ++kc) cs[kc] = 0.f;
#pragma unroll
    for (int kc = 0; kc < D / 16; ++kc) {
      const bf16x8 o8 = *reinterpret_cast<const bf16x8*>(O + head_off + (size_t)qc * sn + 16 * kc + 8 * h);
      float c = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) c = __builtin_fmaf((float)o8[e], (float)dof[kc][e], c);
      cs[kc] = c;
    }
#pragma unroll
    for (int off = NCS / 2; off >= 1; off >>= 1)
#pragma unroll
      for (int kc = 0; kc < off; ++kc) cs[kc] += cs[kc + off];
    dl = sum_with_partner32(cs[0]);
    if (h == 0 && (!RAGGED || qw + r < N)) delta_out[(size_t)bh * N + qw + r] = dl;
  }
  float pdp = 0.f;                                   // DELTA_MODE: this lane's share of sum_k P dP
  // -delta_i in all 16 accumulator slots of the lane: the third operand of the first dP^T matrix
  // instruction of every key block, which then delivers dP - delta with no vector instruction
  // (Alg. 2: dS = P o (dP - delta)).  Kept opaque so that it stays resident instead of being
  // rebuilt per block.
  f32x16 neg_delta;
#pragma unroll
  for (int i = 0; i < 16; ++i) neg_delta[i] = -dl;
  asm volatile("" : "+v"(neg_delta));
  f32x16 dQt[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) dQt[db][i] = 0.f;

  const int kend = !CAUSAL ? NK : !RAGGED ? q0 + kQPerWG : max(0, min(NK, q0 + kQPerWG + shift));
  const int ntiles = RAGGED ? (kend + kKTile - 1) / kKTile : kend / kKTile;

  loader.template load_rows<RAGGED>(ldsK, Kh, 0, NK, tid);
  loader.template load_rows<RAGGED>(ldsV, Vh, 0, NK, tid);
  wait_vmem();
#pragma unroll
  for (int kc = 0; kc < D / 16; ++kc) { settle(qf[kc]); settle(dof[kc]); }
  settle(l2);
  __syncthreads();

  // One key tile; BUF (which LDS buffer holds it) is a compile-time constant so that every LDS
  // address is a precomputed per-lane offset plus an immediate.
  auto tile_step = [&](auto buf_c, int j) {
    constexpr int buf = decltype(buf_c)::value;
    constexpr int tK = buf * TILE_BYTES;            // byte offsets of this tile's K and V in smem
    constexpr int tV = (2 + buf) * TILE_BYTES;
    // The next tile lands in the other buffer while this one is being processed; its transfer
    // instructions are issued one per step of the first block's score products rather than in one
    // burst behind the barrier.  After the last tile the current one is fetched once more into the
    // idle buffer (harmless; keeps the instruction stream free of branches).
    const int jn = (j + 1 < ntiles) ? j + 1 : j;
    constexpr int NLD = TileLoader<D>::NI;
    const auto pendK = loader.template prepare<RAGGED>(smem + (buf ^ 1) * TILE_BYTES, Kh, jn * kKTile, NK);
    const auto pendV = loader.template prepare<RAGGED>(smem + (2 + (buf ^ 1)) * TILE_BYTES, Vh, jn * kKTile, NK);
    auto issue_part = [&](int i) {
      if (i < NLD) loader.template issue<RAGGED>(pendK, tid, i);
      else if (i < 2 * NLD) loader.template issue<RAGGED>(pendV, tid, i - NLD);
    };
    bool issued = false;
    const int kt0 = j * kKTile;
    if (!CAUSAL || (kt0 <= qw + shift + 31)) {
      // one 32-key block against this wave's 32 queries (one code path: the block that crosses the
      // diagonal only adds a masking step, so that the fragment reads stay next to their matrix
      // instructions instead of being merged in front of a branch)
      auto kblock = [&](int kb, auto first_c) {
        constexpr bool first = decltype(first_c)::value;     // the block that also issues the tile transfer
        const int kb0 = kt0 + 32 * kb;
        // ---- S^T = K_j Q_i^T, dP^T = V_j dO_i^T ; rows = keys, lane = query
        f32x16 s, dp;
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
        for (int kc = 0; kc < D / 16; ++kc) {
          s = mfma32(lds_row8<D>(tK, fo, 32 * kb, kc), qf[kc], s);
          dp = mfma32(lds_row8<D>(tV, fo, 32 * kb, kc), dof[kc], kc == 0 ? neg_delta : dp);
          if (first) issue_part(kc);
        }
        if (first) {
#pragma unroll
          for (int i = D / 16; i < 2 * NLD; ++i) issue_part(i);
          issued = true;
        }
        sched_reads_ahead_of_mfma<D / 8, 1, 4>();
        // element i of this lane is key kb0 + 4h + c with c = 8 (i / 4) + i % 4 a compile-time
        // constant.  Keys in this lane's future (the block crosses the diagonal) and keys past the
        // sequence end get S = -inf: P = exp(-inf) = 0, so they add nothing to dQ.
        if ((CAUSAL && kb0 + 31 > qw + shift) || (RAGGED && kb0 + 32 > NK)) {
          int lim = CAUSAL ? qw + r + shift - kb0 - 4 * h : 0x7fffffff;     // last visible c
          if (RAGGED) lim = min(lim, NK - 1 - kb0 - 4 * h);
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (8 * (i >> 2) + (i & 3) > lim) s[i] = -INFINITY;
        }
        bf16x8 dsf[2];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], c2, -l2));
          if (DELTA_MODE) pdp = __builtin_fmaf(p, dp[i], pdp);
          else dsf[i >> 3][i & 7] = (bf16_t)(p * dp[i]);      // dp already holds dP - delta
        }
        if (!DELTA_MODE) {
          // ---- dQ_i^T += K_j^T dS^T (step 13)
#pragma unroll
          for (int cc = 0; cc < 2; ++cc)
#pragma unroll
            for (int db = 0; db < D / 32; ++db) {
              dQt[db] = mfma32(lds_col8<D>(tK, fo, 32 * kb + 16 * cc, db), dsf[cc], dQt[db]);
            }
          sched_reads_ahead_of_mfma<D / 16, 2, 4>();
        }
      };
#pragma unroll
      for (int kb = 0; kb < kKTile / 32; ++kb) {
        const int kb0 = kt0 + 32 * kb;
        if (CAUSAL && (kb0 > qw + shift + 31)) continue;   // no query of the wave sees a key of the block
        if (RAGGED && kb0 >= NK) continue;                   // nothing but padding
        if (kb == 0) kblock(kb, std::true_type{});
        else kblock(kb, std::false_type{});
      }
    }
    if (!issued) {      // a wave that skipped the tile's first block still has its share of the transfer to issue
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
  if (DELTA_MODE) {
    const float dsum = sum_with_partner32(pdp);      // the partner lane holds the other keys of every block
    if (h == 0 && (!RAGGED || qw + r < N)) delta_out[(size_t)bh * N + qw + r] = dsum;
    continue;
  }
  if constexpr (kCanStage<D / 32>) {
    // the tile buffers are free now (every wave is past the last tile's barrier): they serve as
    // the staging areas of store_rows_staged; the barrier at the top of the part loop keeps the
    // next block's tile transfers from overwriting an area a slower wave is still reading
    auto piece = [&](int db, int g) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = (bf16_t)(dQt[db][4 * g + e] * alpha);
      return o4;
    };
    store_rows_staged<D / 32>(smem, piece, dQ + head_off + (size_t)qw * sn, sn, RAGGED ? N - qw : 32, tid);
  } else if (!RAGGED || qw + r < N) {
    store_acc_T<D / 32>(dQ + head_off + (size_t)(qw + r) * sn, dQt, alpha, h);
  }
  }   // part
}

template <typename KernT>
static hipError_t set_smem(KernT kern, int smem, std::atomic<bool>& done) {
  if (done.load(std::memory_order_acquire)) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e == hipSuccess) done.store(true, std::memory_order_release);
  return e;
}

template <int D, bool CAUSAL, bool RAGGED, bool GROUPED>
static hipError_t launch_dkdv(const void* Q, const void* K, const void* V, const void* dO,
                              const float* LSE, const float* delta, void* dK, void* dV, int BH,
                              int N, float alpha, Layout lay, hipStream_t st) {
  constexpr int NDB = D / 32 / kDSplit<D>;
  constexpr int smem = 4 * kQTile * kLdsD<D> * 2 + 4 * kQTile * (int)sizeof(float) +
                       (kStagedDkDv<D> ? 4 * 32 * kStagePitch<NDB> : 0);
  static std::atomic<bool> set{false};
  auto k = attn_bwd_dkdv_kernel<D, CAUSAL, RAGGED, GROUPED>;
  hipError_t e;
  if ((e = set_smem(k, smem, set)) != hipSuccess) return e;
  const int nkt = ((RAGGED ? lay.Nk : N) + kKeysPerWG - 1) / kKeysPerWG;
  // Under the causal mask: one block per work-group in a balanced order when that grid is at most
  // one and a half rounds of work-groups (measured: beyond that, mirrored pairs of blocks are as
  // fast or 2 % faster for this kernel), mirrored pairs otherwise.
  static std::atomic<int> resident{0};
  static thread_local OrderCache cache;
  const BlockOrder* ord = &kNoOrder;
  if (CAUSAL && kDSplit<D> == 1) {
    const int res = resident_per_cu(k, smem, resident);
    ord = &small_grid_order(cache, (BH / lay.group) * nkt, nkt, res, 3LL * kNumCUs * res / 2);
  }
  const int pairs = (CAUSAL && ord->n == 0) ? 1 : 0;
  hipLaunchKernelGGL(k, dim3((BH / lay.group) * (pairs ? (nkt + 1) / 2 : nkt) * kDSplit<D>), dim3(256), smem, st, (const bf16_t*)Q,
                     (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, LSE, delta,
                     (bf16_t*)dK, (bf16_t*)dV, N, alpha, lay, pairs, *ord);
  return hipGetLastError();
}

template <int D, bool CAUSAL, bool RAGGED, int MODE>
static hipError_t launch_dq(const void* Q, const void* K, const void* V, const void* dO,
                            const float* LSE, const float* delta, const void* O, void* dQ,
                            float* delta_out, int BH, int N, float alpha, Layout lay, hipStream_t st) {
  constexpr int smem = 4 * kKTile * kLdsD<D> * 2;
  static std::atomic<bool> set{false};
  auto k = attn_bwd_dq_kernel<D, CAUSAL, RAGGED, MODE>;
  hipError_t e;
  if ((e = set_smem(k, smem, set)) != hipSuccess) return e;
  // as in the forward: mirrored pairs of query blocks under the causal mask when that still
  // leaves at least two full rounds of work-groups
  const int nqt = (N + kQPerWG - 1) / kQPerWG;
  const int pairs = (CAUSAL && (long long)BH * ((nqt + 1) / 2) >= 1024) ? 1 : 0;
  const int grid = BH * (pairs ? (nqt + 1) / 2 : nqt);
  static std::atomic<int> resident{0};
  static thread_local OrderCache cache;
  const BlockOrder& ord = (CAUSAL && !pairs)
      ? small_grid_order(cache, grid, nqt, resident_per_cu(k, smem, resident), 8 * kMaxOrder) : kNoOrder;
  hipLaunchKernelGGL(k, dim3(grid), dim3(256), smem, st, (const bf16_t*)Q,
                     (const bf16_t*)K, (const bf16_t*)V, (const bf16_t*)dO, LSE, delta,
                     (const bf16_t*)O, (bf16_t*)dQ, delta_out, N, alpha, lay, pairs, ord);
  return hipGetLastError();
}

}  // namespace

hipError_t attn_bwd_dkdv_dispatch(const void* Q, const void* K, const void* V, const void* dO,
                                  const float* LSE, const float* delta, void* dK, void* dV,
                                  int BH, int N, int d, int causal, float alpha, Layout lay,
                                  hipStream_t st) {
  const bool ragged = (N % kKeysPerWG) != 0 || lay.Nk != N;   // the aligned kernels carry no bounds handling
  if (lay.group > 1) {   // grouped queries: the bounds-checking instantiation serves every N
#define CASEG(DD, CC)                                 \
  if (d == DD && (causal != 0) == CC)                 \
    return launch_dkdv<DD, CC, true, true>(Q, K, V, dO, LSE, delta, dK, dV, BH, N, alpha, lay, st);
    CASEG(32, false) CASEG(32, true) CASEG(64, false) CASEG(64, true) CASEG(128, false) CASEG(128, true)
    CASEG(256, false) CASEG(256, true) CASEG(96, false) CASEG(96, true)
#undef CASEG
    return hipErrorInvalidValue;
  }
#define CASE(DD, CC, RR)                                                \
  if (d == DD && (causal != 0) == CC && ragged == RR)                   \
    return launch_dkdv<DD, CC, RR, false>(Q, K, V, dO, LSE, delta, dK, dV, BH, N, alpha, lay, st);
  CASE(32, false, false) CASE(32, false, true) CASE(32, true, false) CASE(32, true, true)
  CASE(64, false, false) CASE(64, false, true) CASE(64, true, false) CASE(64, true, true)
  CASE(128, false, false) CASE(128, false, true) CASE(128, true, false) CASE(128, true, true)
  CASE(256, false, false) CASE(256, false, true) CASE(256, true, false) CASE(256, true, true)
  CASE(96, false, false) CASE(96, false, true) CASE(96, true, false) CASE(96, true, true)
#undef CASE
  return hipErrorInvalidValue;
}

// O == nullptr: delta is given.  Otherwise delta is formed by the kernel from O and dO and also
// written to delta_out (which must then be non-null).
hipError_t attn_bwd_dq_dispatch(const void* Q, const void* K, const void* V, const void* dO,
                                const float* LSE, const float* delta, const void* O, void* dQ,
                                float* delta_out, int BH, int N, int d, int causal, float alpha,
                                Layout lay, hipStream_t st) {
  const bool ragged = (N % kQPerWG) != 0 || lay.Nk != N;
  const bool own = O != nullptr;
#define CASE(DD, CC, RR)                                                \
  if (d == DD && (causal != 0) == CC && ragged == RR)                   \
    return own ? launch_dq<DD, CC, RR, kOwnDelta>(Q, K, V, dO, LSE, nullptr, O, dQ, delta_out, BH, N, alpha, lay, st) \
               : launch_dq<DD, CC, RR, kGivenDelta>(Q, K, V, dO, LSE, delta, nullptr, dQ, nullptr, BH, N, alpha, lay, st);
  CASE(32, false, false) CASE(32, false, true) CASE(32, true, false) CASE(32, true, true)
  CASE(64, false, false) CASE(64, false, true) CASE(64, true, false) CASE(64, true, true)
  CASE(128, false, false) CASE(128, false, true) CASE(128, true, false) CASE(128, true, true)
  CASE(256, false, false) CASE(256, false, true) CASE(256, true, false) CASE(256, true, true)
  CASE(96, false, false) CASE(96, false, true) CASE(96, true, false) CASE(96, true, true)
#undef CASE
  return hipErrorInvalidValue;
}

// delta = rowsum(P o dP) recomputed from Q, K, V, dO and LSE (always the bounds-checking kernels).
hipError_t attn_delta_recompute_dispatch(const void* Q, const void* K, const void* V,
                                         const void* dO, const float* LSE, float* delta_out,
                                         int BH, int N, int d, int causal, float alpha,
                                         Layout lay, hipStream_t st) {
#define CASE(DD, CC)                                  \
  if (d == DD && (causal != 0) == CC)                 \
    return launch_dq<DD, CC, true, kRecomputeDelta>(Q, K, V, dO, LSE, nullptr, nullptr, nullptr, delta_out, BH, N, alpha, lay, st);
  CASE(32, false) CASE(32, true) CASE(64, false) CASE(64, true) CASE(128, false) CASE(128, true)
  CASE(256, false) CASE(256, true) CASE(96, false) CASE(96, true)
#undef CASE
  return hipErrorInvalidValue;
}
