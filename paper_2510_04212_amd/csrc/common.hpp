// Shared device helpers for the gfx950 attention kernels: vector types, the matrix-core
// wrappers, the LDS tile layout (16-byte-chunk XOR swizzle) and cross-lane exchanges.
//
// Matrix-core fragment layouts used throughout (wave64, v_mfma_f32_32x32x16_bf16,
// D[32x32] += A[32x16] * B[16x32]; lane l, r = l & 31, h = l >> 5):
//   A operand: lane holds A[r][8h .. 8h+7]            (8 consecutive k of one row)
//   B operand: lane holds B[8h .. 8h+7][r]            (8 consecutive k of one column)
//   D / C    : register i of lane holds D[8*(i/4) + 4h + (i%4)][r]
// Because the contraction index may be permuted freely as long as A and B agree, a C-layout
// tile can be fed back as a B operand: registers 8c..8c+7 of a lane are the k-slots (h, 0..7)
// of 16-wide k-chunk c, i.e. k-slot (h, j) of chunk c  <->  tile row 16c + 8*(j/4) + 4h + (j%4).
#pragma once
#include "block_order.hpp"
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

#define DEVI __device__ __forceinline__

constexpr float kLog2e = 1.4426950408889634f;

DEVI f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Width of an LDS tile row, in elements, for head size D.  The swizzle and the tile loader work on
// power-of-two rows; D = 96 uses 128-wide rows of which the last 32 columns are never read.
template <int D> constexpr int kLdsD = (D == 96) ? 128 : D;

// Swizzle of the 16-byte chunk index inside one tile row, chosen so that (a) 16 lanes reading
// the same chunk of 16 consecutive rows and (b) a transposing read touching 8 consecutive rows
// x 64 bytes both spread over all 64 LDS banks.
template <int D> DEVI int swz(int row);
template <> DEVI int swz<128>(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
// D = 256: rows are 512 bytes, as at D = 128 every row starts on bank 0: the same permutation of
// the low four chunk-index bits serves (the fifth bit is left alone).
template <> DEVI int swz<256>(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }
// D = 32: a row is 4 chunks (64 bytes), four consecutive rows span the 64 banks once; rows r and
// r + 4 would collide in (a) unless their chunk positions differ.  (b) touches 8 whole rows there.
template <> DEVI int swz<32>(int row) { return (row >> 2) & 3; }
template <> DEVI int swz<64>(int row) {
  int t = row >> 1;
  return ((t & 1) << 2) | (t & 2) | ((t >> 2) & 1);
}

// Byte offset of element (row, col) of a [rows][D] bf16 tile in LDS; col must be a multiple of 4
// for 8-byte accesses and of 8 for 16-byte accesses.
template <int D> DEVI int tile_off(int row, int col) {
  constexpr int DL = kLdsD<D>;
  int chunk = col >> 3;
  return row * (DL * 2) + ((chunk ^ swz<DL>(row)) << 4) + ((col & 7) << 1);
}

// 16-byte natural read: 8 consecutive columns of one row (an A/B fragment whose contraction
// index runs along the tile's columns).
template <int D> DEVI bf16x8 lds_read_row8(const char* tile, int row, int col) {
  return *reinterpret_cast<const bf16x8*>(tile + tile_off<D>(row, col));
}

// Transposing read: returns, for this lane, 4 consecutive ROWS (row0..row0+3) of column
// col0 + (lane & 15).  ds_read_b64_tr_b16 works on groups of 16 lanes: lane i of a group
// supplies the address of 4 consecutive columns (4*(i&3)..) of row (i>>2), and receives
// column i of rows 0..3.  col0 must be a multiple of 16.
template <int D> DEVI s16x4 lds_read_tr4(const char* tile, int row0, int col0, int lane) {
  int i = lane & 15;
  int off = tile_off<D>(row0 + (i >> 2), col0 + ((i & 3) << 2));
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(tile + off));
}

// Fragment whose contraction index runs along the tile's ROWS: k-slots (h, 0..7) of the
// 16-row chunk starting at row_base are rows row_base + 8*(j/4) + 4h + (j%4), j = 0..7;
// the lane's own index (lane & 31) selects column col_base + (lane & 31).
template <int D> DEVI bf16x8 lds_read_col8(const char* tile, int row_base, int col_base, int lane) {
  int h = lane >> 5;
  int c0 = col_base + (lane & 16);
  union { struct { s16x4 lo, hi; } p; bf16x8 v; } u;
  u.p.lo = lds_read_tr4<D>(tile, row_base + 4 * h, c0, lane);
  u.p.hi = lds_read_tr4<D>(tile, row_base + 8 + 4 * h, c0, lane);
  return u.v;
}

// ---- The same two fragment reads with the lane-dependent part of the address precomputed.
// The swizzle only looks at row bits 0..3, so moving a fragment by a multiple of 16 rows adds a
// constant to the byte offset: per lane, D/16 offsets serve every row-major (natural) fragment
// and 2 x D/32 offsets every column-major (transposing) one; the rest folds into the
// instruction's immediate offset when the tile address is a compile-time constant.
// The offsets are made absolute LDS addresses once (frag_offsets_add_base); the fragment readers
// below then address LDS as "per-lane register + compile-time constant", which the compiler
// turns into the instruction's immediate offset.  (With the shared-memory symbol in the address
// expression instead, it re-adds the symbol's address - a link-time value - in a vector
// instruction in front of every read.)
template <int D> struct FragOffsets {
  int row[D / 16];          // natural read of columns 16kc + 8h .. +7 of row (lane & 31)
  int col[2][D / 32];       // transposing reads: rows 4h + 8*half + 0..3, column 32db + (lane & 31)
};
// 32-bit LDS address of a pointer into shared memory
DEVI int lds_address(const void* p) {
  typedef __attribute__((address_space(3))) const char lds_char;
  return (int)(unsigned)(unsigned long)((lds_char*)p);
}
template <int D> DEVI void init_frag_offsets(FragOffsets<D>& fo, int lane) {
  const int r = lane & 31, h = lane >> 5, i = lane & 15;
#pragma unroll
  for (int kc = 0; kc < D / 16; ++kc) fo.row[kc] = tile_off<D>(r, 16 * kc + 8 * h);
#pragma unroll
  for (int half = 0; half < 2; ++half)
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
      fo.col[half][db] = tile_off<D>(4 * h + 8 * half + (i >> 2), 32 * db + (lane & 16) + ((i & 3) << 2));
}
// shared_base: LDS address of the array the tiles live in (lds_address(smem))
// (each sum passes through an empty asm statement: otherwise the compiler, rather than keep it in
// a register, re-adds the base in front of every use)
template <int D> DEVI void frag_offsets_add_base(FragOffsets<D>& fo, int shared_base) {
#pragma unroll
  for (int kc = 0; kc < D / 16; ++kc) {
    fo.row[kc] += shared_base;
    asm volatile("" : "+v"(fo.row[kc]));
  }
#pragma unroll
  for (int half = 0; half < 2; ++half)
#pragma unroll
    for (int db = 0; db < D / 32; ++db) {
      fo.col[half][db] += shared_base;
      asm volatile("" : "+v"(fo.col[half][db]));
    }
}
// `tile`: byte offset of the tile inside the shared-memory array (fo holds absolute addresses).
// rows row_base + (lane & 31), row_base a multiple of 16
template <int D> DEVI bf16x8 lds_row8(int tile, const FragOffsets<D>& fo, int row_base, int kc) {
  typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;
  return *reinterpret_cast<lds_bf16x8*>((unsigned long)(unsigned)(fo.row[kc] + tile + row_base * (kLdsD<D> * 2)));
}
// k-slots = rows row_base + 8*(j/4) + 4h + (j%4), column 32db + (lane & 31); row_base a multiple of 16
template <int D> DEVI bf16x8 lds_col8(int tile, const FragOffsets<D>& fo, int row_base, int db) {
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  union { struct { s16x4 lo, hi; } p; bf16x8 v; } u;
  u.p.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (lds_s16x4*)(unsigned long)(unsigned)(fo.col[0][db] + tile + row_base * (kLdsD<D> * 2)));
  u.p.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
      (lds_s16x4*)(unsigned long)(unsigned)(fo.col[1][db] + tile + row_base * (kLdsD<D> * 2)));
  return u.v;
}

// Value held by the lane 32 positions away (lane ^ 32).
DEVI float partner32(float x) {
  unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0] = {lower-half values in all lanes}, r[1] = {upper-half values in all lanes}
  return (threadIdx.x & 32) ? __uint_as_float(r[0]) : __uint_as_float(r[1]);
}
DEVI float max_with_partner32(float x) {
  unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
DEVI float sum_with_partner32(float x) {
  unsigned u = __float_as_uint(x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Addressing of the bf16 tensors Q, K, V, O, dO, dQ, dK, dV: element (b, h, n, k) lives at
// b*sb + h*sh + n*sn + k (the last dimension is contiguous).  [B,H,N,d] contiguous is
// (H*N*d, N*d, d); [B,N,H,d] is (N*H*d, d, H*d).  float32 per-row tensors (LSE, delta) and the
// optional float32 / int32 outputs are always contiguous [B,H,N(,d)].
// Grouped-query attention: K, V, dK, dV have H / group heads with their own batch / head strides
// (sb_kv, sh_kv); query head h uses key/value head h / group.  group = 1 is ordinary attention.
// Nk: rows of K, V, dK, dV per head.  The kernels' sequence-length argument N counts the queries
// (rows of Q, O, dO, dQ, LSE, delta).  Only the bounds-checking kernel instantiations read Nk
// (the others are used for N == Nk, multiples of the block size); with Nk != N the causal mask
// is aligned at the bottom right: query r sees keys c <= r + (Nk - N).
struct Layout {
  long long sb, sh;
  int sn;
  int H;
  long long sb_kv, sh_kv;
  int group;
  int Nk;
};
// first element of query-side head bh = b*H + h
DEVI size_t head_base(const Layout& lay, int bh) {
  return (size_t)(bh / lay.H) * (size_t)lay.sb + (size_t)(bh % lay.H) * (size_t)lay.sh;
}
// first element of the key/value head that query-side head bh attends to
DEVI size_t head_base_kv(const Layout& lay, int bh) {
  return (size_t)(bh / lay.H) * (size_t)lay.sb_kv + (size_t)((bh % lay.H) / lay.group) * (size_t)lay.sh_kv;
}

// Asynchronous copy of a 64-row x D bf16 tile from global memory straight into swizzled LDS
// (global_load_lds_dwordx4: no registers are involved; completion is tracked by vmcnt).
// One wave-instruction moves 64 x 16 bytes to LDS base + 16*lane, i.e. 1024 consecutive bytes =
// 64/CH whole tile rows; the XOR swizzle is applied on the GLOBAL side: the lane that lands in
// chunk slot s of row r fetches chunk s ^ swz(r) of that row.  256 threads (4 waves).
// The caller must execute wait_vmem() and a barrier before any wave reads the tile.
//
// The instruction is emitted through inline assembly on purpose: when the compiler itself sees a
// pending global->LDS transfer it turns every later LDS wait into "wait for everything"
// (lgkmcnt(0)) and inserts a full vmcnt(0) before the first transposing LDS read, which defeats
// both the fragment read-ahead and the overlap of the transfer with computation.  Hidden from
// its bookkeeping, the transfer only makes the compiler's own vmcnt waits more conservative
// (loads complete in order), and its completion is enforced explicitly by wait_vmem().
// A pointer the caller knows to be the same in every lane, as a scalar-register value (the tile
// loader's instruction takes its base address from scalar registers).
DEVI const bf16_t* wave_uniform(const bf16_t* p) {
  const unsigned long long u = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)u);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(u >> 32));
  return reinterpret_cast<const bf16_t*>(((unsigned long long)hi << 32) | lo);
}

template <int D> struct TileLoader {
  static constexpr int DL = kLdsD<D>;            // LDS row width
  static constexpr int CH = DL / 8;              // 16-byte chunk slots per LDS row
  // source chunk that lands in slot `slot` of LDS row `row`; slots whose chunk lies beyond the D
  // columns (D < DL) re-fetch one of the row's real chunks, which nobody reads
  static DEVI int src_chunk(int slot, int row) {
    const int c = slot ^ swz<DL>(row);
    return (D < DL && c >= D / 8) ? (c & 7) : c;
  }
  static constexpr int RPI = 64 / CH;            // rows per wave-instruction
  static constexpr int NI = 64 / RPI / 4;        // instructions per wave (4 waves share a tile)
  unsigned voff[NI];                             // per-lane byte offset inside the source tile
  unsigned lds_wave;                             // byte offset of this wave's first row in the LDS tile
  int sn;                                        // distance between consecutive rows of the source, in elements
  DEVI void init(int tid, int row_stride) {
    const int wave = tid >> 6, lane = tid & 63;
    sn = row_stride;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int row = (wave * NI + i) * RPI + lane / CH;
      const int c = src_chunk(lane % CH, row);
      voff[i] = (unsigned)(row * sn + c * 8) * 2u;
    }
    lds_wave = (unsigned)(wave * NI * RPI * DL * 2);
  }
  // Same for a source tile of which only the first `valid` rows (1..64) exist: rows beyond them
  // re-read the last valid row, so that nothing is fetched out of bounds and the LDS tile holds
  // finite values everywhere (the kernels mask those rows / columns out).
  DEVI void load_clamped(const char* tile, const bf16_t* src, int valid, int tid) const {
    typedef __attribute__((address_space(3))) const char lds_char;
    const int wave = tid >> 6, lane = tid & 63;
    const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long)((lds_char*)tile) + lds_wave);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int row = (wave * NI + i) * RPI + lane / CH;
      const int c = src_chunk(lane % CH, row);
      const int rc = row < valid ? row : valid - 1;
      const unsigned vo = (unsigned)(rc * sn + c * 8) * 2u;
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(base + (unsigned)(i * RPI * DL * 2)), "v"(vo), "s"(src)
                   : "m0");
    }
  }
  // Tile starting at row `row0` of a tensor with `N` rows (row0 < N).  RAGGED: the tile may
  // reach past row N-1 and is then loaded clamped; otherwise every tile is known to be full.
  template <bool RAGGED>
  DEVI void load_rows(const char* tile, const bf16_t* tensor, int row0, int N, int tid) const {
    const bf16_t* src = wave_uniform(tensor + (size_t)row0 * sn);
    if (!RAGGED || row0 + 64 <= N) load(tile, src);
    else load_clamped(tile, src, N - row0, tid);
  }
  // A tile transfer prepared once (scalar operands) and issued one instruction at a time, so that a
  // caller can spread it over its matrix instructions instead of issuing it in one burst.
  struct Pending { const bf16_t* src; unsigned base; int valid; };
  template <bool RAGGED>
  DEVI Pending prepare(const char* tile, const bf16_t* tensor, int row0, int N) const {
    typedef __attribute__((address_space(3))) const char lds_char;
    Pending p;
    p.src = wave_uniform(tensor + (size_t)row0 * sn);
    p.base = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long)((lds_char*)tile) + lds_wave);
    p.valid = RAGGED ? N - row0 : 64;
    return p;
  }
  // instruction i (0 .. NI-1) of the prepared transfer
  template <bool RAGGED>
  DEVI void issue(const Pending& p, int tid, int i) const {
    unsigned vo = voff[i];
    if (RAGGED && p.valid < 64) {
      const int wave = tid >> 6, lane = tid & 63;
      const int row = (wave * NI + i) * RPI + lane / CH;
      const int c = src_chunk(lane % CH, row);
      const int rc = row < p.valid ? row : p.valid - 1;
      vo = (unsigned)(rc * sn + c * 8) * 2u;
    }
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(p.base + (unsigned)(i * RPI * DL * 2)), "v"(vo), "s"(p.src)
                 : "m0");
  }
  // tile: LDS address of the destination tile; src: first row of the 64-row source tile (wave-uniform)
  DEVI void load(const char* tile, const bf16_t* src) const {
    typedef __attribute__((address_space(3))) const char lds_char;
    const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long)((lds_char*)tile) + lds_wave);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :
                   : "s"(base + (unsigned)(i * RPI * DL * 2)), "v"(voff[i]), "s"(src)
                   : "m0");
    }
  }
};

// s_waitcnt vmcnt(0): every outstanding global load (including loads into LDS) has landed.
DEVI void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// Marks a register value as used at this point, so that the compiler waits HERE for the load that
// produces it rather than at its first real use.  The kernels call it on their register-resident
// fragments right after the explicit wait in front of the tile loop: a compiler-generated
// "vmcnt(n)" left inside the loop (needed in its first pass only) would in every later pass also
// wait for the next tile's global->LDS transfers, which the compiler does not know of, and stall
// the wave at the start of each tile until they have landed.
template <class T> DEVI void settle(T& x) { asm volatile("" : "+v"(x)); }

// Sum of the two bf16 values of a packed pair, added to acc in float32 (v_dot2c_f32_bf16 with
// a (1,1) second operand).
DEVI float add_pair_bf16(bf16x2 p, float acc) {
  bf16x2 one;
  one[0] = (bf16_t)1.0f;
  one[1] = (bf16_t)1.0f;
  return __builtin_amdgcn_fdot2_f32_bf16(p, one, acc, false);
}

// x / l for the many x that share one divisor l (a row's outputs): a reciprocal of l refined by
// one Newton step, then per quotient one product and one residual correction.  The result is the
// correctly rounded quotient up to rare last-bit cases, and exact whenever l is a power of two;
// 4 instructions per quotient instead of the ~10 of a full division.  A subnormal or tiny l (the
// reciprocal instruction takes no subnormal inputs) is handled by scaling numerator and
// denominator by 2^64 first, which is exact.  l = 0 gives NaN.
struct Divisor { float l, r, scale; };
DEVI Divisor make_divisor(float l) {
  const float scale = l < 0x1p-64f ? 0x1p64f : 1.0f;
  const float ls = l * scale;
  const float r0 = __builtin_amdgcn_rcpf(ls);
  return Divisor{ls, __builtin_fmaf(__builtin_fmaf(-ls, r0, 1.0f), r0, r0), scale};
}
DEVI float divide(float x, Divisor d) {
  const float xs = x * d.scale;
  const float q = xs * d.r;
  return __builtin_fmaf(__builtin_fmaf(-q, d.l, xs), d.r, q);
}

// Output rows of a wave that holds a 32-row tile transposed in accumulator layout (lane (r,h) has,
// for its row r, the columns 32db + 8g + 4h .. +3 of every (db, g)): written straight from the
// registers, every store instruction would put 8-byte pieces into 32 different rows.  Instead the
// wave passes the tile through an LDS staging area of its own (32 rows of kStagePitch<NDB> bytes,
// wave w's area following wave w-1's from stage_wave0 on) and stores whole rows, 16 bytes per
// lane with consecutive lanes on consecutive chunks.  No barrier is involved: the area belongs to this wave alone, and the LDS executes one wave's
// accesses in order.  piece(db, g) returns the four bf16 values of that position; rows at or
// beyond rows_valid are not stored.  Needs 64 % (4 NDB) == 0.
template <int NDB> constexpr int kStagePitch = 64 * NDB + 16;   // +16: rows start 4 banks apart
template <int NDB> constexpr bool kCanStage = (64 % (4 * NDB)) == 0;
template <int NDB, class PieceF>
DEVI void store_rows_staged(char* stage_wave0, PieceF&& piece, bf16_t* dst_row0, int sn, int rows_valid, int tid) {
  static_assert(kCanStage<NDB>, "row width");
  constexpr int PITCH = kStagePitch<NDB>;
  constexpr int CPR = 4 * NDB;                  // 16-byte chunks per row
  constexpr int RPI = 64 / CPR;                 // rows per store instruction
  // The thread index goes through a copy the compiler cannot see through: every address below
  // depends on it, and computed from the kernel's own copy they would all be formed before the
  // tile loop and held in registers through it.
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  char* stage = stage_wave0 + (tid >> 6) * (32 * PITCH);
  const int r = lane & 31, h = lane >> 5;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *reinterpret_cast<bf16x4*>(stage + r * PITCH + (32 * db + 8 * g + 4 * h) * 2) = piece(db, g);
  typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
#pragma unroll
  for (int it = 0; it < 32 / RPI; ++it) {
    const int row = it * RPI + lane / CPR, c = lane % CPR;
    const u32x4 v = *reinterpret_cast<const u32x4*>(stage + row * PITCH + c * 16);
    if (row < rows_valid) *reinterpret_cast<u32x4*>(dst_row0 + (size_t)row * sn + c * 8) = v;
  }
}

// Issue-order hints for one scheduling region (basic block) that holds N matrix instructions,
// each fed by PER LDS fragment reads: the reads are issued AHEAD matrix instructions before
// their use, so that LDS latency is covered by matrix-core work instead of stalling the wave.
// (sched_group_barrier masks: 0x008 = MFMA, 0x100 = LDS read.)
template <int N, int PER, int AHEAD_> DEVI void sched_reads_ahead_of_mfma() {
  static_assert(PER == 1 || PER == 2, "PER");
  constexpr int AHEAD = AHEAD_ < N ? AHEAD_ : N;
  __builtin_amdgcn_sched_group_barrier(0x100, AHEAD * PER, 0);
#pragma unroll
  for (int i = 0; i < N - AHEAD; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, PER, 0);
  }
#pragma unroll
  for (int i = 0; i < AHEAD; ++i) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
}

// Work-group index remap: consecutive hardware work-group ids go round-robin over the 8 XCDs
// (each with its own L2).  Give every XCD a contiguous range of logical ids so that the
// work-groups sharing one head's K/V run on the same L2.  Only applied when the grid is a
// multiple of 8 (otherwise the map would not be a bijection).
DEVI int xcd_remap(int id, int n) {
  if ((n & 7) != 0) return id;
  return (id & 7) * (n >> 3) + (id >> 3);
}

// Logical id of a work-group: with an order table (block_order.hpp) the s-th work-group of an XCD
// takes item pos[s] of the XCD's contiguous share of the grid, otherwise the plain remap above.
// The table is a kernel argument, i.e. read with scalar loads.
DEVI int logical_wg(const BlockOrder& ord, int id, int n) {
  if (ord.n == 0) return xcd_remap(id, n);
  return (id & 7) * (n >> 3) + ord.pos[id >> 3];
}

// Rotation of the causal block order of one head, for grids small enough to be resident all at
// once or nearly so (at most `capacity` work-groups, which callers set to 1.5x what the chip
// holds of that kernel: measured, the rotation wins up to one and a half rounds of work-groups;
// from two rounds on, plain heavy-first order does better and is kept).  Blocks of one head differ in
// work by up to nblk : 1.  Work-groups are handed to the CUs of an XCD round-robin, so with a
// fixed heavy-to-light order the j-th work-group of a CU always lands on the same weight class;
// rotating the order by a different amount for each "lap" over the XCD's 32 CUs gives every CU
// a mix.  The rotation depends on the head only, so every block is still visited once.
DEVI int small_grid_rotation(int bh, int nblk, int grid, int capacity) {
  if (grid > capacity || (grid & 7) != 0) return 0;
  const int first = (bh * nblk) % (grid >> 3);     // dispatch sequence number of the head's first block inside its XCD
  return (3 * (first >> 5)) % nblk;
}

// ---- host side of the order table --------------------------------------------------------------
constexpr int kNumCUs = 256;

// Work-groups of `kern` (256 threads, `smem` bytes of dynamic LDS) that a compute unit holds at
// once; asked of the runtime once per kernel instantiation.
template <class KernT>
static int resident_per_cu(KernT kern, int smem, std::atomic<int>& cached) {
  int r = cached.load(std::memory_order_relaxed);
  if (r == 0) {
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&r, reinterpret_cast<const void*>(kern), 256, smem) != hipSuccess || r <= 0) {
      (void)hipGetLastError();   // the answer only steers the block order: not an error of the launch that follows
      r = 1;
    }
    cached.store(r, std::memory_order_relaxed);
  }
  return r;
}

// The table for a causal grid of `grid` one-block work-groups with `nblk` blocks per head; empty
// (n = 0) unless the grid is at most `max_grid`, a multiple of 8, every XCD's share holds whole
// heads and fits the table.  The last table is kept (one per calling thread and kernel
// instantiation), so a training loop computes it once.
struct OrderCache {
  int grid = -1, nblk = -1, resident = -1;
  BlockOrder ord;
};
static const BlockOrder kNoOrder{};
static const BlockOrder& small_grid_order(OrderCache& c, int grid, int nblk, int resident, long long max_grid) {
  if (c.grid != grid || c.nblk != nblk || c.resident != resident) {
    c.grid = grid; c.nblk = nblk; c.resident = resident;
    c.ord.n = 0;
    if ((grid & 7) == 0 && grid <= max_grid) fill_block_order(c.ord, grid >> 3, nblk, resident);
  }
  return c.ord;
}
