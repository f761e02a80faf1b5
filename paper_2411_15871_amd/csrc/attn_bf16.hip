// bf16 causal grouped-query flash attention on the matrix cores, forward and backward.
// Layout: qkv[T, (nq+2nkv)*D] = [q heads | k heads | v heads] (q, k already rotated), o[T, nq*D],
// lse[nq, T] (natural log), delta[nq, T] = rowsum(dO * O).  Tokens are sequence-major; a block
// never crosses a sequence boundary.  D = head_dim is 64 or 128.
// Keys and values are read through AttnGeom: from the packed qkv rows for plain causal attention, or from a
// gathered buffer that also holds the rows of earlier context-parallel ranks (the queries are then the last
// seq - q_off positions of each sequence); dK/dV are written the same way.
//
// All three kernels compute score tiles "transposed" where that keeps per-query statistics
// lane-local: v_mfma_f32_32x32x16_bf16 leaves column j of its result in lane j%32, so
//   forward / dQ : S^T = K Q^T        (column = query  -> running max/sum, lse, delta live in the lane)
//   dK/dV        : S   = Q K^T        (column = key    -> the dK^T, dV^T accumulators keep their column)
// and the probability tile is fed back as the B operand of the next product straight from registers
// (the 8 k-slots of a lane are rows 8*(r/4)+4*(lane/32)+r%4 of two adjacent register quads).  The
// matching A operand (V^T, K^T, dO^T, Q^T: "k" is the token index, the slow dimension in memory)
// comes from LDS through the transposing load ds_read_b64_tr_b16.
//
// 64-token tiles stream global -> LDS directly (see dma.h) through a ring of three slots (two in the
// forward kernel, so that two of its blocks fit a compute unit): the transfer of tile t+2 (t+1) is issued
// right after the barrier that publishes tile t.  A tile is stored
// [token][D] unpadded; the 16-byte chunk c of row r sits at chunk position c ^ swz(r), which makes
// the 16-byte fragment reads (16 consecutive rows, one chunk) and the transposing reads (4
// consecutive rows x 64 bytes) both bank-conflict free for 256-byte rows (D = 128).
// Blocks are launched heaviest first over all heads (the causal work per block grows with its position).
// Long rows of tiles may be cut into chunks whose float32 partial results a small kernel merges in chunk
// order; the chunk length is chosen per launch from a simulation of the launch (pick_chunk below).
// No atomics: dQ is produced per query block, dK/dV per (key block, query head), then the heads of
// a group are added in index order.
#include <map>
#include <mutex>
#include <queue>
#include <tuple>
#include <vector>
#include "common.h"
#include "dma.h"

#define AB_THREADS 256
#define AB_KT 64   // tokens per LDS tile
#define AB_RING 3  // tile slots
#define AB_CH 16   // backward: a block walks at most g.ch 64-token tiles, this many by default (longer causal rows are split
                   // into chunks whose float32 partial results a second kernel adds in chunk order)

// Work split of the backward kernels.  Along the block's own dimension there are ceil(seq/128) blocks;
// block i has tiles_of(i) tiles to walk and is cut into ceil(tiles/ch) chunks (ch is chosen per launch).  A launch index is
// mapped to (block, chunk) heaviest block first; `pair` numbers the (block, chunk) pairs in natural order.
//
// Positions.  seq = keys per sequence (positions 0..seq-1); the queries of a sequence are its positions
// q_off..seq-1 (q_off = 0: every position; otherwise a multiple of 128, so that query blocks and key blocks
// share one grid of 128-position blocks, of which blocks q_off/128.. hold queries).  Query-side arrays (q in qkv,
// o, dout, lse, delta, dq) are indexed by the local token b*(seq-q_off) + position - q_off; keys, values and
// their gradients by b*seq + position in kv / dkv, rows of ldkv / lddkv elements laid out [k heads | v heads].
struct AttnGeom {
  int seq, q_off, nq, nkv;
  const bf16_t* kv; int ldkv;
  bf16_t* dkv; int lddkv;
  int ch;      // backward kernels: 64-token tiles per chunk
  int nq_all;  // nq * batch: a launch index is (pair index) * nq_all + (batch * nq + head), so that the heaviest
               // chunks of every head start first
};
struct ChunkMap { int blk, chunk, pair, chunks; };
__host__ __device__ static inline int dq_tiles(int i, int seq) { int e = (i + 1) * 128; return ((e < seq ? e : seq) + AB_KT - 1) / AB_KT; }
__host__ __device__ static inline int dkv_first(int i, int q_off) { return i * 128 > q_off ? i * 128 : q_off; }  // first query position a key block meets
__host__ __device__ static inline int dkv_tiles(int i, int seq, int q_off) { return (seq - dkv_first(i, q_off) + AB_KT - 1) / AB_KT; }
__host__ __device__ static inline int chunks_of(int tiles, int c) { return (tiles + c - 1) / c; }
static int total_pairs_dq(int seq, int q_off, int c) {
  int n = 0;
  for (int i = q_off / 128; i < (seq + 127) / 128; i++) n += chunks_of(dq_tiles(i, seq), c);
  return n;
}
static int total_pairs_dkv(int seq, int q_off, int c) {
  int n = 0;
  for (int i = 0; i < (seq + 127) / 128; i++) n += chunks_of(dkv_tiles(i, seq, q_off), c);
  return n;
}
template <bool DKV>
__device__ __forceinline__ ChunkMap map_chunk(int id, int seq, int q_off, int total, int c) {
  const int nblk = (seq + 127) / 128;
  ChunkMap m;
  int rem = id, after = 0;  // `after` = pairs of the blocks visited before this one
  if (DKV) {  // heaviest = block 0; natural pair order = visiting order
    int i = 0;
    for (;; i++) { int ch = chunks_of(dkv_tiles(i, seq, q_off), c); if (rem < ch || i == nblk - 1) { m.chunks = ch; break; } rem -= ch; after += ch; }
    m.blk = i; m.chunk = rem; m.pair = after + rem;
  } else {    // heaviest = last block; the first block with queries is q_off/128
    int i = nblk - 1;
    for (;; i--) { int ch = chunks_of(dq_tiles(i, seq), c); if (rem < ch || i == q_off / 128) { m.chunks = ch; break; } rem -= ch; after += ch; }
    m.blk = i; m.chunk = rem; m.pair = total - after - m.chunks + rem;
  }
  return m;
}

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

#define LOG2E 1.4426950408889634f
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

// acc += A * B with the accumulator held in the accumulation half of the register file (AGPRs) for the whole
// tile loop: the long-lived gradient accumulators then cost no ordinary registers and no copies.  (This file
// is built with -amdgpu-mfma-vgpr-form, so the short-lived score tiles that the vector ALU post-processes are
// produced in ordinary registers by the intrinsic, with the compiler's own hazard handling.)  The hardware
// interlocks back-to-back accumulation into the same registers; the wait states the compiler would otherwise
// insert around a matrix instruction are written out by hand, since it cannot see into the assembly statement:
// before the instruction (see mfma_acc) and, before anything else reads an accumulator, mfma_acc_settle().
__device__ __forceinline__ void mfma_acc(f32x16& acc, bf16x8 a, bf16x8 b) {
  // two wait states first: an operand fragment may have been written by the vector ALU (the bf16 packing) in the
  // instruction just before, and a matrix instruction must not read such a register that early
  asm("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// acc = 0, produced by the matrix unit so that the accumulator is born in an AGPR; the trailing wait states let
// the result land before any register copy the compiler may place behind this statement.
__device__ __forceinline__ void mfma_acc_zero(f32x16& acc) {
  const bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
  asm volatile("s_nop 3\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %1, 0\n\ts_nop 15\n\ts_nop 15" : "=a"(acc) : "v"(z));
}
__device__ __forceinline__ void mfma_acc_settle(f32x16 (&a)[2]) {
  asm volatile("s_nop 15\n\ts_nop 15" : "+a"(a[0]), "+a"(a[1]));
}
__device__ __forceinline__ void mfma_acc_settle(f32x16 (&a)[4]) {
  asm volatile("s_nop 15\n\ts_nop 15" : "+a"(a[0]), "+a"(a[1]), "+a"(a[2]), "+a"(a[3]));
}
// The AGPR placement pays where ordinary registers are short (D = 128: 64 or 128 accumulator registers next to
// the operand fragments and two score tiles).  With D = 64 everything fits the ordinary registers, where the
// compiler would only shuttle an AGPR-constrained value back and forth, so those kernels use the intrinsic.
template <int D> __device__ __forceinline__ void acc_zero(f32x16& acc) {
  if constexpr (D == 128) mfma_acc_zero(acc);
  else {
#pragma unroll
    for (int r = 0; r < 16; r++) acc[r] = 0.f;
  }
}
template <int D> __device__ __forceinline__ void acc_mfma(f32x16& acc, bf16x8 a, bf16x8 b) {
  if constexpr (D == 128) mfma_acc(acc, a, b);
  else acc = MFMA(a, b, acc);
}
template <int D, int N> __device__ __forceinline__ void acc_settle(f32x16 (&a)[N]) {
  if constexpr (D == 128) mfma_acc_settle(a);
}


template <int D>
struct ATile {
  static constexpr int LD = D;
  static constexpr int ELEMS = AB_KT * D;
  static constexpr int BYTES = ELEMS * 2;
  static constexpr int CPR = D / 8;   // 16-byte chunks per row
  static constexpr int IPW = D / 32;  // transfers per wave per tile (4 waves)
  __device__ static __forceinline__ int swz(int r) { return (((r & 3) << 2) | ((r >> 2) & 3)) & (CPR - 1); }
  // element offset of (row r, column c), c a multiple of 4
  __device__ static __forceinline__ int off(int r, int c) { return r * LD + ((((c >> 3) ^ swz(r)) << 3) | (c & 7)); }
};

// Per-lane byte offsets (relative to the tile's first row in global memory, row stride ld elements)
// of the chunks this wave transfers; rows >= rows_valid are clamped to the last valid row.
template <int D>
__device__ __forceinline__ void tile_voff(uint32_t (&v)[ATile<D>::IPW], int ld, int wave, int lane, int rows_valid) {
  using TL = ATile<D>;
#pragma unroll
  for (int j = 0; j < TL::IPW; j++) {
    const int p = (wave * TL::IPW + j) * 64 + lane;
    const int row = p / TL::CPR, c = (p % TL::CPR) ^ TL::swz(row);
    v[j] = (uint32_t)(((size_t)min(row, rows_valid - 1) * ld + c * 8) * sizeof(bf16_t));
  }
}
template <int D>
__device__ __forceinline__ void tile_dma(const char* base, const uint32_t (&v)[ATile<D>::IPW], uint32_t lds_tile, int wave) {
#pragma unroll
  for (int j = 0; j < ATile<D>::IPW; j++) dma16_base(base, v[j], lds_tile + (wave * ATile<D>::IPW + j) * 1024);
}

// Byte offsets inside a tile of the two kinds of fragment reads, precomputed per lane.
//   direct: row l32 (+32*mt), columns ks*16 + kg*8 .. +7              -> kdir[ks] (+ mt*32*LD*2)
//   transposed: rows 4*kg + s/4 (+8 for the second read) (+ mt*32 + 16*c), column dt*32 + h16*16 + (s%4)*4
//                                                                      -> tr0[dt], tr1[dt] (+ (mt*32+16c)*LD*2)
// The swizzle of a row only depends on row%16 through bits that the added multiples of 16 (and, for
// the direct reads, 32) leave untouched, so the additions are plain constants.
template <int D>
struct FragAddr {
  int kdir[D / 16], tr0[D / 32], tr1[D / 32];
  __device__ __forceinline__ void init(int lane) {
    using TL = ATile<D>;
    const int l32 = lane & 31, kg = lane >> 5, s16 = lane & 15, h16 = (lane >> 4) & 1;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) kdir[ks] = TL::off(l32, ks * 16 + kg * 8) * 2;
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++) {
      tr0[dt] = TL::off(4 * kg + (s16 >> 2), dt * 32 + h16 * 16 + ((s16 & 3) << 2)) * 2;
      tr1[dt] = TL::off(8 + 4 * kg + (s16 >> 2), dt * 32 + h16 * 16 + ((s16 & 3) << 2)) * 2;
    }
  }
};
// Fragment reads take a per-lane pointer (tile base + precomputed lane offset) and a compile-time
// constant byte offset, which the compiler folds into the offset field of the LDS instruction.
typedef __attribute__((address_space(3))) char lds_char;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
__device__ __forceinline__ bf16x8 lds_frag(const lds_char* lane_ptr, int const_off) {
  return *reinterpret_cast<const lds_bf16x8*>(lane_ptr + const_off);
}
__device__ __forceinline__ bf16x8 lds_frag_tr(const lds_char* lane_ptr0, const lds_char* lane_ptr1, int const_off) {
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(lane_ptr0 + const_off));
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(lane_ptr1 + const_off));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}
// Per-tile lane pointers for one LDS tile.
template <int D>
struct TilePtrs {
  const lds_char* dir[D / 16];
  const lds_char* t0[D / 32];
  const lds_char* t1[D / 32];
  __device__ __forceinline__ void set(const lds_char* tile, const FragAddr<D>& fa) {
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) dir[ks] = tile + fa.kdir[ks];
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++) { t0[dt] = tile + fa.tr0[dt]; t1[dt] = tile + fa.tr1[dt]; }
  }
};
// Registers 8c..8c+7 of a 32x32 result tile as a bf16 B fragment (k-slots = rows 16c+4g+{0..3}, 16c+8+4g+{0..3}).
__device__ __forceinline__ bf16x8 pack_rows(const f32x16& t, int c) {
  bf16x8 f;
#pragma unroll
  for (int i = 0; i < 8; i++) f[i] = (bf16_t)t[8 * c + i];
  return f;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Score tiles of a 64-token LDS tile: acc[mt] = sum over k of T[rows 32 mt .. 32 mt + 31][k] * b[k] (direct fragments
// of the tile behind P against the D-long register fragments b).  A matrix instruction that accumulates into the
// result of the one just before it has to wait for that result, so the products of the independent tiles are
// issued round robin: score_tiles interleaves its two tiles, score_tiles2 the four tiles of two operand pairs
// (the backward kernels' S and dP).  The LDS fragments of step k+1 are requested before the products of step k
// are issued, and the matrix and LDS instructions are pinned in that order (vector-ALU work of the caller may
// still move across), so no product waits for an LDS read issued just before it.
#define SCHED_PIN_MFMA_DS() __builtin_amdgcn_sched_barrier(0x1 | 0x2 | 0x4 | 0x400)  // ALU, VALU, SALU, TRANS may cross
template <int D>
__device__ __forceinline__ void score_tiles(f32x16 (&acc)[2], const TilePtrs<D>& P, const bf16x8 (&b)[D / 16]) {
  using TL = ATile<D>;
  constexpr int KS = D / 16;
  const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 fr[2][4];  // two k-steps (two fragments each) per chunk
  auto fetch = [&](int c) {
#pragma unroll
    for (int i = 0; i < 4; i++) fr[c & 1][i] = lds_frag(P.dir[2 * c + (i >> 1)], (i & 1) * 32 * TL::LD * 2);
  };
  fetch(0);
#pragma unroll
  for (int c = 0; c < KS / 2; c++) {
    if (c + 1 < KS / 2) fetch(c + 1);
    SCHED_PIN_MFMA_DS();
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int ks = 2 * c + (i >> 1), mt = i & 1;
      acc[mt] = MFMA(fr[c & 1][i], b[ks], ks == 0 ? z : acc[mt]);
    }
    SCHED_PIN_MFMA_DS();
  }
}
template <int D>
__device__ __forceinline__ void score_tiles2(f32x16 (&acc0)[2], const TilePtrs<D>& P0, const bf16x8 (&b0)[D / 16],
                                             f32x16 (&acc1)[2], const TilePtrs<D>& P1, const bf16x8 (&b1)[D / 16]) {
  using TL = ATile<D>;
  constexpr int KS = D / 16;
  const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  bf16x8 fr[2][4];  // one k-step of both operand pairs per chunk
  auto fetch = [&](int ks) {
    fr[ks & 1][0] = lds_frag(P0.dir[ks], 0);
    fr[ks & 1][1] = lds_frag(P0.dir[ks], 32 * TL::LD * 2);
    fr[ks & 1][2] = lds_frag(P1.dir[ks], 0);
    fr[ks & 1][3] = lds_frag(P1.dir[ks], 32 * TL::LD * 2);
  };
  fetch(0);
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    if (ks + 1 < KS) fetch(ks + 1);
    SCHED_PIN_MFMA_DS();
    acc0[0] = MFMA(fr[ks & 1][0], b0[ks], ks == 0 ? z : acc0[0]);
    acc0[1] = MFMA(fr[ks & 1][1], b0[ks], ks == 0 ? z : acc0[1]);
    acc1[0] = MFMA(fr[ks & 1][2], b1[ks], ks == 0 ? z : acc1[0]);
    acc1[1] = MFMA(fr[ks & 1][3], b1[ks], ks == 0 ? z : acc1[1]);
    SCHED_PIN_MFMA_DS();
  }
}

// acc[dt] += T[64 x D]^T (transposed fragments of the LDS tile behind P) * src, src = a 64 x 32 score tile held as
// two 32x32 register tiles.  The 64 "k" rows go in four groups of 16 (g = 2*mt + c); the transposed fragments
// of group g+1 are fetched before the products of group g are issued, so no product waits for its own LDS
// read, and between(g) runs after group g's products are issued (independent vector work to overlap them).
template <int D, class F>
__device__ __forceinline__ void acc_tile_tr(f32x16 (&acc)[D / 32], const TilePtrs<D>& P, const f32x16 (&src)[2], F between) {
  using TL = ATile<D>;
  bf16x8 fr[2][D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++) fr[0][dt] = lds_frag_tr(P.t0[dt], P.t1[dt], 0);
#pragma unroll
  for (int g = 0; g < 4; g++) {
    if (g + 1 < 4) {
      const int ro = (g + 1) * 16 * TL::LD * 2;
#pragma unroll
      for (int dt = 0; dt < D / 32; dt++) fr[(g + 1) & 1][dt] = lds_frag_tr(P.t0[dt], P.t1[dt], ro);
    }
    const bf16x8 pf = pack_rows(src[g >> 1], g & 1);
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++) acc_mfma<D>(acc[dt], fr[g & 1][dt], pf);
    between(g);
  }
}

template <int D>
__device__ __forceinline__ void load_row_frags(bf16x8 (&f)[D / 16], const bf16_t* row, bool valid, int kg) {
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    f[ks] = valid ? *reinterpret_cast<const bf16x8*>(row + ks * 16 + kg * 8) : z;
  }
}

// Makes the compiler wait here for the global loads that produced the fragments: their first use would
// otherwise be inside the tile loop, and the wait it would place there (a vmcnt count that knows nothing
// of the asynchronous tile transfers) would drain the transfer ring on every step.
template <int N>
__device__ __forceinline__ void pin_frags(const bf16x8 (&f)[N]) {
#pragma unroll
  for (int i = 0; i < N; i++) asm volatile("" ::"v"(f[i]));
}
__device__ __forceinline__ void pin_scalar(float v) { asm volatile("" ::"v"(v)); }

// ================================================================================ forward
// Work units of the forward kernel: query block i (128 rows) needs fwd_tiles(i) key tiles; with ch > 0 they
// are cut into chunks of ch tiles (ch even, so that every chunk starts at a tile each of the block's waves
// can see), one launch index per (block, chunk), heaviest block first.  A block with a single chunk writes
// o and lse itself; otherwise every chunk writes its unnormalised float32 output rows with their running
// maximum and sum, and a combine kernel merges the chunks in chunk order.
__host__ __device__ static inline int fwd_tiles(int i, int seq) { int e = (i + 1) * 128; return ((e < seq ? e : seq) + AB_KT - 1) / AB_KT; }
__host__ __device__ static inline int fwd_chunks(int i, int seq, int ch) { return ch > 0 ? (fwd_tiles(i, seq) + ch - 1) / ch : 1; }
static int fwd_units(int seq, int q_off, int ch) {
  int n = 0;
  for (int i = q_off / 128; i < (seq + 127) / 128; i++) n += fwd_chunks(i, seq, ch);
  return n;
}

// grid (units * nq * batch); wave w owns query rows i0 + 32w .. +31.  The K and V tiles go through two LDS
// slots each (64 KiB per block at D = 128), so that two blocks fit a compute unit: the matrix work of
// one block's waves then overlaps the softmax arithmetic of the other's.
#define AF_RING 2

// A wave's 32 rows x D columns in the transposed accumulator layout (lane l32 = row, kg = lane / 32; quad (dt, q4) of
// a lane is columns dt*32 + 8*q4 + 4*kg .. +3) leave through a wave-private LDS region so that a lane stores 16 bytes
// of a contiguous row segment instead of 16 (float32) or 8 (bf16) bytes scattered over 32 rows.  16-byte chunks are
// XOR-swizzled by row; quad(dt, q4) returns the four values, row_ptr(r) the destination of row r or nullptr.
// The region must not be in use by any wave (block barrier before the first call).
template <int D, typename Quad, typename RowPtr>
__device__ __forceinline__ void wave_rows_out_f32(float* reg, int lane, Quad quad, RowPtr row_ptr) {
  constexpr int NCH = D / 4;  // 16-byte chunks per row
  const int l32 = lane & 31, kg = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int q4 = 0; q4 < 4; q4++) {
      const int ch = (dt * 32 + 8 * q4 + 4 * kg) >> 2;
      *reinterpret_cast<f32x4*>(reg + l32 * D + ((ch ^ (l32 & (NCH - 1))) << 2)) = quad(dt, q4);
    }
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int it = 0; it < 32 * NCH / 64; it++) {
    const int row = it * (64 / NCH) + lane / NCH, ch = lane % NCH;
    const f32x4 v = *reinterpret_cast<const f32x4*>(reg + row * D + ((ch ^ (row & (NCH - 1))) << 2));
    float* dst = row_ptr(row);
    if (dst != nullptr) *reinterpret_cast<f32x4*>(dst + ch * 4) = v;
  }
}
template <int D, typename Quad, typename RowPtr>
__device__ __forceinline__ void wave_rows_out_bf16(bf16_t* reg, int lane, Quad quad, RowPtr row_ptr) {
  constexpr int NCH = D / 8;  // 16-byte chunks per row
  const int l32 = lane & 31, kg = lane >> 5;
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int q4 = 0; q4 < 4; q4++) {
      const int c0 = dt * 32 + 8 * q4 + 4 * kg;
      const f32x4 v = quad(dt, q4);
      const bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
      *reinterpret_cast<bf16x4*>(reg + l32 * D + ((((c0 >> 3) ^ (l32 & (NCH - 1))) << 3) | (c0 & 4))) = o;
    }
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int it = 0; it < 32 * NCH / 64; it++) {
    const int row = it * (64 / NCH) + lane / NCH, ch = lane % NCH;
    const bf16x8 v = *reinterpret_cast<const bf16x8*>(reg + row * D + ((ch ^ (row & (NCH - 1))) << 3));
    bf16_t* dst = row_ptr(row);
    if (dst != nullptr) *reinterpret_cast<bf16x8*>(dst + ch * 8) = v;
  }
}
#define AF_TAU 8.0f  // log2 of the headroom a row's probabilities may take over its reference maximum
template <int D>
__global__ __launch_bounds__(AB_THREADS, 2) void attn_fwd_bf16_kernel(const AttnGeom g, const bf16_t* __restrict__ qkv,
                                                                   bf16_t* __restrict__ o, float* __restrict__ lse, int T,
                                                                   float scale_log2, int ch, int units,
                                                                   float* __restrict__ part_o, float* __restrict__ part_ml) {
  using TL = ATile<D>;
  extern __shared__ __attribute__((aligned(1024))) char smem[];  // K ring, then V ring
  const lds_char* sm = (const lds_char*)smem;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, kg = lane >> 5;
  const int seq = g.seq, nq = g.nq, nkv = g.nkv, qb0 = g.q_off / 128, ldkv = g.ldkv;
  const int hb = blockIdx.x % g.nq_all, launch = blockIdx.x / g.nq_all;
  const int h = hb % nq, b = hb / nq, hk = h / (nq / nkv);
  const int ld = (nq + 2 * nkv) * D;
  int blk, chunk = 0, nchunks = 1, pair;
  if (ch == 0) {
    pair = units - 1 - launch;
    blk = qb0 + pair;
  } else {  // heaviest block first; `pair` numbers the (block, chunk) units in natural order
    int rem = launch, after = 0;
    blk = (seq + 127) / 128 - 1;
    for (;; blk--) {
      nchunks = fwd_chunks(blk, seq, ch);
      if (rem < nchunks || blk == qb0) break;
      rem -= nchunks;
      after += nchunks;
    }
    chunk = rem;
    pair = units - after - nchunks + rem;
  }
  const int i0 = blk * 128, iw = i0 + wave * 32, iq = iw + l32;  // positions in the sequence
  const size_t ktok0 = (size_t)b * seq;
  const long long qtok0 = (long long)b * (seq - g.q_off) - g.q_off;  // local token of position p = qtok0 + p
  const char* kbase = reinterpret_cast<const char*>(g.kv + ktok0 * ldkv + (size_t)hk * D);
  const char* vbase = reinterpret_cast<const char*>(g.kv + ktok0 * ldkv + (size_t)(nkv + hk) * D);
  const size_t tstride = (size_t)AB_KT * ldkv * sizeof(bf16_t);

  bf16x8 qf[D / 16];
  load_row_frags<D>(qf, qkv + (size_t)(qtok0 + min(iq, seq - 1)) * ld + (size_t)h * D, iq < seq, kg);
  f32x16 ot[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) ot[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  FragAddr<D> fa;
  fa.init(lane);
  uint32_t voff[TL::IPW];
  tile_voff<D>(voff, ldkv, wave, lane, AB_KT);
  const uint32_t ldsK = lds_address(smem), ldsV = ldsK + AF_RING * TL::BYTES;
  const int tiles_all = (min(seq, i0 + 128) + AB_KT - 1) / AB_KT;  // keys needed by this block: [0, 64*tiles_all)
  const int t_begin = chunk * ch, ntiles = ch == 0 ? tiles_all : min(tiles_all, t_begin + ch);  // this unit: [t_begin, ntiles)
  auto issue = [&](int t) {
    const int slot = (t - t_begin) % AF_RING, valid = seq - t * AB_KT;
    if (valid >= AB_KT) {
      tile_dma<D>(kbase + t * tstride, voff, ldsK + slot * TL::BYTES, wave);
      tile_dma<D>(vbase + t * tstride, voff, ldsV + slot * TL::BYTES, wave);
    } else {
      uint32_t vc[TL::IPW];
      tile_voff<D>(vc, ldkv, wave, lane, valid);
      tile_dma<D>(kbase + t * tstride, vc, ldsK + slot * TL::BYTES, wave);
      tile_dma<D>(vbase + t * tstride, vc, ldsV + slot * TL::BYTES, wave);
    }
  };
  pin_frags(qf);
  issue(t_begin);
  int slot = 0;
  for (int t = t_begin; t < ntiles; t++, slot ^= 1) {
    dma_wait<0>();
    __syncthreads();  // tile t is visible; every wave is done with tile t-1, whose slot tile t+1 reuses
    if (t + 1 < ntiles) issue(t + 1);
    const int kb = t * AB_KT;
    if (kb > iw + 31) continue;  // no key of the tile is visible to any row of this wave
    TilePtrs<D> Kp, Vp;
    Kp.set(sm + slot * TL::BYTES, fa);
    Vp.set(sm + (AF_RING + slot) * TL::BYTES, fa);
    f32x16 st[2];
    score_tiles<D>(st, Kp, qf);
    if (kb + AB_KT - 1 > iw) {  // the tile crosses the diagonal for this wave: mask keys above the row
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++)
          if (kb + mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3) > iq) st[mt][r] = -INFINITY;
    }
    float mx = fmaxf(st[0][0], st[1][0]);
#pragma unroll
    for (int r = 1; r < 16; r++) mx = fmaxf(mx, fmaxf(st[0][r], st[1][r]));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    // The reference maximum m of a row moves only when some row of the wave outgrows its reference by more than
    // 2^AF_TAU (then every row takes its true maximum and the accumulators are rescaled); otherwise the tile's
    // probabilities are formed against the old reference and may reach 2^AF_TAU, which float32 sums and the bf16 P
    // fragments hold without loss of relative precision.  The result depends on m only through rounding: the
    // normalisation by l at the end and lse = m + log2 l use the same reference.  After the first few tiles of a row the
    // rescaling (one multiply per accumulator element per tile) almost never runs.
    const float mnew = mx * scale_log2;  // finite from the unit's first tile on: its first key is visible to every row
    float rs = 0.f;
    if (__any(mnew > m + AF_TAU)) {
      const float mn = fmaxf(m, mnew);
      const float alpha = fast_exp2(m - mn);
      l *= alpha;
      m = mn;
#pragma unroll
      for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) ot[dt][r] *= alpha;
    }
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const float p = fast_exp2(fmaf(st[mt][r], scale_log2, -m));
        st[mt][r] = p;
        rs += p;
      }
    rs += __shfl_xor(rs, 32, 64);
    l += rs;
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int c = 0; c < 2; c++) {
        const bf16x8 pf = pack_rows(st[mt], c);
        const int ro = (mt * 32 + 16 * c) * TL::LD * 2;
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++) ot[dt] = MFMA(lds_frag_tr(Vp.t0[dt], Vp.t1[dt], ro), pf, ot[dt]);
      }
  }
  __syncthreads();  // every wave is done with the K/V rings: their LDS serves the output turn
  if (nchunks > 1) {  // partial result of this chunk
    const size_t unit = ((size_t)b * nq + h) * units + pair;
    wave_rows_out_f32<D>(
        reinterpret_cast<float*>(smem) + wave * (32 * D), lane,
        [&](int dt, int q4) { return f32x4{ot[dt][4 * q4], ot[dt][4 * q4 + 1], ot[dt][4 * q4 + 2], ot[dt][4 * q4 + 3]}; },
        [&](int r) { return iw + r < seq ? part_o + (unit * 128 + (iw + r - i0)) * D : nullptr; });
    if (iq < seq && kg == 0) {
      part_ml[(unit * 128 + (iq - i0)) * 2] = m;
      part_ml[(unit * 128 + (iq - i0)) * 2 + 1] = l;
    }
    return;
  }
  const float inv = 1.0f / l;
  wave_rows_out_bf16<D>(
      reinterpret_cast<bf16_t*>(smem) + wave * (32 * D), lane,
      [&](int dt, int q4) {
        return f32x4{ot[dt][4 * q4] * inv, ot[dt][4 * q4 + 1] * inv, ot[dt][4 * q4 + 2] * inv, ot[dt][4 * q4 + 3] * inv};
      },
      [&](int r) { return iw + r < seq ? o + (size_t)(qtok0 + iw + r) * nq * D + (size_t)h * D : nullptr; });
  if (iq < seq && kg == 0) lse[(size_t)h * T + qtok0 + iq] = (m + log2f(l)) * 0.6931471805599453f;
}

// Merges the chunks of the query blocks that were split: with M = max_c m_c, o = sum_c 2^(m_c-M) o_c / L,
// L = sum_c 2^(m_c-M) l_c, lse = (M + log2 L) ln 2; chunks are added in chunk order.
// grid (8 * blocks, nq, batch): a 256-thread block merges 16 rows, a thread D/16 columns of one row.
template <int D>
__global__ __launch_bounds__(256) void attn_fwd_combine_kernel(int seq, int q_off, int nq, int ch, int units, const float* __restrict__ part_o,
                                                               const float* __restrict__ part_ml, bf16_t* __restrict__ o,
                                                               float* __restrict__ lse, int T) {
  const int blk = q_off / 128 + (blockIdx.x >> 3), h = blockIdx.y, b = blockIdx.z;
  const int nchunks = fwd_chunks(blk, seq, ch);
  if (nchunks == 1) return;
  const int r = (blockIdx.x & 7) * 16 + (threadIdx.x >> 4), pos = blk * 128 + r;
  if (pos >= seq) return;
  int pair0 = 0;
  for (int i = q_off / 128; i < blk; i++) pair0 += fwd_chunks(i, seq, ch);
  const size_t unit0 = ((size_t)b * nq + h) * units + pair0;
  constexpr int CPT = D / 16;  // columns per thread
  const int c0 = (threadIdx.x & 15) * CPT;
  const float* ml = part_ml + (unit0 * 128 + r) * 2;
  float M = -INFINITY;
  for (int c = 0; c < nchunks; c++) M = fmaxf(M, ml[(size_t)c * 256]);
  float L = 0.f, acc[CPT];
#pragma unroll
  for (int i = 0; i < CPT; i++) acc[i] = 0.f;
  for (int c = 0; c < nchunks; c++) {
    const float w = exp2f(ml[(size_t)c * 256] - M);
    L += w * ml[(size_t)c * 256 + 1];
    const float* po = part_o + ((unit0 + c) * 128 + r) * D + c0;
#pragma unroll
    for (int i = 0; i < CPT; i += 4) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(po + i);
      acc[i] += w * v[0]; acc[i + 1] += w * v[1]; acc[i + 2] += w * v[2]; acc[i + 3] += w * v[3];
    }
  }
  const float inv = 1.0f / L;
  const size_t tok = (size_t)b * (seq - q_off) + (pos - q_off);
  bf16_t* orow = o + tok * (size_t)nq * D + (size_t)h * D + c0;
#pragma unroll
  for (int i = 0; i < CPT; i += 4) {
    bf16x4 v = {(bf16_t)(acc[i] * inv), (bf16_t)(acc[i + 1] * inv), (bf16_t)(acc[i + 2] * inv), (bf16_t)(acc[i + 3] * inv)};
    *reinterpret_cast<bf16x4*>(orow + i) = v;
  }
  if (c0 == 0) lse[(size_t)h * T + tok] = (M + log2f(L)) * 0.6931471805599453f;
}

// ================================================================================ backward: dQ
// Same tiling as the forward kernel.  dQ^T = sum over key tiles of K^T dS^T, dS^T = P^T (dP^T - delta),
// P^T = exp2(S^T*scale_log2 - lse2), dP^T = V dO^T.
// Every block forms the per-row statistics delta[h,t] = sum_c dO[t,h,c] O[t,h,c] and lse2[h,t] = lse[h,t] log2(e) of its
// own rows itself (a row's two lanes each hold half of dO).  The dK/dV blocks read them from memory: when the dQ blocks
// are launched ahead of them, the block of a query block's first chunk stores them (delta_out != nullptr); when both
// kinds share one launch, attn_bwd_prep_kernel has filled the arrays.
template <int D>
__device__ __forceinline__ void attn_bwd_dq_block(const int bid, const AttnGeom& g, const bf16_t* __restrict__ qkv,
                                                  const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                                  const float* __restrict__ lse, float* __restrict__ lse2_out,
                                                  float* __restrict__ delta_out, bf16_t* __restrict__ dqkv,
                                                  float* __restrict__ part, int pairs, int T, float scale, float scale_log2) {
  using TL = ATile<D>;
  extern __shared__ __attribute__((aligned(1024))) char smem[];  // K ring, then V ring
  const lds_char* sm = (const lds_char*)smem;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, kg = lane >> 5;
  const int seq = g.seq, nq = g.nq, nkv = g.nkv, ldkv = g.ldkv;
  const int hb = bid % g.nq_all;
  const int h = hb % nq, b = hb / nq, hk = h / (nq / nkv);
  const int ld = (nq + 2 * nkv) * D;
  const ChunkMap cm = map_chunk<false>(bid / g.nq_all, seq, g.q_off, pairs, g.ch);
  const int i0 = cm.blk * 128, iw = i0 + wave * 32, iq = iw + l32;
  const size_t ktok0 = (size_t)b * seq;
  const long long qtok0 = (long long)b * (seq - g.q_off) - g.q_off;  // local token of position p = qtok0 + p
  const char* kbase = reinterpret_cast<const char*>(g.kv + ktok0 * ldkv + (size_t)hk * D);
  const char* vbase = reinterpret_cast<const char*>(g.kv + ktok0 * ldkv + (size_t)(nkv + hk) * D);
  const size_t tstride = (size_t)AB_KT * ldkv * sizeof(bf16_t);

  bf16x8 qf[D / 16], dof[D / 16];
  const size_t qrow = (size_t)(qtok0 + min(iq, seq - 1));
  load_row_frags<D>(qf, qkv + qrow * ld + (size_t)h * D, iq < seq, kg);
  load_row_frags<D>(dof, dout + qrow * (size_t)nq * D + (size_t)h * D, iq < seq, kg);
  const float l2 = lse[(size_t)h * T + qrow] * LOG2E;
  float dl = 0.f;
  {
    bf16x8 of[D / 16];
    load_row_frags<D>(of, o + qrow * (size_t)nq * D + (size_t)h * D, iq < seq, kg);
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++)
#pragma unroll
      for (int e = 0; e < 8; e++) dl = fmaf((float)dof[ks][e], (float)of[ks][e], dl);
    dl += __shfl_xor(dl, 32, 64);  // the row's other half (the same number attn_bwd_prep_kernel stores for the dK/dV blocks)
    if (delta_out != nullptr && cm.chunk == 0 && kg == 0 && iq < seq) {  // launched ahead of the dK/dV kernel: store them for it
      delta_out[(size_t)h * T + qrow] = dl;
      lse2_out[(size_t)h * T + qrow] = l2;
    }
  }
  f32x16 dqt[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++) acc_zero<D>(dqt[dt]);

  FragAddr<D> fa;
  fa.init(lane);
  uint32_t voff[TL::IPW];
  tile_voff<D>(voff, ldkv, wave, lane, AB_KT);
  const uint32_t ldsK = lds_address(smem), ldsV = ldsK + AB_RING * TL::BYTES;
  const int t0 = cm.chunk * g.ch, ntiles = min(dq_tiles(cm.blk, seq), t0 + g.ch);  // this block walks key tiles [t0, ntiles)
  auto issue = [&](int t, int slot) {
    const int valid = seq - t * AB_KT;
    if (valid >= AB_KT) {
      tile_dma<D>(kbase + t * tstride, voff, ldsK + slot * TL::BYTES, wave);
      tile_dma<D>(vbase + t * tstride, voff, ldsV + slot * TL::BYTES, wave);
    } else {
      uint32_t vc[TL::IPW];
      tile_voff<D>(vc, ldkv, wave, lane, valid);
      tile_dma<D>(kbase + t * tstride, vc, ldsK + slot * TL::BYTES, wave);
      tile_dma<D>(vbase + t * tstride, vc, ldsV + slot * TL::BYTES, wave);
    }
  };
  pin_frags(qf);
  pin_frags(dof);
  pin_scalar(l2);
  pin_scalar(dl);
  issue(t0, 0);
  if (t0 + 1 < ntiles) issue(t0 + 1, 1);
  int slot = 0;
  for (int t = t0; t < ntiles; t++, slot = slot == AB_RING - 1 ? 0 : slot + 1) {
    if (t + 1 < ntiles) dma_wait<2 * TL::IPW>(); else dma_wait<0>();
    __syncthreads();
    if (t + 2 < ntiles) issue(t + 2, slot == 0 ? AB_RING - 1 : slot - 1);
    const int kb = t * AB_KT;
    if (kb > iw + 31) continue;
    TilePtrs<D> Kp, Vp;
    Kp.set(sm + slot * TL::BYTES, fa);
    Vp.set(sm + (AB_RING + slot) * TL::BYTES, fa);
    f32x16 st[2], dp[2];
    score_tiles2<D>(st, Kp, qf, dp, Vp, dof);
    // P^T from S^T while the dP^T products are still in the matrix pipeline
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int r = 0; r < 16; r++) st[mt][r] = fast_exp2(fmaf(st[mt][r], scale_log2, -l2));
    if (kb + AB_KT - 1 > iw) {
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++)
          if (kb + mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3) > iq) st[mt][r] = 0.f;
    }
    // dS^T = P^T (dP^T - delta), one quarter (8 registers of a tile) ahead of the products that consume it
    auto ds_quarter = [&](int g) {
#pragma unroll
      for (int r = 0; r < 8; r++) st[g >> 1][8 * (g & 1) + r] *= dp[g >> 1][8 * (g & 1) + r] - dl;
    };
    ds_quarter(0);
    acc_tile_tr<D>(dqt, Kp, st, [&](int g) { if (g + 1 < 4) ds_quarter(g + 1); });
  }
  acc_settle<D>(dqt);
  __syncthreads();  // every wave is done with the K/V rings: their LDS serves the output turn
  if (part != nullptr) {  // float32 partial of this chunk: part[batch][head][pair][128 rows][D], unscaled
    float* rows = part + ((((size_t)b * nq + h) * pairs + cm.pair) * 128 + wave * 32) * D;
    wave_rows_out_f32<D>(
        reinterpret_cast<float*>(smem) + wave * (32 * D), lane,
        [&](int dt, int q4) { return f32x4{dqt[dt][4 * q4], dqt[dt][4 * q4 + 1], dqt[dt][4 * q4 + 2], dqt[dt][4 * q4 + 3]}; },
        [&](int r) { return rows + (size_t)r * D; });
  } else {
    wave_rows_out_bf16<D>(
        reinterpret_cast<bf16_t*>(smem) + wave * (32 * D), lane,
        [&](int dt, int q4) {
          return f32x4{dqt[dt][4 * q4] * scale, dqt[dt][4 * q4 + 1] * scale, dqt[dt][4 * q4 + 2] * scale, dqt[dt][4 * q4 + 3] * scale};
        },
        [&](int r) { return iw + r < seq ? dqkv + (size_t)(qtok0 + iw + r) * ld + (size_t)h * D : nullptr; });
  }
}

// dq[token][head] = scale * sum over the chunks of the token's query block (ascending) of the partials.
// grid (16*query blocks, nq, batch), 256 threads: a block owns 8 rows of a query block, thread = (row, 4 columns).
template <int D>
__device__ __forceinline__ void attn_bwd_dq_reduce_block(int bx, int by, int bz, const float* __restrict__ part,
                                                         bf16_t* __restrict__ dqkv, int seq, int q_off, int nq, int nkv, int pairs,
                                                         int cl, float scale) {
  const int i = q_off / 128 + (bx >> 4), r0 = (bx & 15) * 8, h = by, b = bz, ld = (nq + 2 * nkv) * D;
  int base = 0;
  for (int k = q_off / 128; k < i; k++) base += chunks_of(dq_tiles(k, seq), cl);
  const int ch = chunks_of(dq_tiles(i, seq), cl);
  const float* p0 = part + (((size_t)b * nq + h) * pairs + base) * 128 * D;
  for (int e = threadIdx.x; e < 8 * D / 4; e += 256) {
    const int row = r0 + e / (D / 4), c4 = (e % (D / 4)) * 4;
    if (i * 128 + row >= seq) continue;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int c = 0; c < ch; c++) s += __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p0 + ((size_t)c * 128 + row) * D + c4));
    bf16x4 o = {(bf16_t)(s[0] * scale), (bf16_t)(s[1] * scale), (bf16_t)(s[2] * scale), (bf16_t)(s[3] * scale)};
    *reinterpret_cast<bf16x4*>(dqkv + ((size_t)b * (seq - q_off) + (i * 128 + row - q_off)) * ld + (size_t)h * D + c4) = o;
  }
}

// ================================================================================ backward: dK, dV
// grid (pairs * nq * batch): one block per (key block, chunk, query head); wave w owns keys
// j0 + 32w .. +31 and keeps their K, V fragments and the dK^T, dV^T accumulators in registers while
// 64-query tiles of that head's Q and dO stream through LDS.  With grouped heads (nq > nkv) the
// block writes float32 partials part[batch][query head][pair][128 keys][dK | dV] and
// attn_bwd_reduce_kernel (its dK/dV part) adds the group's heads and the key block's chunks in index order; with
// nq == nkv and no block longer than one chunk it writes dK, dV directly.
template <int D>
__device__ __forceinline__ void attn_bwd_dkv_block(const int bid, const AttnGeom& g, const bf16_t* __restrict__ qkv,
                                                   const bf16_t* __restrict__ dout, const float* __restrict__ lse2,
                                                   const float* __restrict__ delta, float* __restrict__ part, int pairs, int T,
                                                   float scale, float scale_log2) {
  using TL = ATile<D>;
  extern __shared__ __attribute__((aligned(1024))) char smem[];  // Q ring, dO ring, lse2 ring, delta ring
  const lds_char* sm = (const lds_char*)smem;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, kg = lane >> 5;
  const int seq = g.seq, nq = g.nq, nkv = g.nkv;
  const int hb = bid % g.nq_all;
  const int hq = hb % nq, b = hb / nq, grp = nq / nkv, hk = hq / grp;
  const int ld = (nq + 2 * nkv) * D, ldo = nq * D;
  const ChunkMap cm = map_chunk<true>(bid / g.nq_all, seq, g.q_off, pairs, g.ch);
  const int j0 = cm.blk * 128, jw = j0 + wave * 32, jk = jw + l32;  // key positions in the sequence (block 0 is the heaviest)
  const int q0 = dkv_first(cm.blk, g.q_off);                        // first query position this key block meets
  const size_t ktok0 = (size_t)b * seq;
  const size_t qtok = (size_t)b * (seq - g.q_off) + (q0 - g.q_off);  // local token of position q0
  const char* qbase = reinterpret_cast<const char*>(qkv + qtok * ld + (size_t)hq * D);
  const char* obase = reinterpret_cast<const char*>(dout + qtok * ldo + (size_t)hq * D);
  const float* lrow = lse2 + (size_t)hq * T + qtok;
  const float* drow = delta + (size_t)hq * T + qtok;
  float* lse_s = reinterpret_cast<float*>(smem + 2 * AB_RING * TL::BYTES);
  float* del_s = lse_s + AB_RING * AB_KT;

  bf16x8 kf[D / 16], vf[D / 16];
  const int jkc = min(jk, seq - 1);
  load_row_frags<D>(kf, g.kv + (ktok0 + jkc) * g.ldkv + (size_t)hk * D, jk < seq, kg);
  load_row_frags<D>(vf, g.kv + (ktok0 + jkc) * g.ldkv + (size_t)(nkv + hk) * D, jk < seq, kg);
  f32x16 dkt[D / 32], dvt[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++) { acc_zero<D>(dkt[dt]); acc_zero<D>(dvt[dt]); }

  FragAddr<D> fa;
  fa.init(lane);
  uint32_t vq[TL::IPW], vo[TL::IPW];
  tile_voff<D>(vq, ld, wave, lane, AB_KT);
  tile_voff<D>(vo, ldo, wave, lane, AB_KT);
  const uint32_t ldsQ = lds_address(smem), ldsO = ldsQ + AB_RING * TL::BYTES;
  const int t0 = cm.chunk * g.ch, ntiles = min(dkv_tiles(cm.blk, seq, g.q_off), t0 + g.ch);  // query tiles q0 + 64*[t0, ntiles)
  const size_t qstride = (size_t)AB_KT * ld * sizeof(bf16_t), ostride = (size_t)AB_KT * ldo * sizeof(bf16_t);
  auto issue = [&](int t, int slot) {
    const int valid = seq - (q0 + t * AB_KT);
    const char* qp = qbase + t * qstride;
    const char* op = obase + t * ostride;
    if (valid >= AB_KT) {
      tile_dma<D>(qp, vq, ldsQ + slot * TL::BYTES, wave);
      tile_dma<D>(op, vo, ldsO + slot * TL::BYTES, wave);
    } else {
      uint32_t vc[TL::IPW];
      tile_voff<D>(vc, ld, wave, lane, valid);
      tile_dma<D>(qp, vc, ldsQ + slot * TL::BYTES, wave);
      tile_voff<D>(vc, ldo, wave, lane, valid);
      tile_dma<D>(op, vc, ldsO + slot * TL::BYTES, wave);
    }
  };
  // per-row statistics of a tile (64 floats each): even waves transfer lse2, odd waves delta (waves 2 and 3
  // repeat what waves 0 and 1 transfer, which keeps the transfer count of all waves equal)
  const uint32_t ldsS = ldsQ + 2 * AB_RING * TL::BYTES + (wave & 1) * AB_RING * AB_KT * sizeof(float);
  const float* srow = (wave & 1) ? drow : lrow;
  pin_frags(kf);
  pin_frags(vf);
  auto issue_stat = [&](int t, int slot) {
    const int row0 = q0 + t * AB_KT;
    dma4_base(srow + t * AB_KT, (uint32_t)((min(row0 + lane, seq - 1) - row0) * sizeof(float)),
              ldsS + slot * AB_KT * sizeof(float));
  };
  issue(t0, 0);
  issue_stat(t0, 0);
  if (t0 + 1 < ntiles) { issue(t0 + 1, 1); issue_stat(t0 + 1, 1); }
  int slot = 0;
  for (int t = t0; t < ntiles; t++, slot = slot == AB_RING - 1 ? 0 : slot + 1) {
    if (t + 1 < ntiles) dma_wait<2 * TL::IPW + 1>(); else dma_wait<0>();
    __syncthreads();
    if (t + 2 < ntiles) { const int ns = slot == 0 ? AB_RING - 1 : slot - 1; issue(t + 2, ns); issue_stat(t + 2, ns); }
    const int qb = q0 + t * AB_KT;
    if (qb + AB_KT - 1 < jw) continue;  // every query of the tile precedes every key of this wave
    TilePtrs<D> Qp, Op;
    Qp.set(sm + slot * TL::BYTES, fa);
    Op.set(sm + (AB_RING + slot) * TL::BYTES, fa);
    const float* ls = lse_s + slot * AB_KT;
    const float* ds = del_s + slot * AB_KT;
    f32x16 st[2], dp[2];
    score_tiles2<D>(st, Qp, kf, dp, Op, vf);
    // P from S (rows 8*q4 + 4*kg + e of each 32-row half) while dP is in the matrix pipeline
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const f32x4 lv = *reinterpret_cast<const f32x4*>(ls + mt * 32 + 8 * q4 + 4 * kg);
#pragma unroll
        for (int e = 0; e < 4; e++) st[mt][4 * q4 + e] = fast_exp2(fmaf(st[mt][4 * q4 + e], scale_log2, -lv[e]));
      }
    if (qb < jw + 32 || qb + AB_KT > seq) {  // diagonal tile, or rows past the end of the sequence
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int qi = qb + mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
          if (qi < jk || qi >= seq) st[mt][r] = 0.f;
        }
    }
    // dV^T += dO^T P; once a quarter of P (8 registers of a tile) is packed for its products, it is turned
    // into dS = P (dP - delta) in place while those products run; then dK^T += Q^T dS.
    acc_tile_tr<D>(dvt, Op, st, [&](int g) {
      const int mt = g >> 1, c = g & 1;
#pragma unroll
      for (int q = 0; q < 2; q++) {
        const f32x4 dv4 = *reinterpret_cast<const f32x4*>(ds + mt * 32 + 8 * (2 * c + q) + 4 * kg);
#pragma unroll
        for (int e = 0; e < 4; e++) st[mt][8 * c + 4 * q + e] *= dp[mt][8 * c + 4 * q + e] - dv4[e];
      }
    });
    acc_tile_tr<D>(dkt, Qp, st, [](int) {});
  }
  acc_settle<D>(dkt);
  acc_settle<D>(dvt);
  __syncthreads();  // every wave is done with the Q/dO rings: their LDS serves the output turn (dK, then dV)
  auto dk_quad = [&](int dt, int q4) {
    return f32x4{dkt[dt][4 * q4] * scale, dkt[dt][4 * q4 + 1] * scale, dkt[dt][4 * q4 + 2] * scale, dkt[dt][4 * q4 + 3] * scale};
  };
  auto dv_quad = [&](int dt, int q4) { return f32x4{dvt[dt][4 * q4], dvt[dt][4 * q4 + 1], dvt[dt][4 * q4 + 2], dvt[dt][4 * q4 + 3]}; };
  if (part != nullptr) {
    float* rows = part + ((((size_t)b * nq + hq) * pairs + cm.pair) * 128 + wave * 32) * (2 * D);
    float* reg = reinterpret_cast<float*>(smem) + wave * (32 * D);
    wave_rows_out_f32<D>(reg, lane, dk_quad, [&](int r) { return rows + (size_t)r * (2 * D); });
    __builtin_amdgcn_wave_barrier();
    wave_rows_out_f32<D>(reg, lane, dv_quad, [&](int r) { return rows + (size_t)r * (2 * D) + D; });
  } else {
    bf16_t* reg = reinterpret_cast<bf16_t*>(smem) + wave * (32 * D);
    wave_rows_out_bf16<D>(reg, lane, dk_quad,
                          [&](int r) { return jw + r < seq ? g.dkv + (ktok0 + jw + r) * g.lddkv + (size_t)hk * D : nullptr; });
    __builtin_amdgcn_wave_barrier();
    wave_rows_out_bf16<D>(reg, lane, dv_quad,
                          [&](int r) { return jw + r < seq ? g.dkv + (ktok0 + jw + r) * g.lddkv + (size_t)(nkv + hk) * D : nullptr; });
  }
}

// One launch for both halves of the backward pass, used when every query head has a key/value head of its own.  Alone,
// each half leaves compute units idle while its longest blocks finish; in one grid the dQ units fill the gaps of the
// dK/dV units and the other way round (measured on MI355X at 2 x 2048 tokens, 8 heads: 122 -> 94 us).  With grouped
// heads the same merge measured slower than two launches (4096 tokens, 4:1 heads: 128 -> 145 us; 8192 tokens, 8:1:
// 594 -> 652 us), so those shapes keep two launches.  Launch index -> (head, unit): units of the two kinds alternate, each kind
// heaviest first, the dK/dV unit (the dearer one) leading; once the shorter list is used up the rest of the longer
// follows.  grid ((pairs_q + pairs_k) * nq * batch).
template <int D>
__global__ __launch_bounds__(AB_THREADS) void attn_bwd_bf16_kernel(const AttnGeom gq, const AttnGeom gk, const bf16_t* __restrict__ qkv,
                                                                   const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                                                   const float* __restrict__ lse, const float* __restrict__ lse2,
                                                                   const float* __restrict__ delta, bf16_t* __restrict__ dqkv,
                                                                   float* __restrict__ part_q, float* __restrict__ part_kv, int pairs_q,
                                                                   int pairs_k, int T, float scale, float scale_log2) {
  const int hb = blockIdx.x % gq.nq_all, u = blockIdx.x / gq.nq_all, both = 2 * min(pairs_q, pairs_k);
  int idx;
  bool dkv;
  if (u < both) { dkv = (u & 1) == 0; idx = u >> 1; }
  else { dkv = pairs_k > pairs_q; idx = u - both / 2; }
  if (dkv) attn_bwd_dkv_block<D>(idx * gk.nq_all + hb, gk, qkv, dout, lse2, delta, part_kv, pairs_k, T, scale, scale_log2);
  else attn_bwd_dq_block<D>(idx * gq.nq_all + hb, gq, qkv, o, dout, lse, nullptr, nullptr, dqkv, part_q, pairs_q, T, scale, scale_log2);
}
// The two halves as launches of their own (dQ first: it stores the row statistics the dK/dV blocks read).
template <int D>
__global__ __launch_bounds__(AB_THREADS) void attn_bwd_dq_bf16_kernel(const AttnGeom g, const bf16_t* __restrict__ qkv,
                                                                      const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                                                      const float* __restrict__ lse, float* __restrict__ lse2,
                                                                      float* __restrict__ delta, bf16_t* __restrict__ dqkv,
                                                                      float* __restrict__ part, int pairs, int T, float scale, float scale_log2) {
  attn_bwd_dq_block<D>((int)blockIdx.x, g, qkv, o, dout, lse, lse2, delta, dqkv, part, pairs, T, scale, scale_log2);
}
template <int D>
__global__ __launch_bounds__(AB_THREADS) void attn_bwd_dkv_bf16_kernel(const AttnGeom g, const bf16_t* __restrict__ qkv,
                                                                       const bf16_t* __restrict__ dout, const float* __restrict__ lse2,
                                                                       const float* __restrict__ delta, float* __restrict__ part,
                                                                       int pairs, int T, float scale, float scale_log2) {
  attn_bwd_dkv_block<D>((int)blockIdx.x, g, qkv, dout, lse2, delta, part, pairs, T, scale, scale_log2);
}

// Per-row statistics of the backward pass for the dK/dV blocks: delta[h,t] = sum_c dO[t,h,c] O[t,h,c] and
// lse2[h,t] = lse[h,t] log2(e).  The sum runs in the order the dQ blocks use for their own copy (two halves of the row,
// each 8 elements out of every 16, one fused multiply-add per element, halves added last), so both kernels work with
// the same numbers.  One thread per (token, head).
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_prep_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dout,
                                                            const float* __restrict__ lse, float* __restrict__ lse2,
                                                            float* __restrict__ delta, int T, int nq) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)T * nq) return;
  const int h = (int)(i % nq);
  const size_t t = i / nq;
  const bf16_t* orow = o + (t * nq + h) * D;
  const bf16_t* drow = dout + (t * nq + h) * D;
  float half[2] = {0.f, 0.f};
#pragma unroll
  for (int kg = 0; kg < 2; kg++)
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) {
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(drow + ks * 16 + kg * 8), b = *reinterpret_cast<const bf16x8*>(orow + ks * 16 + kg * 8);
#pragma unroll
      for (int e = 0; e < 8; e++) half[kg] = fmaf((float)a[e], (float)b[e], half[kg]);
    }
  delta[(size_t)h * T + t] = half[0] + half[1];
  lse2[(size_t)h * T + t] = lse[(size_t)h * T + t] * LOG2E;
}

// dk,dv[token][kv head] = sum over the group's query heads (ascending) and, inside a head, over the
// chunks of the token's key block (ascending) of the float32 partials.
// grid (32*ceil(seq/128), nkv, batch), 256 threads: a block owns 4 rows of a key block, thread = (key row, 4
// columns of [dK | dV]).
template <int D>
__device__ __forceinline__ void attn_bwd_group_reduce_block(int bx, int by, int bz, const float* __restrict__ part, const AttnGeom& g,
                                                            int pairs) {
  const int seq = g.seq, nq = g.nq, nkv = g.nkv;
  const int i = bx >> 5, r0 = (bx & 31) * 4, hk = by, b = bz, grp = nq / nkv;
  int base = 0;
  for (int k = 0; k < i; k++) base += chunks_of(dkv_tiles(k, seq, g.q_off), g.ch);
  const int ch = chunks_of(dkv_tiles(i, seq, g.q_off), g.ch);
  for (int e = threadIdx.x; e < 4 * 2 * D / 4; e += 256) {
    const int row = r0 + e / (2 * D / 4), c4 = (e % (2 * D / 4)) * 4;
    if (i * 128 + row >= seq) continue;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int gh = 0; gh < grp; gh++) {
      const float* p0 = part + (((size_t)b * nq + hk * grp + gh) * pairs + base) * 128 * (2 * D);
      for (int c = 0; c < ch; c++) s += __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p0 + ((size_t)c * 128 + row) * (2 * D) + c4));
    }
    bf16x4 o = {(bf16_t)s[0], (bf16_t)s[1], (bf16_t)s[2], (bf16_t)s[3]};
    bf16_t* dst = g.dkv + ((size_t)b * seq + i * 128 + row) * g.lddkv + (c4 < D ? (size_t)hk * D + c4 : (size_t)(nkv + hk) * D + (c4 - D));
    *reinterpret_cast<bf16x4*>(dst) = o;
  }
}

// Both merges in one launch (they are independent, short and bandwidth-bound): the first nb_q blocks are the
// (x, y, z) = (16 * query blocks, nq, batch) grid of the dQ merge, the rest the (32 * key blocks, nkv, batch) grid of
// the dK/dV merge; either part may be empty.
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_reduce_kernel(const float* __restrict__ part_q, bf16_t* __restrict__ dqkv, int pairs_q,
                                                              int ch_q, float scale, unsigned nb_q, unsigned gqx, unsigned gqy,
                                                              const float* __restrict__ part_kv, const AttnGeom g, int pairs_k,
                                                              unsigned gkx, unsigned gky) {
  unsigned id = blockIdx.x;
  if (id < nb_q) {
    attn_bwd_dq_reduce_block<D>((int)(id % gqx), (int)(id / gqx % gqy), (int)(id / (gqx * gqy)), part_q, dqkv, g.seq, g.q_off, g.nq,
                                g.nkv, pairs_q, ch_q, scale);
  } else {
    id -= nb_q;
    attn_bwd_group_reduce_block<D>((int)(id % gkx), (int)(id / gkx % gky), (int)(id / (gkx * gky)), part_kv, g, pairs_k);
  }
}

// ------------------------------------------------------------------------------------ host side
template <typename K>
static int set_lds(K kernel, size_t bytes) {
  DH_HIP(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return DH_OK;
}

static int attn_num_cus() {  // of the current device
  static int cached[DH_MAX_DEVICES] = {};
  const int dev = dh_device_index();
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) cached[dev] = n;
    else cached[dev] = 256;
    (void)hipGetLastError();
  }
  return cached[dev];
}

// Chunk length of a launch.  The blocks of a launch are (block of 128 positions, chunk) units times nq*batch heads,
// started heaviest first; the hardware hands the next block to the first free compute unit.  That list schedule is
// simulated for each candidate length: a unit costs its tiles plus a fixed overhead, every chunk of a split launch
// costs the traffic of its float32 partial result (written, then read by the merging kernel), and a split launch
// pays for the merging kernels.  The constants are measured on MI355X (microseconds): a compute unit finishes a
// forward tile in 1.45 whether one or two blocks share it, a dQ tile in 1.8, a dK/dV tile in 2.5; HBM moves 4 MB per
// microsecond under this load.
enum { PICK_FWD = 0, PICK_DQ = 1, PICK_DKV = 2 };
struct PickKey {
  int kind, seq, q_off, nq_all, d, grouped, cus;
  bool operator<(const PickKey& o) const {
    return std::tie(kind, seq, q_off, nq_all, d, grouped, cus) < std::tie(o.kind, o.seq, o.q_off, o.nq_all, o.d, o.grouped, o.cus);
  }
};
static double simulate_launch(int kind, int seq, int q_off, int nq_all, int ch, int slots, double t_tile, double t_ovh) {
  const int nblk = (seq + 127) / 128, qb0 = q_off / 128;
  std::priority_queue<double, std::vector<double>, std::greater<double>> free_at;
  for (int i = 0; i < slots; i++) free_at.push(0.0);
  double makespan = 0.0;
  auto run = [&](int tiles) {
    for (int t0 = 0; t0 < tiles; t0 += ch) {
      const double cost = (tiles - t0 < ch ? tiles - t0 : ch) * t_tile + t_ovh;
      for (int h = 0; h < nq_all; h++) {
        const double end = free_at.top() + cost;
        free_at.pop();
        free_at.push(end);
        if (end > makespan) makespan = end;
      }
    }
  };
  if (kind == PICK_DKV) for (int i = 0; i < nblk; i++) run(dkv_tiles(i, seq, q_off));
  else for (int i = nblk - 1; i >= qb0; i--) run(dq_tiles(i, seq));  // forward: the tiles dQ walks
  return makespan;
}
static int pick_chunk(int kind, int seq, int q_off, int nq_all, int d, bool grouped) {
  static std::mutex mu;
  static std::map<PickKey, int> cache;
  const PickKey key{kind, seq, q_off, nq_all, d, grouped ? 1 : 0, attn_num_cus()};
  std::lock_guard<std::mutex> lock(mu);
  auto it = cache.find(key);
  if (it != cache.end()) return it->second;
  const int nblk = (seq + 127) / 128, qb0 = q_off / 128;
  const int max_tiles = kind == PICK_DKV ? dkv_tiles(0, seq, q_off) : dq_tiles(nblk - 1, seq);
  const double t_tile = (kind == PICK_FWD ? 1.45 : kind == PICK_DQ ? 1.8 : 2.5) * d / 128.0, t_ovh = 3.0;
  const double us_per_byte = 2.0 / 4.0e6, t_merge = 12.0;
  static const int cand_fwd[] = {4, 8, 16, 32, 64, 1 << 20}, cand_bwd[] = {4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 1 << 20};
  const int* cand = kind == PICK_FWD ? cand_fwd : cand_bwd;
  const int n_cand = kind == PICK_FWD ? 6 : 12;
  int best = cand[n_cand - 1];
  double best_t = 1e300;
  for (int k = 0; k < n_cand; k++) {
    const int ch = cand[k];
    if (ch < (1 << 20) && ch >= max_tiles) continue;  // same as not splitting
    int units = 0;
    if (kind == PICK_DKV) for (int i = 0; i < nblk; i++) units += chunks_of(dkv_tiles(i, seq, q_off), ch);
    else for (int i = qb0; i < nblk; i++) units += chunks_of(dq_tiles(i, seq), ch);
    const bool split = units > (kind == PICK_DKV ? nblk : nblk - qb0);
    double t = simulate_launch(kind, seq, q_off, nq_all, ch, attn_num_cus(), t_tile, t_ovh);
    double bytes = 0.0;
    if (kind == PICK_FWD) { if (split) bytes = (double)units * (d + 2); }
    else if (kind == PICK_DQ) { if (split) bytes = (double)units * d; }
    else if (split || grouped) bytes = (double)units * 2 * d;
    t += bytes * nq_all * 128 * sizeof(float) * us_per_byte + (split && !(kind == PICK_DKV && grouped) ? t_merge : 0.0);
    if (t < best_t) { best_t = t; best = ch; }
  }
  // When splitting pays at all it is because the launch would leave compute units idle, and then the finest split
  // whose units are still all resident at once balances them best (measured: 4 heads x 4096 tokens, forward 16 -> 10
  // tiles per chunk 48 -> 42 us, backward 24 -> 22 tiles 116 -> 113 us; one more unit than fits costs a second round).
  // Resident blocks per compute unit: forward 2 (4 at D = 64, counted as 2), backward 1 (2 at D = 64).
  if (best < (1 << 20)) {
    const long long resident = (long long)attn_num_cus() * (kind == PICK_FWD || d == 64 ? 2 : 1);
    for (int ch = 8; ch < best; ch += 2) {
      long long units = 0;
      if (kind == PICK_DKV) for (int i = 0; i < nblk; i++) units += chunks_of(dkv_tiles(i, seq, q_off), ch);
      else for (int i = qb0; i < nblk; i++) units += chunks_of(dq_tiles(i, seq), ch);
      if (units * nq_all <= resident) { best = ch; break; }
    }
  }
  cache[key] = best;
  return best;
}

// Tiles per chunk of the forward kernel; 0 = blocks are not split.
static int fwd_chunk_tiles(int batch, int seq, int q_off, int nq, int d) {
  const int ch = pick_chunk(PICK_FWD, seq, q_off, nq * batch, d, false);
  return ch >= (1 << 20) ? 0 : ch;
}
// Tiles per chunk of the dQ and of the dK/dV kernel.
static void bwd_chunk_tiles(int batch, int seq, int q_off, int nq, int nkv, int d, int& ch_q, int& ch_k) {
  ch_q = pick_chunk(PICK_DQ, seq, q_off, nq * batch, d, false);
  ch_k = pick_chunk(PICK_DKV, seq, q_off, nq * batch, d, nq > nkv);
}

// The launchers take the queries' sequence length seq_q and q_off; kv == nullptr selects plain attention (keys and
// values in the packed qkv rows, gradients into the packed dqkv rows).
static int check_geom(int d, int q_off, const void* kv, int ldkv, int nkv) {
  if (d != 64 && d != 128) DH_FAIL(DH_ERR_SHAPE, "attention (bf16): head_dim %d must be 64 or 128", d);
  if (q_off < 0 || q_off % 128) DH_FAIL(DH_ERR_SHAPE, "attention (bf16): the query offset %d must be a non-negative multiple of 128", q_off);
  if (!kv && q_off) DH_FAIL(DH_ERR_INVALID_ARG, "attention (bf16): a query offset needs a key/value buffer");
  if (kv && (ldkv < 2 * nkv * d || ldkv % 8 || ((uintptr_t)kv & 15)))
    DH_FAIL(DH_ERR_SHAPE, "attention (bf16): key/value rows must hold 2*nkv*d elements, be a multiple of 8 long and 16-byte aligned");
  return DH_OK;
}

size_t dh_attn_fwd_bf16_ws_bytes(int batch, int seq_q, int q_off, int nq, int nkv, int d) {
  (void)nkv;
  if (batch * seq_q == 0) return 0;
  const int seq = q_off + seq_q, ch = fwd_chunk_tiles(batch, seq, q_off, nq, d);
  if (ch == 0) return 0;
  return (size_t)batch * nq * fwd_units(seq, q_off, ch) * 128 * ((size_t)d + 2) * sizeof(float);
}

int dh_launch_attn_fwd_bf16(int batch, int seq_q, int nq, int nkv, int d, const bf16_t* qkv, const bf16_t* kv, int ldkv, int q_off,
                            bf16_t* o, float* lse, void* ws, size_t ws_bytes, hipStream_t stream) {
  int rc;
  if ((rc = check_geom(d, q_off, kv, ldkv, nkv))) return rc;
  if (batch * seq_q == 0) return DH_OK;
  const int seq = q_off + seq_q, T = batch * seq_q;
  AttnGeom g;
  g.seq = seq; g.q_off = q_off; g.nq = nq; g.nkv = nkv; g.dkv = nullptr; g.lddkv = 0; g.ch = 0; g.nq_all = nq * batch;
  if (kv) { g.kv = kv; g.ldkv = ldkv; } else { g.kv = qkv + (size_t)nq * d; g.ldkv = (nq + 2 * nkv) * d; }
  const int nblk = (seq + 127) / 128 - q_off / 128;  // blocks that hold queries
  int ch = fwd_chunk_tiles(batch, seq, q_off, nq, d);
  if (ch > 0 && (!ws || ws_bytes < dh_attn_fwd_bf16_ws_bytes(batch, seq_q, q_off, nq, nkv, d))) ch = 0;  // no room for partial results
  const int units = ch > 0 ? fwd_units(seq, q_off, ch) : nblk;
  float* part_o = (float*)ws;
  float* part_ml = ch > 0 ? part_o + (size_t)batch * nq * units * 128 * d : nullptr;
  dim3 grid((unsigned)units * nq * batch), cgrid(nblk * 8, nq, batch);
  const float sl2 = (float)(1.4426950408889634 / sqrt((double)d));
  const size_t lds = 2 * AF_RING * (size_t)AB_KT * d * 2;
  static bool ready_dev[DH_MAX_DEVICES][2] = {};
  bool* ready = ready_dev[dh_device_index()];
  if (d == 128) {
    if (!ready[0]) { if ((rc = set_lds(attn_fwd_bf16_kernel<128>, lds))) return rc; ready[0] = true; }
    attn_fwd_bf16_kernel<128><<<grid, AB_THREADS, lds, stream>>>(g, qkv, o, lse, T, sl2, ch, units, part_o, part_ml);
    DH_LAUNCH_CHECK();
    if (ch > 0) attn_fwd_combine_kernel<128><<<cgrid, 256, 0, stream>>>(seq, q_off, nq, ch, units, part_o, part_ml, o, lse, T);
  } else {
    if (!ready[1]) { if ((rc = set_lds(attn_fwd_bf16_kernel<64>, lds))) return rc; ready[1] = true; }
    attn_fwd_bf16_kernel<64><<<grid, AB_THREADS, lds, stream>>>(g, qkv, o, lse, T, sl2, ch, units, part_o, part_ml);
    DH_LAUNCH_CHECK();
    if (ch > 0) attn_fwd_combine_kernel<64><<<cgrid, 256, 0, stream>>>(seq, q_off, nq, ch, units, part_o, part_ml, o, lse, T);
  }
  DH_LAUNCH_CHECK();
  return DH_OK;
}

// workspace: lse2[nq*T] floats; dK/dV partials [batch][nq][pairs][128][2d] floats when heads are grouped
// or some block needs more than one chunk; dQ partials [batch][nq][pairs][128][d] floats in the latter case
struct BwdLayout {
  size_t o_lse2, o_dkv, o_dq, total;
  int ch_q, ch_k, pq, pk;   // chunk lengths and (block, chunk) pair counts of the dQ and the dK/dV launch
  bool part_q, part_kv;     // whether the launch writes float32 partial results
};
static BwdLayout bwd_ws_layout(int batch, int seq_q, int q_off, int nq, int nkv, int d) {
  BwdLayout L;
  const size_t T = (size_t)batch * seq_q;
  const int seq = q_off + seq_q, nblk = (seq + 127) / 128;
  bwd_chunk_tiles(batch, seq, q_off, nq, nkv, d, L.ch_q, L.ch_k);
  L.pq = total_pairs_dq(seq, q_off, L.ch_q);
  L.pk = total_pairs_dkv(seq, q_off, L.ch_k);
  L.part_q = L.pq > nblk - q_off / 128;
  L.part_kv = nq > nkv || L.pk > nblk;
  size_t cur = 0;
  L.o_lse2 = cur; cur += dh_align_up(nq * T * sizeof(float), 256);
  L.o_dkv = cur; if (L.part_kv) cur += dh_align_up((size_t)batch * nq * L.pk * 128 * 2 * d * sizeof(float), 256);
  L.o_dq = cur; if (L.part_q) cur += dh_align_up((size_t)batch * nq * L.pq * 128 * d * sizeof(float), 256);
  L.total = cur;
  return L;
}

size_t dh_attn_bwd_bf16_ws_bytes(int batch, int seq_q, int q_off, int nq, int nkv, int d) {
  return bwd_ws_layout(batch, seq_q, q_off, nq, nkv, d).total;
}

int dh_launch_attn_bwd_bf16(int batch, int seq_q, int nq, int nkv, int d, const bf16_t* qkv, const bf16_t* kv, int ldkv, int q_off,
                            const bf16_t* o, const bf16_t* dout, const float* lse, bf16_t* dqkv, bf16_t* dkv, int lddkv,
                            float* delta, void* ws, size_t ws_bytes, hipStream_t stream) {
  int rc;
  if ((rc = check_geom(d, q_off, kv, ldkv, nkv))) return rc;
  if (kv && (!dkv || lddkv < 2 * nkv * d || lddkv % 8 || ((uintptr_t)dkv & 15)))
    DH_FAIL(DH_ERR_SHAPE, "attention (bf16): the key/value gradient buffer must match the key/value buffer's layout rules");
  const int T = batch * seq_q, seq = q_off + seq_q;
  if (T == 0) return DH_OK;
  AttnGeom g;
  g.seq = seq; g.q_off = q_off; g.nq = nq; g.nkv = nkv;
  if (kv) { g.kv = kv; g.ldkv = ldkv; g.dkv = dkv; g.lddkv = lddkv; }
  else { g.kv = qkv + (size_t)nq * d; g.dkv = dqkv + (size_t)nq * d; g.ldkv = g.lddkv = (nq + 2 * nkv) * d; }
  const BwdLayout lay = bwd_ws_layout(batch, seq_q, q_off, nq, nkv, d);
  g.nq_all = nq * batch;
  AttnGeom gq_geom = g, gk_geom = g;
  gq_geom.ch = lay.ch_q;
  gk_geom.ch = lay.ch_k;
  if (!ws || ws_bytes < lay.total) DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "attn_bwd: workspace %zu < %zu bytes", ws_bytes, lay.total);
  float* lse2 = (float*)((char*)ws + lay.o_lse2);
  float* part_kv = lay.part_kv ? (float*)((char*)ws + lay.o_dkv) : nullptr;
  float* part_q = lay.part_q ? (float*)((char*)ws + lay.o_dq) : nullptr;
  const float sc = (float)(1.0 / sqrt((double)d)), sl2 = (float)(1.4426950408889634 / sqrt((double)d));
  const int nblk = (seq + 127) / 128, nblk_q = nblk - q_off / 128, pq = lay.pq, pk = lay.pk;
  dim3 gw((unsigned)(pq + pk) * nq * batch), gwq((unsigned)pq * nq * batch), gwk((unsigned)pk * nq * batch), gq(nblk_q * 16, nq, batch),
      gk(nblk * 32, nkv, batch);
  const unsigned nb_q = part_q ? gq.x * gq.y * gq.z : 0, nb_k = part_kv ? gk.x * gk.y * gk.z : 0;
  const size_t lds_dq = 2 * AB_RING * (size_t)AB_KT * d * 2, lds_dkv = lds_dq + 2 * AB_RING * AB_KT * sizeof(float);
  static bool ready_dev[DH_MAX_DEVICES][2] = {};
  bool* ready = ready_dev[dh_device_index()];
#define DH_ATTN_BWD(DD, IDX)                                                                                                   \
  do {                                                                                                                         \
    if (!ready[IDX]) {                                                                                                         \
      if ((rc = set_lds(attn_bwd_bf16_kernel<DD>, lds_dkv)) || (rc = set_lds(attn_bwd_dq_bf16_kernel<DD>, lds_dq)) ||          \
          (rc = set_lds(attn_bwd_dkv_bf16_kernel<DD>, lds_dkv))) return rc;                                                    \
      ready[IDX] = true;                                                                                                       \
    }                                                                                                                          \
    if (nq == nkv) {                                                                                                           \
      attn_bwd_prep_kernel<DD><<<(unsigned)(((size_t)T * nq + 255) / 256), 256, 0, stream>>>(o, dout, lse, lse2, delta, T, nq); \
      DH_LAUNCH_CHECK();                                                                                                       \
      attn_bwd_bf16_kernel<DD><<<gw, AB_THREADS, lds_dkv, stream>>>(gq_geom, gk_geom, qkv, o, dout, lse, lse2, delta, dqkv, part_q, \
                                                                   part_kv, pq, pk, T, sc, sl2);                               \
    } else {                                                                                                                   \
      attn_bwd_dq_bf16_kernel<DD><<<gwq, AB_THREADS, lds_dq, stream>>>(gq_geom, qkv, o, dout, lse, lse2, delta, dqkv, part_q, pq, T, sc, sl2); \
      DH_LAUNCH_CHECK();                                                                                                       \
      attn_bwd_dkv_bf16_kernel<DD><<<gwk, AB_THREADS, lds_dkv, stream>>>(gk_geom, qkv, dout, lse2, delta, part_kv, pk, T, sc, sl2); \
    }                                                                                                                          \
    DH_LAUNCH_CHECK();                                                                                                         \
    if (nb_q + nb_k > 0) {                                                                                                     \
      attn_bwd_reduce_kernel<DD><<<nb_q + nb_k, 256, 0, stream>>>(part_q, dqkv, pq, lay.ch_q, sc, nb_q, gq.x, gq.y, part_kv, gk_geom, pk, \
                                                                 gk.x, gk.y);                                                  \
      DH_LAUNCH_CHECK();                                                                                                       \
    }                                                                                                                          \
  } while (0)
  if (d == 128) DH_ATTN_BWD(128, 0); else DH_ATTN_BWD(64, 1);
#undef DH_ATTN_BWD
  return DH_OK;
}
