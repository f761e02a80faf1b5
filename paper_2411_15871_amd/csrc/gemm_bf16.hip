// bf16 GEMM on the matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//   C[M,N] (+)= opA(A) * opB(B)
// Operand layouts (all row-major):
//   TA = false: A is [M,K] (K contiguous)      TA = true: A is [K,M] (M contiguous)
//   TB = false: B is [K,N] (N contiguous)      TB = true: B is [N,K] (K contiguous)
// The forward projections use (TA=0,TB=0) with weights [in,out]; data gradients (dY * W^T) use
// (TA=0,TB=1); weight gradients (X^T * dY) use (TA=1,TB=0) and add into a float32 buffer.
//
// Tiling.  A block of WM x WN waves owns a BM x BN tile of C; a wave owns (BM/WM) x (BN/WN) as 32x32
// MFMA tiles.  K is consumed BK = 32 at a time through a ring of 4 LDS stages.  Tiles travel global
// -> LDS directly (global_load_lds_dwordx4: each lane moves 16 bytes, a wave fills 1 KiB of consecutive
// LDS), so no registers or LDS-write instructions are spent on staging; the loads of stage s+3 are
// issued right after the barrier that releases stage s, i.e. three K steps of matrix work cover the
// memory latency, and a step only waits (vmcnt) for the oldest stage in flight.
// Because a wave's 1 KiB lands linearly in LDS, bank conflicts are avoided by permuting which global
// 16-byte chunk each lane fetches (XOR swizzle), not by padding:
//   * K-contiguous operand, tile [rows][32]: 4 chunks per row; chunk c of row r sits at position
//     c ^ ((r>>2)&3).  The MFMA fragment read (16 lanes = 16 consecutive rows, one 16-byte chunk each)
//     then touches 16 different 16-byte bank groups.
//   * K-major operand (K is the slow dimension in memory), tile [32][cols]: chunk c of k-row r sits at
//     c ^ ((r&3)<<2).  Fragments come out of LDS through the transposing load ds_read_b64_tr_b16
//     (16 lanes fetch a 4(k) x 16(col) patch, each lane receives the 4 k-values of one column; two
//     such reads make one 8-k fragment); the swizzle puts the 4 k-rows of a patch on disjoint banks.
// Lanes whose chunk lies outside the matrix fetch from a 16-byte zero constant instead, which
// zero-fills ragged edges without branches.
// The tile -> block mapping is XCD-aware: consecutive block ids go round-robin to the 8 XCDs, so
// block b works on logical tile (b%8)*ceil(tiles/8) + b/8, and logical tiles are ordered in groups
// of 4 tile-rows, column by column; each XCD's L2 then serves a compact 4 x n patch of tiles.
// Split-K (grid.y > 1) writes float32 partial tiles to a workspace that a second kernel adds in
// split order, so results never depend on scheduling (no atomics anywhere).
// Requirements: N % 8 == 0 and every contiguous operand dimension % 8 == 0 (16-byte chunks).
#include <algorithm>
#include "common.h"

#define GB_BK 32
#define GB_STAGES 4

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

__device__ __attribute__((aligned(16))) const uint32_t dh_zero_chunk[4] = {0, 0, 0, 0};

enum { EPI_STORE_BF16 = 0, EPI_ACC_F32 = 1, EPI_PARTIAL_F32 = 2, EPI_TAIL_F32 = 3 };

struct GemmArgs {
  int M, N, K;
  const bf16_t* A;
  const bf16_t* B;
  void* C;  // bf16 (EPI_STORE_BF16), float (EPI_ACC_F32) or float partial base (EPI_PARTIAL_F32)
  int epi;
  int kt_per_split;  // K tiles handled by one split
  int tiles_m, tiles_n, tiles_per_xcd;
  const bf16_t* bias;          // optional [N], added before the bf16 store
  const int32_t* group_rows;   // grouped GEMM: device array of row counts (blockIdx.z = group), else nullptr
  int group_mode;              // 0/1: groups split M (A and C rows), B per group; 2: groups split K, C per group
  // Modes 0/1 are issued as two launches: part 1 with the large tile, part 2 with the 128x128 tile.  When the groups'
  // large tiles would leave the last round of tiles over the compute units nearly empty (the row counts are data), part 1
  // keeps only each group's whole large-tile rows and part 2 takes the remainders; otherwise part 1 does everything.
  int group_part, n_groups, part1_bm, part1_bn, cus;
  // Tail launch: when the tile count leaves the last round over the compute units less than half full, those tiles
  // are issued apart with K split over blockIdx.y, so that the round is short; tile_first = launch index of this
  // launch's first tile; EPI_TAIL_F32 writes tile-local float32 partials [split][tile][BM][BN].
  int tile_first;
  // SwiGLU fused into the epilogue (whole tiles only, bf16 result).  GLU_FWD: the GEMM is the gate/up projection with
  // N = 2*glu_f columns [gate | up]; a tile takes 128 gate columns and the 128 up columns of the same outputs (its B
  // panel is fetched from two places), stores both to C and gate*sigmoid(gate)*up to glu_out [M, glu_f].
  // GLU_BWD: the GEMM yields dA [M, N = glu_f]; instead of storing it the epilogue reads gate/up from glu_in
  // [M, 2*glu_f] and stores d(gate), d(up) to C [M, 2*glu_f].  Element arithmetic: swiglu_*_elem, as the row-wise kernels.
  int glu_mode, glu_f;
  const bf16_t* glu_in;
  bf16_t* glu_out;
  // An all-reduce stand-in carried along (Sec. 6.3, Table 7's closing remark: computation and communication in one kernel,
  // their shares of the machine fixed inside it instead of left to the dispatcher): the first ar_blocks thread blocks of
  // the launch stream the payload -- they hold their compute units for as long as the transfer lasts --, the tiles
  // follow.  0 = none.
  int ar_blocks;
};
// The stand-in's operands travel as a kernel argument of their own: GemmArgs is edited by the grouped path and lives in
// registers, the partial pointers are indexed at run time and stay in the argument segment.
struct GemmAr {
  int ranks;
  size_t n8;
  bf16_t* out;
  PartPtrs parts;
};
enum { GLU_NONE = 0, GLU_FWD = 1, GLU_BWD = 2 };

// Launch index -> tile coordinates.  XCD-aware: launch indices go round-robin over the 8 XCDs, each XCD owns a
// contiguous range of the logical tile order, which walks the tiles in bands of 4 tile rows.
__device__ __forceinline__ bool tile_of_launch(int idx, int tiles_m, int tiles_n, int tiles_per_xcd, int& tm, int& tn) {
  if ((idx >> 3) >= tiles_per_xcd) return false;  // grouped launches: grid sized for the largest group
  const int logical = (idx & 7) * tiles_per_xcd + (idx >> 3);
  if (logical >= tiles_m * tiles_n) return false;
  const int group = logical / (4 * tiles_n);
  const int rows_in_group = min(4, tiles_m - group * 4);
  const int in_group = logical - group * 4 * tiles_n;
  tm = group * 4 + in_group % rows_in_group;
  tn = in_group / rows_in_group;
  return true;
}

// Whether the remainders go to part 2: decided from the device-side row counts, the same way by both launches.
__device__ __forceinline__ bool grouped_split_remainders(const GemmArgs& g) {
  int full = 0, bulk = 0;
  const int tn = (g.N + g.part1_bn - 1) / g.part1_bn;
  for (int i = 0; i < g.n_groups; i++) {
    const int r = g.group_rows[i];
    full += (r + g.part1_bm - 1) / g.part1_bm * tn;
    bulk += r / g.part1_bm * tn;
  }
  const int tail = full % g.cus;  // tiles of the last, partly filled round
  return tail != 0 && tail * 4 < g.cus && bulk <= full / g.cus * g.cus;
}

// One 16-byte chunk per lane, global -> LDS.  lds_wave_base must be wave-uniform.  Written as inline
// assembly so that the compiler does not order later LDS reads behind the transfer with a full
// vmcnt(0) wait (it cannot tell the stages apart); the kernel waits for the transfers itself, once per
// K step, before the barrier that publishes a stage.
__device__ __forceinline__ void dma16(const void* gptr, bf16_t* lds_wave_base) {
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_wave_base;
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}

// Same with a wave-uniform 64-bit base (SGPR pair) and a per-lane 32-bit byte offset: the offsets of a
// tile do not change from one K step to the next, only the base advances.
__device__ __forceinline__ void dma16_base(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}

// Per-lane byte offsets of this wave's chunks relative to the tile origin (row r0, k = tile start).
// Rows/columns beyond the matrix are clamped to the last valid one: they only feed rows/columns of C
// that are never stored.  (K must not be clamped; ragged K tiles take issue_tile below.)
// half_jump != 0 (K-major only, whole tiles): the tile's second half of columns lies half_jump columns further on.
template <int ROWS, int NWAVES, bool KMAJOR>
__device__ __forceinline__ void tile_offsets(uint32_t (&voff)[ROWS * GB_BK / 8 / 64 / NWAVES], int r0, int R, int K, int wave,
                                             int lane, int half_jump = 0) {
  constexpr int IPW = ROWS * GB_BK / 8 / 64 / NWAVES;
#pragma unroll
  for (int j = 0; j < IPW; j++) {
    const int p = (wave * IPW + j) * 64 + lane;
    if (KMAJOR) {
      constexpr int CPR = ROWS / 8;
      const int kr = p / CPR, c = (p % CPR) ^ ((kr & 3) << 2);
      int col = min(r0 + c * 8, R - 8) - r0;
      if (half_jump != 0) col = c * 8 + (c * 8 >= ROWS / 2 ? half_jump : 0);
      voff[j] = (uint32_t)(((size_t)kr * R + col) * sizeof(bf16_t));
    } else {
      const int row = p >> 2, c = (p & 3) ^ ((row >> 2) & 3);
      const int rr = min(r0 + row, R - 1) - r0;
      voff[j] = (uint32_t)(((size_t)rr * K + c * 8) * sizeof(bf16_t));
    }
  }
}

// Issues this wave's share of one operand tile (general path with per-chunk bounds checks).  ROWS = tile extent along the operand's non-K
// dimension; KMAJOR = memory rows are k.  R/K = full matrix extents (non-K dimension, K dimension).
template <int ROWS, int NWAVES, bool KMAJOR>
__device__ __forceinline__ void issue_tile(bf16_t* lds_tile, const bf16_t* __restrict__ base, int r0, int k0, int R, int K,
                                           int wave, int lane) {
  constexpr int INSTS = ROWS * GB_BK / 8 / 64;  // wave-level loads per tile
  static_assert(INSTS % NWAVES == 0, "tile must split evenly over the waves");
  constexpr int IPW = INSTS / NWAVES;
#pragma unroll
  for (int j = 0; j < IPW; j++) {
    const int inst = wave * IPW + j;
    const int p = inst * 64 + lane;  // chunk position inside the LDS tile
    const bf16_t* src;
    if (KMAJOR) {
      constexpr int CPR = ROWS / 8;
      const int kr = p / CPR, c = (p % CPR) ^ ((kr & 3) << 2);
      const int k = k0 + kr, r = r0 + c * 8;
      src = (k < K && r < R) ? base + (size_t)k * R + r : reinterpret_cast<const bf16_t*>(dh_zero_chunk);
    } else {
      const int row = p >> 2, c = (p & 3) ^ ((row >> 2) & 3);
      const int r = r0 + row, k = k0 + c * 8;
      src = (r < R && k < K) ? base + (size_t)r * K + k : reinterpret_cast<const bf16_t*>(dh_zero_chunk);
    }
    dma16(src, lds_tile + inst * 512);
  }
}

// Fragment (8 consecutive k of one row) from a K-contiguous tile.
__device__ __forceinline__ bf16x8 frag_kc(const bf16_t* tile, int row, int kchunk) {
  return *reinterpret_cast<const bf16x8*>(tile + row * GB_BK + ((kchunk ^ ((row >> 2) & 3)) << 3));
}
// Fragment from a K-major tile [GB_BK][COLS]: k0..k0+7 of column c16 + s (s = lane%16, c16 % 16 == 0).
template <int COLS>
__device__ __forceinline__ bf16x8 frag_km(const bf16_t* tile, int k0, int c16, int s) {
  const int kr = k0 + (s >> 2);                 // k0 % 8 == 0, so (kr & 3) == (s >> 2) for both reads
  const int col = c16 + ((s & 3) << 2);
  const int off = kr * COLS + ((((col >> 3) ^ ((kr & 3) << 2)) << 3) | (col & 7));
  const bf16_t* p0 = tile + off;
  const bf16_t* p1 = p0 + 4 * COLS;             // k-row + 4: same (kr & 3), same swizzle
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(__attribute__((address_space(3))) void*)p0);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(__attribute__((address_space(3))) void*)p1);
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16_kernel(GemmArgs g, const GemmAr ar) {
  constexpr int NW = WM * WN;
  if (g.ar_blocks > 0 && blockIdx.x < (unsigned)g.ar_blocks) {  // this block is a share of the stand-in, not a tile
    if (blockIdx.y == 0 && blockIdx.z == 0)
      allreduce_span<bf16_t>(ar.parts, ar.ranks, ar.out, ar.n8, (size_t)blockIdx.x * blockDim.x + threadIdx.x,
                             (size_t)g.ar_blocks * blockDim.x);
    return;
  }
  if (g.group_rows != nullptr) {
    // Grouped: the groups' rows lie behind one another; this block's group is blockIdx.z.  The row
    // counts are data (expert routing), so the extents are fixed up here from device memory and the
    // grid is sized for the largest possible group; surplus blocks leave at the tile check below.
    int row0 = 0;
    for (int i = 0; i < (int)blockIdx.z; i++) row0 += g.group_rows[i];
    int rows = g.group_rows[blockIdx.z];
    if (g.group_part != 0) {
      const bool split = grouped_split_remainders(g);
      if (g.group_part == 1) {
        if (split) rows -= rows % g.part1_bm;
      } else {
        if (!split) return;
        row0 += rows - rows % g.part1_bm;
        rows %= g.part1_bm;
      }
    }
    if (rows == 0) return;
    if (g.group_mode == 2) {
      g.A += (size_t)row0 * g.M;
      g.B += (size_t)row0 * g.N;
      g.C = reinterpret_cast<float*>(g.C) + (size_t)blockIdx.z * g.M * g.N;
      g.K = rows;
      g.kt_per_split = (rows + GB_BK - 1) / GB_BK;
    } else {
      g.A += (size_t)row0 * g.K;
      g.B += (size_t)blockIdx.z * g.K * g.N;
      g.C = reinterpret_cast<bf16_t*>(g.C) + (size_t)row0 * g.N;
      g.M = rows;
      g.tiles_m = (rows + BM - 1) / BM;
      g.tiles_per_xcd = (g.tiles_m * g.tiles_n + 7) / 8;
    }
  }
  constexpr int WTM = BM / WM, WTN = BN / WN, MT = WTM / 32, NT = WTN / 32;
  constexpr int A_ELEMS = BM * GB_BK, B_ELEMS = BN * GB_BK, STAGE = A_ELEMS + B_ELEMS;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  int tm, tn;
  if (!tile_of_launch((int)blockIdx.x - g.ar_blocks + g.tile_first, g.tiles_m, g.tiles_n, g.tiles_per_xcd, tm, tn)) return;
  const int m0 = tm * BM, n0 = tn * BN;
  const bool glu_fwd = !TA && !TB && BN == 256 && g.glu_mode == GLU_FWD;
  const int nb0 = glu_fwd ? tn * (BN / 2) : n0;  // first column of the tile's B panel (its first half, if fused)
  const int nkt_total = (g.K + GB_BK - 1) / GB_BK;
  const int kt_begin = blockIdx.y * g.kt_per_split;
  const int kt_end = min(nkt_total, kt_begin + g.kt_per_split);

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; i++)
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  constexpr int IPA = BM * GB_BK / 8 / 64 / NW, IPB = BN * GB_BK / 8 / 64 / NW, IPS = IPA + IPB;
  uint32_t voa[IPA], vob[IPB];
  tile_offsets<BM, NW, TA>(voa, m0, g.M, g.K, wave, lane);
  tile_offsets<BN, NW, !TB>(vob, n0, g.N, g.K, wave, lane, glu_fwd ? g.glu_f - BN / 2 : 0);
  // tile origins at k = 0 and the byte stride of one K step
  const char* a0 = reinterpret_cast<const char*>(g.A + (TA ? (size_t)m0 : (size_t)m0 * g.K));
  const char* b0 = reinterpret_cast<const char*>(g.B + (TB ? (size_t)n0 * g.K : (size_t)nb0));
  const size_t sa = (TA ? (size_t)GB_BK * g.M : (size_t)GB_BK) * sizeof(bf16_t);
  const size_t sb = (TB ? (size_t)GB_BK : (size_t)GB_BK * g.N) * sizeof(bf16_t);
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
  auto issue_full = [&](int stage, const char* ab, const char* bb) {  // full K tile: precomputed offsets, uniform base
    const uint32_t la = lds0 + (uint32_t)(stage * STAGE * sizeof(bf16_t)) + wave * IPA * 1024;
    const uint32_t lb = lds0 + (uint32_t)((stage * STAGE + A_ELEMS) * sizeof(bf16_t)) + wave * IPB * 1024;
#pragma unroll
    for (int j = 0; j < IPA; j++) dma16_base(ab, voa[j], la + j * 1024);
#pragma unroll
    for (int j = 0; j < IPB; j++) dma16_base(bb, vob[j], lb + j * 1024);
  };
  auto issue = [&](int kt) {
    const int stage = (kt - kt_begin) % GB_STAGES;
    if ((kt + 1) * GB_BK <= g.K) {
      issue_full(stage, a0 + (size_t)kt * sa, b0 + (size_t)kt * sb);
    } else {
      bf16_t* st = smem + stage * STAGE;
      issue_tile<BM, NW, TA>(st, g.A, m0, kt * GB_BK, g.M, g.K, wave, lane);
      issue_tile<BN, NW, !TB>(st + A_ELEMS, g.B, n0, kt * GB_BK, g.N, g.K, wave, lane);
    }
  };
  const int l32 = lane & 31, kg = lane >> 5, s16 = lane & 15, h16 = (lane >> 4) & 1;
  struct Frags {
    bf16x8 a[MT], b[NT];
  };
  auto load_frags = [&](Frags& f, int stage, int ks) {
    const bf16_t* As = smem + stage * STAGE;
    const bf16_t* Bs = As + A_ELEMS;
#pragma unroll
    for (int i = 0; i < MT; i++) {
      if (TA) f.a[i] = frag_km<BM>(As, ks * 16 + kg * 8, wm0 + i * 32 + h16 * 16, s16);
      else f.a[i] = frag_kc(As, wm0 + i * 32 + l32, ks * 2 + kg);
    }
#pragma unroll
    for (int j = 0; j < NT; j++) {
      if (!TB) f.b[j] = frag_km<BN>(Bs, ks * 16 + kg * 8, wn0 + j * 32 + h16 * 16, s16);
      else f.b[j] = frag_kc(Bs, wn0 + j * 32 + l32, ks * 2 + kg);
    }
  };
  // operands swapped: the result tile is C^T, so a lane holds 4 consecutive columns of one row
  auto mma = [&](const Frags& f) {
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
      for (int j = 0; j < NT; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.b[j], f.a[i], acc[i][j], 0, 0, 0);
  };
  static_assert(GB_BK == 32, "the step below is written for two 16-wide MFMA sub-steps per stage");

#pragma unroll
  for (int s = 0; s < GB_STAGES - 1; s++)
    if (kt_begin + s < kt_end) issue(kt_begin + s);

  // Step `it` works on K tile kt_begin+it held in stage it%4.  The fragments of its first sub-step were
  // read at the end of step it-1; the step reads the second sub-step's fragments, multiplies the first,
  // then waits until stage it+1 has landed (the GB_STAGES-2 younger stages may stay in flight) and
  // passes the barrier -- after which every wave is also done reading stage it-1 --, issues the
  // transfer of tile it+3 into that buffer, reads the first fragments of stage it+1 and multiplies the
  // second sub-step.  The matrix cores thus have work queued across the barrier and the LDS latency.
  const int n = kt_end - kt_begin;
  const int n_full = min(kt_end, g.K / GB_BK) - kt_begin;  // leading steps whose tile is a full K tile
  Frags f0, f1;
  if (n > 0) {
    if (n > GB_STAGES - 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((GB_STAGES - 2) * IPS) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    load_frags(f0, 0, 0);
  }
  int it = 0;
  {
    // steady state, four steps per trip so that stage numbers are constants; every tile issued here
    // (up to it+6) is a full tile inside this block's K range
    const char* ap = a0 + (size_t)(kt_begin + GB_STAGES - 1) * sa;
    const char* bp = b0 + (size_t)(kt_begin + GB_STAGES - 1) * sb;
    for (; it + 2 * GB_STAGES - 1 <= n_full; it += GB_STAGES) {
#pragma unroll
      for (int u = 0; u < GB_STAGES; u++) {
        load_frags(f1, u, 1);
        mma(f0);
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"((GB_STAGES - 3) * IPS) : "memory");
        __syncthreads();
        issue_full((u + GB_STAGES - 1) % GB_STAGES, ap, bp);
        ap += sa;
        bp += sb;
        load_frags(f0, (u + 1) % GB_STAGES, 0);
        mma(f1);
      }
    }
  }
  for (; it < n; it++) {  // tail (and short K ranges): same steps with the checks spelled out
    load_frags(f1, it % GB_STAGES, 1);
    mma(f0);
    if (it + 1 < n) {
      if (it + GB_STAGES - 2 < n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"((GB_STAGES - 3) * IPS) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (it + GB_STAGES - 1 < n) issue(kt_begin + it + GB_STAGES - 1);
      load_frags(f0, (it + 1) % GB_STAGES, 0);
    }
    mma(f1);
  }

  // Epilogue.  acc[i][j][4q+e] = C[row][col], row = lane%32, col = 8q + 4*(lane/32) + e within the 32x32 tile.
  float* Cf = reinterpret_cast<float*>(g.C);
  bf16_t* Cb = reinterpret_cast<bf16_t*>(g.C);
  if (g.epi == EPI_PARTIAL_F32) Cf += (size_t)blockIdx.y * g.M * g.N;
  if (g.epi == EPI_TAIL_F32) {  // whole tile, tile-local layout (rows/columns beyond the matrix are never read back)
    Cf += ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * (BM * BN);
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
      for (int j = 0; j < NT; j++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *reinterpret_cast<f32x4*>(Cf + (size_t)(wm0 + i * 32 + l32) * BN + wn0 + j * 32 + 8 * q + 4 * kg) = v;
        }
    return;
  }
  if (g.epi == EPI_STORE_BF16 && m0 + BM <= g.M && n0 + BN <= g.N) {
    // Whole tile, bf16 result: the wave turns its part of C around in LDS (the ring is free now) so that a lane
    // stores 16 bytes and a store instruction covers 8 rows of 128 contiguous bytes, instead of 8 bytes per lane
    // scattered over 32 rows.  Wave-private region [WTM rows][64 columns], 16-byte chunks XOR-swizzled by row.
    static_assert(WTN == 64, "a row of the wave's part is 128 bytes");
    __syncthreads();
    bf16_t* reg = smem + wave * (WTM * WTN);
#pragma unroll
    for (int i = 0; i < MT; i++)
#pragma unroll
      for (int j = 0; j < NT; j++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const int row = i * 32 + l32, c0 = j * 32 + 8 * q + 4 * kg;
          f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          if (g.bias != nullptr) {
            const bf16x4 bb = *reinterpret_cast<const bf16x4*>(g.bias + n0 + wn0 + c0);
            v += f32x4{(float)bb[0], (float)bb[1], (float)bb[2], (float)bb[3]};
          }
          const bf16x4 o = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
          *reinterpret_cast<bf16x4*>(reg + row * WTN + ((((c0 >> 3) ^ (row & 7)) << 3) | (c0 & 4))) = o;
        }
    __builtin_amdgcn_wave_barrier();
    if (glu_fwd) {
      // the wave's 64 columns are gate columns (first two wave columns) or up columns (last two) of outputs nb0 + ...
      const int cb = nb0 + (wn0 < BN / 2 ? wn0 : g.glu_f - BN / 2 + wn0);
#pragma unroll
      for (int it = 0; it < WTM / 8; it++) {
        const int row = it * 8 + (lane >> 3), ch = lane & 7;
        const bf16x8 o = *reinterpret_cast<const bf16x8*>(reg + row * WTN + ((ch ^ (row & 7)) << 3));
        *reinterpret_cast<bf16x8*>(Cb + (size_t)(m0 + wm0 + row) * g.N + cb + ch * 8) = o;
      }
      // gate and up of one output sit in the regions of waves two wave columns apart: once every wave has written,
      // each wave combines half of the rows of its pair (the values as stored, i.e. rounded to bf16)
      __syncthreads();
      const int pw = (wave % WN) & 1, hi = (wave % WN) >> 1;
      const bf16_t* rg = smem + ((wave / WN) * WN + pw) * (WTM * WTN);
      const bf16_t* ru = rg + 2 * (WTM * WTN);
#pragma unroll
      for (int it = 0; it < WTM / 16; it++) {
        const int row = hi * (WTM / 2) + it * 8 + (lane >> 3), ch = lane & 7;
        const bf16x8 gv = *reinterpret_cast<const bf16x8*>(rg + row * WTN + ((ch ^ (row & 7)) << 3));
        const bf16x8 uv = *reinterpret_cast<const bf16x8*>(ru + row * WTN + ((ch ^ (row & 7)) << 3));
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 8; e++) o[e] = (bf16_t)swiglu_fwd_elem((float)gv[e], (float)uv[e]);
        *reinterpret_cast<bf16x8*>(g.glu_out + (size_t)(m0 + wm0 + row) * g.glu_f + nb0 + pw * WTN + ch * 8) = o;
      }
      return;
    }
    if (g.glu_mode == GLU_BWD) {
      // gate/up of 8 row groups are fetched together (the accumulators' registers are free by now), so that the
      // epilogue waits for memory twice, not once per row group
      constexpr int NB = 8;
      static_assert((WTM / 8) % NB == 0, "row groups come in batches");
#pragma unroll
      for (int it0 = 0; it0 < WTM / 8; it0 += NB) {
        bf16x8 gv[NB], uv[NB];
#pragma unroll
        for (int u = 0; u < NB; u++) {
          const int row = (it0 + u) * 8 + (lane >> 3), ch = lane & 7;
          const size_t r2 = (size_t)(m0 + wm0 + row) * (2 * (size_t)g.glu_f) + n0 + wn0 + ch * 8;
          gv[u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(g.glu_in + r2));
          uv[u] = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(g.glu_in + r2 + g.glu_f));
        }
#pragma unroll
        for (int u = 0; u < NB; u++) {
          const int row = (it0 + u) * 8 + (lane >> 3), ch = lane & 7;
          const size_t r2 = (size_t)(m0 + wm0 + row) * (2 * (size_t)g.glu_f) + n0 + wn0 + ch * 8;
          const bf16x8 o = *reinterpret_cast<const bf16x8*>(reg + row * WTN + ((ch ^ (row & 7)) << 3));
          bf16x8 dg, du;
#pragma unroll
          for (int e = 0; e < 8; e++) {
            float a, b;
            swiglu_bwd_elem((float)gv[u][e], (float)uv[u][e], (float)o[e], a, b);
            dg[e] = (bf16_t)a;
            du[e] = (bf16_t)b;
          }
          *reinterpret_cast<bf16x8*>(Cb + r2) = dg;
          *reinterpret_cast<bf16x8*>(Cb + r2 + g.glu_f) = du;
        }
      }
      return;
    }
#pragma unroll
    for (int it = 0; it < WTM / 8; it++) {
      const int row = it * 8 + (lane >> 3), ch = lane & 7;
      const bf16x8 o = *reinterpret_cast<const bf16x8*>(reg + row * WTN + ((ch ^ (row & 7)) << 3));
      *reinterpret_cast<bf16x8*>(Cb + (size_t)(m0 + wm0 + row) * g.N + n0 + wn0 + ch * 8) = o;
    }
    return;
  }
  if (g.epi != EPI_STORE_BF16 && m0 + BM <= g.M && n0 + BN <= g.N) {
    // Whole tile, float32 result (accumulate or partial): the same turn through LDS, one 32-column tile column j at a
    // time (wave-private region [WTM rows][32 floats], 16-byte chunks XOR-swizzled by row), so that a lane reads /
    // adds / writes 16 bytes of a 128-byte row segment.
    __syncthreads();
    float* reg = reinterpret_cast<float*>(smem_raw) + wave * (WTM * 32);
#pragma unroll
    for (int j = 0; j < NT; j++) {
      if (j > 0) __builtin_amdgcn_wave_barrier();  // the region's previous contents have been read
#pragma unroll
      for (int i = 0; i < MT; i++)
#pragma unroll
        for (int q = 0; q < 4; q++) {
          const int row = i * 32 + l32, ch = 2 * q + kg;
          const f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *reinterpret_cast<f32x4*>(reg + row * 32 + ((ch ^ (row & 7)) << 2)) = v;
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int it = 0; it < WTM / 8; it++) {
        const int row = it * 8 + (lane >> 3), ch = lane & 7;
        const f32x4 v = *reinterpret_cast<const f32x4*>(reg + row * 32 + ((ch ^ (row & 7)) << 2));
        f32x4* p = reinterpret_cast<f32x4*>(Cf + (size_t)(m0 + wm0 + row) * g.N + n0 + wn0 + j * 32 + ch * 4);
        if (g.epi == EPI_ACC_F32) *p = *p + v;
        else *p = v;
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < MT; i++) {
    const int row = m0 + wm0 + i * 32 + l32;
    if (row >= g.M) continue;
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const int col = n0 + wn0 + j * 32 + 8 * q + 4 * kg;
        if (col >= g.N) continue;  // N % 8 == 0: a group of 4 columns is entirely in or out
        const size_t o = (size_t)row * g.N + col;
        f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
        if (g.epi == EPI_STORE_BF16) {
          if (g.bias != nullptr) {
            const bf16x4 bb = *reinterpret_cast<const bf16x4*>(g.bias + col);
            v += f32x4{(float)bb[0], (float)bb[1], (float)bb[2], (float)bb[3]};
          }
          bf16x4 b = {(bf16_t)v[0], (bf16_t)v[1], (bf16_t)v[2], (bf16_t)v[3]};
          *reinterpret_cast<bf16x4*>(Cb + o) = b;
        } else if (g.epi == EPI_ACC_F32) {
          f32x4* p = reinterpret_cast<f32x4*>(Cf + o);
          *p = *p + v;
        } else {
          *reinterpret_cast<f32x4*>(Cf + o) = v;
        }
      }
  }
}

// Adds the split-K partials in split order; writes bf16 or accumulates into float32.
__global__ void splitk_reduce_kernel(const float* __restrict__ part, int splits, size_t mn, void* __restrict__ C, int epi,
                                     const bf16_t* __restrict__ bias, int N) {
  size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= mn) return;
  f32x4 s = *reinterpret_cast<const f32x4*>(part + i);
  for (int z = 1; z < splits; z++) s += *reinterpret_cast<const f32x4*>(part + (size_t)z * mn + i);
  if (epi == EPI_STORE_BF16) {
    if (bias != nullptr) {
      const bf16x4 bb = *reinterpret_cast<const bf16x4*>(bias + i % N);
      s += f32x4{(float)bb[0], (float)bb[1], (float)bb[2], (float)bb[3]};
    }
    bf16x4 o = {(bf16_t)s[0], (bf16_t)s[1], (bf16_t)s[2], (bf16_t)s[3]};
    *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(C) + i) = o;
  } else {
    f32x4* c = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(C) + i);
    *c = *c + s;
  }
}

// Adds the tail tiles' K splits in split order and applies the final epilogue.  grid (BM*BN/4/256, tail tiles).
template <int BM, int BN>
__global__ __launch_bounds__(256) void tail_reduce_kernel(const float* __restrict__ part, int splits, GemmArgs g, int final_epi) {
  int tm, tn;
  if (!tile_of_launch((int)blockIdx.y + g.tile_first, g.tiles_m, g.tiles_n, g.tiles_per_xcd, tm, tn)) return;
  const int e = (blockIdx.x * 256 + threadIdx.x) * 4, r = e / BN, c = e % BN;
  const int row = tm * BM + r, col = tn * BN + c;
  if (row >= g.M || col >= g.N) return;
  const size_t tile_elems = (size_t)BM * BN, n_tail = gridDim.y;
  f32x4 s = *reinterpret_cast<const f32x4*>(part + blockIdx.y * tile_elems + e);
  for (int z = 1; z < splits; z++) s += *reinterpret_cast<const f32x4*>(part + ((size_t)z * n_tail + blockIdx.y) * tile_elems + e);
  const size_t o = (size_t)row * g.N + col;
  if (final_epi == EPI_STORE_BF16) {
    if (g.bias != nullptr) {
      const bf16x4 bb = *reinterpret_cast<const bf16x4*>(g.bias + col);
      s += f32x4{(float)bb[0], (float)bb[1], (float)bb[2], (float)bb[3]};
    }
    bf16x4 b = {(bf16_t)s[0], (bf16_t)s[1], (bf16_t)s[2], (bf16_t)s[3]};
    *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(g.C) + o) = b;
  } else {
    f32x4* p = reinterpret_cast<f32x4*>(reinterpret_cast<float*>(g.C) + o);
    *p = *p + s;
  }
}

// ------------------------------------------------------------------------------------ host side
struct GemmPlan {
  int cfg;  // 0: 256x256 (8 waves), 1: 128x128 (4 waves), 2: 256x128 (4 waves)
  int bm, bn, splits, kt_per_split;
  int tail_tiles, tail_splits, tail_kt;  // tail launch (0 tiles = none): its tiles, K splits and K tiles per split
};

static int num_cus() {  // of the current device
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

// Tile and split-K choice.  256x256 tiles when they give most compute units a block; else 256x128 when that gives
// most units exactly one block (one 4-wave block per unit measured faster than two 128x128 blocks sharing a unit, for
// row-major A: 4096x1792x4096 with B transposed 84 -> 72 us); else 128x128;
// if a single wave of blocks still leaves units idle and K is long, split K (bounded by the
// workspace) so that about one block per unit exists.
static GemmPlan choose_plan(bool ta, int M, int N, int K, size_t ws_bytes) {
  const int cus = num_cus();
  auto tiles = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
  GemmPlan p;
  if (tiles(256, 256) * 2 >= cus) { p.cfg = 0; p.bm = 256; p.bn = 256; }
  else if (!ta && tiles(256, 128) <= cus && tiles(256, 128) * 4 >= (long long)cus * 3) { p.cfg = 2; p.bm = 256; p.bn = 128; }
  else { p.cfg = 1; p.bm = 128; p.bn = 128; }
  const int nkt = (K + GB_BK - 1) / GB_BK;
  const long long t = tiles(p.bm, p.bn);
  int splits = 1;
  if (t * 4 <= cus * 3 && nkt >= 32) {
    splits = (int)(cus / t);
    if (splits > nkt / 16) splits = nkt / 16;
    const size_t per = (size_t)M * N * sizeof(float);
    if (per == 0 || ws_bytes / per < (size_t)splits) splits = per ? (int)(ws_bytes / per) : 1;
    if (splits < 2) splits = 1;
  }
  p.kt_per_split = nkt == 0 ? 1 : (nkt + splits - 1) / splits;
  p.splits = nkt == 0 ? 1 : (nkt + p.kt_per_split - 1) / p.kt_per_split;
  // Tail: more than one round of 256x256 tiles whose last round is at most half full -> split those tiles' K so that
  // the last round takes 1/splits of a round (plus a small ordered reduction) instead of a whole one.
  p.tail_tiles = p.tail_splits = p.tail_kt = 0;
  const int tail = (int)(t % cus);
  if (p.cfg == 0 && p.splits == 1 && t > cus && tail > 0 && tail * 2 <= cus && nkt >= 64) {
    int ts = cus / tail;
    if (ts > 8) ts = 8;
    if (ts > nkt / 16) ts = nkt / 16;
    const size_t per = (size_t)(tail + 7) * p.bm * p.bn * sizeof(float);  // the launch index range is padded to a multiple of 8
    if (ws_bytes / per < (size_t)ts) ts = (int)(ws_bytes / per);
    if (ts >= 2) {
      p.tail_tiles = tail;
      p.tail_kt = (nkt + ts - 1) / ts;
      p.tail_splits = (nkt + p.tail_kt - 1) / p.tail_kt;
    }
  }
  return p;
}

// Launch indices of the tail launch: from the first index of the last round to the end of the (padded) index range.
static void tail_range(int M, int N, const GemmPlan& p, int& first, int& count) {
  const long long t = (long long)((M + p.bm - 1) / p.bm) * ((N + p.bn - 1) / p.bn);
  first = (int)(t / num_cus()) * num_cus();
  count = (int)((t + 7) / 8 * 8) - first;
}

size_t dh_gemm_bf16_ws_bytes(bool ta, bool tb, int M, int N, int K) {
  (void)tb;
  GemmPlan p = choose_plan(ta, M, N, K, (size_t)-1);
  if (p.tail_tiles > 0) {
    int first, count;
    tail_range(M, N, p, first, count);
    return (size_t)count * p.tail_splits * p.bm * p.bn * sizeof(float);
  }
  return p.splits > 1 ? (size_t)p.splits * M * N * sizeof(float) : 0;
}

template <int BM, int BN, int WM, int WN, bool TA, bool TB>
static int launch_cfg(GemmArgs g, int splits, hipStream_t stream, int n_groups = 1, int tile_first = 0, int n_tiles = -1,
                      const GemmAr* ar = nullptr) {
  constexpr size_t LDS_BYTES = GB_STAGES * (size_t)(BM + BN) * GB_BK * sizeof(bf16_t);
  static bool attr_set[DH_MAX_DEVICES] = {};  // the attribute belongs to the kernel's code object on one device
  const int dev = dh_device_index();
  if (!attr_set[dev]) {
    DH_HIP(hipFuncSetAttribute((const void*)gemm_bf16_kernel<BM, BN, WM, WN, TA, TB>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES));
    attr_set[dev] = true;
  }
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = (g.N + BN - 1) / BN;
  g.tiles_per_xcd = (g.tiles_m * g.tiles_n + 7) / 8;
  g.tile_first = tile_first;
  dim3 grid((n_tiles >= 0 ? n_tiles : g.tiles_per_xcd * 8) + g.ar_blocks, splits, n_groups);
  GemmAr none;
  none.ranks = 0; none.n8 = 0; none.out = nullptr;
  for (int r = 0; r < DH_MAX_RANKS; r++) none.parts.p[r] = nullptr;
  gemm_bf16_kernel<BM, BN, WM, WN, TA, TB><<<grid, 64 * WM * WN, LDS_BYTES, stream>>>(g, ar ? *ar : none);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

template <bool TA, bool TB>
static int launch_layout(const GemmArgs& g, const GemmPlan& p, hipStream_t stream, int n_groups = 1, int tile_first = 0,
                         int n_tiles = -1, int splits = 0, const GemmAr* ar = nullptr) {
  if (splits == 0) splits = p.splits;
  if (p.cfg == 0) return launch_cfg<256, 256, 2, 4, TA, TB>(g, splits, stream, n_groups, tile_first, n_tiles, ar);
  if (p.cfg == 2) return launch_cfg<256, 128, 2, 2, TA, TB>(g, splits, stream, n_groups, tile_first, n_tiles, ar);
  return launch_cfg<128, 128, 2, 2, TA, TB>(g, splits, stream, n_groups, tile_first, n_tiles, ar);
}
template <typename... Args>
static int launch_any(bool ta, bool tb, Args... args) {
  if (!ta && !tb) return launch_layout<false, false>(args...);
  if (!ta && tb) return launch_layout<false, true>(args...);
  return launch_layout<true, false>(args...);
}


int dh_launch_gemm_bf16(bool ta, bool tb, int M, int N, int K, const bf16_t* A, const bf16_t* B, void* C,
                        bool out_f32_accumulate, const bf16_t* bias, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (M < 0 || N < 0 || K < 0) DH_FAIL(DH_ERR_SHAPE, "gemm: negative dimension");
  if (N % 8 || (ta ? M : K) % 8 || (tb ? K : N) % 8)
    DH_FAIL(DH_ERR_SHAPE, "gemm (bf16): N and the contiguous operand dimensions must be multiples of 8 (M=%d N=%d K=%d ta=%d tb=%d)", M, N, K, ta, tb);
  if (ta && tb) DH_FAIL(DH_ERR_UNSUPPORTED, "gemm (bf16): trans_a with trans_b is not used by the layer and not built");
  if (bias && out_f32_accumulate) DH_FAIL(DH_ERR_INVALID_ARG, "gemm (bf16): a bias goes with a bf16 result only");
  if (M == 0 || N == 0) return DH_OK;
  if ((long long)M * N >= (1ll << 40) || (long long)M * K >= (1ll << 40)) DH_FAIL(DH_ERR_SHAPE, "gemm: matrix too large");
  GemmPlan p = choose_plan(ta, M, N, K, ws ? ws_bytes : 0);
  GemmArgs g;
  g.M = M; g.N = N; g.K = K; g.A = A; g.B = B;
  g.kt_per_split = p.kt_per_split;
  g.tiles_m = g.tiles_n = g.tiles_per_xcd = 0;
  g.bias = bias; g.group_rows = nullptr; g.group_mode = 0;
  g.group_part = 0; g.n_groups = 1; g.part1_bm = g.part1_bn = 256; g.cus = 0; g.tile_first = 0;
  g.glu_mode = GLU_NONE; g.glu_f = 0; g.glu_in = nullptr; g.glu_out = nullptr; g.ar_blocks = 0;
  const int final_epi = out_f32_accumulate ? EPI_ACC_F32 : EPI_STORE_BF16;
  int rc;
  if (p.tail_tiles > 0) {  // whole rounds with the final epilogue, then the last round's tiles with K split, then their sum
    int first, count;
    tail_range(M, N, p, first, count);
    g.C = C; g.epi = final_epi;
    if ((rc = launch_any(ta, tb, g, p, stream, 1, 0, first, 1))) return rc;
    GemmArgs gt = g;
    gt.C = ws; gt.epi = EPI_TAIL_F32; gt.kt_per_split = p.tail_kt;
    if ((rc = launch_any(ta, tb, gt, p, stream, 1, first, count, p.tail_splits))) return rc;
    gt.C = C;
    gt.tiles_m = (M + p.bm - 1) / p.bm; gt.tiles_n = (N + p.bn - 1) / p.bn;
    gt.tiles_per_xcd = (gt.tiles_m * gt.tiles_n + 7) / 8;
    gt.tile_first = first;
    tail_reduce_kernel<256, 256><<<dim3(256 * 256 / 4 / 256, count), 256, 0, stream>>>((const float*)ws, p.tail_splits, gt, final_epi);
    DH_LAUNCH_CHECK();
    return DH_OK;
  }
  if (p.splits > 1) { g.C = ws; g.epi = EPI_PARTIAL_F32; } else { g.C = C; g.epi = final_epi; }
  if ((rc = launch_any(ta, tb, g, p, stream))) return rc;
  if (p.splits > 1) {
    const size_t mn = (size_t)M * N;  // multiple of 8 because N is
    splitk_reduce_kernel<<<(unsigned)((mn / 4 + 255) / 256), 256, 0, stream>>>((const float*)ws, p.splits, mn, C, final_epi, bias, N);
    DH_LAUNCH_CHECK();
  }
  return DH_OK;
}

// GEMM with an all-reduce stand-in in the same launch.  ar_blocks counts 256-thread blocks, as dh_comm_standin's
// n_blocks does; the launch's blocks are 256 or 512 threads, so the same number of threads streams the payload.
bool dh_gemm_ar_fits(bool ta, bool tb, int M, int N, int K) {
  if (M <= 0 || N <= 0 || K <= 0 || (ta && tb) || N % 8 || (ta ? M : K) % 8 || (tb ? K : N) % 8) return false;
  const GemmPlan p = choose_plan(ta, M, N, K, (size_t)-1);
  return p.splits == 1 && p.tail_tiles == 0;
}
int dh_launch_gemm_bf16_ar(bool ta, bool tb, int M, int N, int K, const bf16_t* A, const bf16_t* B, void* C, bool out_f32_accumulate,
                           int n_ranks, const void* const* parts, bf16_t* ar_out, size_t ar_elems, int ar_blocks, hipStream_t stream) {
  if (!dh_gemm_ar_fits(ta, tb, M, N, K)) DH_FAIL(DH_ERR_UNSUPPORTED, "gemm+allreduce: M=%d N=%d K=%d does not run as a single launch", M, N, K);
  if (n_ranks < 1 || n_ranks > DH_MAX_RANKS || ar_blocks < 1 || ar_blocks > 65536 || ar_elems % 8 || ar_elems == 0)
    DH_FAIL(DH_ERR_INVALID_ARG, "gemm+allreduce: n_ranks %d, n_blocks %d, elements %zu", n_ranks, ar_blocks, ar_elems);
  const GemmPlan p = choose_plan(ta, M, N, K, (size_t)-1);
  GemmArgs g;
  g.M = M; g.N = N; g.K = K; g.A = A; g.B = B; g.C = C;
  g.epi = out_f32_accumulate ? EPI_ACC_F32 : EPI_STORE_BF16;
  g.kt_per_split = p.kt_per_split;
  g.tiles_m = g.tiles_n = g.tiles_per_xcd = 0;
  g.bias = nullptr; g.group_rows = nullptr; g.group_mode = 0;
  g.group_part = 0; g.n_groups = 1; g.part1_bm = g.part1_bn = 256; g.cus = 0; g.tile_first = 0;
  g.glu_mode = GLU_NONE; g.glu_f = 0; g.glu_in = nullptr; g.glu_out = nullptr;
  const int threads = p.cfg == 0 ? 512 : 256;
  const size_t n8 = ar_elems / 8, want = (n8 + threads - 1) / threads;
  size_t nb = ((size_t)ar_blocks * 256 + threads - 1) / threads;
  if (nb > want) nb = want;
  g.ar_blocks = (int)nb;
  GemmAr ar;
  ar.ranks = n_ranks; ar.n8 = n8; ar.out = ar_out;
  for (int r = 0; r < DH_MAX_RANKS; r++) ar.parts.p[r] = r < n_ranks ? parts[r] : nullptr;
  return launch_any(ta, tb, g, p, stream, 1, 0, -1, 0, (const GemmAr*)&ar);
}

// Gate/up projection with SwiGLU in its epilogue: gu[T, 2F] = x[T, H] * Wgu[H, 2F] (columns [gate | up]) and
// a[T, F] = gate * sigmoid(gate) * up computed from the stored (rounded) values -- the same bits as
// dh_launch_gemm_bf16 followed by the row-wise kernel.  Fits when the plain GEMM would be one launch of whole 256x256
// tiles and F is a multiple of 128 (a tile = 128 gate + the 128 matching up columns).
bool dh_glu_fwd_fits(int T, int F, int H) {
  if (T <= 0 || F <= 0 || H <= 0 || T % 256 || F % 128 || H % GB_BK) return false;
  const GemmPlan p = choose_plan(false, T, 2 * F, H, (size_t)-1);
  return p.cfg == 0 && p.splits == 1 && p.tail_tiles == 0;
}
int dh_launch_gemm_swiglu_fwd_bf16(int T, int F, int H, const bf16_t* x, const bf16_t* Wgu, bf16_t* gu, bf16_t* a, hipStream_t stream) {
  if (!dh_glu_fwd_fits(T, F, H)) DH_FAIL(DH_ERR_SHAPE, "gemm+swiglu forward: T=%d F=%d H=%d does not fit the fused kernel", T, F, H);
  GemmArgs g;
  g.M = T; g.N = 2 * F; g.K = H; g.A = x; g.B = Wgu; g.C = gu; g.epi = EPI_STORE_BF16;
  g.kt_per_split = H / GB_BK;
  g.tiles_m = g.tiles_n = g.tiles_per_xcd = 0;
  g.bias = nullptr; g.group_rows = nullptr; g.group_mode = 0;
  g.group_part = 0; g.n_groups = 1; g.part1_bm = g.part1_bn = 256; g.cus = 0; g.tile_first = 0;
  g.glu_mode = GLU_FWD; g.glu_f = F; g.glu_in = nullptr; g.glu_out = a; g.ar_blocks = 0;
  return launch_cfg<256, 256, 2, 4, false, false>(g, 1, stream);
}

// Data gradient of the down projection with SwiGLU's backward in its epilogue: dA = dY[T, H] * Wd[F, H]^T is not
// stored; dgu[T, 2F] = (d gate | d up) from dA (rounded to bf16 as the stored dA would be) and gu[T, 2F] -- the same
// bits as the GEMM followed by the row-wise kernel.  Fits when the plain GEMM would be one launch of whole tiles.
bool dh_glu_bwd_fits(int T, int F, int H) {
  if (T <= 0 || F <= 0 || H <= 0 || F % 8 || H % 8) return false;
  const GemmPlan p = choose_plan(false, T, F, H, (size_t)-1);
  return p.splits == 1 && p.tail_tiles == 0 && T % p.bm == 0 && F % p.bn == 0;
}
int dh_launch_gemm_swiglu_bwd_bf16(int T, int F, int H, const bf16_t* dy, const bf16_t* Wd, const bf16_t* gu, bf16_t* dgu, hipStream_t stream) {
  if (!dh_glu_bwd_fits(T, F, H)) DH_FAIL(DH_ERR_SHAPE, "gemm+swiglu backward: T=%d F=%d H=%d does not fit the fused kernel", T, F, H);
  const GemmPlan p = choose_plan(false, T, F, H, (size_t)-1);
  GemmArgs g;
  g.M = T; g.N = F; g.K = H; g.A = dy; g.B = Wd; g.C = dgu; g.epi = EPI_STORE_BF16;
  g.kt_per_split = p.kt_per_split;
  g.tiles_m = g.tiles_n = g.tiles_per_xcd = 0;
  g.bias = nullptr; g.group_rows = nullptr; g.group_mode = 0;
  g.group_part = 0; g.n_groups = 1; g.part1_bm = g.part1_bn = 256; g.cus = 0; g.tile_first = 0;
  g.glu_mode = GLU_BWD; g.glu_f = F; g.glu_in = gu; g.glu_out = nullptr; g.ar_blocks = 0;
  return launch_layout<false, true>(g, p, stream);
}

// Grouped GEMM with device-side row counts (expert routing is data): group z owns group_rows[z] consecutive
// rows, max_rows bounds any group (the grid is sized for it).  mode 0: C[rows,dim_b] = A[rows,dim_a] B_z[dim_a,dim_b];
// mode 1: C[rows,dim_b] = A[rows,dim_a] B_z[dim_b,dim_a]^T; mode 2: C_z[dim_a,dim_b] += A[rows,dim_a]^T B[rows,dim_b]
// (float32).  No split-K: every group is one launch slice of the same grid.
int dh_launch_gemm_grouped_bf16(int mode, int n_groups, const int32_t* group_rows, int max_rows, int dim_a, int dim_b,
                                const bf16_t* A, const bf16_t* B, void* C, hipStream_t stream) {
  if (dim_a % 8 || dim_b % 8) DH_FAIL(DH_ERR_SHAPE, "gemm_grouped (bf16): feature dimensions must be multiples of 8 (%d, %d)", dim_a, dim_b);
  if (max_rows == 0) return DH_OK;
  GemmArgs g;
  g.A = A; g.B = B; g.C = C;
  g.bias = nullptr; g.group_rows = group_rows; g.group_mode = mode;
  g.tiles_m = g.tiles_n = g.tiles_per_xcd = 0;
  g.group_part = 0; g.n_groups = n_groups; g.part1_bm = g.part1_bn = 256; g.cus = num_cus(); g.tile_first = 0;
  g.glu_mode = GLU_NONE; g.glu_f = 0; g.glu_in = nullptr; g.glu_out = nullptr; g.ar_blocks = 0;
  const int avg = std::max(1, max_rows / n_groups);
  GemmPlan p;
  if (mode == 2) { g.M = dim_a; g.N = dim_b; g.K = max_rows; p = choose_plan(true, dim_a, dim_b, avg, 0); }
  else { g.M = max_rows; g.N = dim_b; g.K = dim_a; p = choose_plan(false, avg, dim_b, dim_a, 0); }
  p.splits = 1;
  g.kt_per_split = (g.K + GB_BK - 1) / GB_BK;
  g.epi = mode == 2 ? EPI_ACC_F32 : EPI_STORE_BF16;
  if (mode == 2) return launch_layout<true, false>(g, p, stream, n_groups);
  if (p.cfg != 0 || n_groups > 64)  // small tiles already, or too many groups for the in-kernel row scan: one launch
    return mode == 0 ? launch_layout<false, false>(g, p, stream, n_groups) : launch_layout<false, true>(g, p, stream, n_groups);
  g.group_part = 1;
  int rc = mode == 0 ? launch_layout<false, false>(g, p, stream, n_groups) : launch_layout<false, true>(g, p, stream, n_groups);
  if (rc != DH_OK) return rc;
  g.group_part = 2;
  g.M = std::min(max_rows, g.part1_bm - 1);  // a remainder is shorter than a large tile
  p.cfg = 1; p.bm = p.bn = 128;
  return mode == 0 ? launch_layout<false, false>(g, p, stream, n_groups) : launch_layout<false, true>(g, p, stream, n_groups);
}
