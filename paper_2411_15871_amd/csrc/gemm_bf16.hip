// bf16 GEMM on the matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//   C[M,N] (+)= opA(A) * opB(B)
// Operand layouts (all row-major):
//   TA = false: A is [M,K] (K contiguous)      TA = true: A is [K,M] (M contiguous)
//   TB = false: B is [K,N] (N contiguous)      TB = true: B is [N,K] (K contiguous)
// The forward projections use (TA=0,TB=0) with weights [in,out]; data gradients (dY * W^T) use
// (TA=0,TB=1); weight gradients (X^T * dY) use (TA=1,TB=0) and add into a float32 buffer.
//
// A 256-thread block (4 waves, 2x2) owns a BM x BN tile of C; a wave owns (BM/2) x (BN/2) as
// 32x32 MFMA tiles.  K is consumed BK = 64 at a time through double-buffered LDS: while the matrix
// cores work on stage s the next tile travels global -> registers -> LDS stage s^1, one barrier per
// step.  The MFMA wants, per lane, 8 consecutive k of one row (A) or one column (B):
//   * operands whose K is contiguous are stored [row][BK+8] and read with one 16-byte LDS read
//     (the 8-element pad spreads 16 consecutive rows over all banks);
//   * operands whose K is the slow dimension are stored as they come, [k][rows+32], and read with
//     the transposing LDS load ds_read_b64_tr_b16: 16 lanes fetch a 4(k) x 16(row) patch and each
//     gets the 4 k-values of one row -- two such reads make one 8-k fragment.  The 32-element pad
//     puts 4 consecutive k-rows on disjoint banks.
// Split-K (grid.z > 1) writes float32 partial tiles to a workspace that a second kernel adds in
// split order, so results never depend on scheduling (no atomics anywhere).
// Requirements: K-contiguous operands need K % 8 == 0, M/N-contiguous ones need M % 8 / N % 8 == 0
// (16-byte loads); otherwise any size, edges are zero-filled / predicated.
#include "common.h"

#define GB_BK 64
#define GB_THREADS 256

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ bf16x8 lds_read_direct(const bf16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }

// Two transposing reads -> the 8 k-values (k0..k0+7) of row `m` for this lane.  `tile` is [k][ld].
// Lane s of each 16-lane group points at (k0 + s/4, m16 + 4*(s%4)) and receives row m16 + s.
__device__ __forceinline__ bf16x8 lds_read_tr(const bf16_t* tile, int ld, int k0, int m16, int s) {
  const bf16_t* p0 = tile + (k0 + (s >> 2)) * ld + m16 + ((s & 3) << 2);
  const bf16_t* p1 = p0 + 4 * ld;
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(__attribute__((address_space(3))) void*)p0);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(__attribute__((address_space(3))) void*)p1);
  typedef __attribute__((ext_vector_type(8))) short s16x8;
  s16x8 r = __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, r);
}

enum { EPI_STORE_BF16 = 0, EPI_ACC_F32 = 1, EPI_PARTIAL_F32 = 2 };

struct GemmArgs {
  int M, N, K;
  const bf16_t* A;
  const bf16_t* B;
  void* C;         // bf16 (EPI_STORE_BF16), float (EPI_ACC_F32) or float partial base (EPI_PARTIAL_F32)
  int epi;
  int kt_per_split;  // K tiles handled by one grid.z slice
};

template <int BM, int BN, bool TA, bool TB>
struct GemmTile {
  // LDS footprint of one stage, in elements.  A is K-contiguous when !TA, B when TB.
  static constexpr int A_LD = TA ? (BM + 32) : (GB_BK + 8);
  static constexpr int A_ELEMS = TA ? GB_BK * A_LD : BM * A_LD;
  static constexpr int B_LD = TB ? (GB_BK + 8) : (BN + 32);
  static constexpr int B_ELEMS = TB ? BN * B_LD : GB_BK * B_LD;
  static constexpr int STAGE = A_ELEMS + B_ELEMS;
  static constexpr size_t LDS_BYTES = 2 * (size_t)STAGE * sizeof(bf16_t);
  static constexpr int A_CHUNKS = BM * GB_BK / 8 / GB_THREADS;  // 16-byte chunks per thread
  static constexpr int B_CHUNKS = BN * GB_BK / 8 / GB_THREADS;
};

// Global -> register fetch of one operand tile.  ROWS = extent of the tile along the operand's
// non-K dimension, KMAJOR = memory rows are k (the non-K dimension is contiguous).
template <int ROWS, int NCH, bool KMAJOR>
__device__ __forceinline__ void fetch_tile(bf16x8 (&reg)[NCH], const bf16_t* __restrict__ base, int r0, int k0, int R,
                                           int K) {
  // base[(r, k)] = KMAJOR ? base[k*R + r] : base[r*K + k]
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    int id = threadIdx.x + i * GB_THREADS;
    bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (KMAJOR) {
      int k = k0 + id / (ROWS / 8), r = r0 + (id % (ROWS / 8)) * 8;
      if (k < K && r < R) v = *reinterpret_cast<const bf16x8*>(base + (size_t)k * R + r);
    } else {
      int r = r0 + id / (GB_BK / 8), k = k0 + (id % (GB_BK / 8)) * 8;
      if (r < R && k < K) v = *reinterpret_cast<const bf16x8*>(base + (size_t)r * K + k);
    }
    reg[i] = v;
  }
}

template <int ROWS, int NCH, bool KMAJOR, int LD>
__device__ __forceinline__ void stash_tile(const bf16x8 (&reg)[NCH], bf16_t* lds) {
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    int id = threadIdx.x + i * GB_THREADS;
    int off = KMAJOR ? (id / (ROWS / 8)) * LD + (id % (ROWS / 8)) * 8 : (id / (GB_BK / 8)) * LD + (id % (GB_BK / 8)) * 8;
    *reinterpret_cast<bf16x8*>(lds + off) = reg[i];
  }
}

template <int BM, int BN, bool TA, bool TB>
__global__ __launch_bounds__(GB_THREADS) void gemm_bf16_kernel(GemmArgs g) {
  using TL = GemmTile<BM, BN, TA, TB>;
  constexpr int WTM = BM / 2, WTN = BN / 2, MT = WTM / 32, NT = WTN / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm0 = (wave >> 1) * WTM, wn0 = (wave & 1) * WTN;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int nkt_total = (g.K + GB_BK - 1) / GB_BK;
  const int kt_begin = blockIdx.z * g.kt_per_split;
  const int kt_end = min(nkt_total, kt_begin + g.kt_per_split);

  f32x16 acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; i++)
#pragma unroll
    for (int j = 0; j < NT; j++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

  bf16x8 ra[TL::A_CHUNKS], rb[TL::B_CHUNKS];
  if (kt_begin < kt_end) {
    fetch_tile<BM, TL::A_CHUNKS, TA>(ra, g.A, m0, kt_begin * GB_BK, g.M, g.K);
    fetch_tile<BN, TL::B_CHUNKS, !TB>(rb, g.B, n0, kt_begin * GB_BK, g.N, g.K);
    stash_tile<BM, TL::A_CHUNKS, TA, TL::A_LD>(ra, smem);
    stash_tile<BN, TL::B_CHUNKS, !TB, TL::B_LD>(rb, smem + TL::A_ELEMS);
  }
  __syncthreads();

  const int l32 = lane & 31, kg = lane >> 5, s16 = lane & 15, h16 = (lane >> 4) & 1;
  for (int kt = kt_begin; kt < kt_end; kt++) {
    const int st = (kt - kt_begin) & 1;
    const bf16_t* As = smem + st * TL::STAGE;
    const bf16_t* Bs = As + TL::A_ELEMS;
    const bool more = kt + 1 < kt_end;
    if (more) {
      fetch_tile<BM, TL::A_CHUNKS, TA>(ra, g.A, m0, (kt + 1) * GB_BK, g.M, g.K);
      fetch_tile<BN, TL::B_CHUNKS, !TB>(rb, g.B, n0, (kt + 1) * GB_BK, g.N, g.K);
    }
#pragma unroll
    for (int ks = 0; ks < GB_BK / 16; ks++) {
      bf16x8 fa[MT], fb[NT];
#pragma unroll
      for (int i = 0; i < MT; i++) {
        if (TA) fa[i] = lds_read_tr(As, TL::A_LD, ks * 16 + kg * 8, wm0 + i * 32 + h16 * 16, s16);
        else fa[i] = lds_read_direct(As + (wm0 + i * 32 + l32) * TL::A_LD + ks * 16 + kg * 8);
      }
#pragma unroll
      for (int j = 0; j < NT; j++) {
        if (!TB) fb[j] = lds_read_tr(Bs, TL::B_LD, ks * 16 + kg * 8, wn0 + j * 32 + h16 * 16, s16);
        else fb[j] = lds_read_direct(Bs + (wn0 + j * 32 + l32) * TL::B_LD + ks * 16 + kg * 8);
      }
#pragma unroll
      for (int i = 0; i < MT; i++)
#pragma unroll
        for (int j = 0; j < NT; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      bf16_t* nx = smem + (st ^ 1) * TL::STAGE;
      stash_tile<BM, TL::A_CHUNKS, TA, TL::A_LD>(ra, nx);
      stash_tile<BN, TL::B_CHUNKS, !TB, TL::B_LD>(rb, nx + TL::A_ELEMS);
    }
    __syncthreads();
  }

  // Epilogue.  acc[i][j][r] is C[row][col] with row = 8*(r/4) + 4*(lane/32) + r%4, col = lane%32.
  float* Cf = reinterpret_cast<float*>(g.C);
  bf16_t* Cb = reinterpret_cast<bf16_t*>(g.C);
  if (g.epi == EPI_PARTIAL_F32) Cf += (size_t)blockIdx.z * g.M * g.N;
#pragma unroll
  for (int i = 0; i < MT; i++)
#pragma unroll
    for (int j = 0; j < NT; j++) {
      int col = n0 + wn0 + j * 32 + l32;
      if (col >= g.N) continue;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        int row = m0 + wm0 + i * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);
        if (row >= g.M) continue;
        size_t o = (size_t)row * g.N + col;
        float v = acc[i][j][r];
        if (g.epi == EPI_STORE_BF16) Cb[o] = (bf16_t)v;
        else if (g.epi == EPI_ACC_F32) Cf[o] += v;
        else Cf[o] = v;
      }
    }
}

// Adds the split-K partials in split order; writes bf16 or accumulates into float32.
__global__ void splitk_reduce_kernel(const float* __restrict__ part, int splits, size_t mn, void* __restrict__ C, int epi) {
  size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= mn) return;
  float4 s = *reinterpret_cast<const float4*>(part + i);
  for (int z = 1; z < splits; z++) {
    float4 v = *reinterpret_cast<const float4*>(part + (size_t)z * mn + i);
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  if (epi == EPI_STORE_BF16) {
    bf16x4 o = {(bf16_t)s.x, (bf16_t)s.y, (bf16_t)s.z, (bf16_t)s.w};
    *reinterpret_cast<bf16x4*>(reinterpret_cast<bf16_t*>(C) + i) = o;
  } else {
    float4* c = reinterpret_cast<float4*>(reinterpret_cast<float*>(C) + i);
    float4 o = *c;
    o.x += s.x; o.y += s.y; o.z += s.z; o.w += s.w;
    *c = o;
  }
}

// ------------------------------------------------------------------------------------ host side
struct GemmPlan {
  int bm, bn, splits, kt_per_split;
};

static int g_num_cus = 0;
static int num_cus() {
  if (g_num_cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
      g_num_cus = n;
    else
      g_num_cus = 256;
  }
  return g_num_cus;
}

// Tile and split-K choice: prefer the largest tile that still gives every compute unit a block;
// when even 128x128 tiles leave units idle and K is long, split K (bounded by the workspace).
static GemmPlan choose_plan(int M, int N, int K, size_t ws_bytes) {
  const int cus = num_cus();
  auto tiles = [&](int bm, int bn) { return (long long)((M + bm - 1) / bm) * ((N + bn - 1) / bn); };
  GemmPlan p;
  if (tiles(256, 256) >= cus * 3 / 4) { p.bm = 256; p.bn = 256; }
  else if (tiles(256, 128) >= cus * 3 / 4) { p.bm = 256; p.bn = 128; }
  else { p.bm = 128; p.bn = 128; }
  int nkt = (K + GB_BK - 1) / GB_BK;
  long long t = tiles(p.bm, p.bn);
  int splits = 1;
  if (t < cus * 3 / 4 && nkt >= 8) {
    splits = (int)((cus + t - 1) / t);
    if (splits > nkt / 4) splits = nkt / 4;
    size_t per = (size_t)M * N * sizeof(float);
    if (per == 0 || ws_bytes / per < (size_t)splits) splits = per ? (int)(ws_bytes / per) : 1;
    if (splits < 2) splits = 1;
  }
  p.splits = splits;
  p.kt_per_split = (nkt + splits - 1) / splits;
  p.splits = nkt == 0 ? 1 : (nkt + p.kt_per_split - 1) / p.kt_per_split;
  if (p.kt_per_split == 0) p.kt_per_split = 1;
  return p;
}

size_t dh_gemm_bf16_ws_bytes(bool ta, bool tb, int M, int N, int K) {
  (void)ta; (void)tb;
  GemmPlan p = choose_plan(M, N, K, (size_t)-1);
  return p.splits > 1 ? (size_t)p.splits * M * N * sizeof(float) : 0;
}

template <int BM, int BN, bool TA, bool TB>
static int launch_cfg(const GemmArgs& g, int splits, hipStream_t stream) {
  using TL = GemmTile<BM, BN, TA, TB>;
  static bool attr_set = false;
  if (!attr_set) {
    DH_HIP(hipFuncSetAttribute((const void*)gemm_bf16_kernel<BM, BN, TA, TB>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)TL::LDS_BYTES));
    attr_set = true;
  }
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, splits);
  gemm_bf16_kernel<BM, BN, TA, TB><<<grid, GB_THREADS, TL::LDS_BYTES, stream>>>(g);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

template <bool TA, bool TB>
static int launch_layout(const GemmArgs& g, const GemmPlan& p, hipStream_t stream) {
  if (p.bm == 256 && p.bn == 256) return launch_cfg<256, 256, TA, TB>(g, p.splits, stream);
  if (p.bm == 256 && p.bn == 128) return launch_cfg<256, 128, TA, TB>(g, p.splits, stream);
  return launch_cfg<128, 128, TA, TB>(g, p.splits, stream);
}

int dh_launch_gemm_bf16(bool ta, bool tb, int M, int N, int K, const bf16_t* A, const bf16_t* B, void* C,
                        bool out_f32_accumulate, void* ws, size_t ws_bytes, hipStream_t stream) {
  if (M < 0 || N < 0 || K < 0) DH_FAIL(DH_ERR_SHAPE, "gemm: negative dimension");
  if ((ta ? M : K) % 8 || (tb ? K : N) % 8)
    DH_FAIL(DH_ERR_SHAPE, "gemm (bf16): contiguous dimensions must be multiples of 8 (M=%d N=%d K=%d ta=%d tb=%d)", M, N, K, ta, tb);
  if (M == 0 || N == 0) return DH_OK;
  GemmPlan p = choose_plan(M, N, K, ws ? ws_bytes : 0);
  GemmArgs g;
  g.M = M; g.N = N; g.K = K; g.A = A; g.B = B;
  g.kt_per_split = p.kt_per_split;
  int final_epi = out_f32_accumulate ? EPI_ACC_F32 : EPI_STORE_BF16;
  if (p.splits > 1) { g.C = ws; g.epi = EPI_PARTIAL_F32; } else { g.C = C; g.epi = final_epi; }
  int rc;
  if (!ta && !tb) rc = launch_layout<false, false>(g, p, stream);
  else if (!ta && tb) rc = launch_layout<false, true>(g, p, stream);
  else if (ta && !tb) rc = launch_layout<true, false>(g, p, stream);
  else DH_FAIL(DH_ERR_UNSUPPORTED, "gemm (bf16): trans_a with trans_b is not used by the layer and not built");
  if (rc != DH_OK) return rc;
  if (p.splits > 1) {
    size_t mn = (size_t)M * N;  // multiple of 8 because N is
    splitk_reduce_kernel<<<(unsigned)((mn / 4 + 255) / 256), 256, 0, stream>>>((const float*)ws, p.splits, mn, C, final_epi);
    DH_LAUNCH_CHECK();
  }
  return DH_OK;
}
