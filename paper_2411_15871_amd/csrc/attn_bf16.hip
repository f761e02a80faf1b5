// bf16 causal grouped-query flash attention on the matrix cores, forward and backward.
// Layout: qkv[T, (nq+2nkv)*D] = [q heads | k heads | v heads] (q, k already rotated), o[T, nq*D],
// lse[nq, T] (natural log), delta[nq, T] = rowsum(dO * O).  Tokens are sequence-major; a block
// never crosses a sequence boundary.  D = head_dim is 64 or 128.
//
// All three kernels compute score tiles "transposed" where that keeps per-query statistics
// lane-local: v_mfma_f32_32x32x16_bf16 leaves column j of its result in lane j%32, so
//   forward / dQ : S^T = K Q^T        (column = query  -> running max/sum, lse, delta live in the lane)
//   dK/dV        : S   = Q K^T        (column = key    -> the dK^T, dV^T accumulators keep their column)
// and the probability tile can be fed back as the B operand of the next product straight from
// registers (the 8 k-slots of a lane are rows 8*(r/4)+4*(lane/32)+r%4 of two adjacent register
// quads).  The matching A operand (V^T, K^T, dO^T, Q^T: "k" is the token index, which is the slow
// dimension in memory) comes from LDS through the transposing load ds_read_b64_tr_b16.
// No atomics: dQ is produced per query block, dK/dV per key block, each summed in a fixed order.
#include "common.h"

#define AB_THREADS 256
#define AB_KT 64  // tokens per LDS tile

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// A 64-token tile is stored [token][D] without padding; the 16-byte chunk c of row r sits at chunk
// position c ^ swz(r).  With 256-byte rows (D = 128) this makes both access patterns conflict-free:
// the 16-byte reads of 16 consecutive rows at one chunk index (swz is a bijection on r%16) and the
// transposing reads of 4 consecutive rows x 64 bytes (r%4 lands in the upper two chunk bits).
template <int D>
struct ATile {
  static constexpr int LD = D;
  static constexpr int ELEMS = AB_KT * LD;  // one 64-token tile
  static constexpr int CHUNKS = AB_KT * D / 8 / AB_THREADS;
  static constexpr int CPR = D / 8;         // chunks per row
  __device__ static __forceinline__ int swz(int r) { return (((r & 3) << 2) | ((r >> 2) & 3)) & (CPR - 1); }
  // element offset of (row r, column c) for c a multiple of 4 (stays inside one chunk)
  __device__ static __forceinline__ int off(int r, int c) { return r * LD + ((((c >> 3) ^ swz(r)) << 3) | (c & 7)); }
};

// fetch a [64 tokens][D] tile (row stride ld elements) into registers; rows >= limit read as zero.
template <int D>
__device__ __forceinline__ void afetch(bf16x8 (&reg)[ATile<D>::CHUNKS], const bf16_t* __restrict__ base, int ld, int row0,
                                       int limit) {
#pragma unroll
  for (int i = 0; i < ATile<D>::CHUNKS; i++) {
    int id = threadIdx.x + i * AB_THREADS;
    int r = row0 + id / (D / 8), c = (id % (D / 8)) * 8;
    bf16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (r < limit) v = *reinterpret_cast<const bf16x8*>(base + (size_t)r * ld + c);
    reg[i] = v;
  }
}
template <int D>
__device__ __forceinline__ void astash(const bf16x8 (&reg)[ATile<D>::CHUNKS], bf16_t* lds) {
#pragma unroll
  for (int i = 0; i < ATile<D>::CHUNKS; i++) {
    int id = threadIdx.x + i * AB_THREADS;
    *reinterpret_cast<bf16x8*>(lds + ATile<D>::off(id / (D / 8), (id % (D / 8)) * 8)) = reg[i];
  }
}
// A/B fragment whose 8 k-values are contiguous in the tile row: row `r`, columns c0..c0+7.
template <int D>
__device__ __forceinline__ bf16x8 frag_direct(const bf16_t* tile, int r, int c0) {
  return *reinterpret_cast<const bf16x8*>(tile + ATile<D>::off(r, c0));
}
// Fragment whose k runs down the tile's rows: column c16+s (s = lane%16), rows ka..ka+3 and kb..kb+3.
template <int D>
__device__ __forceinline__ bf16x8 frag_tr(const bf16_t* tile, int ka, int kb, int c16, int s) {
  const bf16_t* p0 = tile + ATile<D>::off(ka + (s >> 2), c16 + ((s & 3) << 2));
  const bf16_t* p1 = tile + ATile<D>::off(kb + (s >> 2), c16 + ((s & 3) << 2));
  s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(__attribute__((address_space(3))) void*)p0);
  s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(__attribute__((address_space(3))) void*)p1);
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7));
}
// Registers 8c..8c+7 of a 32x32 result tile as a bf16 B fragment (k-slots = rows 16c+4g+{0..3}, 16c+8+4g+{0..3}).
__device__ __forceinline__ bf16x8 pack_rows(const f32x16& t, int c) {
  bf16x8 f;
#pragma unroll
  for (int i = 0; i < 8; i++) f[i] = (bf16_t)t[8 * c + i];
  return f;
}

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0)

// ================================================================================ forward
// grid (ceil(seq/128), nq, batch); wave w owns query rows i0 + 32w .. +31.
template <int D>
__global__ __launch_bounds__(AB_THREADS, 2) void attn_fwd_bf16_kernel(int seq, int nq, int nkv, const bf16_t* __restrict__ qkv,
                                                                   bf16_t* __restrict__ o, float* __restrict__ lse, int T,
                                                                   float scale_log2) {
  using TL = ATile<D>;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[TL::ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[TL::ELEMS];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, kg = lane >> 5, s16 = lane & 15, h16 = (lane >> 4) & 1;
  const int h = blockIdx.y, b = blockIdx.z, hk = h / (nq / nkv);
  const int ld = (nq + 2 * nkv) * D;
  const int i0 = blockIdx.x * 128, iw = i0 + wave * 32, iq = iw + l32;  // positions within the sequence
  const size_t tok0 = (size_t)b * seq;
  const bf16_t* kbase = qkv + tok0 * ld + (size_t)(nq + hk) * D;
  const bf16_t* vbase = qkv + tok0 * ld + (size_t)(nq + nkv + hk) * D;

  bf16x8 qf[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    qf[ks] = iq < seq ? *reinterpret_cast<const bf16x8*>(qkv + (tok0 + iq) * ld + (size_t)h * D + ks * 16 + kg * 8) : z;
  }
  f32x16 ot[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) ot[dt][r] = 0.f;
  float m = -INFINITY, l = 0.f;

  const int kend = min(seq, i0 + 128);  // keys needed by this block: [0, kend)
  bf16x8 rk[TL::CHUNKS], rv[TL::CHUNKS];
  afetch<D>(rk, kbase, ld, 0, seq);
  afetch<D>(rv, vbase, ld, 0, seq);
  astash<D>(rk, Ks);
  astash<D>(rv, Vs);
  __syncthreads();
  for (int kb = 0; kb < kend; kb += AB_KT) {
    const bool more = kb + AB_KT < kend;
    if (more) {
      afetch<D>(rk, kbase, ld, kb + AB_KT, seq);
      afetch<D>(rv, vbase, ld, kb + AB_KT, seq);
    }
    if (kb <= iw + 31) {  // some key of the tile is visible to some row of this wave
      f32x16 st[2];
#pragma unroll
      for (int mt = 0; mt < 2; mt++) {
#pragma unroll
        for (int r = 0; r < 16; r++) st[mt][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < D / 16; ks++) st[mt] = MFMA(frag_direct<D>(Ks, mt * 32 + l32, ks * 16 + kg * 8), qf[ks], st[mt]);
      }
      const bool diag = kb + AB_KT - 1 > iw;
      float mx = -INFINITY;
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float s = st[mt][r] * scale_log2;
          if (diag && kb + mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3) > iq) s = -INFINITY;
          st[mt][r] = s;
          mx = fmaxf(mx, s);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float mn = fmaxf(m, mx);
      const float alpha = exp2f(m - mn);
      float rs = 0.f;
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float p = exp2f(st[mt][r] - mn);
          st[mt][r] = p;
          rs += p;
        }
      rs += __shfl_xor(rs, 32, 64);
      l = l * alpha + rs;
      m = mn;
#pragma unroll
      for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) ot[dt][r] *= alpha;
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          bf16x8 pf = pack_rows(st[mt], c);
          const int ka = mt * 32 + 16 * c + 4 * kg;
#pragma unroll
          for (int dt = 0; dt < D / 32; dt++) ot[dt] = MFMA(frag_tr<D>(Vs, ka, ka + 8, dt * 32 + h16 * 16, s16), pf, ot[dt]);
        }
    }
    __syncthreads();
    if (more) {
      astash<D>(rk, Ks);
      astash<D>(rv, Vs);
    }
    __syncthreads();
  }
  if (iq < seq) {
    const float inv = 1.0f / l;
    bf16_t* orow = o + (tok0 + iq) * (size_t)nq * D + (size_t)h * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        bf16x4 v;
#pragma unroll
        for (int i = 0; i < 4; i++) v[i] = (bf16_t)(ot[dt][4 * q4 + i] * inv);
        *reinterpret_cast<bf16x4*>(orow + dt * 32 + 8 * q4 + 4 * kg) = v;
      }
    if (kg == 0) lse[(size_t)h * T + tok0 + iq] = (m + log2f(l)) * 0.6931471805599453f;
  }
}

// ================================================================================ backward: dQ
// Same tiling as the forward kernel.  dQ^T = sum over key tiles of K^T dS^T, dS^T = P^T (dP^T - delta),
// P^T = exp2(S^T*scale_log2 - lse*log2e), dP^T = V dO^T.
template <int D>
__global__ __launch_bounds__(AB_THREADS) void attn_bwd_dq_bf16_kernel(int seq, int nq, int nkv, const bf16_t* __restrict__ qkv,
                                                                      const bf16_t* __restrict__ dout,
                                                                      const float* __restrict__ lse,
                                                                      const float* __restrict__ delta,
                                                                      bf16_t* __restrict__ dqkv, int T, float scale,
                                                                      float scale_log2) {
  using TL = ATile<D>;
  __shared__ __attribute__((aligned(16))) bf16_t Ks[TL::ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t Vs[TL::ELEMS];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, kg = lane >> 5, s16 = lane & 15, h16 = (lane >> 4) & 1;
  const int h = blockIdx.y, b = blockIdx.z, hk = h / (nq / nkv);
  const int ld = (nq + 2 * nkv) * D;
  const int i0 = blockIdx.x * 128, iw = i0 + wave * 32, iq = iw + l32;
  const size_t tok0 = (size_t)b * seq;
  const bf16_t* kbase = qkv + tok0 * ld + (size_t)(nq + hk) * D;
  const bf16_t* vbase = qkv + tok0 * ld + (size_t)(nq + nkv + hk) * D;

  bf16x8 qf[D / 16], dof[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    qf[ks] = iq < seq ? *reinterpret_cast<const bf16x8*>(qkv + (tok0 + iq) * ld + (size_t)h * D + ks * 16 + kg * 8) : z;
    dof[ks] = iq < seq ? *reinterpret_cast<const bf16x8*>(dout + (tok0 + iq) * (size_t)nq * D + (size_t)h * D + ks * 16 + kg * 8) : z;
  }
  const float lse2 = iq < seq ? lse[(size_t)h * T + tok0 + iq] * 1.4426950408889634f : 0.f;
  const float dl = iq < seq ? delta[(size_t)h * T + tok0 + iq] : 0.f;
  f32x16 dqt[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) dqt[dt][r] = 0.f;

  const int kend = min(seq, i0 + 128);
  bf16x8 rk[TL::CHUNKS], rv[TL::CHUNKS];
  afetch<D>(rk, kbase, ld, 0, seq);
  afetch<D>(rv, vbase, ld, 0, seq);
  astash<D>(rk, Ks);
  astash<D>(rv, Vs);
  __syncthreads();
  for (int kb = 0; kb < kend; kb += AB_KT) {
    const bool more = kb + AB_KT < kend;
    if (more) {
      afetch<D>(rk, kbase, ld, kb + AB_KT, seq);
      afetch<D>(rv, vbase, ld, kb + AB_KT, seq);
    }
    if (kb <= iw + 31) {
      f32x16 st[2], dp[2];
#pragma unroll
      for (int mt = 0; mt < 2; mt++) {
#pragma unroll
        for (int r = 0; r < 16; r++) { st[mt][r] = 0.f; dp[mt][r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < D / 16; ks++) {
          st[mt] = MFMA(frag_direct<D>(Ks, mt * 32 + l32, ks * 16 + kg * 8), qf[ks], st[mt]);
          dp[mt] = MFMA(frag_direct<D>(Vs, mt * 32 + l32, ks * 16 + kg * 8), dof[ks], dp[mt]);
        }
      }
      const bool diag = kb + AB_KT - 1 > iw;
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float p = exp2f(st[mt][r] * scale_log2 - lse2);
          if (diag && kb + mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3) > iq) p = 0.f;
          st[mt][r] = p * (dp[mt][r] - dl);
        }
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          bf16x8 df = pack_rows(st[mt], c);
          const int ka = mt * 32 + 16 * c + 4 * kg;
#pragma unroll
          for (int dt = 0; dt < D / 32; dt++) dqt[dt] = MFMA(frag_tr<D>(Ks, ka, ka + 8, dt * 32 + h16 * 16, s16), df, dqt[dt]);
        }
    }
    __syncthreads();
    if (more) {
      astash<D>(rk, Ks);
      astash<D>(rv, Vs);
    }
    __syncthreads();
  }
  if (iq < seq) {
    bf16_t* row = dqkv + (tok0 + iq) * ld + (size_t)h * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        bf16x4 v;
#pragma unroll
        for (int i = 0; i < 4; i++) v[i] = (bf16_t)(dqt[dt][4 * q4 + i] * scale);
        *reinterpret_cast<bf16x4*>(row + dt * 32 + 8 * q4 + 4 * kg) = v;
      }
  }
}

// ================================================================================ backward: dK, dV
// grid (ceil(seq/128), nq, batch): one block per (key block, query head); wave w owns keys
// j0 + 32w .. +31 and keeps their K, V fragments and the dK^T, dV^T accumulators in registers while
// 64-query tiles of that head's Q and dO stream through LDS.  With grouped heads (nq > nkv) the
// block writes float32 partials part[query head][token][dK | dV] and attn_bwd_group_reduce_kernel
// adds the group's heads in index order; with nq == nkv it writes dK, dV directly.
template <int D>
__global__ __launch_bounds__(AB_THREADS) void attn_bwd_dkv_bf16_kernel(int seq, int nq, int nkv, const bf16_t* __restrict__ qkv,
                                                                       const bf16_t* __restrict__ dout,
                                                                       const float* __restrict__ lse,
                                                                       const float* __restrict__ delta,
                                                                       bf16_t* __restrict__ dqkv, float* __restrict__ part,
                                                                       int T, float scale, float scale_log2) {
  using TL = ATile<D>;
  __shared__ __attribute__((aligned(16))) bf16_t Qs[TL::ELEMS];
  __shared__ __attribute__((aligned(16))) bf16_t Os[TL::ELEMS];
  __shared__ float lse_s[AB_KT], del_s[AB_KT];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, kg = lane >> 5, s16 = lane & 15, h16 = (lane >> 4) & 1;
  const int hq = blockIdx.y, b = blockIdx.z, grp = nq / nkv, hk = hq / grp;
  const int ld = (nq + 2 * nkv) * D;
  const int j0 = blockIdx.x * 128, jw = j0 + wave * 32, jk = jw + l32;  // key positions within the sequence
  const size_t tok0 = (size_t)b * seq;

  bf16x8 kf[D / 16], vf[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++) {
    bf16x8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    kf[ks] = jk < seq ? *reinterpret_cast<const bf16x8*>(qkv + (tok0 + jk) * ld + (size_t)(nq + hk) * D + ks * 16 + kg * 8) : z;
    vf[ks] = jk < seq ? *reinterpret_cast<const bf16x8*>(qkv + (tok0 + jk) * ld + (size_t)(nq + nkv + hk) * D + ks * 16 + kg * 8) : z;
  }
  f32x16 dkt[D / 32], dvt[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
    for (int r = 0; r < 16; r++) { dkt[dt][r] = 0.f; dvt[dt][r] = 0.f; }

  const int qstart = j0 / AB_KT * AB_KT;
  const int total = (seq - qstart + AB_KT - 1) / AB_KT;  // query tiles
  bf16x8 rq[TL::CHUNKS], ro[TL::CHUNKS];
  float rl = 0.f, rd = 0.f;
  auto fetch = [&](int it) {
    int qb = qstart + it * AB_KT;
    afetch<D>(rq, qkv + tok0 * ld + (size_t)hq * D, ld, qb, seq);
    afetch<D>(ro, dout + tok0 * (size_t)nq * D + (size_t)hq * D, nq * D, qb, seq);
    if (threadIdx.x < AB_KT) {
      int qi = qb + threadIdx.x;
      rl = qi < seq ? lse[(size_t)hq * T + tok0 + qi] * 1.4426950408889634f : 0.f;
      rd = qi < seq ? delta[(size_t)hq * T + tok0 + qi] : 0.f;
    }
  };
  auto stash = [&]() {
    astash<D>(rq, Qs);
    astash<D>(ro, Os);
    if (threadIdx.x < AB_KT) { lse_s[threadIdx.x] = rl; del_s[threadIdx.x] = rd; }
  };
  if (total > 0) { fetch(0); stash(); }
  __syncthreads();
  for (int it = 0; it < total; it++) {
    const int qb = qstart + it * AB_KT;
    const bool more = it + 1 < total;
    if (more) fetch(it + 1);
    if (qb + AB_KT - 1 >= jw) {  // some query of the tile sees some key of this wave
      f32x16 st[2], dp[2];
#pragma unroll
      for (int mt = 0; mt < 2; mt++) {
#pragma unroll
        for (int r = 0; r < 16; r++) { st[mt][r] = 0.f; dp[mt][r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < D / 16; ks++) {
          st[mt] = MFMA(frag_direct<D>(Qs, mt * 32 + l32, ks * 16 + kg * 8), kf[ks], st[mt]);
          dp[mt] = MFMA(frag_direct<D>(Os, mt * 32 + l32, ks * 16 + kg * 8), vf[ks], dp[mt]);
        }
      }
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int qr = mt * 32 + 8 * (r >> 2) + 4 * kg + (r & 3);  // row within the tile
          const int qi = qb + qr;
          float p = exp2f(st[mt][r] * scale_log2 - lse_s[qr]);
          if (qi < jk || qi >= seq) p = 0.f;
          dp[mt][r] = p * (dp[mt][r] - del_s[qr]);
          st[mt][r] = p;
        }
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int c = 0; c < 2; c++) {
          bf16x8 pf = pack_rows(st[mt], c), df = pack_rows(dp[mt], c);
          const int ka = mt * 32 + 16 * c + 4 * kg;
#pragma unroll
          for (int dt = 0; dt < D / 32; dt++) {
            dvt[dt] = MFMA(frag_tr<D>(Os, ka, ka + 8, dt * 32 + h16 * 16, s16), pf, dvt[dt]);
            dkt[dt] = MFMA(frag_tr<D>(Qs, ka, ka + 8, dt * 32 + h16 * 16, s16), df, dkt[dt]);
          }
        }
    }
    __syncthreads();
    if (more) stash();
    __syncthreads();
  }
  if (jk < seq && part != nullptr) {
    float* prow = part + ((size_t)hq * T + tok0 + jk) * (2 * D);  // hq = hk*grp + head-in-group
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        f32x4 a, c;
#pragma unroll
        for (int i = 0; i < 4; i++) { a[i] = dkt[dt][4 * q4 + i] * scale; c[i] = dvt[dt][4 * q4 + i]; }
        *reinterpret_cast<f32x4*>(prow + dt * 32 + 8 * q4 + 4 * kg) = a;
        *reinterpret_cast<f32x4*>(prow + D + dt * 32 + 8 * q4 + 4 * kg) = c;
      }
  } else if (jk < seq) {
    bf16_t* krow = dqkv + (tok0 + jk) * ld + (size_t)(nq + hk) * D;
    bf16_t* vrow = dqkv + (tok0 + jk) * ld + (size_t)(nq + nkv + hk) * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; dt++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        bf16x4 a, c;
#pragma unroll
        for (int i = 0; i < 4; i++) {
          a[i] = (bf16_t)(dkt[dt][4 * q4 + i] * scale);
          c[i] = (bf16_t)dvt[dt][4 * q4 + i];
        }
        *reinterpret_cast<bf16x4*>(krow + dt * 32 + 8 * q4 + 4 * kg) = a;
        *reinterpret_cast<bf16x4*>(vrow + dt * 32 + 8 * q4 + 4 * kg) = c;
      }
  }
}

// dk,dv[token][kv head] = sum over the group's query heads (ascending) of the float32 partials
// part[query head][token][dK | dV].
template <int D>
__global__ void attn_bwd_group_reduce_kernel(const float* __restrict__ part, bf16_t* __restrict__ dqkv, int T, int nq,
                                             int nkv) {
  const int grp = nq / nkv, ld = (nq + 2 * nkv) * D;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // over T * nkv * (2D/4)
  const int per_tok = 2 * D / 4;
  if (idx >= (size_t)T * nkv * per_tok) return;
  int c4 = (int)(idx % per_tok) * 4;
  int hk = (int)((idx / per_tok) % nkv);
  size_t tok = idx / ((size_t)per_tok * nkv);
  f32x4 s = {0.f, 0.f, 0.f, 0.f};
  for (int g = 0; g < grp; g++) s += *reinterpret_cast<const f32x4*>(part + (((size_t)hk * grp + g) * T + tok) * (2 * D) + c4);
  bf16x4 o = {(bf16_t)s[0], (bf16_t)s[1], (bf16_t)s[2], (bf16_t)s[3]};
  bf16_t* dst = dqkv + tok * ld + (c4 < D ? (size_t)(nq + hk) * D + c4 : (size_t)(nq + nkv + hk) * D + (c4 - D));
  *reinterpret_cast<bf16x4*>(dst) = o;
}

// ------------------------------------------------------------------------------------ host side
int dh_launch_attn_delta_bf16(int T, int nq, int d, const bf16_t* o, const bf16_t* dout, float* delta, hipStream_t stream);

int dh_launch_attn_fwd_bf16(int batch, int seq, int nq, int nkv, int d, const bf16_t* qkv, bf16_t* o, float* lse,
                            hipStream_t stream) {
  if (d != 64 && d != 128) DH_FAIL(DH_ERR_SHAPE, "attention (bf16): head_dim %d must be 64 or 128", d);
  if (batch * seq == 0) return DH_OK;
  dim3 grid((seq + 127) / 128, nq, batch);
  float sl2 = (float)(1.4426950408889634 / sqrt((double)d));
  if (d == 128) attn_fwd_bf16_kernel<128><<<grid, AB_THREADS, 0, stream>>>(seq, nq, nkv, qkv, o, lse, batch * seq, sl2);
  else attn_fwd_bf16_kernel<64><<<grid, AB_THREADS, 0, stream>>>(seq, nq, nkv, qkv, o, lse, batch * seq, sl2);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

size_t dh_attn_bwd_bf16_ws_bytes(int batch, int seq, int nq, int nkv, int d) {
  return nq > nkv ? (size_t)nq * batch * seq * 2 * d * sizeof(float) : 0;
}

int dh_launch_attn_bwd_bf16(int batch, int seq, int nq, int nkv, int d, const bf16_t* qkv, const bf16_t* o,
                            const bf16_t* dout, const float* lse, bf16_t* dqkv, float* delta, void* ws, size_t ws_bytes,
                            hipStream_t stream) {
  if (d != 64 && d != 128) DH_FAIL(DH_ERR_SHAPE, "attention (bf16): head_dim %d must be 64 or 128", d);
  int T = batch * seq;
  if (T == 0) return DH_OK;
  size_t need = dh_attn_bwd_bf16_ws_bytes(batch, seq, nq, nkv, d);
  if (need > 0 && (!ws || ws_bytes < need)) DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "attn_bwd: workspace %zu < %zu bytes", ws_bytes, need);
  float* part = need > 0 ? (float*)ws : nullptr;
  int rc = dh_launch_attn_delta_bf16(T, nq, d, o, dout, delta, stream);
  if (rc != DH_OK) return rc;
  float sc = (float)(1.0 / sqrt((double)d)), sl2 = (float)(1.4426950408889634 / sqrt((double)d));
  dim3 gq((seq + 127) / 128, nq, batch), gk((seq + 127) / 128, nq, batch);
  const unsigned nred = (unsigned)(((size_t)T * nkv * (2 * d / 4) + 255) / 256);
  if (d == 128) {
    attn_bwd_dq_bf16_kernel<128><<<gq, AB_THREADS, 0, stream>>>(seq, nq, nkv, qkv, dout, lse, delta, dqkv, T, sc, sl2);
    DH_LAUNCH_CHECK();
    attn_bwd_dkv_bf16_kernel<128><<<gk, AB_THREADS, 0, stream>>>(seq, nq, nkv, qkv, dout, lse, delta, dqkv, part, T, sc, sl2);
    if (part) { DH_LAUNCH_CHECK(); attn_bwd_group_reduce_kernel<128><<<nred, 256, 0, stream>>>(part, dqkv, T, nq, nkv); }
  } else {
    attn_bwd_dq_bf16_kernel<64><<<gq, AB_THREADS, 0, stream>>>(seq, nq, nkv, qkv, dout, lse, delta, dqkv, T, sc, sl2);
    DH_LAUNCH_CHECK();
    attn_bwd_dkv_bf16_kernel<64><<<gk, AB_THREADS, 0, stream>>>(seq, nq, nkv, qkv, dout, lse, delta, dqkv, part, T, sc, sl2);
    if (part) { DH_LAUNCH_CHECK(); attn_bwd_group_reduce_kernel<64><<<nred, 256, 0, stream>>>(part, dqkv, T, nq, nkv); }
  }
  DH_LAUNCH_CHECK();
  return DH_OK;
}
