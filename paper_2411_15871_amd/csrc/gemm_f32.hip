// float32 GEMM for the fp32 configuration: C[M,N] (+)= opA(A) * opB(B) with plain FMA arithmetic.
// 64x64 output tile per 256-thread block, 4x4 outputs per thread, K consumed 16 at a time through
// LDS.  The sum over K runs in index order in one accumulator per output, so results do not depend
// on scheduling.  Any M, N, K >= 0 is accepted (edges are predicated).
#include "common.h"

#define F32_BM 64
#define F32_BN 64
#define F32_BK 16

template <bool TA, bool TB>
__global__ __launch_bounds__(256) void gemm_f32_kernel(int M, int N, int K, const float* __restrict__ A,
                                                       const float* __restrict__ B, float* __restrict__ C, int accumulate) {
  __shared__ float As[F32_BK][F32_BM + 4];
  __shared__ float Bs[F32_BK][F32_BN + 4];
  const int tid = threadIdx.x;
  const int tx = tid % 16, ty = tid / 16;
  const int m0 = blockIdx.y * F32_BM, n0 = blockIdx.x * F32_BN;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += F32_BK) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      int idx = tid + i * 256;
      int m, k;
      if (TA) { k = idx / F32_BM; m = idx % F32_BM; } else { m = idx / F32_BK; k = idx % F32_BK; }
      int gm = m0 + m, gk = k0 + k;
      float v = 0.f;
      if (gm < M && gk < K) v = TA ? A[(size_t)gk * M + gm] : A[(size_t)gm * K + gk];
      As[k][m] = v;
      int n;
      if (TB) { n = idx / F32_BK; k = idx % F32_BK; } else { k = idx / F32_BN; n = idx % F32_BN; }
      int gn = n0 + n;
      gk = k0 + k;
      v = 0.f;
      if (gn < N && gk < K) v = TB ? B[(size_t)gn * K + gk] : B[(size_t)gk * N + gn];
      Bs[k][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < F32_BK; k++) {
      float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
      float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
      float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; i++) {
    int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      size_t o = (size_t)gm * N + gn;
      C[o] = accumulate ? C[o] + acc[i][j] : acc[i][j];
    }
  }
}

int dh_launch_gemm_f32(bool ta, bool tb, int M, int N, int K, const float* A, const float* B, float* C,
                       bool accumulate, hipStream_t stream) {
  if (M == 0 || N == 0) return DH_OK;
  dim3 grid((N + F32_BN - 1) / F32_BN, (M + F32_BM - 1) / F32_BM), block(256);
  if (!ta && !tb) gemm_f32_kernel<false, false><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate);
  else if (!ta && tb) gemm_f32_kernel<false, true><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate);
  else if (ta && !tb) gemm_f32_kernel<true, false><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate);
  else gemm_f32_kernel<true, true><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate);
  DH_LAUNCH_CHECK();
  return DH_OK;
}
