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
                                                       const float* __restrict__ B, float* __restrict__ C, int accumulate,
                                                       const float* __restrict__ bias, const int32_t* __restrict__ group_rows,
                                                       int group_mode) {
  __shared__ float As[F32_BK][F32_BM + 4];
  __shared__ float Bs[F32_BK][F32_BN + 4];
  if (group_rows != nullptr) {  // grouped: blockIdx.z = group, its rows follow those of the groups before it
    int row0 = 0;
    for (int i = 0; i < (int)blockIdx.z; i++) row0 += group_rows[i];
    const int rows = group_rows[blockIdx.z];
    if (group_mode == 2) {  // weight gradient: the group's rows are the K range
      A += (size_t)row0 * M; B += (size_t)row0 * N; C += (size_t)blockIdx.z * M * N; K = rows;
    } else {
      A += (size_t)row0 * K; B += (size_t)blockIdx.z * K * N; C += (size_t)row0 * N; M = rows;
    }
    if (rows == 0 || (int)blockIdx.y * F32_BM >= M) return;
  }
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
      const float v = bias ? acc[i][j] + bias[gn] : acc[i][j];
      C[o] = accumulate ? C[o] + v : v;
    }
  }
}

int dh_launch_gemm_f32(bool ta, bool tb, int M, int N, int K, const float* A, const float* B, float* C,
                       bool accumulate, const float* bias, hipStream_t stream) {
  if (M == 0 || N == 0) return DH_OK;
  dim3 grid((N + F32_BN - 1) / F32_BN, (M + F32_BM - 1) / F32_BM), block(256);
  if (!ta && !tb) gemm_f32_kernel<false, false><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate, bias, nullptr, 0);
  else if (!ta && tb) gemm_f32_kernel<false, true><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate, bias, nullptr, 0);
  else if (ta && !tb) gemm_f32_kernel<true, false><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate, bias, nullptr, 0);
  else gemm_f32_kernel<true, true><<<grid, block, 0, stream>>>(M, N, K, A, B, C, accumulate, bias, nullptr, 0);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

// Grouped form: see dh_launch_gemm_grouped_bf16.  max_rows bounds every group's row count (grid size).
int dh_launch_gemm_grouped_f32(int mode, int n_groups, const int32_t* group_rows, int max_rows, int dim_a, int dim_b,
                               const float* A, const float* B, float* C, hipStream_t stream) {
  if (max_rows == 0) return DH_OK;
  if (mode == 0) {
    dim3 grid((dim_b + F32_BN - 1) / F32_BN, (max_rows + F32_BM - 1) / F32_BM, n_groups);
    gemm_f32_kernel<false, false><<<grid, 256, 0, stream>>>(max_rows, dim_b, dim_a, A, B, C, 0, nullptr, group_rows, 0);
  } else if (mode == 1) {
    dim3 grid((dim_b + F32_BN - 1) / F32_BN, (max_rows + F32_BM - 1) / F32_BM, n_groups);
    gemm_f32_kernel<false, true><<<grid, 256, 0, stream>>>(max_rows, dim_b, dim_a, A, B, C, 0, nullptr, group_rows, 1);
  } else {
    dim3 grid((dim_b + F32_BN - 1) / F32_BN, (dim_a + F32_BM - 1) / F32_BM, n_groups);
    gemm_f32_kernel<true, false><<<grid, 256, 0, stream>>>(dim_a, dim_b, max_rows, A, B, C, 1, nullptr, group_rows, 2);
  }
  DH_LAUNCH_CHECK();
  return DH_OK;
}
