// float32 causal grouped-query attention, forward and backward, for the fp32 configuration.
// Straightforward wave-per-row kernels (no matrix cores): a 64-lane wave owns one query row (or,
// for dK/dV, one key row), walks the other side 64 rows at a time with one row per lane for the
// dot products, and keeps head_dim/64 output columns per lane.  All sums run in a fixed order.
// Layout: qkv[T, (nq+2nkv)*d] = [q heads | k heads | v heads], o[T, nq*d], lse[nq, T],
// delta[nq, T]; tokens are sequence-major and attention never crosses a sequence boundary.
// Keys and values come from kv[batch*(q_off+seq), ldkv] = [k heads | v heads] per row: the packed qkv rows
// themselves for plain attention (q_off = 0), or a gathered buffer whose first q_off rows per sequence belong to
// earlier context-parallel ranks; query i of a sequence sits at position q_off + i.  dK/dV go to dkv likewise.
#include "common.h"

#define AF_MAXC 4  // head_dim <= 256

__device__ __forceinline__ float dot_row(const float* __restrict__ a_lds, const float* __restrict__ b, int d) {
  float s = 0.f;
  for (int c = 0; c < d; c += 4) {
    float4 v = *reinterpret_cast<const float4*>(b + c);
    s = fmaf(a_lds[c], v.x, s);
    s = fmaf(a_lds[c + 1], v.y, s);
    s = fmaf(a_lds[c + 2], v.z, s);
    s = fmaf(a_lds[c + 3], v.w, s);
  }
  return s;
}

__global__ __launch_bounds__(64) void attn_fwd_f32_kernel(int seq, int nq, int nkv, int d, const float* __restrict__ qkv,
                                                          const float* __restrict__ kv, int ldkv, int q_off,
                                                          float* __restrict__ o, float* __restrict__ lse, int T) {
  __shared__ float qs[256];
  const int lane = threadIdx.x;
  const int row = blockIdx.x, h = blockIdx.y;
  const int hk = h / (nq / nkv);
  const int ld = (nq + 2 * nkv) * d;
  const int last = q_off + row % seq;  // position of this query = last key it sees
  const float scale = 1.0f / sqrtf((float)d);
  for (int c = lane; c < d; c += 64) qs[c] = qkv[(size_t)row * ld + h * d + c] * scale;
  __syncthreads();
  const float* kbase = kv + (size_t)(row / seq) * (q_off + seq) * ldkv + (size_t)hk * d;  // key row 0 of this sequence
  const float* vbase = kbase + (size_t)nkv * d;
  float m = -INFINITY, l = 0.f, acc[AF_MAXC] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 <= last; j0 += 64) {
    int j = j0 + lane;
    float s = (j <= last) ? dot_row(qs, kbase + (size_t)j * ldkv, d) : -INFINITY;
    float mn = fmaxf(m, wave_max(s));
    float p = (j <= last) ? expf(s - mn) : 0.f;
    float alpha = expf(m - mn);
    l = l * alpha + wave_sum(p);
    m = mn;
#pragma unroll
    for (int c = 0; c < AF_MAXC; c++) acc[c] *= alpha;
    int cnt = min(64, last - j0 + 1);
    for (int jj = 0; jj < cnt; jj++) {
      float pj = __shfl(p, jj, 64);
      const float* vr = vbase + (size_t)(j0 + jj) * ldkv;
#pragma unroll
      for (int c = 0; c < AF_MAXC; c++)
        if (lane + 64 * c < d) acc[c] = fmaf(pj, vr[lane + 64 * c], acc[c]);
    }
  }
#pragma unroll
  for (int c = 0; c < AF_MAXC; c++)
    if (lane + 64 * c < d) o[(size_t)row * nq * d + h * d + lane + 64 * c] = acc[c] / l;
  if (lane == 0) lse[(size_t)h * T + row] = m + logf(l);
}

// delta[h, t] = sum_c dout[t,h,c] * o[t,h,c]
template <typename T>
__global__ __launch_bounds__(64) void attn_delta_kernel(int nq, int d, const T* __restrict__ o, const T* __restrict__ dout,
                                                        float* __restrict__ delta, int Ttok) {
  const int row = blockIdx.x, h = blockIdx.y;
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += 64) {
    size_t i = (size_t)row * nq * d + h * d + c;
    s += to_f32(o[i]) * to_f32(dout[i]);
  }
  s = wave_sum(s);
  if (threadIdx.x == 0) delta[(size_t)h * Ttok + row] = s;
}

__global__ __launch_bounds__(64) void attn_bwd_dq_f32_kernel(int seq, int nq, int nkv, int d, const float* __restrict__ qkv,
                                                             const float* __restrict__ kv, int ldkv, int q_off,
                                                             const float* __restrict__ dout, const float* __restrict__ lse,
                                                             const float* __restrict__ delta, float* __restrict__ dqkv, int T) {
  __shared__ float qs[256], dos[256];
  const int lane = threadIdx.x;
  const int row = blockIdx.x, h = blockIdx.y;
  const int hk = h / (nq / nkv);
  const int ld = (nq + 2 * nkv) * d;
  const int last = q_off + row % seq;
  const float scale = 1.0f / sqrtf((float)d);
  for (int c = lane; c < d; c += 64) {
    qs[c] = qkv[(size_t)row * ld + h * d + c] * scale;
    dos[c] = dout[(size_t)row * nq * d + h * d + c];
  }
  __syncthreads();
  const float* kbase = kv + (size_t)(row / seq) * (q_off + seq) * ldkv + (size_t)hk * d;
  const float* vbase = kbase + (size_t)nkv * d;
  const float L = lse[(size_t)h * T + row], D = delta[(size_t)h * T + row];
  float acc[AF_MAXC] = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = 0; j0 <= last; j0 += 64) {
    int j = j0 + lane;
    float ds = 0.f;
    if (j <= last) {
      float p = expf(dot_row(qs, kbase + (size_t)j * ldkv, d) - L);
      ds = p * (dot_row(dos, vbase + (size_t)j * ldkv, d) - D);
    }
    int cnt = min(64, last - j0 + 1);
    for (int jj = 0; jj < cnt; jj++) {
      float dj = __shfl(ds, jj, 64);
      const float* kr = kbase + (size_t)(j0 + jj) * ldkv;
#pragma unroll
      for (int c = 0; c < AF_MAXC; c++)
        if (lane + 64 * c < d) acc[c] = fmaf(dj, kr[lane + 64 * c], acc[c]);
    }
  }
#pragma unroll
  for (int c = 0; c < AF_MAXC; c++)
    if (lane + 64 * c < d) dqkv[(size_t)row * ld + h * d + lane + 64 * c] = acc[c] * scale;
}

__global__ __launch_bounds__(64) void attn_bwd_dkv_f32_kernel(int seq, int nq, int nkv, int d, const float* __restrict__ qkv,
                                                              const float* __restrict__ kv, int ldkv, int q_off,
                                                              const float* __restrict__ dout, const float* __restrict__ lse,
                                                              const float* __restrict__ delta, float* __restrict__ dkv, int lddkv, int T) {
  __shared__ float ks[256], vs[256];
  const int lane = threadIdx.x;
  const int row = blockIdx.x, hk = blockIdx.y;  // key row (of the batch*(q_off+seq) key rows), kv head
  const int g = nq / nkv;
  const int ld = (nq + 2 * nkv) * d;
  const int S = q_off + seq, b = row / S, pos = row % S;
  const int first = b * seq + max(pos - q_off, 0);  // first query token that sees this key
  const int send = (b + 1) * seq;                  // one past the last query token of this sequence
  const float scale = 1.0f / sqrtf((float)d);
  for (int c = lane; c < d; c += 64) {
    ks[c] = kv[(size_t)row * ldkv + hk * d + c] * scale;
    vs[c] = kv[(size_t)row * ldkv + (nkv + hk) * d + c];
  }
  __syncthreads();
  float dk[AF_MAXC] = {0.f, 0.f, 0.f, 0.f}, dv[AF_MAXC] = {0.f, 0.f, 0.f, 0.f};
  for (int h = hk * g; h < (hk + 1) * g; h++) {
    for (int i0 = first; i0 < send; i0 += 64) {
      int i = i0 + lane;
      float p = 0.f, ds = 0.f;
      if (i < send) {
        p = expf(dot_row(ks, qkv + (size_t)i * ld + h * d, d) - lse[(size_t)h * T + i]);
        ds = p * (dot_row(vs, dout + (size_t)i * nq * d + h * d, d) - delta[(size_t)h * T + i]);
      }
      int cnt = min(64, send - i0);
      for (int ii = 0; ii < cnt; ii++) {
        float pi = __shfl(p, ii, 64), di = __shfl(ds, ii, 64);
        const float* qr = qkv + (size_t)(i0 + ii) * ld + h * d;
        const float* dor = dout + (size_t)(i0 + ii) * nq * d + h * d;
#pragma unroll
        for (int c = 0; c < AF_MAXC; c++)
          if (lane + 64 * c < d) {
            dv[c] = fmaf(pi, dor[lane + 64 * c], dv[c]);
            dk[c] = fmaf(di, qr[lane + 64 * c], dk[c]);
          }
      }
    }
  }
#pragma unroll
  for (int c = 0; c < AF_MAXC; c++)
    if (lane + 64 * c < d) {
      dkv[(size_t)row * lddkv + hk * d + lane + 64 * c] = dk[c] * scale;
      dkv[(size_t)row * lddkv + (nkv + hk) * d + lane + 64 * c] = dv[c];
    }
}

int dh_launch_attn_fwd_f32(int batch, int seq, int nq, int nkv, int d, const float* qkv, const float* kv, int ldkv,
                           int q_off, float* o, float* lse, hipStream_t stream) {
  int T = batch * seq;
  if (d > 256 || d % 4) DH_FAIL(DH_ERR_SHAPE, "attention (fp32): head_dim %d must be a multiple of 4, at most 256", d);
  if (T == 0) return DH_OK;
  if (!kv) { kv = qkv + (size_t)nq * d; ldkv = (nq + 2 * nkv) * d; q_off = 0; }
  attn_fwd_f32_kernel<<<dim3(T, nq), 64, 0, stream>>>(seq, nq, nkv, d, qkv, kv, ldkv, q_off, o, lse, T);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

int dh_launch_attn_bwd_f32(int batch, int seq, int nq, int nkv, int d, const float* qkv, const float* kv, int ldkv,
                           int q_off, const float* o, const float* dout, const float* lse, float* dqkv, float* dkv, int lddkv,
                           float* delta, hipStream_t stream) {
  int T = batch * seq;
  if (d > 256 || d % 4) DH_FAIL(DH_ERR_SHAPE, "attention (fp32): head_dim %d must be a multiple of 4, at most 256", d);
  if (T == 0) return DH_OK;
  if (!kv) {
    kv = qkv + (size_t)nq * d; dkv = dqkv + (size_t)nq * d;
    ldkv = lddkv = (nq + 2 * nkv) * d; q_off = 0;
  }
  attn_delta_kernel<float><<<dim3(T, nq), 64, 0, stream>>>(nq, d, o, dout, delta, T);
  DH_LAUNCH_CHECK();
  attn_bwd_dq_f32_kernel<<<dim3(T, nq), 64, 0, stream>>>(seq, nq, nkv, d, qkv, kv, ldkv, q_off, dout, lse, delta, dqkv, T);
  DH_LAUNCH_CHECK();
  attn_bwd_dkv_f32_kernel<<<dim3(batch * (q_off + seq), nkv), 64, 0, stream>>>(seq, nq, nkv, d, qkv, kv, ldkv, q_off, dout, lse, delta,
                                                                               dkv, lddkv, T);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

// Shared with the bf16 path (defined here once).
int dh_launch_attn_delta_bf16(int T, int nq, int d, const bf16_t* o, const bf16_t* dout, float* delta, hipStream_t stream) {
  attn_delta_kernel<bf16_t><<<dim3(T, nq), 64, 0, stream>>>(nq, d, o, dout, delta, T);
  DH_LAUNCH_CHECK();
  return DH_OK;
}
