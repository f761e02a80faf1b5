// Row-wise and element-wise operators of the layer: RMSNorm (with the residual add of the
// bias-dropout-add operator fused in, dropout p = 0), RoPE, SwiGLU, residual add.
// All are HBM-bound: every tensor is read or written exactly once with 16-byte (bf16) or
// 2x16-byte (fp32) accesses per thread; reductions are wave/block reductions in registers.
#include "common.h"

#define ROW_THREADS 256

// ------------------------------------------------------------------------------------ RMSNorm fwd
// One 256-thread block per row.  Thread t owns columns (t + 256*c)*8 .. +7 for c < NCH and keeps
// them in registers between the sum-of-squares pass and the scale pass.
template <typename T, int NCH>
__global__ __launch_bounds__(ROW_THREADS) void rmsnorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                                  const T* __restrict__ gamma, float eps,
                                                                  T* __restrict__ x_out, T* __restrict__ h,
                                                                  float* __restrict__ rstd, int H) {
  __shared__ float red[8];
  const size_t row = blockIdx.x;
  const T* xr = x + row * H;
  Vec8<T> v[NCH];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) {
      v[c].load(xr + col);
      if (res != nullptr) {
        Vec8<T> r;
        r.load(res + row * H + col);
#pragma unroll
        for (int i = 0; i < 8; i++) v[c].v[i] = to_f32(from_f32<T>(v[c].v[i] + r.v[i]));
        v[c].store(x_out + row * H + col);
      }
#pragma unroll
      for (int i = 0; i < 8; i++) ss += v[c].v[i] * v[c].v[i];
    }
  }
  ss = block256_sum(ss, red);
  float r = 1.0f / sqrtf(ss / (float)H + eps);
  if (threadIdx.x == 0) rstd[row] = r;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) {
      Vec8<T> g;
      g.load(gamma + col);
#pragma unroll
      for (int i = 0; i < 8; i++) g.v[i] = g.v[i] * v[c].v[i] * r;
      g.store(h + row * H + col);
    }
  }
}

// ------------------------------------------------------------------------------------ RMSNorm bwd
// Block b handles rows [b*RPB, (b+1)*RPB).  dx = rstd*(gh - xh*mean(gh*xh)) (+ dres), gh = gamma*dy,
// xh = x*rstd.  The next row is already in flight while the current one is reduced.  The gain
// gradient sum_t dy*xh is accumulated per thread over the block's rows and written as one partial
// row per block; two small kernels then add the partial rows in a fixed order (first groups of
// COLSUM_GROUP consecutive rows, then the groups), so the result does not depend on scheduling.
#define NORM_BWD_RPB 8
#define COLSUM_GROUP 32
template <typename T, int NCH>
__global__ __launch_bounds__(ROW_THREADS) void rmsnorm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                  const T* __restrict__ gamma,
                                                                  const float* __restrict__ rstd,
                                                                  const T* __restrict__ dres, T* __restrict__ dx,
                                                                  float* __restrict__ dg_partial, int rows, int H) {
  __shared__ float red[8];
  Vec8<T> g[NCH];
  float dg[NCH][8];
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) g[c].load(gamma + col);
#pragma unroll
    for (int i = 0; i < 8; i++) dg[c][i] = 0.f;
  }
  const size_t row0 = (size_t)blockIdx.x * NORM_BWD_RPB;
  const int nrows = min(NORM_BWD_RPB, rows - (int)row0);
  Vec8<T> ndy[NCH], nx[NCH], nres[NCH];
  auto fetch = [&](size_t row) {
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (threadIdx.x + ROW_THREADS * c) * 8;
      if (col < H) {
        ndy[c].load(dy + row * H + col);
        nx[c].load(x + row * H + col);
        if (dres != nullptr) nres[c].load(dres + row * H + col);
      }
    }
  };
  fetch(row0);
  for (int rr = 0; rr < nrows; rr++) {
    const size_t row = row0 + rr;
    const float r = rstd[row];
    Vec8<T> gh[NCH], xh[NCH], rs[NCH];
#pragma unroll
    for (int c = 0; c < NCH; c++) { gh[c] = ndy[c]; xh[c] = nx[c]; rs[c] = nres[c]; }
    if (rr + 1 < nrows) fetch(row + 1);
    float dot = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (threadIdx.x + ROW_THREADS * c) * 8;
      if (col < H) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
          xh[c].v[i] *= r;
          dg[c][i] += gh[c].v[i] * xh[c].v[i];
          gh[c].v[i] *= g[c].v[i];
          dot += gh[c].v[i] * xh[c].v[i];
        }
      }
    }
    dot = block256_sum(dot, red) / (float)H;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (threadIdx.x + ROW_THREADS * c) * 8;
      if (col < H) {
        Vec8<T> o;
#pragma unroll
        for (int i = 0; i < 8; i++) o.v[i] = r * (gh[c].v[i] - xh[c].v[i] * dot);
        if (dres != nullptr) {
#pragma unroll
          for (int i = 0; i < 8; i++) o.v[i] += rs[c].v[i];
        }
        o.store(dx + row * H + col);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) {
      float4* p = reinterpret_cast<float4*>(dg_partial + (size_t)blockIdx.x * H + col);
      p[0] = make_float4(dg[c][0], dg[c][1], dg[c][2], dg[c][3]);
      p[1] = make_float4(dg[c][4], dg[c][5], dg[c][6], dg[c][7]);
    }
  }
}

// out[grp][col] = sum of partial rows grp*COLSUM_GROUP .. +COLSUM_GROUP-1 (ascending), one thread per column.
__global__ void colsum_group_kernel(const float* __restrict__ partial, float* __restrict__ out, int nrows, int H) {
  int col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= H) return;
  int r0 = blockIdx.y * COLSUM_GROUP, r1 = min(nrows, r0 + COLSUM_GROUP);
  float v[COLSUM_GROUP];
#pragma unroll
  for (int i = 0; i < COLSUM_GROUP; i++) v[i] = r0 + i < r1 ? partial[(size_t)(r0 + i) * H + col] : 0.f;
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < COLSUM_GROUP; i++) s += v[i];
  out[(size_t)blockIdx.y * H + col] = s;
}

// dst[col] += sum_b partial[b][col], b ascending.
__global__ void colsum_accumulate_kernel(const float* __restrict__ partial, float* __restrict__ dst, int nblk, int H) {
  int col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= H) return;
  float s = 0.f;
  for (int b = 0; b < nblk; b++) s += partial[(size_t)b * H + col];
  dst[col] += s;
}

// ------------------------------------------------------------------------------------ RoPE
// In place on heads stored side by side in a row of `row_stride` elements.  A thread rotates 8
// pairs (i, i + d/2).  Angles are formed in double so that position*theta keeps full fp32 accuracy
// at long sequences.
template <typename T>
__global__ void rope_kernel(T* __restrict__ t, int rows, int seq, int n_heads, int d, int row_stride, double log2_base,
                            int inverse) {
  int half = d / 2;
  int chunks = half / 8;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)rows * n_heads * chunks;
  if (idx >= total) return;
  int c = (int)(idx % chunks);
  int head = (int)((idx / chunks) % n_heads);
  size_t row = idx / ((size_t)chunks * n_heads);
  int pos = (int)(row % seq);
  T* pa = t + row * row_stride + (size_t)head * d + c * 8;
  T* pb = pa + half;
  Vec8<T> a, b, oa, ob;
  a.load(pa);
  b.load(pb);
#pragma unroll
  for (int i = 0; i < 8; i++) {
    double theta = exp2(-2.0 * (double)(c * 8 + i) / (double)d * log2_base);
    double sn, cs;
    sincos((double)pos * theta, &sn, &cs);
    float s = inverse ? -(float)sn : (float)sn, co = (float)cs;
    oa.v[i] = a.v[i] * co - b.v[i] * s;
    ob.v[i] = a.v[i] * s + b.v[i] * co;
  }
  oa.store(pa);
  ob.store(pb);
}

// ------------------------------------------------------------------------------------ SwiGLU
template <typename T>
__global__ void swiglu_fwd_kernel(const T* __restrict__ gu, T* __restrict__ a, int rows, int F) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  int chunks = F / 8;
  if (idx >= (size_t)rows * chunks) return;
  size_t row = idx / chunks;
  int col = (int)(idx % chunks) * 8;
  Vec8<T> g, u, o;
  g.load(gu + row * 2 * F + col);
  u.load(gu + row * 2 * F + F + col);
#pragma unroll
  for (int i = 0; i < 8; i++) o.v[i] = g.v[i] / (1.0f + expf(-g.v[i])) * u.v[i];
  o.store(a + row * F + col);
}

template <typename T>
__global__ void swiglu_bwd_kernel(const T* __restrict__ gu, const T* __restrict__ da, T* __restrict__ dgu, int rows, int F) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  int chunks = F / 8;
  if (idx >= (size_t)rows * chunks) return;
  size_t row = idx / chunks;
  int col = (int)(idx % chunks) * 8;
  Vec8<T> g, u, d, og, ou;
  g.load(gu + row * 2 * F + col);
  u.load(gu + row * 2 * F + F + col);
  d.load(da + row * F + col);
#pragma unroll
  for (int i = 0; i < 8; i++) {
    float s = 1.0f / (1.0f + expf(-g.v[i]));
    og.v[i] = d.v[i] * u.v[i] * s * (1.0f + g.v[i] * (1.0f - s));
    ou.v[i] = d.v[i] * g.v[i] * s;
  }
  og.store(dgu + row * 2 * F + col);
  ou.store(dgu + row * 2 * F + F + col);
}

// ------------------------------------------------------------------------------------ residual add
template <typename T>
__global__ void add_kernel(const T* __restrict__ a, const T* __restrict__ b, T* __restrict__ out, size_t n8) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n8) return;
  Vec8<T> x, y;
  x.load(a + idx * 8);
  y.load(b + idx * 8);
#pragma unroll
  for (int i = 0; i < 8; i++) x.v[i] += y.v[i];
  x.store(out + idx * 8);
}

// ------------------------------------------------------------------------------------ host side
static int nch_for(int H) {
  int n = (H + ROW_THREADS * 8 - 1) / (ROW_THREADS * 8);
  return n <= 1 ? 1 : n <= 2 ? 2 : n <= 4 ? 4 : n <= 8 ? 8 : 0;
}

template <typename T>
static int rmsnorm_fwd_t(int rows, int H, const void* x, const void* res, const void* gamma, float eps, void* x_out,
                         void* h, float* rstd, hipStream_t s) {
  int nch = nch_for(H);
  dim3 g(rows), b(ROW_THREADS);
#define GO(N)                                                                                                         \
  rmsnorm_fwd_kernel<T, N><<<g, b, 0, s>>>((const T*)x, (const T*)res, (const T*)gamma, eps, (T*)x_out, (T*)h, rstd, H)
  switch (nch) {
    case 1: GO(1); break;
    case 2: GO(2); break;
    case 4: GO(4); break;
    case 8: GO(8); break;
    default: DH_FAIL(DH_ERR_SHAPE, "rmsnorm: hidden %d too large (max 16384)", H);
  }
#undef GO
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_rmsnorm_fwd(int dtype, int T, int H, const void* x, const void* residual, const void* gamma,
                              float eps, void* x_out, void* h, float* rstd, void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "rmsnorm_fwd: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (T == 0) return DH_OK;
  if (!x || !gamma || !h || !rstd || (residual && !x_out)) DH_FAIL(DH_ERR_INVALID_ARG, "rmsnorm_fwd: null pointer");
  return dtype == DH_BF16 ? rmsnorm_fwd_t<bf16_t>(T, H, x, residual, gamma, eps, x_out, h, rstd, (hipStream_t)stream)
                          : rmsnorm_fwd_t<float>(T, H, x, residual, gamma, eps, x_out, h, rstd, (hipStream_t)stream);
}

template <typename T>
static int rmsnorm_bwd_t(int rows, int H, const void* dy, const void* x, const void* gamma, const float* rstd,
                         const void* dres, void* dx, float* dgamma, float* partial, hipStream_t s) {
  int nch = nch_for(H);
  int nblk = (rows + NORM_BWD_RPB - 1) / NORM_BWD_RPB;
  dim3 g(nblk), b(ROW_THREADS);
#define GO(N)                                                                                                       \
  rmsnorm_bwd_kernel<T, N><<<g, b, 0, s>>>((const T*)dy, (const T*)x, (const T*)gamma, rstd, (const T*)dres, (T*)dx, \
                                           partial, rows, H)
  switch (nch) {
    case 1: GO(1); break;
    case 2: GO(2); break;
    case 4: GO(4); break;
    case 8: GO(8); break;
    default: DH_FAIL(DH_ERR_SHAPE, "rmsnorm: hidden %d too large (max 16384)", H);
  }
#undef GO
  DH_LAUNCH_CHECK();
  const int ngrp = (nblk + COLSUM_GROUP - 1) / COLSUM_GROUP;
  float* grouped = partial + (size_t)nblk * H;
  colsum_group_kernel<<<dim3((H + 255) / 256, ngrp), 256, 0, s>>>(partial, grouped, nblk, H);
  DH_LAUNCH_CHECK();
  colsum_accumulate_kernel<<<(H + 255) / 256, 256, 0, s>>>(grouped, dgamma, ngrp, H);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" size_t dh_rmsnorm_bwd_ws_bytes(int T, int H) {
  size_t nblk = (size_t)(T + NORM_BWD_RPB - 1) / NORM_BWD_RPB;
  size_t ngrp = (nblk + COLSUM_GROUP - 1) / COLSUM_GROUP;
  return (nblk + ngrp) * H * sizeof(float);
}

extern "C" int dh_rmsnorm_bwd(int dtype, int T, int H, const void* dy, const void* x, const void* gamma,
                              const float* rstd, const void* dres, void* dx, float* dgamma, void* ws, size_t ws_bytes,
                              void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "rmsnorm_bwd: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (T == 0) return DH_OK;
  if (!dy || !x || !gamma || !rstd || !dx || !dgamma) DH_FAIL(DH_ERR_INVALID_ARG, "rmsnorm_bwd: null pointer");
  if (!ws || ws_bytes < dh_rmsnorm_bwd_ws_bytes(T, H))
    DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "rmsnorm_bwd: workspace %zu < %zu bytes", ws_bytes, dh_rmsnorm_bwd_ws_bytes(T, H));
  return dtype == DH_BF16
             ? rmsnorm_bwd_t<bf16_t>(T, H, dy, x, gamma, rstd, dres, dx, dgamma, (float*)ws, (hipStream_t)stream)
             : rmsnorm_bwd_t<float>(T, H, dy, x, gamma, rstd, dres, dx, dgamma, (float*)ws, (hipStream_t)stream);
}

extern "C" int dh_rope(int dtype, int T, int seq, int n_heads, int head_dim, int row_stride, float base, int inverse,
                       void* t, void* stream) {
  if (T < 0 || seq <= 0 || n_heads <= 0 || head_dim <= 0 || head_dim % 16 || row_stride % 8 || row_stride < n_heads * head_dim)
    DH_FAIL(DH_ERR_SHAPE, "rope: T=%d seq=%d heads=%d d=%d stride=%d (d must be a multiple of 16)", T, seq, n_heads,
            head_dim, row_stride);
  if (T == 0) return DH_OK;
  if (!t) DH_FAIL(DH_ERR_INVALID_ARG, "rope: null pointer");
  size_t total = (size_t)T * n_heads * (head_dim / 16);
  dim3 g((unsigned)((total + 255) / 256)), b(256);
  double l2b = log2((double)base);
  if (dtype == DH_BF16)
    rope_kernel<bf16_t><<<g, b, 0, (hipStream_t)stream>>>((bf16_t*)t, T, seq, n_heads, head_dim, row_stride, l2b, inverse);
  else
    rope_kernel<float><<<g, b, 0, (hipStream_t)stream>>>((float*)t, T, seq, n_heads, head_dim, row_stride, l2b, inverse);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_swiglu_fwd(int dtype, int T, int F, const void* gu, void* a, void* stream) {
  if (T < 0 || F <= 0 || F % 8) DH_FAIL(DH_ERR_SHAPE, "swiglu_fwd: T=%d F=%d (F must be a positive multiple of 8)", T, F);
  if (T == 0) return DH_OK;
  if (!gu || !a) DH_FAIL(DH_ERR_INVALID_ARG, "swiglu_fwd: null pointer");
  size_t total = (size_t)T * (F / 8);
  dim3 g((unsigned)((total + 255) / 256)), b(256);
  if (dtype == DH_BF16)
    swiglu_fwd_kernel<bf16_t><<<g, b, 0, (hipStream_t)stream>>>((const bf16_t*)gu, (bf16_t*)a, T, F);
  else
    swiglu_fwd_kernel<float><<<g, b, 0, (hipStream_t)stream>>>((const float*)gu, (float*)a, T, F);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_swiglu_bwd(int dtype, int T, int F, const void* gu, const void* da, void* dgu, void* stream) {
  if (T < 0 || F <= 0 || F % 8) DH_FAIL(DH_ERR_SHAPE, "swiglu_bwd: T=%d F=%d (F must be a positive multiple of 8)", T, F);
  if (T == 0) return DH_OK;
  if (!gu || !da || !dgu) DH_FAIL(DH_ERR_INVALID_ARG, "swiglu_bwd: null pointer");
  size_t total = (size_t)T * (F / 8);
  dim3 g((unsigned)((total + 255) / 256)), b(256);
  if (dtype == DH_BF16)
    swiglu_bwd_kernel<bf16_t><<<g, b, 0, (hipStream_t)stream>>>((const bf16_t*)gu, (const bf16_t*)da, (bf16_t*)dgu, T, F);
  else
    swiglu_bwd_kernel<float><<<g, b, 0, (hipStream_t)stream>>>((const float*)gu, (const float*)da, (float*)dgu, T, F);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_add(int dtype, size_t n, const void* a, const void* b, void* out, void* stream) {
  if (n % 8) DH_FAIL(DH_ERR_SHAPE, "add: element count %zu must be a multiple of 8", n);
  if (!a || !b || !out) DH_FAIL(DH_ERR_INVALID_ARG, "add: null pointer");
  if (n == 0) return DH_OK;
  size_t n8 = n / 8;
  dim3 g((unsigned)((n8 + 255) / 256)), bl(256);
  if (dtype == DH_BF16)
    add_kernel<bf16_t><<<g, bl, 0, (hipStream_t)stream>>>((const bf16_t*)a, (const bf16_t*)b, (bf16_t*)out, n8);
  else
    add_kernel<float><<<g, bl, 0, (hipStream_t)stream>>>((const float*)a, (const float*)b, (float*)out, n8);
  DH_LAUNCH_CHECK();
  return DH_OK;
}
