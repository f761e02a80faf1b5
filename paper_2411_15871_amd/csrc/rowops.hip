// Row-wise and element-wise operators of the layer: RMSNorm (with the residual add of the
// bias-dropout-add operator fused in, dropout p = 0), RoPE, SwiGLU, residual add.
// All are HBM-bound: every tensor is read or written exactly once with 16-byte (bf16) or
// 2x16-byte (fp32) accesses per thread; reductions are wave/block reductions in registers.
#include <mutex>
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
// row per block; colsum_finish_kernel then adds the partial rows in an order fixed by the shapes, so the result
// does not depend on scheduling.
// Rows a backward-norm block walks (its partial gain gradient is one row of the column-sum input): 8, fewer for
// short inputs so that a couple of hundred blocks exist.
__host__ __device__ static inline int norm_bwd_rpb(int rows) { return rows >= 4096 ? 8 : rows >= 1024 ? 4 : rows >= 512 ? 2 : 1; }
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
  const int rpb = norm_bwd_rpb(rows);
  const size_t row0 = (size_t)blockIdx.x * rpb;
  const int nrows = min(rpb, rows - (int)row0);
  Raw8<T> ndy[NCH], nx[NCH], nres[NCH];  // the next row, as fetched
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
    Vec8<T> gh[NCH], xh[NCH];
    Raw8<T> rs[NCH];
#pragma unroll
    for (int c = 0; c < NCH; c++) { gh[c].from(ndy[c]); xh[c].from(nx[c]); rs[c] = nres[c]; }
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
          for (int i = 0; i < 8; i++) o.v[i] += rs[c].get(i);
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

// dst[col] += sum over the nrows partial rows of partial[row][col], in an order fixed by the shapes alone: a block owns
// 32 columns, its 8 slices of threads each add a contiguous eighth of the rows in ascending order (16 loads in
// flight), and slice 0 adds the eight sums in slice order.  Columns [0, H0) go to dst0, columns [H0, ld) to dst1.
#define COLSUM_SLICES 8
__global__ __launch_bounds__(256) void colsum_finish_kernel(const float* __restrict__ partial, int nrows, int ld,
                                                            float* __restrict__ dst0, int H0, float* __restrict__ dst1) {
  __shared__ float part[COLSUM_SLICES][32];
  const int c = threadIdx.x & 31, slice = threadIdx.x >> 5, col = blockIdx.x * 32 + c;
  const int per = (nrows + COLSUM_SLICES - 1) / COLSUM_SLICES, r0 = slice * per, r1 = min(nrows, r0 + per);
  float s = 0.f;
  if (col < ld) {
    for (int b0 = r0; b0 < r1; b0 += 16) {
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; i++) v[i] = b0 + i < r1 ? partial[(size_t)(b0 + i) * ld + col] : 0.f;
#pragma unroll
      for (int i = 0; i < 16; i++) s += v[i];
    }
  }
  part[slice][c] = s;
  __syncthreads();
  if (slice == 0 && col < ld) {
    float t = part[0][c];
#pragma unroll
    for (int k = 1; k < COLSUM_SLICES; k++) t += part[k][c];
    if (col < H0) dst0[col] += t;
    else dst1[col - H0] += t;
  }
}

// ------------------------------------------------------------------------------------ RoPE
// In place on heads stored side by side in a row of `row_stride` elements.  A thread rotates 8
// pairs (i, i + d/2).  Angles are formed in double so that position*theta keeps full fp32 accuracy
// at long sequences: theta of the thread's first pair by one double exp2, the next seven by multiplying with
// ratio = base^(-2/d); the angle is reduced to [-pi, pi] in double, and only sine and cosine of the reduced
// angle are taken in float (absolute error ~1e-7).
// ADJACENT: pair i is elements (2i, 2i+1): the thread's 8 pairs are 16 consecutive elements.
template <typename T, bool ADJACENT>
__global__ void rope_kernel(T* __restrict__ t, int rows, int seq, int pos0, int n_heads, int d, int row_stride, double log2_base,
                            double ratio, int inverse) {
  int half = d / 2;
  int chunks = half / 8;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)rows * n_heads * chunks;
  if (idx >= total) return;
  int c = (int)(idx % chunks);
  int head = (int)((idx / chunks) % n_heads);
  size_t row = idx / ((size_t)chunks * n_heads);
  int pos = pos0 + (int)(row % seq);
  T* pa = t + row * row_stride + (size_t)head * d + (ADJACENT ? c * 16 : c * 8);
  T* pb = pa + (ADJACENT ? 8 : half);
  Vec8<T> a, b, oa, ob;
  a.load(pa);
  b.load(pb);
  if (ADJACENT) {  // de-interleave: a = first elements of the 8 pairs, b = second elements
    Vec8<T> lo = a, hi = b;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      a.v[i] = lo.v[2 * i]; b.v[i] = lo.v[2 * i + 1];
      a.v[4 + i] = hi.v[2 * i]; b.v[4 + i] = hi.v[2 * i + 1];
    }
  }
  double theta = exp2(-2.0 * (double)(c * 8) / (double)d * log2_base);
#pragma unroll
  for (int i = 0; i < 8; i++) {
    double ang = (double)pos * theta;
    ang -= 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
    theta *= ratio;
    float sn, co;
    sincosf((float)ang, &sn, &co);
    float s = inverse ? -sn : sn;
    oa.v[i] = a.v[i] * co - b.v[i] * s;
    ob.v[i] = a.v[i] * s + b.v[i] * co;
  }
  if (ADJACENT) {
    Vec8<T> lo, hi;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      lo.v[2 * i] = oa.v[i]; lo.v[2 * i + 1] = ob.v[i];
      hi.v[2 * i] = oa.v[4 + i]; hi.v[2 * i + 1] = ob.v[4 + i];
    }
    oa = lo; ob = hi;
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
  for (int i = 0; i < 8; i++) o.v[i] = swiglu_fwd_elem(g.v[i], u.v[i]);
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
  for (int i = 0; i < 8; i++) swiglu_bwd_elem(g.v[i], u.v[i], d.v[i], og.v[i], ou.v[i]);
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
  int nblk = (rows + norm_bwd_rpb(rows) - 1) / norm_bwd_rpb(rows);
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
  colsum_finish_kernel<<<(H + 31) / 32, 256, 0, s>>>(partial, nblk, H, dgamma, H, nullptr);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" size_t dh_rmsnorm_bwd_ws_bytes(int T, int H) {
  size_t nblk = (size_t)(T + norm_bwd_rpb(T) - 1) / norm_bwd_rpb(T);
  return nblk * H * sizeof(float);
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

// RMSNorm backward for callers that may not allocate (code under stream capture, serving loops): the per-block partial
// rows of the gain gradient live in a library-owned static device array instead of a caller workspace.  Every GPU holds
// its own copy of the array at its own address; the address is looked up once per device, with that device current.
#define DH_NORM_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) float dh_norm_scratch[DH_NORM_SCRATCH_BYTES / sizeof(float)];
static int norm_scratch_ptr(float** out) {
  static float* ptr[DH_MAX_DEVICES] = {};
  static std::mutex mu;
  int dev = 0;
  DH_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= DH_MAX_DEVICES) DH_FAIL(DH_ERR_UNSUPPORTED, "rmsnorm_bwd_noalloc: device index %d above %d", dev, DH_MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lock(mu);
  if (ptr[dev] == nullptr) {
    void* p = nullptr;
    DH_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(dh_norm_scratch)));
    if (p == nullptr) DH_FAIL(DH_ERR_HIP, "rmsnorm_bwd_noalloc: the scratch array has no device address");
    ptr[dev] = (float*)p;
  }
  *out = ptr[dev];
  return DH_OK;
}

extern "C" size_t dh_rmsnorm_bwd_noalloc_max_bytes(void) { return DH_NORM_SCRATCH_BYTES; }

extern "C" int dh_rmsnorm_bwd_noalloc(int dtype, int T, int H, const void* dy, const void* x, const void* gamma,
                                      const float* rstd, const void* dres, void* dx, float* dgamma, void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "rmsnorm_bwd_noalloc: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (dtype != DH_F32 && dtype != DH_BF16) DH_FAIL(DH_ERR_INVALID_ARG, "rmsnorm_bwd_noalloc: dtype %d", dtype);
  if (T == 0) return DH_OK;
  if (!dy || !x || !gamma || !rstd || !dx || !dgamma) DH_FAIL(DH_ERR_INVALID_ARG, "rmsnorm_bwd_noalloc: null pointer");
  const size_t need = dh_rmsnorm_bwd_ws_bytes(T, H);
  if (need > DH_NORM_SCRATCH_BYTES)
    DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "rmsnorm_bwd_noalloc: T=%d H=%d needs %zu bytes of scratch, the static array holds %u", T, H,
            need, DH_NORM_SCRATCH_BYTES);
  float* scratch = nullptr;
  int rc = norm_scratch_ptr(&scratch);
  if (rc) return rc;
  // every partial row the finishing kernel reads is written by this call's first kernel: nothing to clear
  return dtype == DH_BF16 ? rmsnorm_bwd_t<bf16_t>(T, H, dy, x, gamma, rstd, dres, dx, dgamma, scratch, (hipStream_t)stream)
                          : rmsnorm_bwd_t<float>(T, H, dy, x, gamma, rstd, dres, dx, dgamma, scratch, (hipStream_t)stream);
}

extern "C" int dh_rope(int dtype, int T, int seq, int n_heads, int head_dim, int row_stride, float base, int inverse,
                       void* t, void* stream) {
  return dh_rope_at(dtype, T, seq, 0, n_heads, head_dim, row_stride, base, inverse, t, stream);
}

extern "C" int dh_rope_at(int dtype, int T, int seq, int pos0, int n_heads, int head_dim, int row_stride, float base, int inverse,
                          void* t, void* stream) {
  return dh_rope_pairs(dtype, DH_ROPE_HALVES, T, seq, pos0, n_heads, head_dim, row_stride, base, inverse, t, stream);
}

extern "C" int dh_rope_pairs(int dtype, int pairing, int T, int seq, int pos0, int n_heads, int head_dim, int row_stride, float base,
                             int inverse, void* t, void* stream) {
  if (pairing != DH_ROPE_HALVES && pairing != DH_ROPE_ADJACENT) DH_FAIL(DH_ERR_INVALID_ARG, "rope: unknown pairing %d", pairing);
  if (T < 0 || seq <= 0 || pos0 < 0 || n_heads <= 0 || head_dim <= 0 || head_dim % 16 || row_stride % 8 || row_stride < n_heads * head_dim)
    DH_FAIL(DH_ERR_SHAPE, "rope: T=%d seq=%d heads=%d d=%d stride=%d (d must be a multiple of 16)", T, seq, n_heads,
            head_dim, row_stride);
  if (T == 0) return DH_OK;
  if (!t) DH_FAIL(DH_ERR_INVALID_ARG, "rope: null pointer");
  size_t total = (size_t)T * n_heads * (head_dim / 16);
  dim3 g((unsigned)((total + 255) / 256)), b(256);
  const double l2b = log2((double)base), ratio = exp2(-2.0 / (double)head_dim * l2b);
#define GO(TT, ADJ) rope_kernel<TT, ADJ><<<g, b, 0, (hipStream_t)stream>>>((TT*)t, T, seq, pos0, n_heads, head_dim, row_stride, l2b, ratio, inverse)
  if (dtype == DH_BF16) { if (pairing == DH_ROPE_ADJACENT) GO(bf16_t, true); else GO(bf16_t, false); }
  else { if (pairing == DH_ROPE_ADJACENT) GO(float, true); else GO(float, false); }
#undef GO
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

// ------------------------------------------------------------------------------------ LayerNorm fwd
// As the RMSNorm kernel, with mean removal and a shift: optional fused x_out = x + res (+ bias), then
// mu = mean(x_out), rstd = (mean((x_out-mu)^2) + eps)^(-1/2) (two passes over the registers, so the
// variance is formed from centred values), h = gamma*(x_out-mu)*rstd + beta.
template <typename T, int NCH>
__global__ __launch_bounds__(ROW_THREADS) void layernorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ res,
                                                                    const T* __restrict__ res_bias, const T* __restrict__ gamma,
                                                                    const T* __restrict__ beta, float eps, T* __restrict__ x_out,
                                                                    T* __restrict__ h, float* __restrict__ mu_out,
                                                                    float* __restrict__ rstd, int H) {
  __shared__ float red[8];
  const size_t row = blockIdx.x;
  Vec8<T> v[NCH];
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) {
      v[c].load(x + row * H + col);
      if (res != nullptr) {
        Vec8<T> r;
        r.load(res + row * H + col);
        if (res_bias != nullptr) {
          Vec8<T> bb;
          bb.load(res_bias + col);
#pragma unroll
          for (int i = 0; i < 8; i++) r.v[i] += bb.v[i];
        }
#pragma unroll
        for (int i = 0; i < 8; i++) v[c].v[i] = to_f32(from_f32<T>(v[c].v[i] + r.v[i]));
        v[c].store(x_out + row * H + col);
      }
#pragma unroll
      for (int i = 0; i < 8; i++) sum += v[c].v[i];
    }
  }
  const float mu = block256_sum(sum, red) / (float)H;
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) {
#pragma unroll
      for (int i = 0; i < 8; i++) {
        v[c].v[i] -= mu;
        ss += v[c].v[i] * v[c].v[i];
      }
    }
  }
  ss = block256_sum(ss, red);
  const float r = 1.0f / sqrtf(ss / (float)H + eps);
  if (threadIdx.x == 0) { mu_out[row] = mu; rstd[row] = r; }
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) {
      Vec8<T> g, b;
      g.load(gamma + col);
      b.load(beta + col);
#pragma unroll
      for (int i = 0; i < 8; i++) g.v[i] = g.v[i] * v[c].v[i] * r + b.v[i];
      g.store(h + row * H + col);
    }
  }
}

// ------------------------------------------------------------------------------------ LayerNorm bwd
// dx = rstd*(gh - mean(gh) - xh*mean(gh*xh)) (+ dres), gh = gamma*dy, xh = (x-mu)*rstd.  Per block one
// partial row [dgamma | dbeta] of 2H floats, reduced in fixed order by the column-sum kernels.
template <typename T, int NCH>
__global__ __launch_bounds__(ROW_THREADS) void layernorm_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                                    const T* __restrict__ gamma, const float* __restrict__ mu,
                                                                    const float* __restrict__ rstd, const T* __restrict__ dres,
                                                                    T* __restrict__ dx, float* __restrict__ partial, int rows, int H) {
  __shared__ float red[8];
  Vec8<T> g[NCH];
  float dg[NCH][8], db[NCH][8];
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) g[c].load(gamma + col);
#pragma unroll
    for (int i = 0; i < 8; i++) dg[c][i] = db[c][i] = 0.f;
  }
  const int rpb = norm_bwd_rpb(rows);
  const size_t row0 = (size_t)blockIdx.x * rpb;
  const int nrows = min(rpb, rows - (int)row0);
  Raw8<T> ndy[NCH], nx[NCH], nres[NCH];  // the next row, as fetched
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
    const float r = rstd[row], m = mu[row];
    Vec8<T> gh[NCH], xh[NCH];
    Raw8<T> rs[NCH];
#pragma unroll
    for (int c = 0; c < NCH; c++) { gh[c].from(ndy[c]); xh[c].from(nx[c]); rs[c] = nres[c]; }
    if (rr + 1 < nrows) fetch(row + 1);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (threadIdx.x + ROW_THREADS * c) * 8;
      if (col < H) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
          xh[c].v[i] = (xh[c].v[i] - m) * r;
          dg[c][i] += gh[c].v[i] * xh[c].v[i];
          db[c][i] += gh[c].v[i];
          gh[c].v[i] *= g[c].v[i];
          s1 += gh[c].v[i];
          s2 += gh[c].v[i] * xh[c].v[i];
        }
      }
    }
    s1 = block256_sum(s1, red) / (float)H;
    s2 = block256_sum(s2, red) / (float)H;
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      int col = (threadIdx.x + ROW_THREADS * c) * 8;
      if (col < H) {
        Vec8<T> o;
#pragma unroll
        for (int i = 0; i < 8; i++) o.v[i] = r * (gh[c].v[i] - s1 - xh[c].v[i] * s2);
        if (dres != nullptr) {
#pragma unroll
          for (int i = 0; i < 8; i++) o.v[i] += rs[c].get(i);
        }
        o.store(dx + row * H + col);
      }
    }
  }
#pragma unroll
  for (int c = 0; c < NCH; c++) {
    int col = (threadIdx.x + ROW_THREADS * c) * 8;
    if (col < H) {
      float4* p = reinterpret_cast<float4*>(partial + (size_t)blockIdx.x * 2 * H + col);
      p[0] = make_float4(dg[c][0], dg[c][1], dg[c][2], dg[c][3]);
      p[1] = make_float4(dg[c][4], dg[c][5], dg[c][6], dg[c][7]);
      float4* q = reinterpret_cast<float4*>(partial + (size_t)blockIdx.x * 2 * H + H + col);
      q[0] = make_float4(db[c][0], db[c][1], db[c][2], db[c][3]);
      q[1] = make_float4(db[c][4], db[c][5], db[c][6], db[c][7]);
    }
  }
}

// ------------------------------------------------------------------------------------ GeLU (tanh form, erf form)
// 0.5 (1 + tanh u) = sigmoid(2u), so the tanh form is x * sigmoid(2u), u = sqrt(2/pi) (x + 0.044715 x^3): one
// exponential per element; its derivative is s + x s (1 - s) 2 u', s = sigmoid(2u).
__device__ __forceinline__ float gelu_tanh_inner(float x) { return 0.7978845608028654f * (x + 0.044715f * x * x * x); }
__device__ __forceinline__ float gelu_sigmoid2u(float x) { return 1.0f / (1.0f + expf(-2.0f * gelu_tanh_inner(x))); }

template <typename T, bool ERF>
__global__ void gelu_fwd_kernel(const T* __restrict__ f, T* __restrict__ a, size_t n8) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n8) return;
  Vec8<T> x;
  x.load(f + idx * 8);
#pragma unroll
  for (int i = 0; i < 8; i++)
    x.v[i] = ERF ? 0.5f * x.v[i] * (1.0f + erff(x.v[i] * 0.7071067811865476f))
                 : x.v[i] * gelu_sigmoid2u(x.v[i]);
  x.store(a + idx * 8);
}

template <typename T, bool ERF>
__global__ void gelu_bwd_kernel(const T* __restrict__ f, const T* __restrict__ da, T* __restrict__ df, size_t n8) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n8) return;
  Vec8<T> x, d;
  x.load(f + idx * 8);
  d.load(da + idx * 8);
#pragma unroll
  for (int i = 0; i < 8; i++) {
    const float v = x.v[i];
    if (ERF) {  // Phi(v) + v phi(v)
      d.v[i] *= 0.5f * (1.0f + erff(v * 0.7071067811865476f)) + v * 0.3989422804014327f * expf(-0.5f * v * v);
    } else {
      const float sg = gelu_sigmoid2u(v);
      d.v[i] *= sg + v * sg * (1.0f - sg) * 2.0f * 0.7978845608028654f * (1.0f + 3.0f * 0.044715f * v * v);
    }
  }
  d.store(df + idx * 8);
}

// ------------------------------------------------------------------------------------ bias + residual, column sums
// out[t,:] = a[t,:] + b[t,:] + bias[:]
template <typename T>
__global__ void bias_residual_add_kernel(const T* __restrict__ a, const T* __restrict__ b, const T* __restrict__ bias,
                                         T* __restrict__ out, size_t n8, int chunks) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n8) return;
  Vec8<T> x, y, z;
  x.load(a + idx * 8);
  y.load(b + idx * 8);
  z.load(bias + (idx % chunks) * 8);
#pragma unroll
  for (int i = 0; i < 8; i++) x.v[i] += y.v[i] + z.v[i];
  x.store(out + idx * 8);
}

// partial[by][col] = sum of rows by*rpb .. +rpb-1 of x (ascending); a thread owns 8 columns and keeps 8 rows'
// loads in flight.  Short inputs (the row shard of sequence parallelism) take fewer rows per block so that the
// launch still covers the chip.
static inline int colsum_rows_per_block(int T) { return T >= 2048 ? 32 : 8; }
template <typename T>
__global__ __launch_bounds__(256) void colsum_rows_kernel(const T* __restrict__ x, float* __restrict__ partial, int rows, int N,
                                                          int rpb) {
  const int col = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (col >= N) return;
  const int r0 = blockIdx.y * rpb, r1 = min(rows, r0 + rpb);
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = r0; r < r1; r += 8) {
    Raw8<T> raw[8];
#pragma unroll
    for (int u = 0; u < 8; u++)
      if (r + u < r1) raw[u].load(x + (size_t)(r + u) * N + col);
#pragma unroll
    for (int u = 0; u < 8; u++)
      if (r + u < r1) {
        Vec8<T> v;
        v.from(raw[u]);
#pragma unroll
        for (int i = 0; i < 8; i++) s[i] += v.v[i];
      }
  }
  float4* p = reinterpret_cast<float4*>(partial + (size_t)blockIdx.y * N + col);
  p[0] = make_float4(s[0], s[1], s[2], s[3]);
  p[1] = make_float4(s[4], s[5], s[6], s[7]);
}

// ------------------------------------------------------------------------------------ host side (GPT-style operators)
extern "C" int dh_layernorm_fwd(int dtype, int T, int H, const void* x, const void* residual, const void* residual_bias,
                                const void* gamma, const void* beta, float eps, void* x_out, void* h, float* mu, float* rstd,
                                void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "layernorm_fwd: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (T == 0) return DH_OK;
  if (!x || !gamma || !beta || !h || !mu || !rstd || (residual && !x_out) || (residual_bias && !residual))
    DH_FAIL(DH_ERR_INVALID_ARG, "layernorm_fwd: null pointer (a residual bias needs a residual)");
  const int nch = nch_for(H);
  hipStream_t s = (hipStream_t)stream;
#define GO(TT, N)                                                                                                           \
  layernorm_fwd_kernel<TT, N><<<T, ROW_THREADS, 0, s>>>((const TT*)x, (const TT*)residual, (const TT*)residual_bias,         \
                                                        (const TT*)gamma, (const TT*)beta, eps, (TT*)x_out, (TT*)h, mu, rstd, H)
#define GO2(N) do { if (dtype == DH_BF16) GO(bf16_t, N); else GO(float, N); } while (0)
  switch (nch) {
    case 1: GO2(1); break;
    case 2: GO2(2); break;
    case 4: GO2(4); break;
    case 8: GO2(8); break;
    default: DH_FAIL(DH_ERR_SHAPE, "layernorm: hidden %d too large (max 16384)", H);
  }
#undef GO2
#undef GO
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" size_t dh_layernorm_bwd_ws_bytes(int T, int H) { return dh_rmsnorm_bwd_ws_bytes(T, 2 * H); }

extern "C" int dh_layernorm_bwd(int dtype, int T, int H, const void* dy, const void* x, const void* gamma, const float* mu,
                                const float* rstd, const void* dres, void* dx, float* dgamma, float* dbeta, void* ws,
                                size_t ws_bytes, void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "layernorm_bwd: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (T == 0) return DH_OK;
  if (!dy || !x || !gamma || !mu || !rstd || !dx || !dgamma || !dbeta) DH_FAIL(DH_ERR_INVALID_ARG, "layernorm_bwd: null pointer");
  if (!ws || ws_bytes < dh_layernorm_bwd_ws_bytes(T, H))
    DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "layernorm_bwd: workspace %zu < %zu bytes", ws_bytes, dh_layernorm_bwd_ws_bytes(T, H));
  const int nch = nch_for(H);
  const int nblk = (T + norm_bwd_rpb(T) - 1) / norm_bwd_rpb(T);
  float* partial = (float*)ws;
  hipStream_t s = (hipStream_t)stream;
#define GO(TT, N)                                                                                                          \
  layernorm_bwd_kernel<TT, N><<<nblk, ROW_THREADS, 0, s>>>((const TT*)dy, (const TT*)x, (const TT*)gamma, mu, rstd,         \
                                                           (const TT*)dres, (TT*)dx, partial, T, H)
#define GO2(N) do { if (dtype == DH_BF16) GO(bf16_t, N); else GO(float, N); } while (0)
  switch (nch) {
    case 1: GO2(1); break;
    case 2: GO2(2); break;
    case 4: GO2(4); break;
    case 8: GO2(8); break;
    default: DH_FAIL(DH_ERR_SHAPE, "layernorm: hidden %d too large (max 16384)", H);
  }
#undef GO2
#undef GO
  DH_LAUNCH_CHECK();
  colsum_finish_kernel<<<(2 * H + 31) / 32, 256, 0, s>>>(partial, nblk, 2 * H, dgamma, H, dbeta);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_gelu_fwd(int dtype, size_t n, const void* f, void* a, void* stream) {
  return dh_gelu_fwd_form(dtype, DH_GELU_TANH, n, f, a, stream);
}
extern "C" int dh_gelu_bwd(int dtype, size_t n, const void* f, const void* da, void* df, void* stream) {
  return dh_gelu_bwd_form(dtype, DH_GELU_TANH, n, f, da, df, stream);
}

extern "C" int dh_gelu_fwd_form(int dtype, int form, size_t n, const void* f, void* a, void* stream) {
  if (form != DH_GELU_TANH && form != DH_GELU_ERF) DH_FAIL(DH_ERR_INVALID_ARG, "gelu: unknown form %d", form);
  if (n % 8) DH_FAIL(DH_ERR_SHAPE, "gelu_fwd: element count %zu must be a multiple of 8", n);
  if (n == 0) return DH_OK;
  if (!f || !a) DH_FAIL(DH_ERR_INVALID_ARG, "gelu_fwd: null pointer");
  const size_t n8 = n / 8;
  dim3 g((unsigned)((n8 + 255) / 256)), b(256);
#define GO(TT, E) gelu_fwd_kernel<TT, E><<<g, b, 0, (hipStream_t)stream>>>((const TT*)f, (TT*)a, n8)
  if (dtype == DH_BF16) { if (form == DH_GELU_ERF) GO(bf16_t, true); else GO(bf16_t, false); }
  else { if (form == DH_GELU_ERF) GO(float, true); else GO(float, false); }
#undef GO
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_gelu_bwd_form(int dtype, int form, size_t n, const void* f, const void* da, void* df, void* stream) {
  if (form != DH_GELU_TANH && form != DH_GELU_ERF) DH_FAIL(DH_ERR_INVALID_ARG, "gelu: unknown form %d", form);
  if (n % 8) DH_FAIL(DH_ERR_SHAPE, "gelu_bwd: element count %zu must be a multiple of 8", n);
  if (n == 0) return DH_OK;
  if (!f || !da || !df) DH_FAIL(DH_ERR_INVALID_ARG, "gelu_bwd: null pointer");
  const size_t n8 = n / 8;
  dim3 g((unsigned)((n8 + 255) / 256)), b(256);
#define GO(TT, E) gelu_bwd_kernel<TT, E><<<g, b, 0, (hipStream_t)stream>>>((const TT*)f, (const TT*)da, (TT*)df, n8)
  if (dtype == DH_BF16) { if (form == DH_GELU_ERF) GO(bf16_t, true); else GO(bf16_t, false); }
  else { if (form == DH_GELU_ERF) GO(float, true); else GO(float, false); }
#undef GO
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_bias_residual_add(int dtype, int T, int H, const void* a, const void* b, const void* bias, void* out,
                                    void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "bias_residual_add: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (T == 0) return DH_OK;
  if (!a || !b || !bias || !out) DH_FAIL(DH_ERR_INVALID_ARG, "bias_residual_add: null pointer");
  const size_t n8 = (size_t)T * (H / 8);
  dim3 g((unsigned)((n8 + 255) / 256)), bl(256);
  if (dtype == DH_BF16)
    bias_residual_add_kernel<bf16_t><<<g, bl, 0, (hipStream_t)stream>>>((const bf16_t*)a, (const bf16_t*)b, (const bf16_t*)bias, (bf16_t*)out, n8, H / 8);
  else
    bias_residual_add_kernel<float><<<g, bl, 0, (hipStream_t)stream>>>((const float*)a, (const float*)b, (const float*)bias, (float*)out, n8, H / 8);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" size_t dh_colsum_ws_bytes(int T, int N) {
  const size_t rpb = colsum_rows_per_block(T);
  const size_t nblk = ((size_t)T + rpb - 1) / rpb;
  return nblk * N * sizeof(float);
}

extern "C" int dh_colsum(int dtype, int T, int N, const void* x, float* out, void* ws, size_t ws_bytes, void* stream) {
  if (T < 0 || N <= 0 || N % 8) DH_FAIL(DH_ERR_SHAPE, "colsum: T=%d N=%d (N must be a positive multiple of 8)", T, N);
  if (T == 0) return DH_OK;
  if (!x || !out) DH_FAIL(DH_ERR_INVALID_ARG, "colsum: null pointer");
  if (!ws || ws_bytes < dh_colsum_ws_bytes(T, N)) DH_FAIL(DH_ERR_WORKSPACE_TOO_SMALL, "colsum: workspace %zu < %zu bytes", ws_bytes, dh_colsum_ws_bytes(T, N));
  const int rpb = colsum_rows_per_block(T);
  const int nblk = (T + rpb - 1) / rpb;
  float* partial = (float*)ws;
  hipStream_t s = (hipStream_t)stream;
  dim3 g((N / 8 + 255) / 256, nblk);
  if (dtype == DH_BF16) colsum_rows_kernel<bf16_t><<<g, 256, 0, s>>>((const bf16_t*)x, partial, T, N, rpb);
  else colsum_rows_kernel<float><<<g, 256, 0, s>>>((const float*)x, partial, T, N, rpb);
  DH_LAUNCH_CHECK();
  colsum_finish_kernel<<<(N + 31) / 32, 256, 0, s>>>(partial, nblk, N, out, N, nullptr);
  DH_LAUNCH_CHECK();
  return DH_OK;
}
