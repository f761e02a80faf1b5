// Shared declarations of libdhelix's HIP sources (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/dhelix.h"

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

// ---- error plumbing (host) -------------------------------------------------------------------
int dh_set_error(int code, const char* fmt, ...);
#define DH_FAIL(code, ...) return dh_set_error(code, __VA_ARGS__)
// Host-side state cached per device (kernel attributes, compute-unit counts): index of the current device.
constexpr int DH_MAX_DEVICES = 64;
static inline int dh_device_index() {
  int d = 0;
  if (hipGetDevice(&d) != hipSuccess || d < 0 || d >= DH_MAX_DEVICES) d = 0;
  return d;
}

#define DH_HIP(expr)                                                                     \
  do {                                                                                   \
    hipError_t _e = (expr);                                                              \
    if (_e != hipSuccess)                                                                \
      return dh_set_error(DH_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(_e));    \
  } while (0)
#define DH_LAUNCH_CHECK()                                                                \
  do {                                                                                   \
    hipError_t _e = hipGetLastError();                                                   \
    if (_e != hipSuccess)                                                                \
      return dh_set_error(DH_ERR_HIP, "kernel launch failed: %s", hipGetErrorString(_e));\
  } while (0)

static inline size_t dh_elem_size(int dtype) { return dtype == DH_BF16 ? 2 : 4; }
static inline size_t dh_align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- device helpers ----------------------------------------------------------------------------
// bf16 <-> fp32.  Conversion to bf16 rounds to nearest even.
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return (bf16_t)v; }

// 8 elements as they lie in memory (16 bytes of bf16, 32 of float): what a kernel holds for data fetched ahead of
// its use, converted to float (Vec8) only when the row's turn comes.
template <typename T> struct Raw8;
template <> struct Raw8<float> {
  f32x4 a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const f32x4*>(p);
    b = *reinterpret_cast<const f32x4*>(p + 4);
  }
  __device__ __forceinline__ float get(int i) const { return i < 4 ? a[i] : b[i - 4]; }
};
template <> struct Raw8<bf16_t> {
  bf16x8 t;
  __device__ __forceinline__ void load(const bf16_t* p) { t = *reinterpret_cast<const bf16x8*>(p); }
  __device__ __forceinline__ float get(int i) const { return (float)t[i]; }
};

// 8-element vector of the storage type, loaded/stored with the widest access.
template <typename T> struct Vec8;
template <> struct Vec8<float> {
  float v[8];
  __device__ __forceinline__ void from(const Raw8<float>& r) {
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = r.get(i);
  }
  __device__ __forceinline__ void load(const float* p) {
    const float4* q = reinterpret_cast<const float4*>(p);
    float4 a = q[0], b = q[1];
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
  __device__ __forceinline__ void store(float* p) const {
    float4* q = reinterpret_cast<float4*>(p);
    q[0] = make_float4(v[0], v[1], v[2], v[3]);
    q[1] = make_float4(v[4], v[5], v[6], v[7]);
  }
  __device__ __forceinline__ void load_stream(const float* p) {
    const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p) + 1);
    v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3]; v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
  }
  __device__ __forceinline__ void store_stream(float* p) const {
    const f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
    __builtin_nontemporal_store(a, reinterpret_cast<f32x4*>(p));
    __builtin_nontemporal_store(b, reinterpret_cast<f32x4*>(p) + 1);
  }
};
template <> struct Vec8<bf16_t> {
  float v[8];
  __device__ __forceinline__ void from(const Raw8<bf16_t>& r) {
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = r.get(i);
  }
  __device__ __forceinline__ void load(const bf16_t* p) {
    bf16x8 t = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = (float)t[i];
  }
  __device__ __forceinline__ void store(bf16_t* p) const {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; i++) t[i] = (bf16_t)v[i];
    *reinterpret_cast<bf16x8*>(p) = t;
  }
  // Streaming forms for data that is touched once (collective payloads): non-temporal accesses, so that the
  // lines do not displace the operand panels a co-running GEMM keeps in L2.
  __device__ __forceinline__ void load_stream(const bf16_t* p) {
    bf16x8 t = __builtin_nontemporal_load(reinterpret_cast<const bf16x8*>(p));
#pragma unroll
    for (int i = 0; i < 8; i++) v[i] = (float)t[i];
  }
  __device__ __forceinline__ void store_stream(bf16_t* p) const {
    bf16x8 t;
#pragma unroll
    for (int i = 0; i < 8; i++) t[i] = (bf16_t)v[i];
    __builtin_nontemporal_store(t, reinterpret_cast<bf16x8*>(p));
  }
};

// SwiGLU element arithmetic with every rounding spelled out (no contraction into fused multiply-adds), so that the
// row-wise kernels and the GEMM epilogues that fuse them give the same bits.
__device__ __forceinline__ float swiglu_fwd_elem(float g, float u) {
  return __fmul_rn(__fdiv_rn(g, __fadd_rn(1.0f, expf(-g))), u);
}
__device__ __forceinline__ void swiglu_bwd_elem(float g, float u, float d, float& dg, float& du) {
  const float s = __fdiv_rn(1.0f, __fadd_rn(1.0f, expf(-g)));
  const float gs = __fmul_rn(g, s);  // g * sigmoid(g)
  dg = __fmul_rn(__fmul_rn(__fmul_rn(d, u), s), __fadd_rn(1.0f, __fmul_rn(g, __fsub_rn(1.0f, s))));
  du = __fmul_rn(d, gs);
}

// All-reduce stand-in: out = sum over the n_ranks partial buffers, added in rank order in float32.  A thread handles the
// 8-element vectors first, first + stride, ... below n8; shared by the stand-in kernel and the GEMM launches that carry
// a stand-in along (the same bits either way).
#define DH_MAX_RANKS 16
struct PartPtrs {
  const void* p[DH_MAX_RANKS];
};
template <typename T>
__device__ __forceinline__ void allreduce_span(const PartPtrs& parts, int n_ranks, T* __restrict__ out, size_t n8, size_t first,
                                               size_t stride) {
  for (size_t i = first; i < n8; i += stride) {
    Vec8<T> acc;
    acc.load_stream((const T*)parts.p[0] + i * 8);
    for (int r = 1; r < n_ranks; r++) {
      Vec8<T> v;
      v.load_stream((const T*)parts.p[r] + i * 8);
#pragma unroll
      for (int k = 0; k < 8; k++) acc.v[k] += v.v[k];
    }
    acc.store_stream(out + i * 8);
  }
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over a 256-thread block; every thread gets the result.  red: 8 floats of LDS.
__device__ __forceinline__ float block256_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// ---- internal launchers (host, defined in the .hip files) ------------------------------------
// All return a dh_status and only enqueue work on `stream`.
// bias: optional [N] in the operand type, added to a result that is stored (not accumulated).
int dh_launch_gemm_f32(bool ta, bool tb, int M, int N, int K, const float* A, const float* B, float* C,
                       bool accumulate, const float* bias, hipStream_t stream);
int dh_launch_gemm_bf16(bool ta, bool tb, int M, int N, int K, const bf16_t* A, const bf16_t* B, void* C,
                        bool out_f32_accumulate, const bf16_t* bias, void* ws, size_t ws_bytes, hipStream_t stream);
int dh_launch_gemm_grouped_f32(int mode, int n_groups, const int32_t* group_rows, int max_rows, int dim_a, int dim_b,
                               const float* A, const float* B, float* C, hipStream_t stream);
int dh_launch_gemm_grouped_bf16(int mode, int n_groups, const int32_t* group_rows, int max_rows, int dim_a, int dim_b,
                                const bf16_t* A, const bf16_t* B, void* C, hipStream_t stream);
size_t dh_gemm_bf16_ws_bytes(bool ta, bool tb, int M, int N, int K);
// A bf16 GEMM launch that carries an all-reduce stand-in along: the first ar_blocks*256/(block size) thread blocks of the
// launch stream the payload (elems bf16 elements, n_ranks partials), the others compute the GEMM's tiles.  *_fits: the
// GEMM is a single launch without workspace.
bool dh_gemm_ar_fits(bool ta, bool tb, int M, int N, int K);
int dh_launch_gemm_bf16_ar(bool ta, bool tb, int M, int N, int K, const bf16_t* A, const bf16_t* B, void* C, bool out_f32_accumulate,
                           int n_ranks, const void* const* parts, bf16_t* ar_out, size_t ar_elems, int ar_blocks, hipStream_t stream);
// SwiGLU fused into the epilogue of the gate/up projection (forward) and of the down projection's data gradient
// (backward); *_fits says whether the shapes allow it (otherwise: the GEMM, then the row-wise kernel).
bool dh_glu_fwd_fits(int T, int F, int H);
int dh_launch_gemm_swiglu_fwd_bf16(int T, int F, int H, const bf16_t* x, const bf16_t* Wgu, bf16_t* gu, bf16_t* a, hipStream_t stream);
bool dh_glu_bwd_fits(int T, int F, int H);
int dh_launch_gemm_swiglu_bwd_bf16(int T, int F, int H, const bf16_t* dy, const bf16_t* Wd, const bf16_t* gu, bf16_t* dgu, hipStream_t stream);
// Attention launchers: seq = queries per sequence; kv == nullptr selects plain causal attention over the packed
// qkv rows, otherwise keys/values come from kv[batch*(q_off+seq), ldkv] and their gradients go to dkv likewise.
int dh_launch_attn_fwd_f32(int batch, int seq, int nq, int nkv, int d, const float* qkv, const float* kv, int ldkv,
                           int q_off, float* o, float* lse, hipStream_t stream);
int dh_launch_attn_bwd_f32(int batch, int seq, int nq, int nkv, int d, const float* qkv, const float* kv, int ldkv,
                           int q_off, const float* o, const float* dout, const float* lse, float* dqkv, float* dkv, int lddkv,
                           float* delta, hipStream_t stream);
int dh_launch_attn_fwd_bf16(int batch, int seq, int nq, int nkv, int d, const bf16_t* qkv, const bf16_t* kv, int ldkv, int q_off,
                            bf16_t* o, float* lse, void* ws, size_t ws_bytes, hipStream_t stream);
size_t dh_attn_fwd_bf16_ws_bytes(int batch, int seq, int q_off, int nq, int nkv, int d);
int dh_launch_attn_bwd_bf16(int batch, int seq, int nq, int nkv, int d, const bf16_t* qkv, const bf16_t* kv, int ldkv, int q_off,
                            const bf16_t* o, const bf16_t* dout, const float* lse, bf16_t* dqkv, bf16_t* dkv, int lddkv,
                            float* delta, void* ws, size_t ws_bytes, hipStream_t stream);
size_t dh_attn_bwd_bf16_ws_bytes(int batch, int seq, int q_off, int nq, int nkv, int d);
