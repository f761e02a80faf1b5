// Error reporting and the generic single-operator entry points of libdhelix.
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include "common.h"

static thread_local char g_err[512] = "";

int dh_set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

extern "C" const char* dh_last_error(void) { return g_err; }

extern "C" int dh_gemm_bias(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, const void* B,
                            const void* bias, void* C, int out_f32_accumulate, void* ws, size_t ws_bytes, void* stream) {
  if (M < 0 || N < 0 || K < 0) DH_FAIL(DH_ERR_SHAPE, "gemm: negative dimension");
  if (M > 0 && N > 0 && (!C || (K > 0 && (!A || !B)))) DH_FAIL(DH_ERR_INVALID_ARG, "gemm: null pointer");
  if (bias && out_f32_accumulate) DH_FAIL(DH_ERR_INVALID_ARG, "gemm: a bias goes with a stored result only");
  if (dtype == DH_F32)
    return dh_launch_gemm_f32(trans_a != 0, trans_b != 0, M, N, K, (const float*)A, (const float*)B, (float*)C,
                              out_f32_accumulate != 0, (const float*)bias, (hipStream_t)stream);
  if (dtype == DH_BF16)
    return dh_launch_gemm_bf16(trans_a != 0, trans_b != 0, M, N, K, (const bf16_t*)A, (const bf16_t*)B, C,
                               out_f32_accumulate != 0, (const bf16_t*)bias, ws, ws_bytes, (hipStream_t)stream);
  DH_FAIL(DH_ERR_INVALID_ARG, "gemm: unknown dtype %d", dtype);
}

extern "C" int dh_gemm(int dtype, int trans_a, int trans_b, int M, int N, int K, const void* A, const void* B, void* C,
                       int out_f32_accumulate, void* ws, size_t ws_bytes, void* stream) {
  return dh_gemm_bias(dtype, trans_a, trans_b, M, N, K, A, B, nullptr, C, out_f32_accumulate, ws, ws_bytes, stream);
}

extern "C" int dh_gemm_grouped(int dtype, int mode, int n_groups, const int32_t* group_rows, int max_rows, int dim_a, int dim_b,
                               const void* A, const void* B, void* C, void* stream) {
  if (mode < 0 || mode > 2 || n_groups < 1 || n_groups > 64 || max_rows < 0 || dim_a <= 0 || dim_b <= 0)
    DH_FAIL(DH_ERR_INVALID_ARG, "gemm_grouped: mode=%d groups=%d max_rows=%d dims=%d,%d", mode, n_groups, max_rows, dim_a, dim_b);
  if (max_rows == 0) return DH_OK;
  if (!group_rows || !A || !B || !C) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_grouped: null pointer");
  if (dtype == DH_F32)
    return dh_launch_gemm_grouped_f32(mode, n_groups, group_rows, max_rows, dim_a, dim_b, (const float*)A, (const float*)B,
                                      (float*)C, (hipStream_t)stream);
  if (dtype == DH_BF16)
    return dh_launch_gemm_grouped_bf16(mode, n_groups, group_rows, max_rows, dim_a, dim_b, (const bf16_t*)A, (const bf16_t*)B, C,
                                       (hipStream_t)stream);
  DH_FAIL(DH_ERR_INVALID_ARG, "gemm_grouped: unknown dtype %d", dtype);
}

extern "C" int dh_gemm_allreduce_fits(int trans_a, int trans_b, int M, int N, int K) {
  return dh_gemm_ar_fits(trans_a != 0, trans_b != 0, M, N, K) ? 1 : 0;
}

extern "C" int dh_gemm_allreduce(int trans_a, int trans_b, int M, int N, int K, const void* A, const void* B, void* C,
                                 int out_f32_accumulate, int n_ranks, const void* const* parts, void* ar_out, size_t ar_elems,
                                 int n_blocks, void* stream) {
  if (!dh_gemm_ar_fits(trans_a != 0, trans_b != 0, M, N, K))
    DH_FAIL(DH_ERR_UNSUPPORTED, "gemm_allreduce: M=%d N=%d K=%d ta=%d tb=%d does not run as a single launch", M, N, K, trans_a, trans_b);
  if (!A || !B || !C || !parts || !ar_out) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_allreduce: null pointer");
  if (n_ranks < 1 || n_ranks > DH_MAX_RANKS) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_allreduce: n_ranks %d outside 1..%d", n_ranks, DH_MAX_RANKS);
  if (n_blocks < 1 || n_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_allreduce: n_blocks %d outside 1..65536", n_blocks);
  if (ar_elems == 0 || ar_elems % 8) DH_FAIL(DH_ERR_SHAPE, "gemm_allreduce: element count %zu must be a positive multiple of 8", ar_elems);
  if ((uintptr_t)ar_out & 15) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_allreduce: ar_out must be 16-byte aligned");
  for (int r = 0; r < n_ranks; r++)
    if (!parts[r] || ((uintptr_t)parts[r] & 15)) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_allreduce: partial %d is null or not 16-byte aligned", r);
  return dh_launch_gemm_bf16_ar(trans_a != 0, trans_b != 0, M, N, K, (const bf16_t*)A, (const bf16_t*)B, C, out_f32_accumulate != 0,
                                n_ranks, parts, (bf16_t*)ar_out, ar_elems, n_blocks, (hipStream_t)stream);
}

extern "C" int dh_gemm_swiglu_fwd_fits(int T, int F, int H) { return dh_glu_fwd_fits(T, F, H) ? 1 : 0; }
extern "C" int dh_gemm_swiglu_bwd_fits(int T, int F, int H) { return dh_glu_bwd_fits(T, F, H) ? 1 : 0; }

extern "C" int dh_gemm_swiglu_fwd(int T, int F, int H, const void* x, const void* w_gate_up, void* gu, void* a, void* stream) {
  if (!dh_glu_fwd_fits(T, F, H)) DH_FAIL(DH_ERR_UNSUPPORTED, "gemm_swiglu_fwd: T=%d F=%d H=%d does not fit the fused kernel", T, F, H);
  if (!x || !w_gate_up || !gu || !a) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_swiglu_fwd: null pointer");
  return dh_launch_gemm_swiglu_fwd_bf16(T, F, H, (const bf16_t*)x, (const bf16_t*)w_gate_up, (bf16_t*)gu, (bf16_t*)a, (hipStream_t)stream);
}

extern "C" int dh_gemm_swiglu_bwd(int T, int F, int H, const void* dy, const void* w_down, const void* gu, void* dgu, void* stream) {
  if (!dh_glu_bwd_fits(T, F, H)) DH_FAIL(DH_ERR_UNSUPPORTED, "gemm_swiglu_bwd: T=%d F=%d H=%d does not fit the fused kernel", T, F, H);
  if (!dy || !w_down || !gu || !dgu) DH_FAIL(DH_ERR_INVALID_ARG, "gemm_swiglu_bwd: null pointer");
  return dh_launch_gemm_swiglu_bwd_bf16(T, F, H, (const bf16_t*)dy, (const bf16_t*)w_down, (const bf16_t*)gu, (bf16_t*)dgu, (hipStream_t)stream);
}

extern "C" size_t dh_gemm_workspace_bytes(int dtype, int trans_a, int trans_b, int M, int N, int K) {
  if (dtype != DH_BF16 || M <= 0 || N <= 0 || K <= 0) return 0;
  return dh_gemm_bf16_ws_bytes(trans_a != 0, trans_b != 0, M, N, K);
}

static int check_attn(const char* who, int batch, int seq, int nq, int nkv, int d) {
  if (batch < 0 || seq < 0 || nq <= 0 || nkv <= 0 || nq % nkv || d <= 0 || d % 8)
    DH_FAIL(DH_ERR_SHAPE, "%s: batch=%d seq=%d nq=%d nkv=%d d=%d", who, batch, seq, nq, nkv, d);
  return DH_OK;
}

extern "C" size_t dh_attn_fwd_workspace_bytes(int dtype, int batch, int seq, int nq, int nkv, int d) {
  return dh_attn_ctx_fwd_workspace_bytes(dtype, batch, seq, 0, nq, nkv, d);
}

extern "C" size_t dh_attn_ctx_fwd_workspace_bytes(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d) {
  if (dtype != DH_BF16 || batch <= 0 || seq <= 0 || q_off < 0 || nq <= 0 || nkv <= 0 || d <= 0) return 0;
  return dh_attn_fwd_bf16_ws_bytes(batch, seq, q_off, nq, nkv, d);
}

extern "C" int dh_attn_fwd(int dtype, int batch, int seq, int nq, int nkv, int d, const void* qkv, void* o, float* lse,
                           void* ws, size_t ws_bytes, void* stream) {
  int rc = check_attn("attn_fwd", batch, seq, nq, nkv, d);
  if (rc) return rc;
  if (batch * seq > 0 && (!qkv || !o || !lse)) DH_FAIL(DH_ERR_INVALID_ARG, "attn_fwd: null pointer");
  if (dtype == DH_F32)
    return dh_launch_attn_fwd_f32(batch, seq, nq, nkv, d, (const float*)qkv, nullptr, 0, 0, (float*)o, lse, (hipStream_t)stream);
  if (dtype == DH_BF16)
    return dh_launch_attn_fwd_bf16(batch, seq, nq, nkv, d, (const bf16_t*)qkv, nullptr, 0, 0, (bf16_t*)o, lse, ws, ws_bytes,
                                   (hipStream_t)stream);
  DH_FAIL(DH_ERR_INVALID_ARG, "attn_fwd: unknown dtype %d", dtype);
}

extern "C" int dh_attn_ctx_fwd(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d, const void* qkv, const void* kv,
                               void* o, float* lse, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_attn("attn_ctx_fwd", batch, seq, nq, nkv, d);
  if (rc) return rc;
  if (q_off < 0) DH_FAIL(DH_ERR_SHAPE, "attn_ctx_fwd: negative query offset");
  if (batch * seq > 0 && (!qkv || !kv || !o || !lse)) DH_FAIL(DH_ERR_INVALID_ARG, "attn_ctx_fwd: null pointer");
  if (dtype == DH_F32)
    return dh_launch_attn_fwd_f32(batch, seq, nq, nkv, d, (const float*)qkv, (const float*)kv, 2 * nkv * d, q_off, (float*)o, lse,
                                  (hipStream_t)stream);
  if (dtype == DH_BF16)
    return dh_launch_attn_fwd_bf16(batch, seq, nq, nkv, d, (const bf16_t*)qkv, (const bf16_t*)kv, 2 * nkv * d, q_off, (bf16_t*)o, lse,
                                   ws, ws_bytes, (hipStream_t)stream);
  DH_FAIL(DH_ERR_INVALID_ARG, "attn_ctx_fwd: unknown dtype %d", dtype);
}

extern "C" size_t dh_attn_bwd_workspace_bytes(int dtype, int batch, int seq, int nq, int nkv, int d) {
  return dh_attn_ctx_bwd_workspace_bytes(dtype, batch, seq, 0, nq, nkv, d);
}

extern "C" size_t dh_attn_ctx_bwd_workspace_bytes(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d) {
  if (dtype != DH_BF16 || batch <= 0 || seq <= 0 || q_off < 0 || nq <= 0 || nkv <= 0 || d <= 0) return 0;
  return dh_attn_bwd_bf16_ws_bytes(batch, seq, q_off, nq, nkv, d);
}

extern "C" int dh_attn_bwd(int dtype, int batch, int seq, int nq, int nkv, int d, const void* qkv, const void* o,
                           const void* dout, const float* lse, void* dqkv, float* delta, void* ws, size_t ws_bytes,
                           void* stream) {
  int rc = check_attn("attn_bwd", batch, seq, nq, nkv, d);
  if (rc) return rc;
  if (batch * seq > 0 && (!qkv || !o || !dout || !lse || !dqkv || !delta)) DH_FAIL(DH_ERR_INVALID_ARG, "attn_bwd: null pointer");
  if (dtype == DH_F32)
    return dh_launch_attn_bwd_f32(batch, seq, nq, nkv, d, (const float*)qkv, nullptr, 0, 0, (const float*)o, (const float*)dout, lse,
                                  (float*)dqkv, nullptr, 0, delta, (hipStream_t)stream);
  if (dtype == DH_BF16)
    return dh_launch_attn_bwd_bf16(batch, seq, nq, nkv, d, (const bf16_t*)qkv, nullptr, 0, 0, (const bf16_t*)o, (const bf16_t*)dout,
                                   lse, (bf16_t*)dqkv, nullptr, 0, delta, ws, ws_bytes, (hipStream_t)stream);
  DH_FAIL(DH_ERR_INVALID_ARG, "attn_bwd: unknown dtype %d", dtype);
}

extern "C" int dh_attn_ctx_bwd(int dtype, int batch, int seq, int q_off, int nq, int nkv, int d, const void* qkv, const void* kv,
                               const void* o, const void* dout, const float* lse, void* dqkv, void* dkv, float* delta, void* ws,
                               size_t ws_bytes, void* stream) {
  int rc = check_attn("attn_ctx_bwd", batch, seq, nq, nkv, d);
  if (rc) return rc;
  if (q_off < 0) DH_FAIL(DH_ERR_SHAPE, "attn_ctx_bwd: negative query offset");
  if (batch * seq > 0 && (!qkv || !kv || !o || !dout || !lse || !dqkv || !dkv || !delta))
    DH_FAIL(DH_ERR_INVALID_ARG, "attn_ctx_bwd: null pointer");
  if (dtype == DH_F32)
    return dh_launch_attn_bwd_f32(batch, seq, nq, nkv, d, (const float*)qkv, (const float*)kv, 2 * nkv * d, q_off, (const float*)o,
                                  (const float*)dout, lse, (float*)dqkv, (float*)dkv, 2 * nkv * d, delta, (hipStream_t)stream);
  if (dtype == DH_BF16)
    return dh_launch_attn_bwd_bf16(batch, seq, nq, nkv, d, (const bf16_t*)qkv, (const bf16_t*)kv, 2 * nkv * d, q_off, (const bf16_t*)o,
                                   (const bf16_t*)dout, lse, (bf16_t*)dqkv, (bf16_t*)dkv, 2 * nkv * d, delta, ws, ws_bytes,
                                   (hipStream_t)stream);
  DH_FAIL(DH_ERR_INVALID_ARG, "attn_ctx_bwd: unknown dtype %d", dtype);
}
