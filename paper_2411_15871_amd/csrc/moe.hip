// Mixture-of-experts operators (paper Sec. 6.1: top-2 gating; Table 2: Router, Permute, AlltoAll,
// Group-GEMM): router, stable permutation plan, row gathers (permute, all-to-all stand-in), weighted
// combine and their backward forms.  All index work is integer and deterministic: rows are grouped by
// expert with a stable counting sort (expert ascending, then token, then k), nothing uses atomics.
#include "common.h"

// ------------------------------------------------------------------------------------ router (M1)
// One thread per token.  Top-2 by logit, ties to the lower expert id; the two kept probabilities are the
// softmax over the two kept logits: p0 = 1/(1+exp(l1-l0)), p1 = 1-p0 computed as exp(l1-l0)/(1+exp(l1-l0)).
__global__ void moe_route_kernel(int T, int E, const float* __restrict__ logits, int32_t* __restrict__ idx,
                                 float* __restrict__ prob) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  const float* l = logits + (size_t)t * E;
  int i0 = 0, i1 = -1;
  float v0 = l[0], v1 = -INFINITY;
  for (int e = 1; e < E; e++) {
    float v = l[e];
    if (v > v0) { i1 = i0; v1 = v0; i0 = e; v0 = v; }
    else if (v > v1) { i1 = e; v1 = v; }
  }
  float d = expf(v1 - v0);
  idx[2 * t] = i0;
  idx[2 * t + 1] = i1;
  prob[2 * t] = 1.0f / (1.0f + d);
  prob[2 * t + 1] = d / (1.0f + d);
}

// dlogits[t,e] = p_k (dp_k - sum_j p_j dp_j) for the two kept experts, 0 elsewhere.
__global__ void moe_route_bwd_kernel(int T, int E, const float* __restrict__ dprob, const int32_t* __restrict__ idx,
                                     const float* __restrict__ prob, float* __restrict__ dlogits) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  float p0 = prob[2 * t], p1 = prob[2 * t + 1], g0 = dprob[2 * t], g1 = dprob[2 * t + 1];
  float s = p0 * g0 + p1 * g1;
  float* dl = dlogits + (size_t)t * E;
  for (int e = 0; e < E; e++) dl[e] = 0.f;
  dl[idx[2 * t]] = p0 * (g0 - s);
  dl[idx[2 * t + 1]] = p1 * (g1 - s);
}

// ------------------------------------------------------------------------------------ permutation plan (M2, M3)
// Block e ranks the assignments (a = 2t+k, ascending) that chose expert e: thread i owns a contiguous
// slice of assignments, counts its matches, the block scans the counts, then the thread hands out ranks.
__global__ __launch_bounds__(256) void moe_rank_kernel(int n_assign, const int32_t* __restrict__ idx, int32_t* __restrict__ rank,
                                                       int32_t* __restrict__ counts) {
  __shared__ int part[256];
  const int e = blockIdx.x, tid = threadIdx.x;
  const int per = (n_assign + 255) / 256, a0 = min(n_assign, tid * per), a1 = min(n_assign, a0 + per);
  int c = 0;
  for (int a = a0; a < a1; a++) c += idx[a] == e;
  part[tid] = c;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {  // inclusive Hillis-Steele scan
    int v = tid >= off ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  int r = part[tid] - c;
  for (int a = a0; a < a1; a++)
    if (idx[a] == e) rank[a] = r++;
  if (tid == 255) counts[e] = part[255];
}

// Single block: prefix sums over the experts.  offsets[e] = first send row of expert e (send order = expert
// ascending); recv_start[e] = first receive row of expert e (receive order = [local expert][source rank],
// logical expert e = source*n_local + local); group_rows[le] = rows of local expert le.
__global__ void moe_offsets_kernel(int E, int n_local, const int32_t* __restrict__ counts, int32_t* __restrict__ offsets,
                                   int32_t* __restrict__ recv_start, int32_t* __restrict__ group_rows) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  int acc = 0;
  for (int e = 0; e < E; e++) { offsets[e] = acc; acc += counts[e]; }
  offsets[E] = acc;
  acc = 0;
  for (int le = 0; le < n_local; le++) {
    int g = 0;
    for (int src = 0; src < E / n_local; src++) {
      int e = src * n_local + le;
      recv_start[e] = acc;
      acc += counts[e];
      g += counts[e];
    }
    group_rows[le] = g;
  }
}

// dest[a] = send row of assignment a; src_tok[row] = its token; send_of_recv[j] = send row copied to receive
// row j; recv_of_send = the inverse.
__global__ void moe_tables_kernel(int n_assign, const int32_t* __restrict__ idx, const int32_t* __restrict__ rank,
                                  const int32_t* __restrict__ offsets, const int32_t* __restrict__ recv_start,
                                  int32_t* __restrict__ dest, int32_t* __restrict__ src_tok, int32_t* __restrict__ send_of_recv,
                                  int32_t* __restrict__ recv_of_send) {
  int a = blockIdx.x * blockDim.x + threadIdx.x;
  if (a >= n_assign) return;
  int e = idx[a], r = rank[a];
  int row = offsets[e] + r, rr = recv_start[e] + r;
  dest[a] = row;
  src_tok[row] = a >> 1;
  send_of_recv[rr] = row;
  recv_of_send[row] = rr;
}

// ------------------------------------------------------------------------------------ row movement
// out[r,:] = in[map[r],:]  (token permute, all-to-all stand-in in both directions).  One wave per row chunk.
template <typename T>
__global__ __launch_bounds__(256) void gather_rows_kernel(int n_rows, int H, const T* __restrict__ in, const int32_t* __restrict__ map,
                                                          T* __restrict__ out) {
  const int chunks = H / 8;
  const size_t total = (size_t)n_rows * chunks, stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const size_t r = i / chunks;
    const int c = (int)(i % chunks) * 8;
    Vec8<T> v;
    v.load(in + (size_t)map[r] * H + c);
    v.store(out + r * H + c);
  }
}

// y[t,:] = w0*yp[dest[t,0],:] + w1*yp[dest[t,1],:] (+ res[t,:]); weights = prob[t,:] or 1 when prob == nullptr.
template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(int Ttok, int H, const T* __restrict__ yp, const int32_t* __restrict__ dest,
                                                      const float* __restrict__ prob, const T* __restrict__ res, T* __restrict__ y) {
  const int chunks = H / 8;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)Ttok * chunks) return;
  const size_t t = i / chunks;
  const int c = (int)(i % chunks) * 8;
  const float w0 = prob ? prob[2 * t] : 1.f, w1 = prob ? prob[2 * t + 1] : 1.f;
  Vec8<T> a, b;
  a.load(yp + (size_t)dest[2 * t] * H + c);
  b.load(yp + (size_t)dest[2 * t + 1] * H + c);
#pragma unroll
  for (int k = 0; k < 8; k++) a.v[k] = w0 * a.v[k] + w1 * b.v[k];
  if (res != nullptr) {
    b.load(res + t * H + c);
#pragma unroll
    for (int k = 0; k < 8; k++) a.v[k] += b.v[k];
  }
  a.store(y + t * H + c);
}

// Backward of the weighted combine: dyp[dest[t,k],:] = prob[t,k]*dy[t,:]; dprob[t,k] = <dy[t,:], yp[dest[t,k],:]>.
// One 256-thread block per token.
template <typename T>
__global__ __launch_bounds__(256) void combine_bwd_kernel(int H, const T* __restrict__ dy, const T* __restrict__ yp,
                                                          const int32_t* __restrict__ dest, const float* __restrict__ prob,
                                                          T* __restrict__ dyp, float* __restrict__ dprob) {
  __shared__ float red[8];
  const size_t t = blockIdx.x;
  const int r0 = dest[2 * t], r1 = dest[2 * t + 1];
  const float p0 = prob[2 * t], p1 = prob[2 * t + 1];
  float d0 = 0.f, d1 = 0.f;
  for (int c = threadIdx.x * 8; c < H; c += 256 * 8) {
    Vec8<T> g, a, b, o0, o1;
    g.load(dy + t * H + c);
    a.load(yp + (size_t)r0 * H + c);
    b.load(yp + (size_t)r1 * H + c);
#pragma unroll
    for (int k = 0; k < 8; k++) {
      d0 += g.v[k] * a.v[k];
      d1 += g.v[k] * b.v[k];
      o0.v[k] = p0 * g.v[k];
      o1.v[k] = p1 * g.v[k];
    }
    o0.store(dyp + (size_t)r0 * H + c);
    o1.store(dyp + (size_t)r1 * H + c);
  }
  d0 = block256_sum(d0, red);
  d1 = block256_sum(d1, red);
  if (threadIdx.x == 0) { dprob[2 * t] = d0; dprob[2 * t + 1] = d1; }
}

// ------------------------------------------------------------------------------------ host side
extern "C" int dh_moe_route(int T, int E, const float* logits, int32_t* idx, float* prob, void* stream) {
  if (T < 0 || E < 2 || E > 256) DH_FAIL(DH_ERR_SHAPE, "moe_route: T=%d E=%d (E must be 2..256)", T, E);
  if (T == 0) return DH_OK;
  if (!logits || !idx || !prob) DH_FAIL(DH_ERR_INVALID_ARG, "moe_route: null pointer");
  moe_route_kernel<<<(T + 255) / 256, 256, 0, (hipStream_t)stream>>>(T, E, logits, idx, prob);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_moe_route_bwd(int T, int E, const float* dprob, const int32_t* idx, const float* prob, float* dlogits,
                                void* stream) {
  if (T < 0 || E < 2 || E > 256) DH_FAIL(DH_ERR_SHAPE, "moe_route_bwd: T=%d E=%d (E must be 2..256)", T, E);
  if (T == 0) return DH_OK;
  if (!dprob || !idx || !prob || !dlogits) DH_FAIL(DH_ERR_INVALID_ARG, "moe_route_bwd: null pointer");
  moe_route_bwd_kernel<<<(T + 255) / 256, 256, 0, (hipStream_t)stream>>>(T, E, dprob, idx, prob, dlogits);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_moe_plan(int T, int E, int n_local, const int32_t* idx, const dh_moe_tables* tb, void* stream) {
  if (T < 0 || E < 2 || E > 256 || n_local < 1 || E % n_local) DH_FAIL(DH_ERR_SHAPE, "moe_plan: T=%d E=%d n_local=%d", T, E, n_local);
  if (!tb || !tb->rank || !tb->dest || !tb->src_tok || !tb->send_of_recv || !tb->recv_of_send || !tb->counts || !tb->offsets ||
      !tb->recv_start || !tb->group_rows || (T > 0 && !idx))
    DH_FAIL(DH_ERR_INVALID_ARG, "moe_plan: null pointer");
  const int n = 2 * T;
  hipStream_t s = (hipStream_t)stream;
  moe_rank_kernel<<<E, 256, 0, s>>>(n, idx, tb->rank, tb->counts);
  DH_LAUNCH_CHECK();
  moe_offsets_kernel<<<1, 64, 0, s>>>(E, n_local, tb->counts, tb->offsets, tb->recv_start, tb->group_rows);
  DH_LAUNCH_CHECK();
  if (n > 0) {
    moe_tables_kernel<<<(n + 255) / 256, 256, 0, s>>>(n, idx, tb->rank, tb->offsets, tb->recv_start, tb->dest, tb->src_tok,
                                                      tb->send_of_recv, tb->recv_of_send);
    DH_LAUNCH_CHECK();
  }
  return DH_OK;
}

extern "C" int dh_moe_gather_rows(int dtype, int n_rows, int H, const void* in, const int32_t* map, void* out, int n_blocks,
                                  void* stream) {
  if (n_rows < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "moe_gather_rows: rows=%d H=%d (H must be a positive multiple of 8)", n_rows, H);
  if (n_blocks < 0 || n_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "moe_gather_rows: n_blocks %d outside 0..65536", n_blocks);
  if (n_rows == 0) return DH_OK;
  if (!in || !map || !out) DH_FAIL(DH_ERR_INVALID_ARG, "moe_gather_rows: null pointer");
  size_t want = ((size_t)n_rows * (H / 8) + 255) / 256, cap = n_blocks > 0 ? (size_t)n_blocks : 4096;
  unsigned grid = (unsigned)(want < cap ? want : cap);
  if (dtype == DH_BF16) gather_rows_kernel<bf16_t><<<grid, 256, 0, (hipStream_t)stream>>>(n_rows, H, (const bf16_t*)in, map, (bf16_t*)out);
  else gather_rows_kernel<float><<<grid, 256, 0, (hipStream_t)stream>>>(n_rows, H, (const float*)in, map, (float*)out);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_moe_combine(int dtype, int T, int H, const void* yp, const int32_t* dest, const float* prob,
                              const void* residual, void* y, void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "moe_combine: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (T == 0) return DH_OK;
  if (!yp || !dest || !y) DH_FAIL(DH_ERR_INVALID_ARG, "moe_combine: null pointer");
  unsigned grid = (unsigned)(((size_t)T * (H / 8) + 255) / 256);
  if (dtype == DH_BF16) combine_kernel<bf16_t><<<grid, 256, 0, (hipStream_t)stream>>>(T, H, (const bf16_t*)yp, dest, prob, (const bf16_t*)residual, (bf16_t*)y);
  else combine_kernel<float><<<grid, 256, 0, (hipStream_t)stream>>>(T, H, (const float*)yp, dest, prob, (const float*)residual, (float*)y);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_moe_combine_bwd(int dtype, int T, int H, const void* dy, const void* yp, const int32_t* dest, const float* prob,
                                  void* dyp, float* dprob, void* stream) {
  if (T < 0 || H <= 0 || H % 8) DH_FAIL(DH_ERR_SHAPE, "moe_combine_bwd: T=%d H=%d (H must be a positive multiple of 8)", T, H);
  if (T == 0) return DH_OK;
  if (!dy || !yp || !dest || !prob || !dyp || !dprob) DH_FAIL(DH_ERR_INVALID_ARG, "moe_combine_bwd: null pointer");
  if (dtype == DH_BF16)
    combine_bwd_kernel<bf16_t><<<T, 256, 0, (hipStream_t)stream>>>(H, (const bf16_t*)dy, (const bf16_t*)yp, dest, prob, (bf16_t*)dyp, dprob);
  else
    combine_bwd_kernel<float><<<T, 256, 0, (hipStream_t)stream>>>(H, (const float*)dy, (const float*)yp, dest, prob, (float*)dyp, dprob);
  DH_LAUNCH_CHECK();
  return DH_OK;
}
