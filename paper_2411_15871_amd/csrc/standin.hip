// One-GPU stand-ins for the collectives of the layer's critical path (tensor-parallel all-reduce,
// sequence-parallel all-gather and reduce-scatter) and for the Send/Recv exchanges of context parallelism.
// A stand-in moves the collective's payload through HBM: the reductions read the n_ranks partial
// buffers and write their sum, the all-gather copies the n_ranks shards behind one another.  It is meant to run on a stream restricted to a few compute units,
// so the grid is small and grid-strided: each thread streams 16-byte vectors.
#include "common.h"

template <typename T>
__global__ __launch_bounds__(256) void allreduce_kernel(PartPtrs parts, int n_ranks, T* __restrict__ out, size_t n8) {
  allreduce_span<T>(parts, n_ranks, out, n8, (size_t)blockIdx.x * blockDim.x + threadIdx.x, (size_t)gridDim.x * blockDim.x);
}

// out = [parts[0] | parts[1] | ... ], each part n8 vectors of 8 elements.
template <typename T>
__global__ __launch_bounds__(256) void allgather_kernel(PartPtrs parts, int n_ranks, T* __restrict__ out, size_t n8) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t total = n8 * n_ranks;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int r = (int)(i / n8);
    const size_t j = i - (size_t)r * n8;
    Vec8<T> v;
    v.load((const T*)parts.p[r] + j * 8);
    v.store(out + i * 8);
  }
}

extern "C" int dh_comm_standin(int kind, int n_ranks, const void* const* parts, void* out, size_t elems, int dtype,
                               int n_blocks, void* stream) {
  if (kind != DH_COMM_ALLREDUCE && kind != DH_COMM_ALLGATHER && kind != DH_COMM_REDUCESCATTER && kind != DH_COMM_A2A_DISPATCH &&
      kind != DH_COMM_A2A_COMBINE)
    DH_FAIL(DH_ERR_UNSUPPORTED, "comm_standin: kind %d not supported", kind);
  if (dtype != DH_F32 && dtype != DH_BF16) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: dtype %d", dtype);
  // an equal-split all-to-all seen from the receiving rank moves what an all-gather moves: one block from every rank
  if (kind == DH_COMM_A2A_DISPATCH || kind == DH_COMM_A2A_COMBINE) kind = DH_COMM_ALLGATHER;
  if (n_ranks < 1 || n_ranks > DH_MAX_RANKS) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: n_ranks %d outside 1..%d", n_ranks, DH_MAX_RANKS);
  if (elems % 8) DH_FAIL(DH_ERR_SHAPE, "comm_standin: element count %zu must be a multiple of 8", elems);
  if (!parts || !out) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: null pointer");
  if ((uintptr_t)out & 15) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: out must be 16-byte aligned");
  if (n_blocks < 0 || n_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: n_blocks %d outside 0..65536", n_blocks);
  PartPtrs pp;
  for (int r = 0; r < n_ranks; r++) {
    if (!parts[r]) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: partial %d is null", r);
    if ((uintptr_t)parts[r] & 15) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: partial %d must be 16-byte aligned", r);
    pp.p[r] = parts[r];
  }
  if (elems == 0) return DH_OK;
  size_t n8 = elems / 8;
  size_t want = (n8 * (kind == DH_COMM_ALLGATHER ? n_ranks : 1) + 255) / 256;
  size_t cap = n_blocks > 0 ? (size_t)n_blocks : 2048;
  unsigned grid = (unsigned)(want < cap ? want : cap);
  if (kind == DH_COMM_ALLGATHER) {
    if (dtype == DH_BF16)
      allgather_kernel<bf16_t><<<grid, 256, 0, (hipStream_t)stream>>>(pp, n_ranks, (bf16_t*)out, n8);
    else
      allgather_kernel<float><<<grid, 256, 0, (hipStream_t)stream>>>(pp, n_ranks, (float*)out, n8);
    DH_LAUNCH_CHECK();
    return DH_OK;
  }
  if (dtype == DH_BF16)
    allreduce_kernel<bf16_t><<<grid, 256, 0, (hipStream_t)stream>>>(pp, n_ranks, (bf16_t*)out, n8);
  else
    allreduce_kernel<float><<<grid, 256, 0, (hipStream_t)stream>>>(pp, n_ranks, (float*)out, n8);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

// ------------------------------------------------------------------------------------ context parallelism
// Send/Recv stand-in of a ring exchange: every move copies `rows` rows of `width` elements per sequence from
// src to dst, each side with its own row pitch, rows per sequence and first row inside the sequence.
struct CpMoves {
  int n;
  dh_cp_move m[DH_MAX_RANKS];
};

template <typename T>
__global__ __launch_bounds__(256) void cp_exchange_kernel(CpMoves mv, int batch, int rows, int w8) {
  const size_t per = (size_t)batch * rows * w8, total = per * mv.n, stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int k = (int)(i / per);
    const size_t j = i - (size_t)k * per;
    const int c = (int)(j % w8);
    const size_t t = j / w8;
    const int b = (int)(t / rows), r = (int)(t % rows);
    const dh_cp_move& m = mv.m[k];
    Vec8<T> v;
    v.load_stream((const T*)m.src + ((size_t)b * m.src_seq_rows + m.src_row0 + r) * m.src_ld + c * 8);
    v.store_stream((T*)m.dst + ((size_t)b * m.dst_seq_rows + m.dst_row0 + r) * m.dst_ld + c * 8);
  }
}

extern "C" int dh_cp_exchange(int dtype, int n_moves, const dh_cp_move* moves, int batch, int rows, int width, int n_blocks,
                              void* stream) {
  if (dtype != DH_F32 && dtype != DH_BF16) DH_FAIL(DH_ERR_INVALID_ARG, "cp_exchange: dtype %d", dtype);
  if (n_moves < 0 || n_moves > DH_MAX_RANKS) DH_FAIL(DH_ERR_INVALID_ARG, "cp_exchange: n_moves %d outside 0..%d", n_moves, DH_MAX_RANKS);
  if (batch < 0 || rows < 0 || width < 0 || width % 8) DH_FAIL(DH_ERR_SHAPE, "cp_exchange: batch %d rows %d width %d (width: multiple of 8)", batch, rows, width);
  if (n_blocks < 0 || n_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "cp_exchange: n_blocks %d outside 0..65536", n_blocks);
  if (n_moves == 0 || batch * rows == 0 || width == 0) return DH_OK;
  if (!moves) DH_FAIL(DH_ERR_INVALID_ARG, "cp_exchange: null pointer");
  CpMoves mv;
  mv.n = n_moves;
  for (int k = 0; k < n_moves; k++) {
    const dh_cp_move& m = moves[k];
    if (!m.src || !m.dst) DH_FAIL(DH_ERR_INVALID_ARG, "cp_exchange: move %d has a null pointer", k);
    if (m.src_ld < width || m.dst_ld < width || m.src_ld % 8 || m.dst_ld % 8 || m.src_row0 < 0 || m.dst_row0 < 0 ||
        m.src_row0 + rows > m.src_seq_rows || m.dst_row0 + rows > m.dst_seq_rows)
      DH_FAIL(DH_ERR_SHAPE, "cp_exchange: move %d does not fit its buffers", k);
    if (((uintptr_t)m.src | (uintptr_t)m.dst) & 15) DH_FAIL(DH_ERR_INVALID_ARG, "cp_exchange: move %d is not 16-byte aligned", k);
    mv.m[k] = m;
  }
  const size_t want = ((size_t)n_moves * batch * rows * (width / 8) + 255) / 256, cap = n_blocks > 0 ? (size_t)n_blocks : 2048;
  const unsigned grid = (unsigned)(want < cap ? want : cap);
  if (dtype == DH_BF16) cp_exchange_kernel<bf16_t><<<grid, 256, 0, (hipStream_t)stream>>>(mv, batch, rows, width / 8);
  else cp_exchange_kernel<float><<<grid, 256, 0, (hipStream_t)stream>>>(mv, batch, rows, width / 8);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

// out rows = own rows + the peers' rows, added in index order in float32 (the key/value gradient a rank keeps:
// its own contribution plus what the later ranks send back).
template <typename T>
__global__ __launch_bounds__(256) void cp_grad_reduce_kernel(dh_cp_move own, PartPtrs peers, int n_peers, int batch, int rows, int w8) {
  const size_t total = (size_t)batch * rows * w8, stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int c = (int)(i % w8);
    const size_t t = i / w8;
    const int b = (int)(t / rows), r = (int)(t % rows);
    Vec8<T> acc;
    acc.load_stream((const T*)own.src + ((size_t)b * own.src_seq_rows + own.src_row0 + r) * own.src_ld + c * 8);
    for (int k = 0; k < n_peers; k++) {
      Vec8<T> v;
      v.load_stream((const T*)peers.p[k] + i * 8);
#pragma unroll
      for (int e = 0; e < 8; e++) acc.v[e] += v.v[e];
    }
    acc.store((T*)own.dst + ((size_t)b * own.dst_seq_rows + own.dst_row0 + r) * own.dst_ld + c * 8);
  }
}

extern "C" int dh_cp_grad_reduce(int dtype, const dh_cp_move* own, int n_peers, const void* const* peers, int batch, int rows,
                                 int width, int n_blocks, void* stream) {
  if (dtype != DH_F32 && dtype != DH_BF16) DH_FAIL(DH_ERR_INVALID_ARG, "cp_grad_reduce: dtype %d", dtype);
  if (n_peers < 0 || n_peers > DH_MAX_RANKS) DH_FAIL(DH_ERR_INVALID_ARG, "cp_grad_reduce: n_peers %d outside 0..%d", n_peers, DH_MAX_RANKS);
  if (batch < 0 || rows < 0 || width < 0 || width % 8) DH_FAIL(DH_ERR_SHAPE, "cp_grad_reduce: batch %d rows %d width %d", batch, rows, width);
  if (n_blocks < 0 || n_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "cp_grad_reduce: n_blocks %d outside 0..65536", n_blocks);
  if (batch * rows == 0 || width == 0) return DH_OK;
  if (!own || !own->src || !own->dst || (n_peers > 0 && !peers)) DH_FAIL(DH_ERR_INVALID_ARG, "cp_grad_reduce: null pointer");
  if (own->src_ld < width || own->dst_ld < width || own->src_ld % 8 || own->dst_ld % 8 || own->src_row0 < 0 || own->dst_row0 < 0 ||
      own->src_row0 + rows > own->src_seq_rows || own->dst_row0 + rows > own->dst_seq_rows)
    DH_FAIL(DH_ERR_SHAPE, "cp_grad_reduce: the own rows do not fit their buffers");
  if (((uintptr_t)own->src | (uintptr_t)own->dst) & 15) DH_FAIL(DH_ERR_INVALID_ARG, "cp_grad_reduce: buffers must be 16-byte aligned");
  PartPtrs pp;
  for (int k = 0; k < n_peers; k++) {
    if (!peers[k] || ((uintptr_t)peers[k] & 15)) DH_FAIL(DH_ERR_INVALID_ARG, "cp_grad_reduce: peer %d is null or misaligned", k);
    pp.p[k] = peers[k];
  }
  const size_t want = ((size_t)batch * rows * (width / 8) + 255) / 256, cap = n_blocks > 0 ? (size_t)n_blocks : 2048;
  const unsigned grid = (unsigned)(want < cap ? want : cap);
  if (dtype == DH_BF16) cp_grad_reduce_kernel<bf16_t><<<grid, 256, 0, (hipStream_t)stream>>>(*own, pp, n_peers, batch, rows, width / 8);
  else cp_grad_reduce_kernel<float><<<grid, 256, 0, (hipStream_t)stream>>>(*own, pp, n_peers, batch, rows, width / 8);
  DH_LAUNCH_CHECK();
  return DH_OK;
}

extern "C" int dh_stream_create_masked(int n_cus, void** stream) {
  if (!stream) DH_FAIL(DH_ERR_INVALID_ARG, "stream_create_masked: null pointer");
  int dev = 0;
  DH_HIP(hipGetDevice(&dev));
  hipDeviceProp_t prop;
  DH_HIP(hipGetDeviceProperties(&prop, dev));
  int total = prop.multiProcessorCount;
  if (n_cus < 1 || n_cus > total) DH_FAIL(DH_ERR_INVALID_ARG, "stream_create_masked: n_cus %d outside 1..%d", n_cus, total);
  // Enable n_cus bits spread evenly over the device's compute-unit index range.
  uint32_t mask[32] = {0};
  int words = (total + 31) / 32;
  for (int i = 0; i < n_cus; i++) {
    int cu = (int)(((long long)i * total) / n_cus);
    mask[cu / 32] |= 1u << (cu % 32);
  }
  hipStream_t s = nullptr;
  hipError_t e = hipExtStreamCreateWithCUMask(&s, (uint32_t)words, mask);
  if (e != hipSuccess) {
    (void)hipGetLastError();  // do not leave the failure behind for the caller's next HIP call
    return dh_set_error(DH_ERR_UNSUPPORTED, "compute-unit masks are not available on this system (%s)", hipGetErrorString(e));
  }
  *stream = (void*)s;
  return DH_OK;
}

extern "C" int dh_stream_destroy(void* stream) {
  if (!stream) return DH_OK;
  DH_HIP(hipStreamDestroy((hipStream_t)stream));
  return DH_OK;
}
