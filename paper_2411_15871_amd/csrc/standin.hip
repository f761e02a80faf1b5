// One-GPU stand-ins for the collectives of the layer's critical path (tensor-parallel all-reduce,
// sequence-parallel all-gather and reduce-scatter).
// A stand-in moves the collective's payload through HBM: the reductions read the n_ranks partial
// buffers and write their sum, the all-gather copies the n_ranks shards behind one another.  It is meant to run on a stream restricted to a few compute units,
// so the grid is small and grid-strided: each thread streams 16-byte vectors.
#include "common.h"

#define DH_MAX_RANKS 16
struct PartPtrs {
  const void* p[DH_MAX_RANKS];
};

template <typename T>
__global__ __launch_bounds__(256) void allreduce_kernel(PartPtrs parts, int n_ranks, T* __restrict__ out, size_t n8) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
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
  if (kind != DH_COMM_ALLREDUCE && kind != DH_COMM_ALLGATHER && kind != DH_COMM_REDUCESCATTER)
    DH_FAIL(DH_ERR_UNSUPPORTED, "comm_standin: kind %d not supported", kind);
  if (n_ranks < 1 || n_ranks > DH_MAX_RANKS) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: n_ranks %d outside 1..%d", n_ranks, DH_MAX_RANKS);
  if (elems % 8) DH_FAIL(DH_ERR_SHAPE, "comm_standin: element count %zu must be a multiple of 8", elems);
  if (!parts || !out) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: null pointer");
  if (n_blocks < 0 || n_blocks > 65536) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: n_blocks %d outside 0..65536", n_blocks);
  PartPtrs pp;
  for (int r = 0; r < n_ranks; r++) {
    if (!parts[r]) DH_FAIL(DH_ERR_INVALID_ARG, "comm_standin: partial %d is null", r);
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
