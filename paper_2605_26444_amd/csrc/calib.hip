// Measurement aids: read-only kernels that move the same bytes as the head without computing anything.
// They give the ceiling this chip reaches for one launch of a given size and access pattern (a
// contiguous stream, or whole rows fetched through an id list), which is what the head kernels are
// compared with besides the 8 TB/s specification.  Not part of the method.
#include "common.h"

namespace nanospec {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t fold(const u32x4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

// Every workgroup reads one contiguous piece of 256 * 16 * U bytes, U loads in flight per lane.
template <int U>
__global__ __launch_bounds__(256) void calib_stream_kernel(const u32x4* __restrict__ p, int64_t n16, uint32_t* __restrict__ sink) {
  const int64_t base = (int64_t)blockIdx.x * (256 * U) + threadIdx.x;
  u32x4 v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int64_t i = base + (int64_t)u * 256;
    v[u] = i < n16 ? p[i] : u32x4{0u, 0u, 0u, 0u};
  }
  uint32_t acc = 0;
#pragma unroll
  for (int u = 0; u < U; ++u) acc ^= fold(v[u]);
  if (acc == 0x9e3779b9u) sink[threadIdx.x] = acc;          // practically never true; keeps the loads alive
}

// One wavefront per listed row, the row's 16-byte pieces spread over the lanes, NL loads in flight.
template <int NL>
__global__ __launch_bounds__(256) void calib_gather_kernel(const char* __restrict__ W, int64_t row_bytes,
                                                           const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev,
                                                           int32_t V, uint32_t* __restrict__ sink) {
  const int row = (blockIdx.x * 256 + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (row >= n_dev[0]) return;
  int64_t id = ids[row];
  id = id < 0 ? 0 : (id >= V ? V - 1 : id);
  const u32x4* r = reinterpret_cast<const u32x4*>(W + id * row_bytes);
  const int pieces = (int)(row_bytes >> 4);
  uint32_t acc = 0;
  for (int p0 = 0; p0 < pieces; p0 += 64 * NL) {
    u32x4 v[NL];
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int i = p0 + u * 64 + lane;
      v[u] = i < pieces ? r[i] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int u = 0; u < NL; ++u) acc ^= fold(v[u]);
  }
  if (acc == 0x9e3779b9u) sink[threadIdx.x] = acc;
}

hipError_t launch_calib_stream(const void* buf, int64_t bytes, void* sink, hipStream_t s) {
  constexpr int U = 8;
  const int64_t n16 = bytes / 16;
  const int64_t blocks = (n16 + 256 * U - 1) / (256 * U);
  if (blocks < 1 || blocks > 0x7fffffff) return hipErrorInvalidValue;
  calib_stream_kernel<U><<<(unsigned)blocks, 256, 0, s>>>(static_cast<const u32x4*>(buf), n16, static_cast<uint32_t*>(sink));
  return hipGetLastError();
}

hipError_t launch_calib_gather(const void* W, int32_t V, int32_t d, const int32_t* ids, const int32_t* n_dev, int32_t cap,
                               void* sink, hipStream_t s) {
  calib_gather_kernel<8><<<(cap + 3) / 4, 256, 0, s>>>(static_cast<const char*>(W), (int64_t)d * 2, ids, n_dev, V,
                                                       static_cast<uint32_t*>(sink));
  return hipGetLastError();
}

}  // namespace nanospec
