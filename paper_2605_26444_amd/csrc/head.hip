// LM-head projection onto a gathered set of rows (paper Sec. 3.1: Eq. 1 restricted to I_t) and onto
// all rows (Eq. 1, the dense comparison point).  The rows are read straight from W_head inside the
// projection; no packed copy is made.
#include "common.h"

namespace nanospec {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ float dot8(const u32x4 w, const u32x4 h, float acc) {
  acc = fmaf(bf_lo(w.x), bf_lo(h.x), acc);
  acc = fmaf(bf_hi(w.x), bf_hi(h.x), acc);
  acc = fmaf(bf_lo(w.y), bf_lo(h.y), acc);
  acc = fmaf(bf_hi(w.y), bf_hi(h.y), acc);
  acc = fmaf(bf_lo(w.z), bf_lo(h.z), acc);
  acc = fmaf(bf_hi(w.z), bf_hi(h.z), acc);
  acc = fmaf(bf_lo(w.w), bf_lo(h.w), acc);
  acc = fmaf(bf_hi(w.w), bf_hi(h.w), acc);
  return acc;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
  return x;
}

// Any-shape fallback: one wavefront per gathered row, hidden rows re-read through the caches in
// tiles of MT.  Correct for every (M, d % 8 == 0); the tuned kernels below take the common shapes.
template <int MT>
__global__ __launch_bounds__(256) void head_generic_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H,
                                                           const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev,
                                                           int n_fixed, int M, int d, int64_t ld, int64_t ids_stride,
                                                           float* __restrict__ logits) {
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = n_dev ? n_dev[b] : n_fixed;
  const int j = blockIdx.x * 4 + wave;
  if (j >= n) return;
  const int64_t row = ids ? ids[b * ids_stride + j] : j;
  const uint16_t* w = W + row * d;
  for (int m0 = 0; m0 < M; m0 += MT) {
    float acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) acc[t] = 0.f;
    for (int c = lane * 8; c < d; c += 512) {
      const u32x4 wv = *reinterpret_cast<const u32x4*>(w + c);
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        if (m0 + t < M) {
          const u32x4 hv = *reinterpret_cast<const u32x4*>(H + ((int64_t)b * M + m0 + t) * d + c);
          acc[t] = dot8(wv, hv, acc[t]);
        }
      }
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const float s = wave_sum(acc[t]);
      if (lane == 0 && m0 + t < M) logits[((int64_t)b * M + m0 + t) * ld + j] = s;
    }
  }
}

hipError_t launch_head(const void* W, const void* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed,
                       int32_t cap_rows, int32_t batch, int32_t M, int32_t d, int64_t ld_logits, int64_t ids_stride,
                       float* logits, float* partial, int64_t partial_bytes, hipStream_t s) {
  (void)partial;
  (void)partial_bytes;
  dim3 grid((cap_rows + 3) / 4, 1, batch);
  head_generic_kernel<8><<<grid, 256, 0, s>>>(static_cast<const uint16_t*>(W), static_cast<const uint16_t*>(H), ids,
                                              n_dev, n_fixed, M, d, ld_logits, ids_stride, logits);
  return hipGetLastError();
}

}  // namespace nanospec
