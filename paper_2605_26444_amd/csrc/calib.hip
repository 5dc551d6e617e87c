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

// The few-hidden-rows head on the vector ALUs instead of the matrix cores, for measurement: the arithmetic unit is
// the only thing that differs from head_quad_kernel's largest shape.  A workgroup of sixteen wavefronts owns
// sixteen rows: wavefront (kq, rg) takes rows 4*rg .. 4*rg+3 and K-quarter kq; a lane loads 16 bytes (8 columns)
// of each row per 512-column chunk -- one fully coalesced 1 KB instruction per row and chunk, all in flight
// together --, the hidden rows sit in LDS in their natural layout, every lane multiplies its 8 columns with the
// 8 hidden rows (bf16 widened to fp32 by a shift or a mask, fused multiply-add), the 32 per-lane sums are folded
// across the wavefront by a halving butterfly and the four K-quarters are added in fixed order through LDS.
template <int NCH>   // 512-column chunks per K-quarter: d = 2048 * NCH
__global__ __launch_bounds__(1024) void head_valu_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H,
                                                         const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev,
                                                         int V, int M, int64_t ld, float* __restrict__ logits) {
  constexpr int d = 2048 * NCH, QK = 512 * NCH, MH = 8;
  extern __shared__ __attribute__((aligned(16))) char hs[];            // H [8][d] bf16, then the K-quarter sums
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int kq = w & 3, rg = w >> 2;
  const int j0 = blockIdx.x * 16 + rg * 4;
  const int4 idv = *reinterpret_cast<const int4*>(ids + j0);            // capacity-bounded
  const int n = n_dev[0];
  for (int i = threadIdx.x; i < MH * d / 8; i += 1024) {                // hidden rows past M: zeros
    const int m = i / (d / 8);
    reinterpret_cast<u32x4*>(hs)[i] = m < M ? reinterpret_cast<const u32x4*>(H)[i] : u32x4{0u, 0u, 0u, 0u};
  }
  const int idr[4] = {idv.x, idv.y, idv.z, idv.w};
  u32x4 wv[4][NCH];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    int64_t row = idr[r] < 0 ? 0 : (idr[r] >= V ? V - 1 : idr[r]);
    row = j0 + r < n ? row : 0;
#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) wv[r][ch] = *reinterpret_cast<const u32x4*>(W + row * d + kq * QK + ch * 512 + lane * 8);
  }
  __syncthreads();
  float acc[4 * MH];
#pragma unroll
  for (int i = 0; i < 4 * MH; ++i) acc[i] = 0.f;
#pragma unroll
  for (int ch = 0; ch < NCH; ++ch) {
    float wf[4][8];                                                      // this chunk's weights widened once, used by all hidden rows
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const uint32_t wu[4] = {wv[r][ch].x, wv[r][ch].y, wv[r][ch].z, wv[r][ch].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        wf[r][2 * i] = __uint_as_float(wu[i] << 16);
        wf[r][2 * i + 1] = __uint_as_float(wu[i] & 0xffff0000u);
      }
    }
#pragma unroll
    for (int m = 0; m < MH; ++m) {
      const u32x4 hv = *reinterpret_cast<const u32x4*>(hs + ((int64_t)m * d + kq * QK + ch * 512 + lane * 8) * 2);
      const uint32_t hu[4] = {hv.x, hv.y, hv.z, hv.w};
      float hf[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        hf[2 * i] = __uint_as_float(hu[i] << 16);
        hf[2 * i + 1] = __uint_as_float(hu[i] & 0xffff0000u);
      }
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[r * MH + m] = fmaf(wf[r][i], hf[i], acc[r * MH + m]);
      __builtin_amdgcn_sched_barrier(0);                                 // one hidden row's operands at a time (registers)
    }
  }
  // fold the 32 sums across the 64 lanes: at each step a lane keeps half of its values and adds its partner's
  // copies of them; after xor 32, 16, 8, 4, 2 one value is left, shared with lane ^ 1
  int cnt = 4 * MH;
#pragma unroll
  for (int o = 32; o >= 2; o >>= 1) {
    cnt >>= 1;
    const bool upper = (lane & o) != 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (i < cnt) {
        const float keep = upper ? acc[i + cnt] : acc[i];
        const float give = upper ? acc[i] : acc[i + cnt];
        acc[i] = keep + __shfl_xor(give, o);
      }
    }
  }
  float x = acc[0] + __shfl_xor(acc[0], 1);
  // lane l holds value index v = bit-reversed choice: bit for step o is set iff (lane & o): index = sum over steps
  int v = 0;
  {
    int c = 4 * MH;
#pragma unroll
    for (int o = 32; o >= 2; o >>= 1) {
      c >>= 1;
      if (lane & o) v += c;
    }
  }
  float* red = reinterpret_cast<float*>(hs + (int64_t)MH * d * 2);       // [16 waves][32]
  if ((lane & 1) == 0) red[w * 32 + v] = x;
  __syncthreads();
  if (threadIdx.x < 4 * 32) {
    const int g = threadIdx.x >> 5, vv = threadIdx.x & 31, r = vv / MH, m = vv % MH;
    const int j = blockIdx.x * 16 + g * 4 + r;
    if (j < n && m < M) {
      const float* rr = red + (g * 4) * 32 + vv;
      logits[(int64_t)m * ld + j] = ((rr[0] + rr[32]) + rr[64]) + rr[96];
    }
  }
}

hipError_t launch_calib_valu_head(const void* W, const void* H, int32_t V, int32_t d, int32_t M, const int32_t* ids,
                                  const int32_t* n_dev, int32_t cap, float* logits, hipStream_t s) {
  const int lds = 8 * d * 2 + 16 * 32 * 4;
  const dim3 grid((cap + 15) / 16);
  const uint16_t* Wp = static_cast<const uint16_t*>(W);
  const uint16_t* Hp = static_cast<const uint16_t*>(H);
  if (d == 4096) head_valu_kernel<2><<<grid, 1024, lds, s>>>(Wp, Hp, ids, n_dev, V, M, cap, logits);
  else if (d == 2048) head_valu_kernel<1><<<grid, 1024, lds, s>>>(Wp, Hp, ids, n_dev, V, M, cap, logits);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t calib_configure_device() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(head_valu_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(head_valu_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  return e;
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
