// Draft-token selection (paper Alg. 1, SelectDraftTokens(z', I); operator T_K of Sec. 3.2):
// the k largest logits of every row, ordered by value descending then global id ascending, mapped
// from the position in the active list back to the global token id.
//
// A wavefront finds its k best by k rounds of a shuffle arg-max over per-lane candidates held in
// registers; the wavefronts' winners meet in LDS and one wavefront repeats the rounds over them.
// Rows longer than one workgroup's reach are cut into chunks whose winners a second kernel merges.
#include <limits.h>

#include "common.h"

namespace nanospec {

__device__ __forceinline__ bool better(float v1, int i1, float v2, int i2) {
  return v1 > v2 || (v1 == v2 && i1 < i2);
}

// k rounds over the EPT (value, index) pairs each lane holds; `mask` marks the live ones.
// Round r's winner is handed to emit(r, value, index) by every lane (index INT_MAX: none left).
template <int EPT, typename Emit>
__device__ __forceinline__ void wave_topk(const float (&val)[EPT], const int (&idx)[EPT], uint32_t mask, int k, Emit emit) {
  for (int r = 0; r < k; ++r) {
    float bv = -INFINITY;
    int bi = INT_MAX, be = -1;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      if (((mask >> e) & 1u) && better(val[e], idx[e], bv, bi)) {
        bv = val[e];
        bi = idx[e];
        be = e;
      }
    }
    const int mine = bi;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o);
      const int oi = __shfl_xor(bi, o);
      if (better(ov, oi, bv, bi)) {
        bv = ov;
        bi = oi;
      }
    }
    if (be >= 0 && mine == bi) mask &= ~(1u << be);
    emit(r, bv, bi);
  }
}

// One workgroup selects the k best of elements [c*CH, (c+1)*CH) of row (b, m), CH = EPT*THREADS.
// FINAL: write global ids / values; else write (value, position) candidates for the merge kernel.
template <int EPT, int THREADS, bool FINAL>
__global__ __launch_bounds__(THREADS) void topk_select_kernel(const float* __restrict__ logits, int64_t ld,
                                                             const int32_t* __restrict__ ids, int64_t ids_stride,
                                                             const int32_t* __restrict__ n_dev, int n_fixed, int M, int k,
                                                             int32_t* __restrict__ out_ids, float* __restrict__ out_vals,
                                                             float* __restrict__ cand_val, int32_t* __restrict__ cand_idx) {
  constexpr int NW = THREADS / 64;
  constexpr int CE = (NW * kMaxK + 63) / 64;
  __shared__ float s_val[NW * kMaxK];
  __shared__ int s_idx[NW * kMaxK];
  const int c = blockIdx.x, m = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = n_dev ? n_dev[b] : n_fixed;
  const int64_t row = (int64_t)b * M + m;
  const float* src = logits + row * ld;
  const int base = c * (EPT * THREADS);

  float val[EPT];
  int idx[EPT];
  uint32_t mask = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = base + e * THREADS + tid;
    idx[e] = j;
    val[e] = -INFINITY;
    if (j < n) {
      val[e] = src[j];
      mask |= 1u << e;
    }
  }
  wave_topk<EPT>(val, idx, mask, k, [&](int r, float v, int i) {
    if (lane == 0) {
      s_val[wave * k + r] = v;
      s_idx[wave * k + r] = i;
    }
  });
  __syncthreads();
  if (wave != 0) return;
  float cv[CE];
  int ci[CE];
  uint32_t cm = 0;
#pragma unroll
  for (int e = 0; e < CE; ++e) {
    const int q = e * 64 + lane;
    cv[e] = -INFINITY;
    ci[e] = INT_MAX;
    if (q < NW * k && s_idx[q] != INT_MAX) {
      cv[e] = s_val[q];
      ci[e] = s_idx[q];
      cm |= 1u << e;
    }
  }
  wave_topk<CE>(cv, ci, cm, k, [&](int r, float v, int i) {
    if (lane == 0) {
      if (FINAL) {
        const int64_t o = row * k + r;
        out_ids[o] = (i == INT_MAX) ? -1 : (ids ? ids[b * ids_stride + i] : i);
        if (out_vals) out_vals[o] = (i == INT_MAX) ? -INFINITY : v;
      } else {
        const int64_t o = (row * gridDim.x + c) * k + r;
        cand_val[o] = v;
        cand_idx[o] = (i == INT_MAX) ? -1 : i;
      }
    }
  });
}

// Merge the per-chunk winners of one row: at most nchunks*k <= 1024 candidates, 256 threads.
__global__ __launch_bounds__(256) void topk_merge_kernel(const float* __restrict__ cand_val, const int32_t* __restrict__ cand_idx,
                                                         int nchunks, const int32_t* __restrict__ ids, int64_t ids_stride,
                                                         int M, int k, int32_t* __restrict__ out_ids,
                                                         float* __restrict__ out_vals) {
  constexpr int NW = 4, EPT = 4, CE = (NW * kMaxK + 63) / 64;
  __shared__ float s_val[NW * kMaxK];
  __shared__ int s_idx[NW * kMaxK];
  const int m = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = (int64_t)b * M + m;
  const int total = nchunks * k;
  float val[EPT];
  int idx[EPT];
  uint32_t mask = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int q = e * 256 + tid;
    val[e] = -INFINITY;
    idx[e] = INT_MAX;
    if (q < total) {
      const int i = cand_idx[row * total + q];
      if (i >= 0) {
        val[e] = cand_val[row * total + q];
        idx[e] = i;
        mask |= 1u << e;
      }
    }
  }
  wave_topk<EPT>(val, idx, mask, k, [&](int r, float v, int i) {
    if (lane == 0) {
      s_val[wave * k + r] = v;
      s_idx[wave * k + r] = i;
    }
  });
  __syncthreads();
  if (wave != 0) return;
  float cv[CE];
  int ci[CE];
  uint32_t cm = 0;
#pragma unroll
  for (int e = 0; e < CE; ++e) {
    const int q = e * 64 + lane;
    cv[e] = -INFINITY;
    ci[e] = INT_MAX;
    if (q < NW * k && s_idx[q] != INT_MAX) {
      cv[e] = s_val[q];
      ci[e] = s_idx[q];
      cm |= 1u << e;
    }
  }
  wave_topk<CE>(cv, ci, cm, k, [&](int r, float v, int i) {
    if (lane == 0) {
      const int64_t o = row * k + r;
      out_ids[o] = (i == INT_MAX) ? -1 : (ids ? ids[b * ids_stride + i] : i);
      if (out_vals) out_vals[o] = (i == INT_MAX) ? -INFINITY : v;
    }
  });
}

static int chunks_for(int32_t cap) { return (cap + kTopkChunk - 1) / kTopkChunk; }

int64_t topk_workspace_bytes(int32_t cap, int32_t rows, int32_t k) {
  if (cap <= 4096) return 0;
  return (int64_t)rows * chunks_for(cap) * k * 8;
}

hipError_t launch_topk(const float* logits, int64_t ld, const int32_t* ids, int64_t ids_stride, const int32_t* n_dev,
                       int32_t n_fixed, int32_t cap, int32_t batch, int32_t M, int32_t k, int32_t* out_ids,
                       float* out_vals, char* ws, int64_t ws_bytes, hipStream_t s) {
  if (cap <= 4096) {
    topk_select_kernel<4, 1024, true><<<dim3(1, M, batch), 1024, 0, s>>>(logits, ld, ids, ids_stride, n_dev, n_fixed, M, k,
                                                                       out_ids, out_vals, nullptr, nullptr);
    return hipGetLastError();
  }
  const int nch = chunks_for(cap);
  const int64_t need = topk_workspace_bytes(cap, batch * M, k);
  if (nch * k > 1024 || ws == nullptr || ws_bytes < need) return hipErrorInvalidValue;
  float* cv = reinterpret_cast<float*>(ws);
  int32_t* ci = reinterpret_cast<int32_t*>(ws + need / 2);
  topk_select_kernel<16, 1024, false><<<dim3(nch, M, batch), 1024, 0, s>>>(logits, ld, ids, ids_stride, n_dev, n_fixed, M,
                                                                         k, nullptr, nullptr, cv, ci);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  topk_merge_kernel<<<dim3(1, M, batch), 256, 0, s>>>(cv, ci, nch, ids, ids_stride, M, k, out_ids, out_vals);
  return hipGetLastError();
}

}  // namespace nanospec
