// Several sequences in one batch (multi-sequence serving; Sec. 4.6 notes that the per-sequence cost of the method
// adds up over the batch): sequences that draw from one token distribution hold many of the same ids, and the
// per-sequence head fetches such a row once per sequence that holds it.  Here the active sets are split:
//   * an id held by at least min_share sequences is a *shared* row -- listed once (ascending, at most shared_cap
//     of them), fetched once and multiplied with the hidden rows of all sequences; a sequence that does not hold
//     it simply has no column for it;
//   * everything else stays on a per-sequence list and goes through the per-sequence head as before.
// Every (sequence, active id) pair is covered by exactly one of the two parts and its logit lands in the column
// the id has in that sequence's ascending active list, so the logits have the layout of nanospec_sparse_head and
// the selection applies unchanged.
#include "common.h"

namespace nanospec {

constexpr int kListThreads = 1024;

// One wavefront per bitmap word: lane q looks at sequence q's word (window bitmap | T bitmap); 32 ballots count,
// for every bit, the sequences that hold the id.
__global__ __launch_bounds__(1024) void union_count_kernel(VocabPtrs p, UnionPtrs u, int batch) {
  const int lane = threadIdx.x & 63;
  const int w = blockIdx.x * 16 + (threadIdx.x >> 6);
  if (w >= p.nwords) return;
  int cnt[32];
#pragma unroll
  for (int i = 0; i < 32; ++i) cnt[i] = 0;
  for (int b0 = 0; b0 < batch; b0 += 64) {
    const int b = b0 + lane;
    uint32_t word = 0u;
    if (b < batch) word = p.wbit[(size_t)b * p.nwords + w] | p.tbit[(size_t)b * p.nwords + w];
#pragma unroll
    for (int i = 0; i < 32; ++i) cnt[i] += __popcll(__ballot((word >> i) & 1u));
  }
  uint32_t pop = 0u;
#pragma unroll
  for (int i = 0; i < 32; ++i) pop |= (cnt[i] >= u.min_share ? 1u : 0u) << i;
  if (lane == 0) {
    u.shared_bits[w] = pop;
    u.shared_cnt[w] = __popc(pop);
  }
}

// exclusive rank of `pred` among the workgroup's threads in thread order, and the workgroup total; sc: 17 ints of LDS
__device__ __forceinline__ int list_rank(bool pred, int* sc, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(pred);
  const int before = __popcll(bal & ((1ull << lane) - 1ull));
  __syncthreads();                                   // sc may still be read from the previous call
  if (lane == 0) sc[wave] = __popcll(bal);
  __syncthreads();
  int off = 0, tot = 0;
  for (int w = 0; w < kListThreads / 64; ++w) {
    const int t = sc[w];
    off += w < wave ? t : 0;
    tot += t;
  }
  *total = tot;
  return off + before;
}

// One workgroup per sequence.  Every workgroup scans the per-word counts of shared ids (a few thousand words) into
// LDS so that the rank of a shared id is one look-up; workgroup 0 also writes the shared list.  Then the
// sequence's ascending id list is walked once: a shared id records its position in the sequence's column table,
// any other id is appended to the sequence's own list together with its position.
__global__ __launch_bounds__(kListThreads) void union_lists_kernel(VocabPtrs p, UnionPtrs u, int groups) {
  extern __shared__ int pre[];                       // [nwords] exclusive prefix of shared_cnt, then 32 ints of scratch
  int* sc = pre + p.nwords;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x;
  int base = 0;
  for (int w0 = 0; w0 < p.nwords; w0 += kListThreads) {
    const int w = w0 + tid;
    const int c = w < p.nwords ? u.shared_cnt[w] : 0;
    int incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o);
      if (lane >= o) incl += t;
    }
    __syncthreads();
    if (lane == 63) sc[wave] = incl;
    __syncthreads();
    int off = 0, tot = 0;
    for (int ww = 0; ww < kListThreads / 64; ++ww) {
      const int t = sc[ww];
      off += ww < wave ? t : 0;
      tot += t;
    }
    if (w < p.nwords) pre[w] = base + off + incl - c;
    base += tot;
  }
  const int ns = base < u.shared_cap ? base : u.shared_cap;     // shared rows that fit the list
  __syncthreads();
  if (b == 0) {
    for (int w = tid; w < p.nwords; w += kListThreads) {
      uint32_t bits = u.shared_bits[w];
      int r = pre[w];
      while (bits && r < u.shared_cap) {
        const int i = __ffs(bits) - 1;
        u.shared_ids[r++] = w * 32 + i;
        bits &= bits - 1u;
      }
    }
    for (int g = tid; g < groups; g += kListThreads) u.shared_n[g] = ns;
  }
  int32_t* mypos = u.shared_pos + (size_t)b * u.shared_cap;
  for (int r = tid; r < u.shared_cap; r += kListThreads) mypos[r] = -1;
  __syncthreads();                                   // the -1s are out (one workgroup, one L1) before positions overwrite some
  const int n = p.n[b];
  const int32_t* ids = p.ids + (size_t)b * p.cap;
  int32_t* rid = u.rest_ids + (size_t)b * p.cap;
  int32_t* rpos = u.rest_pos + (size_t)b * p.cap;
  int nrest = 0;
  for (int j0 = 0; j0 < n; j0 += kListThreads) {
    const int j = j0 + tid;
    int id = 0;
    bool rest = false;
    if (j < n) {
      id = ids[j];
      const uint32_t bits = u.shared_bits[id >> 5];
      const int r = pre[id >> 5] + __popc(bits & ((1u << (id & 31)) - 1u));
      if (((bits >> (id & 31)) & 1u) && r < u.shared_cap) mypos[r] = j;
      else rest = true;
    }
    int tot;
    const int r = list_rank(rest, sc, &tot);
    if (rest) {
      rid[nrest + r] = id;
      rpos[nrest + r] = j;
    }
    nrest += tot;
  }
  if (tid == 0) u.rest_n[b] = nrest;
}

__global__ __launch_bounds__(256) void union_reset_kernel(UnionPtrs u, int batch, int cap, int groups) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x, stride = (int64_t)gridDim.x * 256;
  for (int64_t x = i; x < (int64_t)batch * cap; x += stride) {
    u.rest_ids[x] = 0;
    u.rest_pos[x] = -1;
  }
  for (int64_t x = i; x < (int64_t)batch * u.shared_cap; x += stride) u.shared_pos[x] = -1;
  for (int64_t x = i; x < u.shared_cap; x += stride) u.shared_ids[x] = 0;
  for (int64_t x = i; x < batch; x += stride) u.rest_n[x] = 0;
  for (int64_t x = i; x < groups; x += stride) u.shared_n[x] = 0;
}

hipError_t union_configure_device() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(union_lists_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

hipError_t launch_union_reset(const nanospec_state* st, hipStream_t s) {
  union_reset_kernel<<<256, 256, 0, s>>>(st->un, st->batch, st->vp.cap, st->un_groups);
  return hipGetLastError();
}

hipError_t launch_union_build(const nanospec_state* st, hipStream_t s) {
  union_count_kernel<<<(st->vp.nwords + 15) / 16, 1024, 0, s>>>(st->vp, st->un, st->batch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  union_lists_kernel<<<st->batch, kListThreads, (st->vp.nwords + 32) * 4, s>>>(st->vp, st->un, st->un_groups);
  return hipGetLastError();
}

}  // namespace nanospec
