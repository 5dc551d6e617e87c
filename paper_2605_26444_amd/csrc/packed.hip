// The paper's own system design as a component (Sec. 3.3 "Avoiding sparse computation via asynchronous
// gathering"; the weight-gather row of Table 4; the repacked-weights row of Table 6): a pre-allocated packed
// buffer holds one copy of every active row; after a vocabulary update only the rows of ids that entered the
// active set are copied in -- on a stream of the caller's choice, so that the copy hides behind the draft
// backbone -- and the head is a dense product on the packed buffer.
//
// Slots are stable: an id keeps its slot while it stays active, a leaving id frees its slot, an entering id
// takes the lowest free one.  Slot order is therefore not id order; the head kernels write the logits of the row
// in slot s to the column out_pos[s] = position of that id in the ascending active list, so logits come out in
// exactly the layout of nanospec_sparse_head and the selection (ties by lower id) applies unchanged.
#include "common.h"

namespace nanospec {

constexpr int kSyncThreads = 1024;

// exclusive rank of `pred` among the workgroup's threads in thread order, and the workgroup total; sc: 17 ints of LDS
__device__ __forceinline__ int block_rank(bool pred, int* sc, int* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long bal = __ballot(pred);
  const int before = __popcll(bal & ((1ull << lane) - 1ull));
  __syncthreads();                                   // sc may still be read from the previous call
  if (lane == 0) sc[wave] = __popcll(bal);
  __syncthreads();
  int off = 0, tot = 0;
  for (int w = 0; w < kSyncThreads / 64; ++w) {
    const int t = sc[w];
    off += w < wave ? t : 0;
    tot += t;
  }
  *total = tot;
  return off + before;
}

// One workgroup: bring slot tables in line with the active list of sequence 0.
//   1. every slot whose id is no longer active (window bitmap | T bitmap) is freed;
//   2. the free slots are listed in ascending order;
//   3. every active id without a slot takes the next free one and goes on the copy list;
//   4. out_pos[slot] = position of the slot's id in the ascending list; hi = slots that may hold a row.
__global__ __launch_bounds__(kSyncThreads) void packed_sync_kernel(VocabPtrs p, PackedPtrs k) {
  __shared__ int sc[32];
  const int tid = threadIdx.x;
  const int n = p.n[0], cap = k.cap;
  int nfree = 0;
  for (int s0 = 0; s0 < cap; s0 += kSyncThreads) {
    const int s = s0 + tid;
    bool isfree = false;
    if (s < cap) {
      const int id = k.slot_id[s];
      isfree = id < 0;
      if (id >= 0) {
        const uint32_t bits = p.wbit[id >> 5] | p.tbit[id >> 5];
        if (!((bits >> (id & 31)) & 1u)) {
          k.slot_of[id] = -1;
          k.slot_id[s] = -1;
          k.out_pos[s] = -1;
          isfree = true;
        }
      }
    }
    int tot;
    const int r = block_rank(isfree, sc, &tot);
    if (isfree) k.free_list[nfree + r] = s;
    nfree += tot;
  }
  __syncthreads();                                   // free_list and slot_of are complete (one workgroup, one L1)
  int ncopy = 0, top = -1;
  for (int j0 = 0; j0 < n; j0 += kSyncThreads) {
    const int j = j0 + tid;
    int id = -1, sl = -1;
    if (j < n) {
      id = p.ids[j];
      sl = k.slot_of[id];
    }
    const bool fresh = j < n && sl < 0;
    int tot;
    const int r = block_rank(fresh, sc, &tot);
    if (fresh) {
      sl = k.free_list[ncopy + r];                   // n <= cap and every active id holds one slot: there is one
      k.slot_of[id] = sl;
      k.slot_id[sl] = id;
      k.copy_list[2 * (ncopy + r)] = id;
      k.copy_list[2 * (ncopy + r) + 1] = sl;
    }
    if (j < n) k.out_pos[sl] = j;
    top = max(top, sl);
    ncopy += tot;
  }
  // highest slot in use
  for (int o = 32; o > 0; o >>= 1) top = max(top, __shfl_xor(top, o));
  __syncthreads();
  if ((tid & 63) == 0) sc[tid >> 6] = top;
  __syncthreads();
  if (tid == 0) {
    int t = -1;
    for (int w = 0; w < kSyncThreads / 64; ++w) t = max(t, sc[w]);
    k.scal[0] = t + 1;                               // hi
    k.scal[1] = ncopy;
  }
}

// Copy the listed rows W[id] -> buf[slot]: the weight-gather kernel.  Workgroup x takes list entries x, x + grid, ...
__global__ __launch_bounds__(256) void packed_copy_kernel(const uint4* __restrict__ W, PackedPtrs k, int row_vec /* 16-byte pieces per row */) {
  const int ncopy = k.scal[1];
  uint4* buf = reinterpret_cast<uint4*>(k.buf);
  for (int e = blockIdx.x; e < ncopy; e += gridDim.x) {
    const int64_t id = k.copy_list[2 * e], sl = k.copy_list[2 * e + 1];
    const uint4* src = W + id * row_vec;
    uint4* dst = buf + sl * row_vec;
    for (int i = threadIdx.x; i < row_vec; i += 256) dst[i] = src[i];
  }
}

__global__ __launch_bounds__(256) void packed_reset_kernel(PackedPtrs k, int V) {
  const int i = blockIdx.x * 256 + threadIdx.x, stride = gridDim.x * 256;
  for (int v = i; v < V; v += stride) k.slot_of[v] = -1;
  for (int s = i; s < k.cap; s += stride) {
    k.slot_id[s] = -1;
    k.out_pos[s] = -1;
  }
  if (i == 0) {
    k.scal[0] = 0;
    k.scal[1] = 0;
  }
}

hipError_t launch_packed_reset(const nanospec_state* st, hipStream_t s) {
  packed_reset_kernel<<<256, 256, 0, s>>>(st->pk, st->V);
  return hipGetLastError();
}

hipError_t launch_packed_gather(const nanospec_state* st, const void* W, hipStream_t s) {
  packed_sync_kernel<<<1, kSyncThreads, 0, s>>>(st->vp, st->pk);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int grid = st->pk.cap < 1024 ? st->pk.cap : 1024;
  packed_copy_kernel<<<grid, 256, 0, s>>>(static_cast<const uint4*>(W), st->pk, st->d / 8);
  return hipGetLastError();
}

}  // namespace nanospec
