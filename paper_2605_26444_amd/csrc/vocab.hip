// Context-aware active vocabulary kept on the GPU (paper Sec. 3.2 Eq. 2-4, Sec. 3.3 "GPU-resident
// state management").
//
// Per sequence the state is: a ring of the last `window` stream ids, a multiplicity counter per
// token id (how many times it occurs inside the window), a window bitmap (counter > 0), a bitmap of
// the extra candidate set T, and the compacted ascending id list I with its count.  One workgroup
// per sequence applies an update in ONE launch: counters are adjusted with atomics for every id that
// leaves or enters the window; the decrement that reaches zero clears the bit and, after a barrier,
// every entering id sets it (so an id that is evicted and re-appended in the same call ends up
// correct whatever order the atomics landed in), and the union bitmap is compacted with popcounts
// and a workgroup prefix scan.  Both bitmaps live in LDS during the kernel.  A short append that leaves T
// alone -- the decoding step -- does not rebuild the list: it patches it in place (vocab_apply_incremental).
// The paper's other description of the same state -- a first-in first-out queue of at most `window`
// distinct ids -- is the second half of this file (vocab_fifo_kernel).
#include <limits.h>

#include "common.h"

namespace nanospec {

__global__ __launch_bounds__(256) void vocab_clear_kernel(VocabPtrs p, int batch) {
  const size_t tid = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t ncnt = (size_t)batch * p.V;
  for (size_t i = tid; i < ncnt; i += stride) p.cnt[i] = 0u;
  const size_t nbit = (size_t)batch * p.nwords;
  for (size_t i = tid; i < nbit; i += stride) {
    p.wbit[i] = 0u;
    p.tbit[i] = 0u;
  }
  for (size_t i = tid; i < (size_t)batch; i += stride) {
    p.n[i] = 0;
    p.pos[i] = 0;
    p.fill[i] = 0;
  }
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_add_int(int x) {
  return x + __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xf, false);   // lanes without a source add 0
}

// inclusive prefix sum over the 64 lanes: Hillis-Steele inside each row of 16 (row_shr 1/2/4/8), then the
// row totals carried across (row_bcast:15 into rows 1 and 3, row_bcast:31 into rows 2 and 3)
__device__ __forceinline__ int wave_incl_scan(int x, int /*lane*/) {
  x = dpp_add_int<0x111, 0xf>(x);
  x = dpp_add_int<0x112, 0xf>(x);
  x = dpp_add_int<0x114, 0xf>(x);
  x = dpp_add_int<0x118, 0xf>(x);
  x = dpp_add_int<0x142, 0xa>(x);
  x = dpp_add_int<0x143, 0xc>(x);
  return x;
}

// Ascending compaction of a bitmap held in LDS: popcount per thread, workgroup exclusive scan,
// emission in id order.  word4(i) yields bitmap words i..i+3 (i a multiple of 4); out[0..total) receives
// the ids (at most cap are stored).  Every thread of the workgroup must call it, after a barrier that
// separates it from any earlier use of sc; returns the number of set bits.  A thread's words (4 for
// vocabularies up to 131072 ids, 8 up to 262144) stay in registers between the count and the emission.
template <typename Word4Fn>
__device__ __forceinline__ int compact_bitmap(Word4Fn word4, int nwords, int32_t* out, int cap, int* sc, int tid) {
  const int lane = tid & 63, wave = tid >> 6;
  const int wpt = (((nwords + kVocabThreads - 1) / kVocabThreads) + 3) & ~3;
  const int w0 = tid * wpt;
  constexpr int kKeep = 8;
  uint32_t keep[kKeep];
  int mine = 0;
#pragma unroll
  for (int c = 0; c < kKeep / 4; ++c) {
    const int i = w0 + 4 * c;
    uint4 x = make_uint4(0, 0, 0, 0);
    if (4 * c < wpt && i < nwords) x = word4(i);
    keep[4 * c] = x.x;
    keep[4 * c + 1] = x.y;
    keep[4 * c + 2] = x.z;
    keep[4 * c + 3] = x.w;
    mine += __popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w);
  }
  for (int i = w0 + kKeep; i < w0 + wpt && i < nwords; i += 4) {   // vocabularies above 262144 ids
    const uint4 x = word4(i);
    mine += __popc(x.x) + __popc(x.y) + __popc(x.z) + __popc(x.w);
  }
  const int incl = wave_incl_scan(mine, lane);
  if (lane == 63) sc[wave] = incl;
  __syncthreads();
  int off = incl - mine, total = 0;
#pragma unroll
  for (int w = 0; w < kVocabThreads / 64; w += 4) {
    const int4 t = *reinterpret_cast<const int4*>(sc + w);
    off += (w < wave ? t.x : 0) + (w + 1 < wave ? t.y : 0) + (w + 2 < wave ? t.z : 0) + (w + 3 < wave ? t.w : 0);
    total += t.x + t.y + t.z + t.w;
  }
  // Emission costs one trip round a short loop per set bit and wavefront-wide per word (the lane with the
  // most bits sets the pace), on a workgroup whose sixteen wavefronts share four SIMDs: it is bound by
  // instruction issue, so the loop is kept to the bare minimum -- two words at a time as one 64-bit
  // value, an unsigned 32-bit list index (base register + offset addressing), and the capacity test
  // hoisted out (the list fits unless T is larger than the state was created for).
  uint32_t uo = (uint32_t)off;
  const bool fits = total <= cap;
  auto emit2 = [&](uint32_t lo, uint32_t hi, int base) {
    unsigned long long x = ((unsigned long long)hi << 32) | lo;
    if (fits) {
      while (x) {
        out[uo++] = base + __ffsll((long long)x) - 1;
        x &= x - 1ull;
      }
    } else {
      while (x) {
        if (uo < (uint32_t)cap) out[uo] = base + __ffsll((long long)x) - 1;
        ++uo;
        x &= x - 1ull;
      }
    }
  };
#pragma unroll
  for (int q = 0; q < kKeep; q += 2) emit2(keep[q], keep[q + 1], (w0 + q) * 32);   // words past the end are zero
  for (int i = w0 + kKeep; i < w0 + wpt && i < nwords; i += 4) {
    const uint4 x = word4(i);
    emit2(x.x, x.y, i * 32);
    emit2(x.z, x.w, (i + 2) * 32);
  }
  return total;
}

// One stream update of sequence b (Eq. 3 then Eq. 4): append src[0..a), evict what leaves the window,
// optionally replace T, rebuild the ascending active list.  wb/tb are the LDS copies of the bitmaps
// (their stores have been issued by this workgroup; the body's first barrier completes them before
// any bit is changed), sc 16 ints of LDS scratch.
__device__ __forceinline__ void vocab_apply_body(const VocabPtrs& p, int b, const int32_t* src, int a,
                                                 const int32_t* ts, int nt, int replace_T, uint32_t* wb, uint32_t* tb,
                                                 int* sc, int bad) {
  const int tid = threadIdx.x;
  const int nwords = p.nwords, V = p.V, W = p.window;
  uint32_t* gw = p.wbit + (size_t)b * nwords;
  uint32_t* gt = p.tbit + (size_t)b * nwords;
  uint32_t* cnt = p.cnt + (size_t)b * V;
  int32_t* ring = p.ring + (size_t)b * W;

  const int pos = p.pos[b], fill = p.fill[b];
  const int skip = a > W ? a - W : 0;      // ids that enter and leave the window within this call
  const int ae = a - skip;
  int n_evict = fill + ae - W;
  if (n_evict < 0) n_evict = 0;
  int oldest = pos - fill;
  if (oldest < 0) oldest += W;

  // Leaving ids first: -1 on the counter with a returning atomic; the decrement that brings a
  // counter to zero (whichever thread performs it) clears the window bit.  Entering ids get their +1
  // without waiting for the result: they are inside the window afterwards whatever the order of the
  // two atomics was, so their bit is simply set -- after the barrier, so that a clear of the same id
  // by the eviction pass cannot come last.
  // The LDS bitmaps were filled by other threads just before this call: the first pass keeps its result
  // in a register until a barrier has made those copies complete; later passes (appends longer than
  // the workgroup) clear directly.
  {
    int e0 = -1;
    if (tid < n_evict) {
      int slot = oldest + tid;
      if (slot >= W) slot -= W;
      const int e = ring[slot];
      if (e >= 0 && atomicSub(&cnt[e], 1u) == 1u) e0 = e;
    }
    __syncthreads();
    if (e0 >= 0) atomicAnd(&wb[e0 >> 5], ~(1u << (e0 & 31)));
  }
  for (int i = tid + kVocabThreads; i < n_evict; i += kVocabThreads) {
    int slot = oldest + i;
    if (slot >= W) slot -= W;
    const int e = ring[slot];
    if (e >= 0) {
      const uint32_t old = atomicSub(&cnt[e], 1u);
      if (old == 1u) atomicAnd(&wb[e >> 5], ~(1u << (e & 31)));
    }
  }
  for (int i = tid; i < skip; i += kVocabThreads) bad |= ((unsigned)src[i] >= (unsigned)V);
  __syncthreads();   // every ring slot about to be overwritten has been read, every clear is done

  for (int i = tid; i < ae; i += kVocabThreads) {
    const int v = src[skip + i];
    const bool ok = (unsigned)v < (unsigned)V;
    if (ok) {
      atomicAdd(&cnt[v], 1u);
      atomicOr(&wb[v >> 5], 1u << (v & 31));
    } else {
      bad = 1;
    }
    int slot = pos + i;
    if (slot >= W) slot -= W;
    ring[slot] = ok ? v : -1;
  }
  if (replace_T) {
    for (int i = tid; i < nt; i += kVocabThreads) {
      const int t = ts[i];
      if ((unsigned)t < (unsigned)V) atomicOr(&tb[t >> 5], 1u << (t & 31));
      else bad = 1;
    }
  }
  __syncthreads();

  // compaction of (window | T)
  const int total = compact_bitmap(
      [&](int i) {
        const uint4 a = *reinterpret_cast<const uint4*>(wb + i), c = *reinterpret_cast<const uint4*>(tb + i);
        return make_uint4(a.x | c.x, a.y | c.y, a.z | c.z, a.w | c.w);
      }, nwords, p.ids + (size_t)b * p.cap, p.cap, sc, tid);
  // bitmaps back to HBM
  for (int i = tid * 4; i < nwords; i += kVocabThreads * 4) {
    *reinterpret_cast<uint4*>(gw + i) = *reinterpret_cast<const uint4*>(wb + i);
    if (replace_T) *reinterpret_cast<uint4*>(gt + i) = *reinterpret_cast<const uint4*>(tb + i);
  }
  if (tid == 0) {
    p.n[b] = total < p.cap ? total : p.cap;
    int np = pos + ae;
    if (np >= W) np -= W;
    p.pos[b] = np;
    const int nf = fill + ae;
    p.fill[b] = nf < W ? nf : W;
  }
  if (bad) atomicOr(p.err, (int)NANOSPEC_DEV_BAD_ID);
}

__device__ __forceinline__ void load_bitmaps(const VocabPtrs& p, int b, uint32_t* wb, uint32_t* tb, int replace_T) {
  const uint32_t* gw = p.wbit + (size_t)b * p.nwords;
  const uint32_t* gt = p.tbit + (size_t)b * p.nwords;
  for (int i = threadIdx.x * 4; i < p.nwords; i += kVocabThreads * 4) {
    *reinterpret_cast<uint4*>(wb + i) = *reinterpret_cast<const uint4*>(gw + i);
    *reinterpret_cast<uint4*>(tb + i) = replace_T ? make_uint4(0, 0, 0, 0) : *reinterpret_cast<const uint4*>(gt + i);
  }
}

// A short append (at most kIncMax ids, T untouched) changes the active list in at most 2*kIncMax places,
// so the list is patched instead of rebuilt.  The bitmaps stay in HBM.  The first wavefront does all of
// the bookkeeping: lanes 0..15 take the ring slots that leave the window, lanes 16..31 the appended ids;
// lanes that hold the same id are found by comparing (a handful of readlanes), the first of them reads the
// id's counter, adds the net change and writes it back -- no atomics, nobody else touches this sequence --
// and a counter that becomes or stops being zero flips the window bit.  Such an id leaves / enters the
// active set unless T holds it.  Every thread then moves its four list entries by (entered ids below) -
// (left ids below); an entered id is written by the thread that holds its predecessor.  The result is
// the list a full compaction would give; when nothing entered or left -- the usual case for text that
// repeats itself -- the list is not touched at all.
// Returns false, before anything has been changed, when the list is too close to its capacity (the
// caller then takes the general path); the decision is uniform over the workgroup.
constexpr int kIncMax = 16;
constexpr int kIncPass = 4 * kVocabThreads;   // list entries per pass
constexpr int kIncLdsInts = 4 * kIncMax + 4;  // LDS the route needs: changes, offsets, four scalars

// The part of a list patch that does not depend on the stream policy.
struct IncScratch {
  int* sC;   // ids that left the active set, then ids that entered it (<= 2*kIncMax)
  int* sO;   // per entered id: (entered ids below it) - (left ids below it)
  int* sN;   // how many left, how many entered, the lowest of them
  __device__ explicit IncScratch(int* sh) : sC(sh), sO(sh + 2 * kIncMax), sN(sh + 4 * kIncMax) {}
};

// First wavefront: lane l holds an id that left the active set (r) and/or one that entered it (av), INT_MAX for
// none; the lists, the rank of every entered id among the changes and the counts go to LDS.
__device__ __forceinline__ void inc_publish(int r, int av, int lane, const IncScratch& sc) {
  int* sC = sc.sC;
  int* sO = sc.sO;
  int* sN = sc.sN;
  const unsigned long long mr = __ballot(r != INT_MAX), ma = __ballot(av != INT_MAX);
  const unsigned long long lower = (1ull << lane) - 1ull;
  const int nR = __popcll(mr);
  if (r != INT_MAX) sC[__popcll(mr & lower)] = r;
  int o = 0, lowest = INT_MAX;
  for (unsigned long long m = mr; m; m &= m - 1ull) {
    const int x = __builtin_amdgcn_readlane(r, __ffsll((long long)m) - 1);
    o -= x < av ? 1 : 0;
    lowest = min(lowest, x);
  }
  for (unsigned long long m = ma; m; m &= m - 1ull) {
    const int x = __builtin_amdgcn_readlane(av, __ffsll((long long)m) - 1);
    o += x < av ? 1 : 0;
    lowest = min(lowest, x);
  }
  if (av != INT_MAX) {
    const int slot = __popcll(ma & lower);
    sC[nR + slot] = av;
    sO[slot] = o;
  }
  if (lane == 0) {
    sN[0] = nR;
    sN[1] = __popcll(ma);
    sN[2] = lowest;
  }
}

// Entries 4*tid .. 4*tid+4 of pass `pass` of the list (the fifth one is the next thread's first), INT_MAX past the end.
__device__ __forceinline__ void inc_mask(int pass, int tid, int n_old, const int4& q, int nx, int (&x)[5]) {
  const int j0 = pass * kIncPass + 4 * tid;
  x[0] = j0 < n_old ? q.x : INT_MAX;
  x[1] = j0 + 1 < n_old ? q.y : INT_MAX;
  x[2] = j0 + 2 < n_old ? q.z : INT_MAX;
  x[3] = j0 + 3 < n_old ? q.w : INT_MAX;
  x[4] = j0 + 4 < n_old ? nx : INT_MAX;
}

// All threads, after the barrier that follows inc_publish: move the list entries (xs = this thread's entries of
// the first pass) and write the entered ids.  Returns the change of the list's length.
__device__ __forceinline__ int inc_patch(int32_t* ids, int cap, int n_old, int (&xs)[5], const IncScratch& sc) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int* sC = sc.sC;
  const int* sO = sc.sO;
  const int* sN = sc.sN;
  const int nR = sN[0], nA = sN[1], lowest = sN[2];
  if (nR + nA) {
    // lane q (mod 32) of every wavefront keeps change q and its offset in registers: the loops below read
    // them with readlane instead of waiting for LDS once per change
    const int chg = sC[lane & (2 * kIncMax - 1)], chgo = sO[lane & (2 * kIncMax - 1)];
    const int passes = n_old / kIncPass + 1;
    for (int pass = 0; pass < passes; ++pass) {
      int4 qn = make_int4(INT_MAX, INT_MAX, INT_MAX, INT_MAX);
      int qnn = INT_MAX;
      if (pass + 1 < passes) {                 // the next pass is read before this one is written
        const int j1 = (pass + 1) * kIncPass + 4 * tid;
        if (j1 < cap) qn = *reinterpret_cast<const int4*>(ids + j1);
        if (j1 + 4 < cap) qnn = ids[j1 + 4];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
      }
      const int j0 = pass * kIncPass + 4 * tid;
      const bool head = j0 == 0;
      if ((xs[0] != INT_MAX && xs[4] > lowest) || head) {   // entries below every change stay where they are; past the end there are none
        // changes below the thread's first entry shift all four alike; a change inside its span (rare: at
        // most one thread per change) is worked out entry by entry on top of that
        int m0 = 0, inside = 0;
        for (int q = 0; q < nR; ++q) {
          const int x = __builtin_amdgcn_readlane(chg, q);
          const int lt0 = x < xs[0] ? 1 : 0;
          m0 -= lt0;
          inside += (x < xs[4] ? 1 : 0) - lt0;
        }
        for (int q = 0; q < nA; ++q) {
          const int x = __builtin_amdgcn_readlane(chg, nR + q);
          const int lt0 = x < xs[0] ? 1 : 0;
          m0 += lt0;
          inside += (x < xs[4] ? 1 : 0) - lt0;
        }
        int mv[4] = {m0, m0, m0, m0};
        bool dead[4] = {false, false, false, false};
        if (inside != 0 || (head && m0 != 0)) {
          for (int q = 0; q < nR; ++q) {
            const int x = __builtin_amdgcn_readlane(chg, q);
            if (x >= xs[0] && x < xs[4]) {
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                mv[i] -= x < xs[i] ? 1 : 0;
                dead[i] = dead[i] || x == xs[i];
              }
            }
          }
          for (int q = 0; q < nA; ++q) {
            const int x = __builtin_amdgcn_readlane(chg, nR + q);
            const int below = __builtin_amdgcn_readlane(chgo, q);
            if (x >= xs[0] && x < xs[4]) {
#pragma unroll
              for (int i = 0; i < 4; ++i) {
                mv[i] += x < xs[i] ? 1 : 0;
                if (xs[i] < x && x < xs[i + 1]) ids[j0 + i + 1 + below] = x;
              }
            }
            if (head && x < xs[0]) ids[below] = x;     // in front of the whole list
          }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (xs[i] != INT_MAX && !dead[i] && mv[i] != 0) ids[j0 + i + mv[i]] = xs[i];
      }
      inc_mask(pass + 1, tid, n_old, qn, qnn, xs);
    }
  }
  return nA - nR;
}

__device__ __forceinline__ bool vocab_apply_incremental(const VocabPtrs& p, int b, const int32_t* src, int a, int* sh) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int V = p.V, W = p.window, cap = p.cap;
  int32_t* ids = p.ids + (size_t)b * cap;
  uint32_t* gw = p.wbit + (size_t)b * p.nwords;
  const uint32_t* gt = p.tbit + (size_t)b * p.nwords;
  uint32_t* cnt = p.cnt + (size_t)b * V;
  int32_t* ring = p.ring + (size_t)b * W;
  // everything that does not depend on the state's scalars is requested first
  const int n_old = p.n[b], pos = p.pos[b], fill = p.fill[b];
  const bool ap = tid >= kIncMax && tid < kIncMax + a;        // this thread appends src[tid - kIncMax]
  int v = -1;
  if (ap) v = src[tid - kIncMax];
  int4 q0 = make_int4(INT_MAX, INT_MAX, INT_MAX, INT_MAX);
  int q0n = INT_MAX;
  if (4 * tid < cap) q0 = *reinterpret_cast<const int4*>(ids + 4 * tid);   // cap is a multiple of 4
  if (4 * tid + 4 < cap) q0n = ids[4 * tid + 4];
  if (n_old + a > cap) return false;
  int xs[5];
  inc_mask(0, tid, n_old, q0, q0n, xs);

  int n_evict = fill + a - W;                // a <= W here
  if (n_evict < 0) n_evict = 0;
  int oldest = pos - fill;
  if (oldest < 0) oldest += W;
  int bad = 0;

  if (tid < 64) {
    int id = -1;
    if (ap) {
      if ((unsigned)v < (unsigned)V) id = v;
      else bad = 1;
    } else if (lane < n_evict) {
      int slot = oldest + lane;
      if (slot >= W) slot -= W;
      id = ring[slot];
    }
    const bool valid = id >= 0;
    uint32_t tw = 0u, oldc = 0u;
    if (valid) {
      tw = gt[id >> 5];
      oldc = cnt[id];
    }
    // net change of this lane's id over all lanes, and whether an earlier lane holds the same id
    int total = 0;
    bool first = true;
    for (int j = 0; j < n_evict; ++j) {
      const bool same = valid && __builtin_amdgcn_readlane(id, j) == id;
      total -= same ? 1 : 0;
      first = first && !(same && j < lane);
    }
    for (int j = kIncMax; j < kIncMax + a; ++j) {
      const bool same = valid && __builtin_amdgcn_readlane(id, j) == id;
      total += same ? 1 : 0;
      first = first && !(same && j < lane);
    }
    if (ap) {
      int slot = pos + (lane - kIncMax);
      if (slot >= W) slot -= W;
      ring[slot] = id;                         // the leaving entries are in registers by now; -1 for an id out of range
    }
    const bool lead = valid && first;
    const uint32_t newc = oldc + (uint32_t)total;
    const uint32_t bit = 1u << (id & 31);
    if (lead && total != 0) cnt[id] = newc;
    const bool left = lead && oldc != 0u && newc == 0u, entered = lead && oldc == 0u && newc != 0u;
    if (left) atomicAnd(&gw[id >> 5], ~bit);   // another lane may own a different bit of the same word
    if (entered) atomicOr(&gw[id >> 5], bit);
    const int r = (left && !(tw & bit)) ? id : INT_MAX;
    const int av = (entered && !(tw & bit)) ? id : INT_MAX;
    inc_publish(r, av, lane, IncScratch(sh));
  }
  __syncthreads();
  const int dn = inc_patch(ids, cap, n_old, xs, IncScratch(sh));
  if (tid == 0) {
    p.n[b] = n_old + dn;
    int np = pos + a;
    if (np >= W) np -= W;
    p.pos[b] = np;
    const int nf = fill + a;
    p.fill[b] = nf < W ? nf : W;
  }
  if (bad) atomicOr(p.err, (int)NANOSPEC_DEV_BAD_ID);
  return true;
}

__global__ __launch_bounds__(kVocabThreads) void vocab_apply_kernel(VocabPtrs p, const int32_t* __restrict__ new_ids,
                                                                    Offsets noff, const int32_t* __restrict__ topk,
                                                                    Offsets toff, int replace_T) {
  extern __shared__ uint32_t lds[];
  const int b = blockIdx.x;
  uint32_t* wb = lds;
  uint32_t* tb = lds + p.nwords;
  int* sc = reinterpret_cast<int*>(tb + p.nwords);   // 16 wave totals
  const int a = noff.v[b + 1] - noff.v[b];
  if (!replace_T && a <= kIncMax && a <= p.window &&
      vocab_apply_incremental(p, b, new_ids + noff.v[b], a, reinterpret_cast<int*>(lds)))
    return;
  load_bitmaps(p, b, wb, tb, replace_T);
  vocab_apply_body(p, b, new_ids + noff.v[b], a, topk + toff.v[b], toff.v[b + 1] - toff.v[b], replace_T, wb, tb, sc, 0);
}

// Eq. 3 with the candidate set built on the device: the ids of cand[b][0..per_seq) (for instance the
// top-k ids of all draft-tree nodes, straight from nanospec_topk_remap's output) are de-duplicated
// through a scratch bitmap in LDS and appended to the stream of sequence b in ascending id order;
// how many are appended is known only on the device.  Entries equal to -1 (top-k padding) are
// skipped; other ids outside [0,V) are skipped and flagged.  T is kept.
__global__ __launch_bounds__(kVocabThreads) void vocab_append_unique_kernel(VocabPtrs p, const int32_t* __restrict__ cand,
                                                                            int per_seq, int64_t stride, int ucap) {
  extern __shared__ uint32_t lds[];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int nwords = p.nwords;
  uint32_t* wb = lds;
  uint32_t* tb = lds + nwords;
  int* sc = reinterpret_cast<int*>(tb + nwords);
  uint32_t* ub = reinterpret_cast<uint32_t*>(sc + 32);
  int32_t* ulist = reinterpret_cast<int32_t*>(ub + nwords);
  load_bitmaps(p, b, wb, tb, 0);
  for (int i = tid * 4; i < nwords; i += kVocabThreads * 4) *reinterpret_cast<uint4*>(ub + i) = make_uint4(0, 0, 0, 0);
  __syncthreads();
  int bad = 0;
  for (int i = tid; i < per_seq; i += kVocabThreads) {
    const int v = cand[b * stride + i];
    if ((unsigned)v < (unsigned)p.V) atomicOr(&ub[v >> 5], 1u << (v & 31));
    else if (v != -1) bad = 1;
  }
  __syncthreads();
  int a = compact_bitmap([&](int i) { return *reinterpret_cast<const uint4*>(ub + i); }, nwords, ulist, ucap, sc, tid);
  a = a < ucap ? a : ucap;
  __syncthreads();
  vocab_apply_body(p, b, ulist, a, nullptr, 0, 0, wb, tb, sc, bad);
}

// ---- second reading of the vocabulary: a first-in first-out queue of at most W distinct ids -------------
// (paper Sec. 3.3: only candidates that are new to the vocabulary are pushed; appendix on vocabulary
// evolution: it grows monotonically up to the capacity and is evicted first-in first-out.)
// The ring holds the members in push order, the window bitmap is the membership test, the
// multiplicity counters are not needed and their memory serves as the staging list of one call.
//
// One call = one batch: the ids that are valid, not members when the call starts and not seen earlier
// in the call, in the order of their first occurrence; at most the last W of them are pushed after
// the oldest members have made room.  src is walked in chunks of one workgroup: a thread's id is new if
// neither bitmap (members, seen-in-this-call) has it and no earlier thread of the chunk holds the same
// id; a ballot + prefix over the wavefronts gives every new id its place in the order.
// wb/tb: LDS bitmaps (stores issued by this workgroup), ub: zeroed LDS bitmap, cl: kVocabThreads ints.
__device__ __forceinline__ void fifo_apply_body(const VocabPtrs& p, int b, const int32_t* src, int a, const int32_t* ts,
                                                int nt, int replace_T, uint32_t* wb, uint32_t* tb, uint32_t* ub, int* sc,
                                                int32_t* cl, int bad) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nwords = p.nwords, V = p.V;
  const int W = p.window < V ? p.window : V;                 // more than V distinct ids cannot exist
  uint32_t* gw = p.wbit + (size_t)b * nwords;
  uint32_t* gt = p.tbit + (size_t)b * nwords;
  int32_t* ring = p.ring + (size_t)b * p.window;
  int32_t* stage = reinterpret_cast<int32_t*>(p.cnt + (size_t)b * V);   // W slots, entry k of the call at k % W
  const int pos = p.pos[b], fill = p.fill[b];

  __syncthreads();                                           // LDS bitmaps complete
  int nF = 0;
  for (int c0 = 0; c0 < a; c0 += kVocabThreads) {
    const int i = c0 + tid;
    const int v = i < a ? src[i] : -1;
    cl[tid] = v;
    __syncthreads();
    const bool ok = (unsigned)v < (unsigned)V;
    if (i < a && !ok) bad = 1;
    bool isnew = ok && !((wb[v >> 5] >> (v & 31)) & 1u) && !((ub[v >> 5] >> (v & 31)) & 1u);
    if (isnew)
      for (int j = 0; j < tid; ++j)
        if (cl[j] == v) {
          isnew = false;
          break;
        }
    const unsigned long long bal = __ballot(isnew);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) sc[wave] = __popcll(bal);
    __syncthreads();
    int off = nF, tot = 0;
    for (int w = 0; w < kVocabThreads / 64; ++w) {
      const int t = sc[w];
      if (w < wave) off += t;
      tot += t;
    }
    nF += tot;
    if (isnew) {
      atomicOr(&ub[v >> 5], 1u << (v & 31));
      const int k = off + before;
      if (k >= nF - W) stage[k % W] = v;                     // older entries of the call can never stay
    }
    __syncthreads();                                         // cl, sc and ub are reused by the next chunk
  }
  const int keep = nF < W ? nF : W;
  int n_evict = fill + keep - W;
  if (n_evict < 0) n_evict = 0;
  int oldest = pos - fill;
  if (oldest < 0) oldest += W;
  for (int i = tid; i < n_evict; i += kVocabThreads) {
    const int e = ring[(oldest + i) % W];
    atomicAnd(&wb[e >> 5], ~(1u << (e & 31)));
  }
  __syncthreads();                                           // slots about to be overwritten have been read
  for (int i = tid; i < keep; i += kVocabThreads) {
    const int v = stage[(nF - keep + i) % W];
    ring[(pos + i) % W] = v;
    atomicOr(&wb[v >> 5], 1u << (v & 31));
  }
  if (replace_T) {
    for (int i = tid; i < nt; i += kVocabThreads) {
      const int t = ts[i];
      if ((unsigned)t < (unsigned)V) atomicOr(&tb[t >> 5], 1u << (t & 31));
      else bad = 1;
    }
  }
  __syncthreads();
  const int total = compact_bitmap(
      [&](int i) {
        const uint4 a = *reinterpret_cast<const uint4*>(wb + i), c = *reinterpret_cast<const uint4*>(tb + i);
        return make_uint4(a.x | c.x, a.y | c.y, a.z | c.z, a.w | c.w);
      }, nwords, p.ids + (size_t)b * p.cap, p.cap, sc, tid);
  for (int i = tid * 4; i < nwords; i += kVocabThreads * 4) {
    *reinterpret_cast<uint4*>(gw + i) = *reinterpret_cast<const uint4*>(wb + i);
    if (replace_T) *reinterpret_cast<uint4*>(gt + i) = *reinterpret_cast<const uint4*>(tb + i);
  }
  if (tid == 0) {
    p.n[b] = total < p.cap ? total : p.cap;
    p.pos[b] = (pos + keep) % W;
    const int nf = fill + keep;
    p.fill[b] = nf < W ? nf : W;
  }
  if (bad) atomicOr(p.err, (int)NANOSPEC_DEV_BAD_ID);
}

// The queue reading's list patch (appends of at most kIncMax ids, T untouched): the first wavefront finds the
// new ids -- valid, not members when the call starts, first occurrence in the call, in call order -- pushes them,
// drops as many of the oldest members as the queue overflows by, and hands the ids that left or entered the
// active set to the same list patch as the window reading.  The membership bitmap stays in HBM.
__device__ __forceinline__ bool fifo_apply_incremental(const VocabPtrs& p, int b, const int32_t* src, int a, int* sh) {
  const int tid = threadIdx.x, lane = tid & 63;
  const int V = p.V, cap = p.cap;
  const int W = p.window < V ? p.window : V;
  int32_t* ids = p.ids + (size_t)b * cap;
  uint32_t* gw = p.wbit + (size_t)b * p.nwords;
  const uint32_t* gt = p.tbit + (size_t)b * p.nwords;
  int32_t* ring = p.ring + (size_t)b * p.window;
  const int n_old = p.n[b], pos = p.pos[b], fill = p.fill[b];
  const bool ap = tid >= kIncMax && tid < kIncMax + a;        // this thread appends src[tid - kIncMax]
  int v = -1;
  if (ap) v = src[tid - kIncMax];
  int4 q0 = make_int4(INT_MAX, INT_MAX, INT_MAX, INT_MAX);
  int q0n = INT_MAX;
  if (4 * tid < cap) q0 = *reinterpret_cast<const int4*>(ids + 4 * tid);
  if (4 * tid + 4 < cap) q0n = ids[4 * tid + 4];
  if (n_old + a > cap) return false;
  int xs[5];
  inc_mask(0, tid, n_old, q0, q0n, xs);
  int oldest = pos - fill;
  if (oldest < 0) oldest += W;
  int bad = 0;
  const IncScratch sc(sh);

  if (tid < 64) {
    // lanes 16..31: the appended ids; lanes 0..15: the oldest members, of which the first n_ev leave -- how
    // many is known only when the new ids have been counted, so all candidates are fetched at once
    int id = -1;
    if (ap) {
      if ((unsigned)v < (unsigned)V) id = v;
      else bad = 1;
    } else if (lane < a && lane < fill) {
      int slot = oldest + lane;
      if (slot >= W) slot -= W;
      id = ring[slot];
    }
    uint32_t tw = 0u, ww = 0u;
    if (id >= 0) {
      tw = gt[id >> 5];
      if (ap) ww = gw[id >> 5];
    }
    const uint32_t bit = 1u << (id & 31);
    bool isnew = ap && id >= 0 && !(ww & bit);
    for (int j = kIncMax; j < kIncMax + a; ++j) {
      const bool same = __builtin_amdgcn_readlane(id, j) == id;
      isnew = isnew && !(same && j < lane);
    }
    const unsigned long long mn = __ballot(isnew);
    const int nF = __popcll(mn);                             // a <= W: all of them stay
    int n_ev = fill + nF - W;
    if (n_ev < 0) n_ev = 0;
    if (isnew) {
      int slot = pos + __popcll(mn & ((1ull << lane) - 1ull));
      if (slot >= W) slot -= W;
      ring[slot] = id;                                       // the members that leave are in registers by now
      atomicOr(&gw[id >> 5], bit);
    }
    const bool leaves = !ap && lane < n_ev && id >= 0;
    if (leaves) atomicAnd(&gw[id >> 5], ~bit);
    const int r = (leaves && !(tw & bit)) ? id : INT_MAX;
    const int av = (isnew && !(tw & bit)) ? id : INT_MAX;
    inc_publish(r, av, lane, sc);
    if (lane == 0) sc.sN[3] = nF;
  }
  __syncthreads();
  const int nF = sc.sN[3];
  const int dn = inc_patch(ids, cap, n_old, xs, sc);
  if (tid == 0) {
    p.n[b] = n_old + dn;
    int np = pos + nF;
    if (np >= W) np -= W;
    p.pos[b] = np;
    const int nf = fill + nF;
    p.fill[b] = nf < W ? nf : W;
  }
  if (bad) atomicOr(p.err, (int)NANOSPEC_DEV_BAD_ID);
  return true;
}

__global__ __launch_bounds__(kVocabThreads) void vocab_fifo_kernel(VocabPtrs p, const int32_t* __restrict__ new_ids,
                                                                   Offsets noff, const int32_t* __restrict__ topk,
                                                                   Offsets toff, int replace_T) {
  extern __shared__ uint32_t lds[];
  const int b = blockIdx.x, tid = threadIdx.x, nwords = p.nwords;
  uint32_t* wb = lds;
  uint32_t* tb = lds + nwords;
  int* sc = reinterpret_cast<int*>(tb + nwords);
  uint32_t* ub = reinterpret_cast<uint32_t*>(sc + 32);
  int32_t* cl = reinterpret_cast<int32_t*>(ub + nwords);
  const int a = noff.v[b + 1] - noff.v[b];
  if (!replace_T && a <= kIncMax && a <= p.window && a <= p.V &&
      fifo_apply_incremental(p, b, new_ids + noff.v[b], a, reinterpret_cast<int*>(lds)))
    return;
  load_bitmaps(p, b, wb, tb, replace_T);
  for (int i = tid * 4; i < nwords; i += kVocabThreads * 4) *reinterpret_cast<uint4*>(ub + i) = make_uint4(0, 0, 0, 0);
  fifo_apply_body(p, b, new_ids + noff.v[b], a, topk + toff.v[b], toff.v[b + 1] - toff.v[b], replace_T, wb, tb, ub, sc, cl, 0);
}

// candidate set built on the device, queue reading: distinct valid candidates in ascending order, then one batch
__global__ __launch_bounds__(kVocabThreads) void vocab_fifo_append_unique_kernel(VocabPtrs p, const int32_t* __restrict__ cand,
                                                                                 int per_seq, int64_t stride, int ucap) {
  extern __shared__ uint32_t lds[];
  const int b = blockIdx.x, tid = threadIdx.x, nwords = p.nwords;
  uint32_t* wb = lds;
  uint32_t* tb = lds + nwords;
  int* sc = reinterpret_cast<int*>(tb + nwords);
  uint32_t* ub = reinterpret_cast<uint32_t*>(sc + 32);
  int32_t* cl = reinterpret_cast<int32_t*>(ub + nwords);
  int32_t* ulist = cl + kVocabThreads;
  load_bitmaps(p, b, wb, tb, 0);
  for (int i = tid * 4; i < nwords; i += kVocabThreads * 4) *reinterpret_cast<uint4*>(ub + i) = make_uint4(0, 0, 0, 0);
  __syncthreads();
  int bad = 0;
  for (int i = tid; i < per_seq; i += kVocabThreads) {
    const int v = cand[b * stride + i];
    if ((unsigned)v < (unsigned)p.V) atomicOr(&ub[v >> 5], 1u << (v & 31));
    else if (v != -1) bad = 1;
  }
  __syncthreads();
  int a = compact_bitmap([&](int i) { return *reinterpret_cast<const uint4*>(ub + i); }, nwords, ulist, ucap, sc, tid);
  a = a < ucap ? a : ucap;
  __syncthreads();
  for (int i = tid * 4; i < nwords; i += kVocabThreads * 4) *reinterpret_cast<uint4*>(ub + i) = make_uint4(0, 0, 0, 0);
  fifo_apply_body(p, b, ulist, a, nullptr, 0, 0, wb, tb, ub, sc, cl, bad);
}

hipError_t vocab_configure(nanospec_state* st) {
  st->vocab_lds_bytes = (2 * st->vp.nwords + 32) * 4;
  if (st->vocab_lds_bytes < kIncLdsInts * 4) st->vocab_lds_bytes = kIncLdsInts * 4;   // the list-patching route's scratch
  // candidates per call are bounded by what is left of the 160 KB of LDS after three bitmaps
  st->unique_cap = (160 * 1024 - 512) / 4 - (3 * st->vp.nwords + 32 + kVocabThreads);
  if (st->unique_cap < st->m_cap * st->k_cap) return hipErrorInvalidValue;
  st->unique_lds_bytes = (3 * st->vp.nwords + 32 + kVocabThreads + st->unique_cap) * 4;
  st->fifo_lds_bytes = (3 * st->vp.nwords + 32 + kVocabThreads) * 4;
  return hipSuccess;
}

// Once per device: every vocabulary kernel may use the chip's whole LDS, whatever vocabulary size a state has
// (a per-state limit would be lowered by the next, smaller state under a live larger one).
hipError_t vocab_configure_device() {
  const void* fns[] = {reinterpret_cast<const void*>(vocab_apply_kernel), reinterpret_cast<const void*>(vocab_append_unique_kernel),
                       reinterpret_cast<const void*>(vocab_fifo_append_unique_kernel), reinterpret_cast<const void*>(vocab_fifo_kernel)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_vocab_clear(const nanospec_state* st, hipStream_t s) {
  size_t work = (size_t)st->batch * st->V;
  int blocks = (int)((work + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  vocab_clear_kernel<<<blocks, 256, 0, s>>>(st->vp, st->batch);
  return hipGetLastError();
}

hipError_t launch_vocab_apply(const nanospec_state* st, const int32_t* d_new, const Offsets& noff,
                              const int32_t* d_topk, const Offsets& toff, int replace_T, hipStream_t s) {
  if (st->policy == NANOSPEC_POLICY_FIFO) {
    vocab_fifo_kernel<<<st->batch, kVocabThreads, st->fifo_lds_bytes, s>>>(st->vp, d_new, noff, d_topk, toff, replace_T);
    return hipGetLastError();
  }
  vocab_apply_kernel<<<st->batch, kVocabThreads, st->vocab_lds_bytes, s>>>(st->vp, d_new, noff, d_topk, toff,
                                                                           replace_T);
  return hipGetLastError();
}

hipError_t launch_vocab_append_unique(const nanospec_state* st, const int32_t* d_cand, int per_seq, int64_t stride,
                                      hipStream_t s) {
  const int ucap = per_seq < st->V ? per_seq : st->V;       // no more distinct ids than candidates or tokens
  if (st->policy == NANOSPEC_POLICY_FIFO) {
    const int flds = (3 * st->vp.nwords + 32 + kVocabThreads + ucap) * 4;
    vocab_fifo_append_unique_kernel<<<st->batch, kVocabThreads, flds, s>>>(st->vp, d_cand, per_seq, stride, ucap);
    return hipGetLastError();
  }
  const int lds = (3 * st->vp.nwords + 32 + ucap) * 4;
  vocab_append_unique_kernel<<<st->batch, kVocabThreads, lds, s>>>(st->vp, d_cand, per_seq, stride, ucap);
  return hipGetLastError();
}

}  // namespace nanospec
