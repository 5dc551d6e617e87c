// Draft-token selection (paper Alg. 1, SelectDraftTokens(z', I); operator T_K of Sec. 3.2):
// the k largest logits of every row, ordered by value descending then global id ascending, mapped
// from the position in the active list back to the global token id.
//
// Every lane keeps a run of consecutive logits in registers, so "lower position" means "lower lane,
// then lower register".  A wavefront extracts its k best in k rounds: a DPP max-reduction of the
// lane maxima, a ballot of the lanes that hold that maximum (the lowest such lane owns the
// lowest-position occurrence), one readlane for the register index, and the winner is blanked.
// The wavefronts' winners meet in LDS in position order and one wavefront repeats the rounds over
// them.  Rows longer than one workgroup's reach are cut into chunks whose winners a second kernel
// merges the same way.  Values of -inf mark "nothing left" (logits are finite by contract).
//
// Fast path in front of the rounds: lane l of wavefront w always holds positions (64w + l)*EPT ..., whatever
// the row's length n, so the logits are requested before n has arrived and masked afterwards.  The nwe
// wavefronts that are at least half full (or the first one) each report their ceil(k/nwe)-th largest lane
// maximum; the smallest report is a lower bound T on the row's k-th largest value (at least k lanes hold
// something >= T), so only elements >= T can be winners.  They are compacted in position order into LDS
// (typically one or two dozen; a DPP prefix sum over the lanes and one over the wavefront totals), every
// thread ranks one candidate against all others while its global id is being fetched, and rank r < k is
// output slot r.  If more than kCandMax elements survive (heavy ties) the kernel falls back to the rounds.
// Measured and not kept: handing out the LDS slots with one atomic counter and breaking ties by position;
// splitting the valid runs evenly over the wavefronts (the layout then depends on n: c2 4.2 against
// 4.1 us, c3 5.0 against 4.6); fetching every lane's 16 ids beside its logits so that the winners' ids
// need no second round trip (4.3-4.4 us on c2); a single-pass threshold -- the smallest maximum of the filled
// 16-lane rows, no rounds -- which lets so many more candidates through that nothing is gained at 3k
// elements (3.74 against 3.72 us) and the 8k-element case falls back to the rounds (12.0 against 6.6 us).
// Half-wavefronts as voters (twice the voters, half the rounds, two thresholds per round) helped only
// the unlucky lengths with a single voting wavefront (1.3k elements: 4.0 against 4.3 us) and cost 0.1-1 us elsewhere.
//
// LSE variants (Sec. 4.2: the draft distribution is the softmax renormalised over the active set):
// the same selection, with the values written as log-probabilities z - log(sum_i exp z_i), i over the
// row's n entries.  The row maximum falls out of the first threshold round, the sum of exp(z - max)
// is taken wavefront by wavefront and added in wavefront order (chunk order in the merge kernel), so
// the result does not depend on timing.
#include <limits.h>

#include "common.h"

namespace nanospec {

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_max(float x) {
  const int ninf = __float_as_int(-INFINITY);
  const int y = __builtin_amdgcn_update_dpp(ninf, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
  return fmaxf(x, __int_as_float(y));
}

// maximum over the 64 lanes, returned in every lane

__device__ __forceinline__ float wave_max(float x) {
  x = dpp_max<0x111, 0xf>(x);   // row_shr:1
  x = dpp_max<0x112, 0xf>(x);   // row_shr:2
  x = dpp_max<0x114, 0xf>(x);   // row_shr:4
  x = dpp_max<0x118, 0xf>(x);   // row_shr:8   -> lane 15 of each row holds the row maximum
  x = dpp_max<0x142, 0xa>(x);   // row_bcast:15 into rows 1 and 3
  x = dpp_max<0x143, 0xc>(x);   // row_bcast:31 into rows 2 and 3 -> lane 63 holds the maximum
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float x) {
  const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, ROW_MASK, 0xf, false);
  return x + __int_as_float(y);
}

// sum over the 64 lanes in a fixed order, returned in every lane
__device__ __forceinline__ float wave_add(float x) {
  x = dpp_add<0x111, 0xf>(x);
  x = dpp_add<0x112, 0xf>(x);
  x = dpp_add<0x114, 0xf>(x);
  x = dpp_add<0x118, 0xf>(x);
  x = dpp_add<0x142, 0xa>(x);
  x = dpp_add<0x143, 0xc>(x);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 63));
}

// v[e] for a lane-varying e in [0, 16): a select tree (4 compares + 15 selects) instead of 16 predicated
// moves.  The elements arrive as sixteen scalars: selects between array elements get folded into a
// lane-varying array index, and that puts the whole array into scratch memory.
__device__ __forceinline__ float sel(bool c, float a, float b) { return c ? a : b; }
__device__ __forceinline__ float pick16(float v0, float v1, float v2, float v3, float v4, float v5, float v6, float v7,
                                        float v8, float v9, float v10, float v11, float v12, float v13, float v14,
                                        float v15, int e) {
  const bool b0 = e & 1, b1 = e & 2, b2 = e & 4, b3 = e & 8;
  const float a0 = sel(b0, v1, v0), a1 = sel(b0, v3, v2), a2 = sel(b0, v5, v4), a3 = sel(b0, v7, v6);
  const float a4 = sel(b0, v9, v8), a5 = sel(b0, v11, v10), a6 = sel(b0, v13, v12), a7 = sel(b0, v15, v14);
  const float c0 = sel(b1, a1, a0), c1 = sel(b1, a3, a2), c2 = sel(b1, a5, a4), c3 = sel(b1, a7, a6);
  return sel(b3, sel(b2, c3, c2), sel(b2, c1, c0));
}

// k rounds over the EPT values each lane holds (position = lane*EPT + register index).
// emit(r, value, position) is called by every lane with wave-uniform arguments; value == -inf
// means that fewer than r+1 elements exist.
template <int EPT, typename Emit>
__device__ __forceinline__ void wave_select(float (&v)[EPT], int k, int lane, Emit emit) {
  for (int r = 0; r < k; ++r) {
    float ml = v[0];
#pragma unroll
    for (int e = 1; e < EPT; ++e) ml = fmaxf(ml, v[e]);
    const float m = wave_max(ml);
    const unsigned long long ball = __ballot(ml == m);
    const int L = ball ? __ffsll(ball) - 1 : 0;
    int ef = 0;
#pragma unroll
    for (int e = EPT - 1; e >= 0; --e) ef = (v[e] == m) ? e : ef;
    const int eL = __builtin_amdgcn_readlane(ef, L);
    emit(r, ball ? m : -INFINITY, L * EPT + eL);
    const bool mine = lane == L;
#pragma unroll
    for (int e = 0; e < EPT; ++e) v[e] = (mine && e == eL) ? -INFINITY : v[e];
  }
}

// One workgroup of NW wavefronts selects the k best of elements [c*CH, (c+1)*CH) of row (b, m),
// CH = NW*64*EPT.  FINAL: write global ids / values; else (value, position) for the merge kernel --
// unless the whole row fits the first chunk (n <= CH, known only on the device): then chunk 0 writes the
// final result itself, the other chunks leave at once and the merge kernel has nothing to do.
constexpr int kLaneCand = 4;   // candidates per lane the owner path keeps in registers

template <int EPT, int NW, bool FINAL, bool LSE>
__global__ __launch_bounds__(64 * NW) void topk_select_kernel(const float* __restrict__ logits, int64_t ld,
                                                             const int32_t* __restrict__ ids, int64_t ids_stride,
                                                             const int32_t* __restrict__ n_dev, int n_fixed, int M, int k,
                                                             int32_t* __restrict__ out_ids, float* __restrict__ out_vals,
                                                             float* __restrict__ cand_val, int32_t* __restrict__ cand_pos,
                                                             float2* __restrict__ cand_ms) {
  constexpr int E2 = (NW * kMaxK + 63) / 64;
  __shared__ float s_val[NW * kMaxK];
  __shared__ int s_pos[NW * kMaxK];
  const int c = blockIdx.x, m = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t row = (int64_t)b * M + m;
  const float* src = logits + row * ld;
  // Position order is (wavefront, lane, register) and does not depend on the row's length, so the logits
  // are requested before the length has arrived: bounded by the row stride, masked by n afterwards.
  const int cbase = c * (NW * 64 * EPT);
  const int p0 = cbase + (wave * 64 + lane) * EPT;         // first position of this lane's run
  float v[EPT];
  if ((ld & 3) == 0) {
#pragma unroll
    for (int e = 0; e < EPT; e += 4) {
      float4 x = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      if (p0 + e < ld) x = *reinterpret_cast<const float4*>(src + p0 + e);   // row stride is a multiple of 4
      v[e] = x.x;
      v[e + 1] = x.y;
      v[e + 2] = x.z;
      v[e + 3] = x.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < EPT; ++e) v[e] = (p0 + e < ld) ? src[p0 + e] : -INFINITY;
  }
  const int n = n_dev ? n_dev[b] : n_fixed;
#pragma unroll
  for (int e = 0; e < EPT; ++e) v[e] = (p0 + e < n) ? v[e] : -INFINITY;
  // Wavefronts that are at least half full (or the first one) vote on the threshold; nwa hold anything at all.
  const int left = n - cbase;
  const int runs = left > 0 ? (left + EPT - 1) / EPT : 0;
  int nwe = (runs + 32) / 64;
  nwe = nwe < 1 ? 1 : (nwe > NW ? NW : nwe);
  int nwa = (runs + 63) / 64;
  nwa = nwa > NW ? NW : nwa;
  const bool fin = FINAL || n <= NW * 64 * EPT;           // uniform over the grid row
  if (!FINAL && fin && c != 0) return;
  float lse = 0.f;                                        // log sum exp of the row (LSE && fin)
  __shared__ float s_thr[NW];
  __shared__ float s_wmax[NW];
  __shared__ float s_sum[NW];
  __shared__ int s_cnt[NW];
  // A wavefront that holds nothing of the row leaves at once (a barrier waits only for the wavefronts that
  // are still running): with sixteen wavefronts on four SIMDs every instruction of an idle one delays the
  // others.  It first leaves the neutral entries the others will read; the first four always stay, for the
  // per-thread chores below (up to kCandMax candidates, k padding slots).
  const int nwl = nwa > 4 ? nwa : (NW < 4 ? NW : 4);      // wavefronts that stay, 0 .. nwl-1
  if (wave >= nwl) {
    if (lane == 0) {
      s_cnt[wave] = 0;
      s_wmax[wave] = -INFINITY;
      s_sum[wave] = 0.f;
    }
    if (lane < k) s_val[wave * k + lane] = -INFINITY;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the entries are in LDS before this wavefront is gone
    return;
  }
  // ---- fast path: threshold from lane maxima, compaction, ranking
  {
    __shared__ __attribute__((aligned(16))) float s_cv[kCandMax + 4];
    __shared__ int s_cp[kCandMax];
    float ml = v[0];
#pragma unroll
    for (int e = 1; e < EPT; ++e) ml = fmaxf(ml, v[e]);
    float x = ml, thr = -INFINITY;
    const int rounds = (k + nwe - 1) / nwe;                // nwe * rounds >= k lanes hold something >= T
    float wmax = -INFINITY, wsum = 0.f;
    for (int r = 0; r < rounds; ++r) {
      thr = wave_max(x);
      if (LSE && r == 0 && wave < nwa) {                    // the first round's result is the wavefront's maximum;
        wmax = thr;                                         // its exp-sum is independent work between the rounds
        const float ref = wmax == -INFINITY ? 0.f : wmax;   // nothing valid here: every term is exp(-inf) = 0
        float se = 0.f;
#pragma unroll
        for (int e = 0; e < EPT; ++e) se += __expf(v[e] - ref);
        wsum = wave_add(se);
      }
      const unsigned long long ball = __ballot(x == thr);
      const int L = ball ? __ffsll(ball) - 1 : 0;
      if (lane == L) x = -INFINITY;
    }
    if (lane == 0) {
      s_thr[wave] = thr;
      if (LSE) {
        s_wmax[wave] = wmax;
        s_sum[wave] = wsum;
      }
    }
    __syncthreads();
    float T = s_thr[0];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) T = fminf(T, ww < nwe ? s_thr[ww] : INFINITY);
    if (LSE) {                                              // wavefront (max, sum) pairs -> the row's, in wavefront order
      const float wm = lane < NW ? s_wmax[lane] : -INFINITY;   // lane ww holds wavefront ww's pair
      float zmax = wave_max(wm);
      zmax = zmax == -INFINITY ? 0.f : zmax;                // empty chunk: every factor below is exp(-inf) = 0
      const float se = wave_add(lane < NW ? s_sum[lane] * expf(wm - zmax) : 0.f);
      if (fin) lse = zmax + logf(se);
      else if (tid == 0) cand_ms[row * gridDim.x + c] = make_float2(zmax, se);
    }
    uint32_t flags = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) flags |= (uint32_t)((p0 + e < n) && (v[e] >= T)) << e;
    const int mine = __popc(flags);
    int incl = mine;                                      // inclusive prefix sum over the lanes, by DPP
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x111, 0xf, 0xf, false);   // row_shr:1
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x112, 0xf, 0xf, false);   // row_shr:2
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x114, 0xf, 0xf, false);   // row_shr:4
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x118, 0xf, 0xf, false);   // row_shr:8
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    incl += __builtin_amdgcn_update_dpp(0, incl, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    const int crowded = __ballot(mine > kLaneCand) != 0ull ? 1 << 20 : 0;   // some lane holds more than the owner path keeps
    if (lane == 63) s_cnt[wave] = incl | crowded;
    __syncthreads();
    int off = incl - mine, C = 0, any_crowded = 0;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) {
      const int t = s_cnt[ww] & 0xfffff;
      any_crowded |= s_cnt[ww] >> 20;
      if (ww < wave) off += t;
      C += t;
    }
    if (EPT == 16 && C <= kCandMax && !any_crowded) {     // uniform over the workgroup
      // Owner path: the lane that holds a candidate asks for its global id at once (up to kLaneCand per
      // lane), the values alone meet in LDS, every thread ranks one of them, and the owner -- whose id has
      // arrived meanwhile -- writes the output slot its candidate's rank names.
      float cval[kLaneCand];
      int cgid[kLaneCand];
      uint32_t f = flags;
#pragma unroll
      for (int j = 0; j < kLaneCand; ++j) {
        cval[j] = 0.f;
        cgid[j] = 0;
        if (__ballot(f != 0u) != 0ull) {                    // some lane of this wavefront has a j-th candidate
          const int e = f ? __ffs(f) - 1 : 0;
          cval[j] = pick16(v[0], v[1], v[2], v[3], v[4], v[5], v[6], v[7], v[8], v[9], v[10], v[11], v[12], v[13], v[14],
                           v[15], e);
          cgid[j] = p0 + e;
          if (f) {
            if (fin && ids) cgid[j] = ids[b * ids_stride + p0 + e];
            s_cv[off + j] = cval[j];
          }
          f &= f - 1u;
        }
      }
      if (tid < 4) s_cv[C + tid] = __builtin_nanf("");     // pads the last group of four; compares false with everything
      if (tid < C) s_cp[tid] = 0;                           // rank of candidate tid, accumulated below
      __syncthreads();
      // Work item (t, g): candidate t against the g-th group of four candidates; t is the fast index
      // (padded to a power of two), so a few dozen candidates are ranked in one sweep of the workgroup.
      const int lg = C <= 1 ? 0 : 32 - __clz(C - 1);
      const int items = ((C + 3) >> 2) << lg;
      for (int w = tid; w < items; w += 64 * nwl) {
        const int t = w & ((1 << lg) - 1), q = (w >> lg) * 4;
        if (t < C) {
          const float val = s_cv[t];
          const float4 o = *reinterpret_cast<const float4*>(&s_cv[q]);
          int r = (o.x > val || (o.x == val && q < t)) ? 1 : 0;         // list order is position order
          r += (o.y > val || (o.y == val && q + 1 < t)) ? 1 : 0;
          r += (o.z > val || (o.z == val && q + 2 < t)) ? 1 : 0;
          r += (o.w > val || (o.w == val && q + 3 < t)) ? 1 : 0;
          if (r) atomicAdd(&s_cp[t], r);
        }
      }
      if (tid >= C && tid < k) {                            // padding slots when fewer than k exist
        if (fin) {
          out_ids[row * k + tid] = -1;
          if (out_vals) out_vals[row * k + tid] = -INFINITY;
        } else {
          cand_val[(row * gridDim.x + c) * k + tid] = -INFINITY;
          cand_pos[(row * gridDim.x + c) * k + tid] = -1;
        }
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < kLaneCand; ++j) {
        const int rank = j < mine ? s_cp[off + j] : k;
        if (rank < k) {
          if (fin) {
            const int64_t o = row * k + rank;
            out_ids[o] = cgid[j];
            if (out_vals) out_vals[o] = (LSE && cval[j] != -INFINITY) ? cval[j] - lse : cval[j];
          } else {
            const int64_t o = (row * gridDim.x + c) * k + rank;
            cand_val[o] = cval[j];
            cand_pos[o] = cgid[j];
          }
        }
      }
      return;
    }
    if (C <= kCandMax) {                                  // uniform over the workgroup
#pragma unroll
      for (int e = 0; e < EPT; ++e)
        if ((flags >> e) & 1u) {
          s_cv[off] = v[e];
          s_cp[off] = p0 + e;
          ++off;
        }
      __syncthreads();
      for (int t = tid; t < (C > k ? C : k); t += 64 * nwl) {
        int64_t o;
        int pos = -1;
        float val = -INFINITY;
        int rank = t;                                       // padding slots when fewer than k exist
        int gid = -1;
        if (t < C) {
          val = s_cv[t];
          pos = s_cp[t];
          if (fin) gid = ids ? ids[b * ids_stride + pos] : pos;   // in flight while the candidate is ranked
          rank = 0;
#pragma unroll 4
          for (int q = 0; q < C; ++q) {
            const float ov = s_cv[q];
            rank += (ov > val || (ov == val && q < t)) ? 1 : 0;   // list order is position order
          }
        }
        if (rank < k) {
          if (fin) {
            o = row * k + rank;
            out_ids[o] = gid;
            if (out_vals) out_vals[o] = (LSE && val != -INFINITY) ? val - lse : val;
          } else {
            o = (row * gridDim.x + c) * k + rank;
            cand_val[o] = val;
            cand_pos[o] = pos;
          }
        }
      }
      return;
    }
  }
  // ---- general path: k rounds per wavefront, then over the wavefronts' winners
  const int wbase = cbase + wave * 64 * EPT;
  wave_select<EPT>(v, k, lane, [&](int r, float val, int pos) {
    if (lane == 0) {
      s_val[wave * k + r] = val;
      s_pos[wave * k + r] = wbase + pos;
    }
  });
  __syncthreads();
  if (wave != 0) return;
  float v2[E2];
#pragma unroll
  for (int e = 0; e < E2; ++e) {
    const int q = lane * E2 + e;
    v2[e] = (q < NW * k) ? s_val[q] : -INFINITY;
  }
  // lane r keeps the r-th winner; ids are looked up and stored by k lanes at once afterwards, so the
  // dependent id loads overlap instead of costing one round trip per rank
  float wval = -INFINITY;
  int wq = 0;
  wave_select<E2>(v2, k, lane, [&](int r, float val, int q) {
    if (lane == r) {
      wval = val;
      wq = q;
    }
  });
  if (lane < k) {
    const bool none = (wval == -INFINITY);
    const int pos = none ? -1 : s_pos[wq];
    if (fin) {
      const int64_t o = row * k + lane;
      out_ids[o] = none ? -1 : (ids ? ids[b * ids_stride + pos] : pos);
      if (out_vals) out_vals[o] = (LSE && !none) ? wval - lse : wval;
    } else {
      const int64_t o = (row * gridDim.x + c) * k + lane;
      cand_val[o] = wval;
      cand_pos[o] = pos;
    }
  }
}

// Merge the per-chunk winners of one row (nchunks*k <= 1024 candidates, in position order).
template <bool LSE>
__global__ __launch_bounds__(64) void topk_merge_kernel(const float* __restrict__ cand_val, const int32_t* __restrict__ cand_pos,
                                                        const float2* __restrict__ cand_ms, int nchunks,
                                                        const int32_t* __restrict__ ids, int64_t ids_stride, int M, int k,
                                                        int32_t* __restrict__ out_ids, float* __restrict__ out_vals,
                                                        const int32_t* __restrict__ n_dev, int n_fixed) {
  constexpr int EPT = 16;
  const int m = blockIdx.y, b = blockIdx.z, lane = threadIdx.x;
  if ((n_dev ? n_dev[b] : n_fixed) <= kTopkChunk) return;   // the first chunk's workgroup has written the result
  const int64_t row = (int64_t)b * M + m;
  const int total = nchunks * k;
  const float* cv = cand_val + row * total;
  const int32_t* cp = cand_pos + row * total;
  float v[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int q = lane * EPT + e;
    v[e] = (q < total) ? cv[q] : -INFINITY;
  }
  float lse = 0.f;
  if (LSE) {                                              // chunk (max, sum) pairs -> one log sum exp, in chunk order
    const float2* ms = cand_ms + row * nchunks;
    float zmax = -INFINITY;
    for (int q = lane; q < nchunks; q += 64) zmax = fmaxf(zmax, ms[q].y > 0.f ? ms[q].x : -INFINITY);
    zmax = wave_max(zmax);
    zmax = zmax == -INFINITY ? 0.f : zmax;
    float se = 0.f;
    for (int q0 = 0; q0 < nchunks; q0 += 64) {
      const int q = q0 + lane;
      float t = 0.f;
      if (q < nchunks && ms[q].y > 0.f) t = ms[q].y * expf(ms[q].x - zmax);
      se += wave_add(t);
    }
    lse = zmax + logf(se);
  }
  float wval = -INFINITY;
  int wq = 0;
  wave_select<EPT>(v, k, lane, [&](int r, float val, int q) {
    if (lane == r) {
      wval = val;
      wq = q;
    }
  });
  if (lane < k) {
    const bool none = (wval == -INFINITY);
    const int pos = none ? -1 : cp[wq];
    const int64_t o = row * k + lane;
    out_ids[o] = none ? -1 : (ids ? ids[b * ids_stride + pos] : pos);
    if (out_vals) out_vals[o] = (LSE && !none) ? wval - lse : wval;
  }
}

static int chunks_for(int32_t cap) { return (cap + kTopkChunk - 1) / kTopkChunk; }

int64_t topk_workspace_bytes(int32_t cap, int32_t rows, int32_t k) {
  if (cap <= kTopkChunk) return 0;
  return (int64_t)rows * chunks_for(cap) * (k * 8 + 8);   // (value, position) per winner + (max, sum) per chunk
}

template <bool LSE>
static hipError_t launch_topk_t(const float* logits, int64_t ld, const int32_t* ids, int64_t ids_stride, const int32_t* n_dev,
                                int32_t n_fixed, int32_t cap, int32_t batch, int32_t M, int32_t k, int32_t* out_ids,
                                float* out_vals, char* ws, int64_t ws_bytes, hipStream_t s) {
  const dim3 rows(1, M, batch);
  if (cap <= 4096) {
    topk_select_kernel<16, 4, true, LSE><<<rows, 256, 0, s>>>(logits, ld, ids, ids_stride, n_dev, n_fixed, M, k, out_ids,
                                                            out_vals, nullptr, nullptr, nullptr);
    return hipGetLastError();
  }
  if (cap <= 8192) {   // eight wavefronts beat sixteen (c3: 6.2 -> 5.0 us, c4: 8.2 -> 5.8 us) and four with 32 logits per lane (5.5, 6.1)
    topk_select_kernel<16, 8, true, LSE><<<rows, 512, 0, s>>>(logits, ld, ids, ids_stride, n_dev, n_fixed, M, k, out_ids,
                                                            out_vals, nullptr, nullptr, nullptr);
    return hipGetLastError();
  }
  if (cap <= kTopkChunk) {
    topk_select_kernel<16, 16, true, LSE><<<rows, 1024, 0, s>>>(logits, ld, ids, ids_stride, n_dev, n_fixed, M, k, out_ids,
                                                              out_vals, nullptr, nullptr, nullptr);
    return hipGetLastError();
  }
  const int nch = chunks_for(cap);
  const int64_t need = topk_workspace_bytes(cap, batch * M, k);
  if (nch * k > 1024 || ws == nullptr || ws_bytes < need) return hipErrorInvalidValue;
  const int64_t slots = (int64_t)batch * M * nch * k;
  float* cv = reinterpret_cast<float*>(ws);
  int32_t* cp = reinterpret_cast<int32_t*>(ws + slots * 4);
  float2* ms = reinterpret_cast<float2*>(ws + slots * 8);
  topk_select_kernel<16, 16, false, LSE><<<dim3(nch, M, batch), 1024, 0, s>>>(logits, ld, ids, ids_stride, n_dev, n_fixed, M,
                                                                            k, out_ids, out_vals, cv, cp, ms);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  topk_merge_kernel<LSE><<<rows, 64, 0, s>>>(cv, cp, ms, nch, ids, ids_stride, M, k, out_ids, out_vals, n_dev, n_fixed);
  return hipGetLastError();
}

hipError_t launch_topk(const float* logits, int64_t ld, const int32_t* ids, int64_t ids_stride, const int32_t* n_dev,
                       int32_t n_fixed, int32_t cap, int32_t batch, int32_t M, int32_t k, int32_t* out_ids,
                       float* out_vals, bool logprob, char* ws, int64_t ws_bytes, hipStream_t s) {
  return logprob ? launch_topk_t<true>(logits, ld, ids, ids_stride, n_dev, n_fixed, cap, batch, M, k, out_ids, out_vals, ws,
                                       ws_bytes, s)
                 : launch_topk_t<false>(logits, ld, ids, ids_stride, n_dev, n_fixed, cap, batch, M, k, out_ids, out_vals, ws,
                                        ws_bytes, s);
}

}  // namespace nanospec
