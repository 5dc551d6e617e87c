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
                                                           float* __restrict__ logits, const int32_t* __restrict__ opos) {
  const int b = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = n_dev ? n_dev[b] : n_fixed;
  const int j = blockIdx.x * 4 + wave;
  if (j >= n) return;
  const int64_t row = ids ? ids[b * ids_stride + j] : j;
  const int jo = opos ? opos[b * ids_stride + j] : j;     // where this row's logits go (a row nobody asks for: nowhere)
  if (jo < 0) return;
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
      if (lane == 0 && m0 + t < M) logits[((int64_t)b * M + m0 + t) * ld + jo] = s;
    }
  }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// sum over the four lanes of a quad, in every lane of it (DPP quad_perm: neighbours 1 apart, then 2 apart)
__device__ __forceinline__ float quad_sum(float x) {
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, true));   // quad_perm:[1,0,3,2]
  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, true));   // quad_perm:[2,3,0,1]
  return x;
}

// Matrix-core kernel for few hidden rows (M <= 16) when d needs several K-iterations: same operand
// layout as head_quad_kernel below, but every wavefront fetches its own hidden-row operands and
// nothing goes through LDS except the final K-slice sum, so the K loop carries no barrier.
// The 16 rows of the A tile of v_mfma_f32_16x16x32_bf16 are 4 gathered rows x 4 column parts, the 16
// columns of the B tile are 4 hidden rows x the same 4 column parts; only the diagonal (part == part)
// 4x4 blocks of the product are kept and summed.  With operand row i = 4*row + part and the part as
// the fastest index, the four lanes of a quad read 64 consecutive bytes of one matrix row and one
// load instruction covers 4 rows x 256 contiguous bytes -- fully coalesced straight into the operand
// registers, for W_head and for the hidden rows alike.  A dot product does not care in which order
// its terms are paired up as long as both operands agree, which they do: both use the same map from
// (lane, step) to column.  The matrix cores run at a quarter of their peak this way, which is still
// several times the arithmetic the HBM stream can feed.
// A workgroup of four wavefronts owns 4*RT rows; wavefront w takes columns [kb + w*128*KS, +128*KS)
// per K-iteration; the four K-slices are summed in fixed order through LDS.
template <int RT, int MT, int KS, int NW, bool FAST>
__global__ __launch_bounds__(64 * NW) void head_quad_private_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H,
                                                        const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev,
                                                        int n_fixed, int V, int M, int d, int64_t ld, int64_t ids_stride,
                                                        float* __restrict__ logits, int seq_first,
                                                        const int32_t* __restrict__ opos) {
  constexpr int ROWS = 4 * RT;
  __shared__ float red[NW][RT * MT * 16];
  // Several sequences: the grid is (sequence, tile) with the sequence fastest, so the workgroups in
  // flight at one time work on the same stretch of the (ascending) id lists of all sequences and the
  // rows the sequences share are fetched from HBM once and then found in L2 / Infinity Cache.
  const int b = seq_first ? blockIdx.x : blockIdx.z;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int j0 = (seq_first ? blockIdx.y : blockIdx.x) * ROWS;
  const int orow = (lane & 15) >> 2, part = lane & 3, q = lane >> 4;   // operand row / column part / k group
  const int coff = w * (128 * KS) + q * 32 + part * 8;                  // + kb + t*128
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  const uint16_t* Hb = H + (int64_t)b * M * d;

  // FAST (chosen by the launcher): d is a whole number of K-iterations, so no load needs a bounds test
  // (hidden rows past M are clamped; their products are never stored) and every address is a per-row base
  // plus a compile-time offset -- two instructions per
  // load instead of a branch and a dozen (the generic form spends ~600 instructions per wavefront on its
  // 32 hidden-row loads before the first weight load is issued).
  auto load_h = [&](int kb, u32x4(&hv)[MT][KS]) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = mt * 4 + orow;
      const uint16_t* hp = Hb + (int64_t)(m < M ? m : M - 1) * d + coff + kb;   // a row past M is a copy, never stored
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        const int c = kb + coff + t * 128;
        if (FAST) hv[mt][t] = *reinterpret_cast<const u32x4*>(hp + t * 128);
        else hv[mt][t] = (c < d && m < M) ? *reinterpret_cast<const u32x4*>(Hb + (int64_t)m * d + c) : zero;
      }
    }
  };
  // Row ids and the row count come through the scalar cache (uniform addresses), issued before any
  // vector load so that nothing queues ahead of them.  The ids are read without waiting for the
  // count: the list is allocated to its capacity, a stale id is clamped into the matrix and its
  // product is never stored.
  int idr[ROWS];
  if (ids) {                                              // one branch around all of them: the loads go out back to back
    const int4* ip = reinterpret_cast<const int4*>(ids + b * ids_stride + j0);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int4 v = ip[rt];
      idr[rt * 4] = v.x;
      idr[rt * 4 + 1] = v.y;
      idr[rt * 4 + 2] = v.z;
      idr[rt * 4 + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int r = 0; r < ROWS; ++r) idr[r] = j0 + r;
  }
  const int n = n_dev ? n_dev[b] : n_fixed;
  // where the logit this thread will store goes: column j, or -- for rows kept in an order of their own -- the
  // column listed for row j (negative: nowhere); asked for now, used after the K loop
  static_assert(RT * MT * 16 <= 64 * NW, "one output per thread");
  int jout = j0 + (threadIdx.x / (MT * 16)) * 4 + (threadIdx.x % 16) / 4;
  if (opos) jout = threadIdx.x < RT * MT * 16 && jout < (int)ids_stride ? opos[b * ids_stride + jout] : -1;
  // A tile past the end leaves before it pulls any hidden rows: the launch is sized by the capacity, and with long
  // rows (this kernel's case) a tile's share of the hidden rows is as many bytes as its weights.  (Measured on the
  // sparsity sweep at d = 8192, capacities 2.6 to 7.4 times the live rows: 10.2 -> 9.7, 16.4 -> 15.7, 31.1 -> 29.2,
  // 109.5 -> 99.5 us; with live rows = capacity nothing changes: 7.02 / 10.7 / 16.9 / 26.2 us at 1000 - 6000 rows.)
  if (j0 >= n) return;
  // hidden rows of the first K-iteration depend on the arguments only: they stream in from L2
  // while the ids are still on their way
  u32x4 hv[MT][KS];
  load_h(0, hv);

  const uint16_t* wrow[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    int64_t row = orow == 0 ? idr[rt * 4] : (orow == 1 ? idr[rt * 4 + 1] : (orow == 2 ? idr[rt * 4 + 2] : idr[rt * 4 + 3]));
    row = row < 0 ? 0 : (row >= V ? V - 1 : row);
    wrow[rt] = W + row * d;
  }

  f32x4 acc[RT][MT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int kb = 0; kb < d; kb += NW * 128 * KS) {
    if (!FAST && kb + w * (128 * KS) >= d) break;
    u32x4 wv[RT][KS];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const uint16_t* wp = wrow[rt] + coff + kb;
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        const int c = kb + coff + t * 128;
        if (FAST) wv[rt][t] = *reinterpret_cast<const u32x4*>(wp + t * 128);
        else wv[rt][t] = (c < d) ? *reinterpret_cast<const u32x4*>(wrow[rt] + c) : zero;
      }
    }
    if (kb != 0) load_h(kb, hv);
    if (FAST) __builtin_amdgcn_sched_barrier(0);            // all loads of the iteration stay in front of its first MFMA
#pragma unroll
    for (int t = 0; t < KS; ++t)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[rt][t]),
                                                               __builtin_bit_cast(bf16x8, hv[mt][t]), acc[rt][mt], 0, 0, 0);
  }

  // result lane l holds product rows 4*(l/16)+v, column l%16: the diagonal block entry is v == l%4;
  // the four parts sit in the four lanes of a quad
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const f32x4 a = acc[rt][mt];
      float x = part == 0 ? a[0] : (part == 1 ? a[1] : (part == 2 ? a[2] : a[3]));
      x = quad_sum(x);
      if (part == 0) red[w][(rt * MT + mt) * 16 + q * 4 + orow] = x;     // (row q of the tile, hidden row orow)
    }
  __syncthreads();
  for (int o = threadIdx.x; o < RT * MT * 16; o += 64 * NW) {
    const int rt = o / (MT * 16), mt = (o / 16) % MT, r = (o % 16) / 4, mm = o % 4;
    const int j = j0 + rt * 4 + r, m = mt * 4 + mm;
    if (j >= n || m >= M || jout < 0) continue;
    float s = red[0][o];
#pragma unroll
    for (int ww = 1; ww < NW; ++ww) s += red[ww][o];
    logits[((int64_t)b * M + m) * ld + jout] = s;
  }
}

template <int RT, int MT, int KS, int NW>
static hipError_t run_quad_private(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed,
                           int32_t cap_rows, int32_t V, int32_t batch, int32_t M, int32_t d, int64_t ld, int64_t ids_stride,
                           float* logits, const int32_t* opos, hipStream_t s) {
  const int tiles = (cap_rows + 4 * RT - 1) / (4 * RT);
  const int seq_first = batch > 1 && tiles <= 65535;
  const dim3 grid = seq_first ? dim3(batch, tiles, 1) : dim3(tiles, 1, batch);
  if (d % (NW * 128 * KS) == 0)
    head_quad_private_kernel<RT, MT, KS, NW, true><<<grid, 64 * NW, 0, s>>>(W, H, ids, n_dev, n_fixed, V, M, d, ld, ids_stride,
                                                                            logits, seq_first, opos);
  else
    head_quad_private_kernel<RT, MT, KS, NW, false><<<grid, 64 * NW, 0, s>>>(W, H, ids, n_dev, n_fixed, V, M, d, ld, ids_stride,
                                                                             logits, seq_first, opos);
  return hipGetLastError();
}

// Matrix-core kernel for few hidden rows (M <= 16).
// The 16 rows of the A tile of v_mfma_f32_16x16x32_bf16 are 4 gathered rows x 4 column parts, the 16
// columns of the B tile are 4 hidden rows x the same 4 column parts; only the diagonal (part == part)
// 4x4 blocks of the product are kept and summed.  With operand row i = 4*row + part and the part as
// the fastest index, the four lanes of a quad read 64 consecutive bytes of one matrix row and one
// load instruction covers 4 rows x 256 contiguous bytes -- fully coalesced straight into the operand
// registers, with no transposition through LDS and no cross-lane reduction of products.  A dot
// product does not care in which order its terms are paired up as long as both operands agree,
// which they do: both use the same map from (lane, step) to column.  The matrix cores run at a
// quarter of their peak this way, still several times the arithmetic the HBM stream can feed.
//
// A workgroup has 4*NRG wavefronts: wavefront (kq, rg) owns rows [4*RT*rg, +4*RT) of the
// workgroup's 4*RT*NRG rows and K-quarter kq of each K-iteration (128*KS columns).  All its weight
// loads of an iteration are put in flight at once.  The hidden rows of a K-quarter are the same for
// every row group, so the NRG wavefronts that share kq each fetch 1/NRG of that slice (already in
// operand layout) and exchange it through LDS: the hidden-row traffic out of L2 shrinks by NRG,
// which is what limits this kernel once the weights stream at HBM speed.  The K-quarters of a row
// group are summed in fixed order through LDS, so a logit's bits do not depend on the row's
// position in the list, on n or on timing.
template <int NRG, int RT, int MT, int KS, bool ONEK>
__global__ __launch_bounds__(256 * NRG) void head_quad_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H,
                                                              const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev,
                                                              int n_fixed, int V, int M, int d, int64_t ld, int64_t ids_stride,
                                                              float* __restrict__ logits, int seq_first,
                                                              const int32_t* __restrict__ opos) {
  constexpr int HI = MT * KS;                      // load instructions per hidden-row K-quarter slice
  constexpr int HPW = (HI + NRG - 1) / NRG;        // of which each sharing wavefront fetches this many
  constexpr int RPG = 4 * RT;                      // rows per row group
  constexpr int NOUT = RT * MT * 16;               // outputs per row group
  static_assert(HI <= 32, "LDS budget: 4*HI KB of hidden-row operands");
  extern __shared__ __attribute__((aligned(16))) char hs[];   // 4*HI KB of hidden-row operands, then the K-quarter sums
  const int b = seq_first ? blockIdx.x : blockIdx.z;      // several sequences: sequence fastest (see head_quad_private_kernel)
  const int tile = seq_first ? blockIdx.y : blockIdx.x;
  const int lane = threadIdx.x & 63;
  const int w = threadIdx.x >> 6;
  const int kq = w & 3, rg = w >> 2;
  const int j0 = (tile * NRG + rg) * RPG;
  const int orow = (lane & 15) >> 2, part = lane & 3, q = lane >> 4;   // operand row / column part / k group
  const int coff = kq * (128 * KS) + q * 32 + part * 8;                // + kb + t*128
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  const uint16_t* Hb = H + (int64_t)b * M * d;

  // Row ids are the first loads issued, so that nothing queues ahead of them, and they are read
  // without waiting for the row count: the list is allocated to its capacity, a stale id is clamped
  // into the matrix and its product is never stored.  (Measured on MI355X: fetching them through
  // the vector path beats the scalar cache here by ~0.5 us, and leaving early on the row count
  // costs ~1.4 us because the hidden-row loads then sink below the wait for the count.)
  // Every load below is unconditional -- out-of-range rows and columns are clamped to valid addresses and
  // masked by arithmetic (row groups past the end all read the first 16 bytes of row 0, which costs next to nothing) -- because a
  // load under a branch makes the outstanding-load count unknowable at compile time: the wait for the
  // ids then becomes a wait for the hidden rows as well, and the weight loads queue behind both.  The row
  // count comes through the vector path too, right behind the ids: scalar loads return out of order, so
  // waiting for a kernel argument would wait for the count before the first hidden-row load is issued.
  int idr[RPG];
  if (ids) {                                              // one 16-byte load per four rows (j0 and the row stride are multiples of 4)
    const int4* ip = reinterpret_cast<const int4*>(ids + b * ids_stride + j0);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
      const int4 v = ip[rt];
      idr[rt * 4] = v.x;
      idr[rt * 4 + 1] = v.y;
      idr[rt * 4 + 2] = v.z;
      idr[rt * 4 + 3] = v.w;
    }
  } else {
#pragma unroll
    for (int r = 0; r < RPG; ++r) idr[r] = j0 + r;
  }
  // (Row groups of 8 rows -- the many-sequence, throughput-bound shape -- keep predicated loads: there
  // the extra address arithmetic costs more than the earlier issue gains; 64 sequences 186 against 179 us.)
  constexpr bool UNCOND = RT == 1;
  int vzero = 0;
  if (UNCOND) asm volatile("" : "+v"(vzero));             // a zero the compiler cannot see through: keeps the load below on the vector path
  const int n = n_dev ? n_dev[b + vzero] : n_fixed;
  // Many sequences (row groups of 8): the launch is sized by the capacity, typically twice the live row count, and
  // the work is throughput-bound -- a workgroup whose rows all lie past the end leaves before it pulls its 64 KB of
  // hidden rows (measured on 64 sequences of 2.3k rows in lists of capacity 5120: a workgroup without rows cost
  // 0.65 of one with rows; 178 -> 130 us).  Measured on top of this and not kept: a workgroup walking 2-8
  // consecutive tiles with the hidden-row operands resident in LDS (125 us at 2 tiles, slower beyond; with the next
  // tile's weight loads issued before the epilogue 136 us; as a kernel of its own with two register sets of weights,
  // every load unconditional and the tile loop fully unrolled, one workgroup per compute unit: 135 us), and handing each of the chip's eight dies one eighth of
  // every sequence's list so that the sequences' copies of a row meet in one L2 (more fabric traffic, not less:
  // every die then needs all sequences' hidden rows in its L2).
  if (!UNCOND && tile * (NRG * RPG) >= n) return;
  // where the logit this thread will store goes (see head_quad_private_kernel); asked for now, used at the end
  static_assert(NOUT <= 256, "one output per thread");
  int jout = -1;
  {
    const int g = threadIdx.x / NOUT, oo = threadIdx.x % NOUT;
    const int j = (tile * NRG + g) * RPG + (oo / (MT * 16)) * 4 + (oo % 16) / 4;
    jout = j;
    if (opos) jout = threadIdx.x < NRG * NOUT && j < (int)ids_stride ? opos[b * ids_stride + j] : -1;
  }

  bool hok[HPW];
  auto load_h = [&](int kb, u32x4(&hv)[HPW]) {
#pragma unroll
    for (int ii = 0; ii < HPW; ++ii) {
      if constexpr (UNCOND) {
        const int i = rg * HPW + ii, ic = i < HI ? i : HI - 1, mt = ic / KS, t = ic % KS;
        const int m = mt * 4 + orow, c = kb + coff + t * 128;
        hok[ii] = m < M && c < d;
        hv[ii] = *reinterpret_cast<const u32x4*>(Hb + (int64_t)(m < M ? m : M - 1) * d + (c < d ? c : 0));
      } else {
        const int i = rg * HPW + ii, mt = i / KS, t = i % KS;
        const int m = mt * 4 + orow, c = kb + coff + t * 128;
        hok[ii] = true;
        hv[ii] = (i < HI && m < M && c < d) ? *reinterpret_cast<const u32x4*>(Hb + (int64_t)m * d + c) : zero;
      }
    }
  };
  // this wavefront's share of the hidden rows of the first K-iteration depends on the arguments
  // only: it streams in from L2 while the ids are still on their way
  u32x4 hv[HPW];
  load_h(0, hv);

  const uint16_t* wrow[RT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    int64_t row = orow == 0 ? idr[rt * 4] : (orow == 1 ? idr[rt * 4 + 1] : (orow == 2 ? idr[rt * 4 + 2] : idr[rt * 4 + 3]));
    row = row < 0 ? 0 : (row >= V ? V - 1 : row);
    if (UNCOND) row = j0 < n ? row : 0;
    wrow[rt] = W + row * d;
  }
  const bool live = j0 < n;                               // a row group past the end reads one 16-byte piece of row 0 over and over

  f32x4 acc[RT][MT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[rt][mt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // ONEK: d <= 512*KS, one K-iteration, straight-line code
  for (int kb = 0; kb < (ONEK ? 1 : d); kb += 512 * KS) {
    if (kb != 0) load_h(kb, hv);
    u32x4 wv[RT][KS];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int t = 0; t < KS; ++t) {
        const int c = kb + coff + t * 128;
        if (UNCOND) wv[rt][t] = *reinterpret_cast<const u32x4*>(wrow[rt] + ((live && c < d) ? c : 0));   // columns past d meet zeros of H
        else wv[rt][t] = (live && c < d) ? *reinterpret_cast<const u32x4*>(wrow[rt] + c) : zero;
      }
    if (UNCOND) __builtin_amdgcn_sched_barrier(0);          // the masking of the hidden rows (a wait for them) stays below the weight loads
    if (kb != 0) __syncthreads();                           // the previous slice has been consumed
#pragma unroll
    for (int ii = 0; ii < HPW; ++ii)
      if (rg * HPW + ii < HI) *reinterpret_cast<u32x4*>(hs + (kq * HI + rg * HPW + ii) * 1024 + lane * 16) = (!UNCOND || hok[ii]) ? hv[ii] : zero;
    __syncthreads();
#pragma unroll
    for (int t = 0; t < KS; ++t)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const bf16x8 bv = *reinterpret_cast<const bf16x8*>(hs + (kq * HI + mt * KS + t) * 1024 + lane * 16);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
          acc[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[rt][t]), bv, acc[rt][mt], 0, 0, 0);
      }
  }

  // result lane l holds product rows 4*(l/16)+v, column l%16: the diagonal block entry is v == l%4;
  // the four parts sit in the four lanes of a quad
  float* red = reinterpret_cast<float*>(hs + 4 * HI * 1024);
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const f32x4 a = acc[rt][mt];
      float x = part == 0 ? a[0] : (part == 1 ? a[1] : (part == 2 ? a[2] : a[3]));
      x = quad_sum(x);
      if (part == 0) red[w * NOUT + (rt * MT + mt) * 16 + q * 4 + orow] = x;   // (tile row q, hidden row orow)
    }
  __syncthreads();
  for (int o = threadIdx.x; o < NRG * NOUT; o += 256 * NRG) {
    const int g = o / NOUT, oo = o % NOUT;
    const int rt = oo / (MT * 16), mt = (oo / 16) % MT, r = (oo % 16) / 4, mm = oo % 4;
    const int j = (tile * NRG + g) * RPG + rt * 4 + r, m = mt * 4 + mm;
    if (j >= n || m >= M || jout < 0) continue;
    const float* rr = red + (g * 4) * NOUT + oo;
    const float s = ((rr[0] + rr[NOUT]) + rr[2 * NOUT]) + rr[3 * NOUT];
    logits[((int64_t)b * M + m) * ld + jout] = s;
  }
}

template <int NRG, int RT, int MT, int KS>
static hipError_t run_quad(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed,
                           int32_t cap_rows, int32_t V, int32_t batch, int32_t M, int32_t d, int64_t ld, int64_t ids_stride,
                           float* logits, const int32_t* opos, hipStream_t s) {
  constexpr int ROWS = 4 * RT * NRG;
  constexpr int LDS = 4 * MT * KS * 1024 + 4 * NRG * (RT * MT * 16) * 4;
  const int tiles = (cap_rows + ROWS - 1) / ROWS;
  const int seq_first = batch > 1 && tiles <= 65535;
  const dim3 grid = seq_first ? dim3(batch, tiles, 1) : dim3(tiles, 1, batch);
  if (d > 512 * KS) return hipErrorInvalidValue;          // callers send longer rows to the K-loop kernel
  head_quad_kernel<NRG, RT, MT, KS, true><<<grid, 256 * NRG, LDS, s>>>(W, H, ids, n_dev, n_fixed, V, M, d, ld, ids_stride, logits, seq_first,
                                                                       opos);
  return hipGetLastError();
}

// Which kernel (all measured on MI355X):
//  * d fits one K-iteration (d <= 512*KS): the shared-hidden-row kernel.  Rows per workgroup follow the
//    row capacity so that small vocabularies still spread over the chip (16 / 8 / 4 rows); with tens
//    of thousands of rows it still wins (dense 128k head, M = 8: 174 us against 188 us barrier-free and
//    184 us for the vendor GEMM library), and for several sequences 2 row groups of 8 rows do best
//    (64 sequences of 2.3k rows: 189 us against 223 us barrier-free).
//  * d needs a K loop: the barrier-free kernel (with a loop the shared form pays two barriers per
//    iteration: 264 us against 118 us at 32k rows of d = 8192, 11.0 against 9.6 us at 1.3k rows).
template <int MT, int KS>
static hipError_t run_quad_auto(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed,
                                int32_t cap_rows, int32_t V, int32_t batch, int32_t M, int32_t d, int64_t ld,
                                int64_t ids_stride, float* logits, const int32_t* opos, hipStream_t s) {
  const int64_t rows = (int64_t)cap_rows * batch;
  if (d > 512 * KS) {
    // (tiles past the end leave at once in this kernel, so what counts is the live rows: 4 rows per workgroup while they
    // fit 256 workgroups -- about 0.8 of the capacity in the workloads here; 7.0 us at 1000 live rows, 10.1 us at 1091)
    if (rows <= 5 * 256) return run_quad_private<1, MT, KS, 4>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
    if (MT <= 2 || rows < 8192) return run_quad_private<2, MT, KS, 4>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
    return run_quad_private<4, MT, KS, 4>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  }
  if (batch > 1 && rows >= 8192) return run_quad<2, 2, MT, KS>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  // 16 / 8 / 4 rows per workgroup: the coarsest shape that still gives every workgroup of the launch (sized by the
  // capacity) a compute unit of its own.  A workgroup without rows costs as much as one with rows here (its loads
  // are unconditional), so one workgroup more than the chip has compute units puts two on one unit and the launch
  // waits for that unit: measured at d = 4096, M = 8, live rows = 0.8 capacity, 8 rows per workgroup: 4.85 us at
  // capacity 2048 (256 workgroups), 6.30 us at 2304 (288); with the earlier thresholds (1440 / 2880 rows) capacity
  // 1280 took 4.88 us (now 4.00) and 2752 took 7.50 us (now 6.52).
  if (rows > 8 * 256) return run_quad<4, 1, MT, KS>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  if (rows > 4 * 256) return run_quad<2, 1, MT, KS>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  return run_quad<1, 1, MT, KS>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
}

// Matrix-core kernel for wide draft trees (16 < M <= 64).  A workgroup owns 64 rows (one 16-row
// tile per wavefront) and works on one 512-column slice of K at a time, so that the hidden rows it
// needs per slice (M x 512) are as many bytes as the weights it streams (64 x 512) instead of four
// times as many.  Weights and hidden rows are loaded with coalesced 1 KB-per-row instructions,
// parked in padded LDS and read back in the operand layout of v_mfma_f32_16x16x32_bf16 (lane = row +
// 16*kgroup, 8 consecutive k per lane; padding keeps the 16 rows on distinct banks); the hidden-row
// slice is shared by the four wavefronts and the next slice's loads are issued before the matrix
// cores start on the current one.
//   LOOPK = true : the workgroup walks all slices and writes logits (many rows: dense head, c5).
//   LOOPK = false: split-K -- slice = blockIdx.y, partial products go to that slice's plane and
//                  head_splitk_reduce_kernel adds the planes in slice order (few rows: the rows
//                  alone cannot fill the chip; deterministic because the order is fixed).
// Bytes between the 1 KB rows of a tile in LDS.  The operand reads take 16 bytes per lane from 16 rows at a
// time; with 16 bytes of padding rows r and r+8 meet in the same banks (SQ_LDS_BANK_CONFLICT: 36 % on top of
// the LDS-active cycles of a launch), with 32 bytes none do (0 conflict cycles; 13.6 -> 13.2 us at M = 64).
constexpr int kTilePad = 32;
//   FAST 1 / 2 (chosen by the launcher): d a whole number of slices, so no load needs a bounds test; hidden
//   rows past M are clamped (1) or do not occur (2: M == 64, sixteen per wavefront) and rows past the end read row 0 instead
//   of being skipped (neither is ever stored), the row count arrives on the vector
//   path behind the ids, and every address is a base plus a lane offset.  The generic form spends ~25
//   instructions and a branch on each of its 32 loads per slice (~860 instructions before the last weight
//   load of the first slice is issued) and, because of the branches, waits for all hidden-row loads
//   before it issues the first weight load.
template <int MT, bool LOOPK, int FAST>
__global__ __launch_bounds__(256) void head_tile64_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H,
                                                          const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev,
                                                          int n_fixed, int V, int M, int d, int64_t ld, int64_t ids_stride,
                                                          float* __restrict__ out, const int32_t* __restrict__ opos,
                                                          int64_t opos_stride, int seq_rows, int row0) {
  constexpr int STRB = 1024 + kTilePad;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int b = blockIdx.z, batch = gridDim.z;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int j0 = blockIdx.x * 64 + w * 16;
  const int S = (d + 511) / 512;
  const int s0 = LOOPK ? 0 : blockIdx.y, s1 = LOOPK ? S : blockIdx.y + 1;
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  char* reg = smem + w * (16 * STRB);

  // one id per lane (capacity-bounded, not waiting for the row count), handed out by readlane
  int myid = j0 + (lane & 15);
  if (ids) myid = ids[b * ids_stride + j0 + (lane & 15)];
  int vzero = 0;
  if (FAST) asm volatile("" : "+v"(vzero));               // keeps the row count's load on the vector path, in order behind the ids
  const int nv = n_dev ? n_dev[b + vzero] : n_fixed;
  // rows kept in an order of their own (LOOPK only): the columns their logits go to, four per lane, asked for now.
  // seq_rows > 0: the list is shared by several sequences of seq_rows hidden rows each and every sequence has
  // its own columns -- hidden row r (counted from row0 on, over the whole launch) belongs to sequence r / seq_rows;
  // those columns are fetched at the end, per hidden row.
  int4 jo4 = make_int4(0, 0, 0, 0);
  if (LOOPK && opos && seq_rows == 0) {
    const int jq = j0 + 4 * (lane >> 4);
    jo4 = jq + 3 < (int)opos_stride ? *reinterpret_cast<const int4*>(opos + b * opos_stride + jq) : make_int4(-1, -1, -1, -1);
  }
  u32x4 hv[16], wv[16];
  int n = nv;
  auto load_slice = [&](int sl) {
    if constexpr (FAST != 0) {
      const uint32_t cb = (uint32_t)(sl * 512 + lane * 8) * 2u;            // byte offset inside a row
      const char* hp = reinterpret_cast<const char*>(H + (int64_t)b * M * d) + cb;
      if constexpr (FAST == 2) {                                          // M == 64: all four wavefronts' hidden rows exist, constant strides
        const char* hw = hp + (int64_t)w * 16 * d * 2;
#pragma unroll
        for (int r = 0; r < 16; ++r) hv[r] = *reinterpret_cast<const u32x4*>(hw + (int64_t)r * d * 2);
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = w * 16 + r;                                         // a hidden row past M is a copy, never stored
          hv[r] = *reinterpret_cast<const u32x4*>(hp + (int64_t)(m < M ? m : M - 1) * d * 2);
        }
      }
      __builtin_amdgcn_sched_barrier(0);                                  // the hidden-row loads go out before the ids are waited for
      n = __builtin_amdgcn_readfirstlane(nv);
      // lane r (mod 16) works out the byte offset of row r once; the wavefront then needs two readlanes,
      // a scalar add and a base-register + lane-offset load per row
      int mrow = myid < 0 ? 0 : (myid >= V ? V - 1 : myid);
      mrow = j0 + (lane & 15) < n ? mrow : 0;                               // rows past the end: row 0, never stored
      const uint64_t ro = (uint64_t)(uint32_t)mrow * (uint64_t)(uint32_t)(d * 2);
      const uint32_t rol = (uint32_t)ro, roh = (uint32_t)(ro >> 32);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint64_t o = ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)roh, r) << 32) |
                           (uint32_t)__builtin_amdgcn_readlane((int)rol, r);
        const char* rp = reinterpret_cast<const char*>(W) + o;
        wv[r] = *reinterpret_cast<const u32x4*>(rp + cb);
      }
      __builtin_amdgcn_sched_barrier(0);                                  // ... and all loads of the slice before anything waits for one
    } else {
      const int c = sl * 512 + lane * 8;
      const bool cok = c < d;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = w * 16 + r;
        hv[r] = (cok && m < M) ? *reinterpret_cast<const u32x4*>(H + ((int64_t)b * M + m) * d + c) : zero;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int64_t row = __builtin_amdgcn_readlane(myid, r);
        row = row < 0 ? 0 : (row >= V ? V - 1 : row);
        wv[r] = (cok && j0 + r < n) ? *reinterpret_cast<const u32x4*>(W + row * d + c) : zero;
      }
    }
  };
  // split-K launches are sized by capacity: tiles past n leave before they pull their hidden-row slice
  // (measured neutral at n close to capacity, and it spares the L2 when n is far below it); the FAST form
  // learns n only with the ids and leaves after its first slice's loads
  if (!FAST && n_dev && (int)blockIdx.x * 64 >= n) return;
  load_slice(s0);
  if (FAST && n_dev && (int)blockIdx.x * 64 >= n) return;
  const int rd_off = (lane & 15) * STRB + (lane >> 4) * 16;
  f32x4 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int sl = s0; sl < s1; ++sl) {
    if (sl != s0) __syncthreads();                          // the previous hidden-row slice has been consumed
#pragma unroll
    for (int r = 0; r < 16; ++r) *reinterpret_cast<u32x4*>(reg + r * STRB + lane * 16) = wv[r];
    bf16x8 av[16];
#pragma unroll
    for (int t = 0; t < 16; ++t) av[t] = *reinterpret_cast<const bf16x8*>(reg + rd_off + t * 64);
#pragma unroll
    for (int r = 0; r < 16; ++r) *reinterpret_cast<u32x4*>(reg + r * STRB + lane * 16) = hv[r];
    __syncthreads();
    if (sl + 1 < s1) load_slice(sl + 1);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if (mt * 16 >= M) break;
      const char* hreg = smem + mt * (16 * STRB);
#pragma unroll
      for (int t = 0; t < 16; ++t) {
        const bf16x8 bv = *reinterpret_cast<const bf16x8*>(hreg + rd_off + t * 64);
        acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[t], bv, acc[mt], 0, 0, 0);
      }
    }
  }
  // result lane l holds rows j0 + 4*(l/16) + v, hidden row 16*mt + l%16
  const int j = j0 + 4 * (lane >> 4);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + (lane & 15);
    if (m >= M || j >= n) continue;
    float* dst = LOOPK ? out + ((int64_t)b * M + m) * ld + j
                       : out + (((int64_t)blockIdx.y * batch + b) * M + m) * ld + j;   // ld = plane row stride
    if (LOOPK && opos) {
      float* rowp = out + ((int64_t)b * M + m) * ld;
      if (seq_rows > 0)
        jo4 = j + 3 < (int)opos_stride ? *reinterpret_cast<const int4*>(opos + (int64_t)((row0 + b * M + m) / seq_rows) * opos_stride + j)
                                       : make_int4(-1, -1, -1, -1);
      const int jo[4] = {jo4.x, jo4.y, jo4.z, jo4.w};
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (j + v < n && jo[v] >= 0) rowp[jo[v]] = acc[mt][v];
    } else if ((ld & 3) == 0 && (LOOPK ? j + 3 < n : true)) {
      *reinterpret_cast<f32x4*>(dst) = acc[mt];
    } else {
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (j + v < n) dst[v] = acc[mt][v];
    }
  }
}

__global__ __launch_bounds__(256) void head_splitk_reduce_kernel(const float* __restrict__ partial, const int32_t* __restrict__ n_dev,
                                                                 int S, int M, int cap, int64_t ld, float* __restrict__ logits,
                                                                 const int32_t* __restrict__ opos) {
  const int b = blockIdx.z, m = blockIdx.y, batch = gridDim.z;
  const int j = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (j >= n_dev[b]) return;
  int4 jo4 = make_int4(0, 0, 0, 0);
  if (opos) jo4 = *reinterpret_cast<const int4*>(opos + (int64_t)b * cap + j);   // j + 3 < cap: cap is a multiple of 64
  const int64_t plane = (int64_t)batch * M * cap;
  const float* p = partial + ((int64_t)b * M + m) * cap + j;
  // eight planes are fetched before the first add so that their latencies overlap; the adds keep slice order
  f32x4 s = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < S; s0 += 8) {
    f32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      v[i] = s0 + i < S ? *reinterpret_cast<const f32x4*>(p + (s0 + i) * plane) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 8; ++i) s += v[i];
  }
  if (opos) {
    float* rowp = logits + ((int64_t)b * M + m) * ld;
    const int jo[4] = {jo4.x, jo4.y, jo4.z, jo4.w};
    const int n = n_dev[b];
#pragma unroll
    for (int v = 0; v < 4; ++v)
      if (j + v < n && jo[v] >= 0) rowp[jo[v]] = s[v];
    return;
  }
  *reinterpret_cast<f32x4*>(logits + ((int64_t)b * M + m) * ld + j) = s;
}

template <int MT>
static hipError_t run_splitk(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_dev, int32_t cap_rows,
                             int32_t V, int32_t batch, int32_t M, int32_t d, int64_t ld, int64_t ids_stride, float* logits,
                             float* partial, int S, const int32_t* opos, hipStream_t s) {
  constexpr int LDS = 4 * 16 * (1024 + kTilePad);
  const int fast = d % 512 != 0 ? 0 : (M == 64 ? 2 : 1);   // 2: every wavefront's sixteen hidden rows exist
  hipError_t e;
  const dim3 grid((cap_rows + 63) / 64, S, batch);
  if (fast == 2) head_tile64_kernel<MT, false, 2><<<grid, 256, LDS, s>>>(W, H, ids, n_dev, 0, V, M, d, cap_rows, ids_stride, partial, nullptr, 0, 0, 0);
  else if (fast == 1) head_tile64_kernel<MT, false, 1><<<grid, 256, LDS, s>>>(W, H, ids, n_dev, 0, V, M, d, cap_rows, ids_stride, partial, nullptr, 0, 0, 0);
  else head_tile64_kernel<MT, false, 0><<<grid, 256, LDS, s>>>(W, H, ids, n_dev, 0, V, M, d, cap_rows, ids_stride, partial, nullptr, 0, 0, 0);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  head_splitk_reduce_kernel<<<dim3((cap_rows / 4 + 255) / 256, M, batch), 256, 0, s>>>(partial, n_dev, S, M, cap_rows, ld,
                                                                                    logits, opos);
  return hipGetLastError();
}

template <int MT>
static hipError_t run_tile64(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed,
                             int32_t cap_rows, int32_t V, int32_t batch, int32_t M, int32_t d, int64_t ld, int64_t ids_stride,
                             float* logits, const int32_t* opos, hipStream_t s) {
  constexpr int LDS = 4 * 16 * (1024 + kTilePad);
  const int fast = d % 512 != 0 ? 0 : (M == 64 ? 2 : 1);   // 2: every wavefront's sixteen hidden rows exist
  const dim3 grid((cap_rows + 63) / 64, 1, batch);
  if (fast == 2) head_tile64_kernel<MT, true, 2><<<grid, 256, LDS, s>>>(W, H, ids, n_dev, n_fixed, V, M, d, ld, ids_stride, logits, opos, ids_stride, 0, 0);
  else if (fast == 1) head_tile64_kernel<MT, true, 1><<<grid, 256, LDS, s>>>(W, H, ids, n_dev, n_fixed, V, M, d, ld, ids_stride, logits, opos, ids_stride, 0, 0);
  else head_tile64_kernel<MT, true, 0><<<grid, 256, LDS, s>>>(W, H, ids, n_dev, n_fixed, V, M, d, ld, ids_stride, logits, opos, ids_stride, 0, 0);
  return hipGetLastError();
}

// Up to 64 hidden rows per sequence in one launch; picks the kernel by M and by how many rows there are.
static hipError_t launch_head_64(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_dev,
                                 int32_t n_fixed, int32_t cap_rows, int32_t V, int32_t batch, int32_t M, int32_t d,
                                 int64_t ld, int64_t ids_stride, float* logits, float* partial, int64_t partial_bytes,
                                 const int32_t* opos, hipStream_t s) {
  if (M <= 4) return run_quad_auto<1, 8>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  if (M <= 8) return run_quad_auto<2, 8>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  // 9..16 hidden rows: 8 loads per row and wavefront when that makes d a single K-iteration (up to 128 KB of
  // LDS for the hidden-row operands), else 4
  if (M <= 12) {
    if (d > 2048 && d <= 4096) return run_quad_auto<3, 8>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
    return run_quad_auto<3, 4>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  }
  if (M <= 16) {
    if (d > 2048 && d <= 4096) return run_quad_auto<4, 8>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
    return run_quad_auto<4, 4>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  }
  // wide trees: split K across workgroups while the rows alone cannot fill the chip
  const int S = (d + 511) / 512;
  const int64_t need = (int64_t)S * batch * M * cap_rows * 4;
  const bool split = n_dev != nullptr && partial != nullptr && S >= 2 && need <= partial_bytes &&
                     (int64_t)cap_rows * batch <= 16384 && cap_rows % 64 == 0 && ld % 4 == 0;
  if (split) {
    if (M <= 32) return run_splitk<2>(W, H, ids, n_dev, cap_rows, V, batch, M, d, ld, ids_stride, logits, partial, S, opos, s);
    return run_splitk<4>(W, H, ids, n_dev, cap_rows, V, batch, M, d, ld, ids_stride, logits, partial, S, opos, s);
  }
  if (M <= 32) return run_tile64<2>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
  return run_tile64<4>(W, H, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld, ids_stride, logits, opos, s);
}

// One row list shared by several sequences (rows that many sequences of a batch hold): every listed row is
// multiplied with all rows_total hidden rows H[rows_total][d] (the sequences' hidden rows back to back, seq_rows
// each), 64 hidden rows per launch group, and the logit of list row j for a hidden row of sequence q goes to
// column opos[q * opos_stride + j] of that hidden row's logits row (nowhere if negative: q does not hold the row).
// n_rep: the list length on the device, once per group (rows_total / 64 + 1 equal entries).  cap_rows % 64 == 0.
template <int MT>
static hipError_t run_shared(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_rep, int32_t cap_rows, int32_t V,
                             int32_t groups, int32_t M, int32_t d, int64_t ld, float* logits, const int32_t* opos, int64_t opos_stride,
                             int32_t seq_rows, int32_t row0, hipStream_t s) {
  constexpr int LDS = 4 * 16 * (1024 + kTilePad);
  const int fast = d % 512 != 0 ? 0 : (M == 64 ? 2 : 1);
  const dim3 grid(cap_rows / 64, 1, groups);
  if (fast == 2) head_tile64_kernel<MT, true, 2><<<grid, 256, LDS, s>>>(W, H, ids, n_rep, 0, V, M, d, ld, 0, logits, opos, opos_stride, seq_rows, row0);
  else if (fast == 1) head_tile64_kernel<MT, true, 1><<<grid, 256, LDS, s>>>(W, H, ids, n_rep, 0, V, M, d, ld, 0, logits, opos, opos_stride, seq_rows, row0);
  else head_tile64_kernel<MT, true, 0><<<grid, 256, LDS, s>>>(W, H, ids, n_rep, 0, V, M, d, ld, 0, logits, opos, opos_stride, seq_rows, row0);
  return hipGetLastError();
}

hipError_t launch_head_shared(const void* W, const void* H, const int32_t* ids, const int32_t* n_rep, int32_t cap_rows, int32_t V,
                              int32_t rows_total, int32_t seq_rows, int32_t d, int64_t ld_logits, float* logits, const int32_t* opos,
                              int64_t opos_stride, hipStream_t s) {
  const uint16_t* Wp = static_cast<const uint16_t*>(W);
  const uint16_t* Hp = static_cast<const uint16_t*>(H);
  if (cap_rows < 64 || cap_rows % 64 != 0 || opos_stride % 4 != 0 || seq_rows < 1 || rows_total < 1) return hipErrorInvalidValue;
  const int groups = rows_total / 64, tail = rows_total % 64;
  if (groups > 0) {
    hipError_t e = run_shared<4>(Wp, Hp, ids, n_rep, cap_rows, V, groups, 64, d, ld_logits, logits, opos, opos_stride, seq_rows, 0, s);
    if (e != hipSuccess) return e;
  }
  if (tail > 0) {                                           // the last, shorter group of hidden rows
    const uint16_t* Ht = Hp + (int64_t)groups * 64 * d;
    float* lt = logits + (int64_t)groups * 64 * ld_logits;
    if (tail <= 32) return run_shared<2>(Wp, Ht, ids, n_rep, cap_rows, V, 1, tail, d, ld_logits, lt, opos, opos_stride, seq_rows, groups * 64, s);
    return run_shared<4>(Wp, Ht, ids, n_rep, cap_rows, V, 1, tail, d, ld_logits, lt, opos, opos_stride, seq_rows, groups * 64, s);
  }
  return hipSuccess;
}

// The dynamic-LDS limit of a kernel is a per-device attribute of the function.  Every instantiation that may ask
// for more than the default 48 KB gets the chip's whole 160 KB once per device -- at nanospec_create or at the
// first stateless call on the device, never in a launch path -- so that no later call can lower it under a live
// state and no asynchronous call makes a runtime call that is not a launch.
constexpr int kLdsLimit = 160 * 1024;

template <int MT, int KS>
static hipError_t configure_quad() {
  const void* fns[] = {reinterpret_cast<const void*>(head_quad_kernel<1, 1, MT, KS, true>),
                       reinterpret_cast<const void*>(head_quad_kernel<2, 1, MT, KS, true>),
                       reinterpret_cast<const void*>(head_quad_kernel<4, 1, MT, KS, true>),
                       reinterpret_cast<const void*>(head_quad_kernel<2, 2, MT, KS, true>)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

template <int MT>
static hipError_t configure_tile64() {
  const void* fns[] = {reinterpret_cast<const void*>(head_tile64_kernel<MT, false, 0>), reinterpret_cast<const void*>(head_tile64_kernel<MT, false, 1>),
                       reinterpret_cast<const void*>(head_tile64_kernel<MT, false, 2>), reinterpret_cast<const void*>(head_tile64_kernel<MT, true, 0>),
                       reinterpret_cast<const void*>(head_tile64_kernel<MT, true, 1>), reinterpret_cast<const void*>(head_tile64_kernel<MT, true, 2>)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t head_configure_device() {
  hipError_t e = configure_quad<1, 8>();
  if (e == hipSuccess) e = configure_quad<2, 8>();
  if (e == hipSuccess) e = configure_quad<3, 8>();
  if (e == hipSuccess) e = configure_quad<3, 4>();
  if (e == hipSuccess) e = configure_quad<4, 8>();
  if (e == hipSuccess) e = configure_quad<4, 4>();
  if (e == hipSuccess) e = configure_tile64<2>();
  if (e == hipSuccess) e = configure_tile64<4>();
  return e;
}

hipError_t launch_head(const void* W, const void* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed,
                       int32_t cap_rows, int32_t V, int32_t batch, int32_t M, int32_t d, int64_t ld_logits, int64_t ids_stride,
                       float* logits, float* partial, int64_t partial_bytes, const int32_t* opos, hipStream_t s) {
  const uint16_t* Wp = static_cast<const uint16_t*>(W);
  const uint16_t* Hp = static_cast<const uint16_t*>(H);
  // more than 16 hidden rows of one sequence: the register-blocked product wherever it is the faster one (many rows: the
  // dense comparison point of wide trees and batches; a few thousand rows: wide trees, instead of split-K + reduce)
  if (wide_supported(M, d, batch, cap_rows))
    return launch_head_wide(W, H, ids, n_dev, n_fixed, cap_rows, V, M, d, ld_logits, logits, opos, s);
  if (M <= 64)
    return launch_head_64(Wp, Hp, ids, n_dev, n_fixed, cap_rows, V, batch, M, d, ld_logits, ids_stride, logits, partial,
                          partial_bytes, opos, s);
  if (batch == 1) {                       // many hidden rows of one sequence: 64 at a time
    for (int m0 = 0; m0 < M; m0 += 64) {
      const int mm = M - m0 < 64 ? M - m0 : 64;
      hipError_t e = launch_head_64(Wp, Hp + (int64_t)m0 * d, ids, n_dev, n_fixed, cap_rows, V, 1, mm, d, ld_logits, ids_stride,
                                    logits + (int64_t)m0 * ld_logits, partial, partial_bytes, opos, s);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  dim3 grid((cap_rows + 3) / 4, 1, batch);
  head_generic_kernel<8><<<grid, 256, 0, s>>>(Wp, Hp, ids, n_dev, n_fixed, M, d, ld_logits, ids_stride, logits, opos);
  return hipGetLastError();
}

}  // namespace nanospec
