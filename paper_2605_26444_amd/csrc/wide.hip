// Eq. 1 of the paper (Sec. 3.1) for many hidden rows at once -- the dense comparison point of a wide draft tree
// (64 hidden rows) and of a batch of sequences (hundreds) -- as a register-blocked matrix-core product.
//
// The kernels of head.hip give every wavefront one 16-row tile of W_head and stream all hidden rows past it: each
// matrix instruction then needs 1.25 KB of operands out of LDS, 2.5 times what LDS delivers at the matrix cores'
// rate, and W_head is read once per 64 hidden rows.  Here a workgroup owns a BM x BN block of the logits (BM rows
// of W_head, BN hidden rows) and walks K in steps of BK columns: both operand blocks of a step are fetched with
// 16-byte loads into registers two steps ahead, parked in padded LDS (two stages, one barrier per step), and every
// wavefront multiplies an (FR*16) x (FH*16) sub-block, so one operand fragment read from LDS feeds FH (or FR)
// matrix instructions.  W_head is read once per BN hidden rows.
#include "common.h"

namespace nanospec {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWidePad = 32;     // bytes between LDS rows: rows r and r+4 share banks, the 16 lanes of a fragment read never meet

// WR x WH wavefronts (4 or 8); a wavefront owns FR x FH fragments of 16 x 16 logits.
//   logits[m][j] for hidden row m < M and list row j < n, row stride ld.  ids == nullptr: rows 0..n-1.
//   opos != nullptr ([opos_len], a multiple of 4 entries): row j's logits go to column opos[j] instead, nowhere if negative.
// d % BK == 0 (checked by the launcher).  Rows past n read row 0, hidden rows past M read row M-1; neither is stored.
// Workgroup order: the chip hands consecutive workgroups to its eight dies in turn and each die has its own L2, so
// the hidden-row blocks of one row block run back to back on one die (blockIdx -> (row block, hidden block) below)
// and find the row block's weights in that L2.
template <int WR, int WH, int FR, int FH, int BK, int D>
__global__ __launch_bounds__(64 * WR * WH) void head_wide_kernel(const uint16_t* __restrict__ W, const uint16_t* __restrict__ H,
                                                        const int32_t* __restrict__ ids, const int32_t* __restrict__ n_dev, int n_fixed,
                                                        int V, int M, int d, int64_t ld, float* __restrict__ logits, int row_blocks,
                                                        int hid_blocks, const int32_t* __restrict__ opos, int opos_len) {
  constexpr int NT = 64 * WR * WH;
  constexpr int BM = WR * FR * 16, BN = WH * FH * 16;
  constexpr int CPR = BK / 8;                      // 16-byte pieces per row and step
  constexpr int RPP = NT / CPR;                    // rows one pass of the workgroup's threads covers
  constexpr int NA = BM / RPP, NB = BN / RPP;      // passes over the W block / the hidden-row block
  constexpr int STR = BK * 2 + kWidePad;           // LDS row stride in bytes
  constexpr int STAGE = (BM + BN) * STR;
  static_assert(BM % RPP == 0 && BN % RPP == 0, "whole passes");
  static_assert(D >= 2 && D % 2 == 0, "step s reads LDS stage s & 1: the unrolled group of D steps must keep that parity");
  extern __shared__ __attribute__((aligned(16))) char smem[];

  // blockIdx -> die x = blockIdx % 8, slot r = blockIdx / 8; hidden block = r % hid_blocks, row block = (r / hid_blocks) * 8 + x
  const int xq = blockIdx.x & 7, xr = blockIdx.x >> 3;
  const int hb = xr % hid_blocks, rb = (xr / hid_blocks) * 8 + xq;
  if (rb >= row_blocks) return;
  const int n = n_dev ? n_dev[0] : n_fixed;
  const int j0 = rb * BM, m0 = hb * BN;
  if (j0 >= n) return;

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int wr = w / WH, wh = w % WH;
  const int pc = tid % CPR, pr = tid / CPR;        // this thread's 16-byte piece and first row of a pass

  // byte offsets of this thread's pieces from W and H (below 4 GB each: checked by the launcher)
  uint32_t aoff[NA], boff[NB];
  int rowv[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int j = j0 + pr + i * RPP;
    rowv[i] = j < n ? j : j0;                      // a row past the end is a copy of the block's first row, never stored
  }
  if (ids) {                                        // one uniform branch around all of them: the loads go out together
#pragma unroll
    for (int i = 0; i < NA; ++i) rowv[i] = ids[rowv[i]];
  }
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    int64_t row = rowv[i];
    row = row < 0 ? 0 : (row >= V ? V - 1 : row);
    aoff[i] = (uint32_t)(row * d * 2 + pc * 16);
  }
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    int m = m0 + pr + i * RPP;
    m = m < M ? m : M - 1;
    boff[i] = (uint32_t)((int64_t)m * d * 2 + pc * 16);
  }
  const char* Wb = reinterpret_cast<const char*>(W);
  const char* Hbase = reinterpret_cast<const char*>(H);

  // D register sets: the loads of step s+D are issued before the matrix work of step s starts, so a load has D
  // steps' time to arrive (one step of matrix work is shorter than an HBM round trip) and D-1 sets -- (D-1) x (BM+BN)
  // x BK x 2 bytes -- are in flight per workgroup all the time
  u32x4 ga[D][NA], gb[D][NB];
  auto fetch = [&](int ks, int set) {
    const uint32_t off = (uint32_t)ks * BK * 2;
#pragma unroll
    for (int i = 0; i < NA; ++i) ga[set][i] = *reinterpret_cast<const u32x4*>(Wb + (aoff[i] + off));
#pragma unroll
    for (int i = 0; i < NB; ++i) gb[set][i] = *reinterpret_cast<const u32x4*>(Hbase + (boff[i] + off));
  };
  auto park = [&](int stage, int set) {
    char* As = smem + stage * STAGE;
    char* Bs = As + BM * STR;
#pragma unroll
    for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4*>(As + (pr + i * RPP) * STR + pc * 16) = ga[set][i];
#pragma unroll
    for (int i = 0; i < NB; ++i) *reinterpret_cast<u32x4*>(Bs + (pr + i * RPP) * STR + pc * 16) = gb[set][i];
  };

  f32x4 acc[FR][FH];
#pragma unroll
  for (int a = 0; a < FR; ++a)
#pragma unroll
    for (int b = 0; b < FH; ++b) acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

  // fragment addresses: lane = row (mod 16) + 16 * k group, 8 consecutive k (16 bytes) per lane
  const int frag_off = (lane & 15) * STR + (lane >> 4) * 16;
  // One step: BK/32 sub-steps of FR x FH matrix instructions.  Operand fragments are asked for one fragment ahead
  // of their use (the next row fragment while the current one's FH instructions run, the next sub-step's hidden-row
  // fragments during the last row fragment), so an LDS round trip is covered by matrix work of the same wavefront.
  auto multiply = [&](int stage) {
    const char* As = smem + stage * STAGE + (wr * FR * 16) * STR + frag_off;
    const char* Bs = smem + stage * STAGE + BM * STR + (wh * FH * 16) * STR + frag_off;
    constexpr int KK = BK / 32;
    if constexpr (WR * WH != 8) {                     // memory-bound shape: the plain order, scheduled by the compiler (205 against 217 us)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        bf16x8 bq[FH];
#pragma unroll
        for (int b = 0; b < FH; ++b) bq[b] = *reinterpret_cast<const bf16x8*>(Bs + b * 16 * STR + kk * 64);
#pragma unroll
        for (int a = 0; a < FR; ++a) {
          const bf16x8 aq = *reinterpret_cast<const bf16x8*>(As + a * 16 * STR + kk * 64);
#pragma unroll
          for (int b = 0; b < FH; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aq, bq[b], acc[a][b], 0, 0, 0);
        }
      }
      return;
    }
    bf16x8 bf[2][FH], af[2];
#pragma unroll
    for (int b = 0; b < FH; ++b) bf[0][b] = *reinterpret_cast<const bf16x8*>(Bs + b * 16 * STR);
    af[0] = *reinterpret_cast<const bf16x8*>(As);
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
      for (int a = 0; a < FR; ++a) {
        const int cur = (kk * FR + a) & 1;
        if (a + 1 < FR) {
          af[cur ^ 1] = *reinterpret_cast<const bf16x8*>(As + (a + 1) * 16 * STR + kk * 64);
        } else if (kk + 1 < KK) {
          af[cur ^ 1] = *reinterpret_cast<const bf16x8*>(As + (kk + 1) * 64);
#pragma unroll
          for (int b = 0; b < FH; ++b) bf[(kk + 1) & 1][b] = *reinterpret_cast<const bf16x8*>(Bs + b * 16 * STR + (kk + 1) * 64);
        }
#pragma unroll
        for (int b = 0; b < FH; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[cur], bf[kk & 1][b], acc[a][b], 0, 0, 0);
      }
    }
    // The order above is the order wanted; left alone, the scheduler puts every fragment read right in front of its
    // first use.  Groups: the LDS reads of the next fragment(s), then FH matrix instructions.  Only for the
    // compute-bound shapes (eight wavefronts): 644 -> 614 us at 512 hidden rows on 256 x 128 logits; the memory-bound
    // four-wavefront shape loses with it (205 -> 218 us at 64 hidden rows).
    if constexpr (WR * WH == 8) {
      __builtin_amdgcn_sched_group_barrier(0x100, FH + 1, 0);
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
#pragma unroll
        for (int a = 0; a < FR; ++a) {
          if (a + 1 < FR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          else if (kk + 1 < KK) __builtin_amdgcn_sched_group_barrier(0x100, FH + 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, FH, 0);
        }
      }
    }
  };

  // Every fetch is unconditional -- past the end the last step is fetched again and never used -- because a load
  // under a branch makes the number of loads in flight unknowable at compile time, and every wait for one register
  // set then becomes a wait for all of them.  Set s % D receives step s + D right after it was parked for step s.
  // D == 2: nk is even (the launcher checks d % (2 * BK) == 0) and the loop body has no branch at all; D = 4, 6, ..: any nk,
  // the steps past the end skip their matrix work (a uniform branch around LDS reads and matrix instructions only).
  const int nk = d / BK;
#pragma unroll
  for (int j = 0; j < D; ++j) fetch(j < nk ? j : nk - 1, j);
  __builtin_amdgcn_sched_barrier(0);
  park(0, 0);
  __syncthreads();
  for (int ks = 0; ks < nk; ks += D) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
      const int st = ks + j;                        // LDS stage j & 1 holds this step, set (j + 1) % D holds (or awaits) the next
      fetch(st + D < nk ? st + D : nk - 1, j);
      __builtin_amdgcn_sched_barrier(0);            // the loads go out before the matrix work, not after it
      if (D == 2 || st < nk) multiply(j & 1);
      park((j + 1) & 1, (j + 1) % D);               // that stage's last readers passed the previous barrier
      __syncthreads();
    }
  }

  // result lane l holds list rows j + v (v = 0..3), j = 4 * (l / 16), of hidden row l % 16 of the fragment
#pragma unroll
  for (int a = 0; a < FR; ++a) {
    const int j = j0 + (wr * FR + a) * 16 + 4 * (lane >> 4);
#pragma unroll
    for (int b = 0; b < FH; ++b) {
      const int m = m0 + (wh * FH + b) * 16 + (lane & 15);
      if (m >= M || j >= n) continue;
      float* dst = logits + (int64_t)m * ld + j;
      if (opos) {                                       // rows kept in an order of their own: list row j's logits go to column opos[j]
        const int4 jo4 = j + 3 < opos_len ? *reinterpret_cast<const int4*>(opos + j) : make_int4(-1, -1, -1, -1);
        const int jo[4] = {jo4.x, jo4.y, jo4.z, jo4.w};
        float* rowp = logits + (int64_t)m * ld;
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (j + v < n && jo[v] >= 0) rowp[jo[v]] = acc[a][b][v];
      } else if ((ld & 3) == 0 && j + 3 < n) {
        *reinterpret_cast<f32x4*>(dst) = acc[a][b];
      } else {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (j + v < n) dst[v] = acc[a][b][v];
      }
    }
  }
}

template <int WR, int WH, int FR, int FH, int BK, int D>
static hipError_t run_wide(const uint16_t* W, const uint16_t* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed, int32_t cap_rows,
                           int32_t V, int32_t M, int32_t d, int64_t ld, float* logits, const int32_t* opos, hipStream_t s) {
  constexpr int BM = WR * FR * 16, BN = WH * FH * 16;
  constexpr int LDS = 2 * (BM + BN) * (BK * 2 + kWidePad);
  const int row_blocks = (cap_rows + BM - 1) / BM, hid_blocks = (M + BN - 1) / BN;
  const int64_t grid = (int64_t)((row_blocks + 7) / 8) * hid_blocks * 8;
  if (grid > 0x7fffffff || (int64_t)V * d * 2 > 0xffffffffll || (int64_t)M * d * 2 > 0xffffffffll) return hipErrorInvalidValue;
  head_wide_kernel<WR, WH, FR, FH, BK, D><<<dim3((unsigned)grid), 64 * WR * WH, LDS, s>>>(W, H, ids, n_dev, n_fixed, V, M, d, ld, logits, row_blocks, hid_blocks, opos, cap_rows / 4 * 4);
  return hipGetLastError();
}

hipError_t wide_configure_device() {
  const void* fns[] = {reinterpret_cast<const void*>(head_wide_kernel<4, 1, 2, 4, 64, 2>), reinterpret_cast<const void*>(head_wide_kernel<4, 2, 4, 4, 64, 2>),
                       reinterpret_cast<const void*>(head_wide_kernel<2, 4, 8, 4, 64, 2>), reinterpret_cast<const void*>(head_wide_kernel<2, 2, 1, 1, 256, 2>)};
  for (const void* f : fns) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Which row capacities the register-blocked product takes (one sequence or the dense head, 16 < M, no column map):
//   at least 16384 rows and d % 128 == 0: the three block shapes of launch_head_wide below;
//   a few thousand rows, M <= 64 and d % 512 == 0: the 32 x 32 shape (no split of K, one launch) from the capacity on
//   at which it beats split-K + reduce (measured at d = 3584, M = 64 / 32, live rows = capacity: 8.9 against 10.7 us
//   at 1000 rows, 11.6 / 11.7 at 2000, 14.9 / 12.3 at 3000, 25.4 / 21.2 at 8000; M = 32: 12.7 / 12.4 at 3000, 17.6 / 13.3
//   at 5000).
bool wide_supported(int32_t M, int32_t d, int32_t batch, int32_t cap_rows) {
  if (batch != 1 || M <= 16) return false;
  if (cap_rows >= 16384) return d % 128 == 0;                    // an even number of 64-column steps
  return M <= 64 && d % 512 == 0 && cap_rows >= (M <= 32 ? 4096 : 2560);
}

// One sequence (or the dense head), more than 16 hidden rows.
//   a few thousand rows (wide draft trees): latency-bound.  32 x 32 logits per workgroup of four wavefronts, 256-column
//     steps (512 bytes of a row per load pass, 64 KB in flight per workgroup) -- the rows alone cannot fill the chip,
//     so the hidden rows are split in two as well.  3000 rows x 64 hidden rows, d = 3584: 12.2 us in one launch against
//     10 + 4 us for split-K and its reduce.  The time is the 458 KB every workgroup pulls through its compute unit's
//     L1 (11.7 us without any matrix work); three or four register sets in flight instead of two: 13.6 / 14.1 us;
//     128-column steps 13.6; 64 x 16 logits 14.9.
//   many rows, up to 64 hidden rows: memory-bound.  128 x 64 logits per workgroup of four wavefronts, 60 KB of LDS, two
//     workgroups per compute unit (dense 152k x 3584 head at 64 hidden rows: 205-219 us, the vendor GEMM 205-208,
//     5.2 TB/s; 256-byte steps with one workgroup per compute unit: 209 us).
//   up to 128: 256 x 128 logits, eight wavefronts of 64 x 64.
//   more: compute-bound.  256 x 256 logits per workgroup, eight wavefronts of 128 x 64 (one fragment read feeds four or
//     eight matrix instructions), all 160 KB of LDS for the two stages.  512 hidden rows on the 128k x 4096 matrix:
//     516-539 us = 1.0 PFLOP/s, the vendor GEMM 510-513.  On the way there: four wavefronts of 128 x 64 on 256 x 128
//     logits 844 us (one wavefront per SIMD: nothing overlaps an LDS round trip), eight of 64 x 64 644 us, with the
//     scheduling groups 614 us, 256 x 256 logits in 32-column steps 553 us.
hipError_t launch_head_wide(const void* W, const void* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed, int32_t cap_rows,
                            int32_t V, int32_t M, int32_t d, int64_t ld, float* logits, const int32_t* opos, hipStream_t s) {
  const uint16_t* Wp = static_cast<const uint16_t*>(W);
  const uint16_t* Hp = static_cast<const uint16_t*>(H);
  if (cap_rows < 16384) return run_wide<2, 2, 1, 1, 256, 2>(Wp, Hp, ids, n_dev, n_fixed, cap_rows, V, M, d, ld, logits, opos, s);
  if (M <= 64) return run_wide<4, 1, 2, 4, 64, 2>(Wp, Hp, ids, n_dev, n_fixed, cap_rows, V, M, d, ld, logits, opos, s);
  if (M <= 128) return run_wide<4, 2, 4, 4, 64, 2>(Wp, Hp, ids, n_dev, n_fixed, cap_rows, V, M, d, ld, logits, opos, s);
  return run_wide<2, 4, 8, 4, 64, 2>(Wp, Hp, ids, n_dev, n_fixed, cap_rows, V, M, d, ld, logits, opos, s);
}

}  // namespace nanospec
