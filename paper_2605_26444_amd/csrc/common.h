// Internal declarations shared by the translation units of libnanospec (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nanospec.h"

namespace nanospec {

constexpr int kVocabThreads = 1024;   // one workgroup per sequence in the vocabulary kernel
constexpr int kTopkThreads = 1024;    // single-pass top-k workgroup
constexpr int kTopkChunk = 16384;     // elements per workgroup in the two-pass top-k
constexpr int kMaxK = 64;
constexpr int kCandMax = 256;          // top-k fast path: most candidates ranked directly

// Per-sequence offsets travel by value in the kernel argument block (no H2D copy, graph-safe).
struct Offsets {
  int32_t v[NANOSPEC_MAX_BATCH + 1];
};

struct VocabPtrs {
  int32_t* ring;        // [batch][window]
  uint32_t* cnt;        // [batch][V]
  uint32_t* wbit;       // [batch][nwords]
  uint32_t* tbit;       // [batch][nwords]
  int32_t* ids;         // [batch][cap]
  int32_t* n;           // [batch]
  int32_t* pos;         // [batch] next ring slot
  int32_t* fill;        // [batch] valid ring entries
  int32_t* err;         // [1] sticky flags
  int32_t V, window, nwords, cap;
};

// Packed-buffer variant (one sequence): slot tables and the row copies.
struct PackedPtrs {
  uint16_t* buf;        // [cap][d] bf16: one row per slot
  int32_t* slot_of;     // [V]   slot that holds the id's row, or -1
  int32_t* slot_id;     // [cap] id whose row the slot holds, or -1
  int32_t* out_pos;     // [cap] position of that id in the ascending active list, or -1
  int32_t* free_list;   // [cap] scratch of one gather: free slots ascending
  int32_t* copy_list;   // [cap][2] scratch of one gather: (id, slot) of the rows to copy
  int32_t* scal;        // [0] slots that may hold a row (highest slot in use + 1), [1] rows on the copy list
  int32_t cap;
};

// Batch-union head (several sequences): rows shared by many sequences, and what is left per sequence.
struct UnionPtrs {
  uint32_t* shared_bits;  // [nwords] bit = id held by at least min_share sequences
  int32_t* shared_cnt;    // [nwords] set bits per word
  int32_t* shared_ids;    // [shared_cap] the lowest shared_cap such ids, ascending
  int32_t* shared_n;      // [groups] their number, repeated once per group of 64 hidden rows
  int32_t* shared_pos;    // [batch][shared_cap] column of shared row r in the sequence's logits, -1 if the sequence lacks it
  int32_t* rest_ids;      // [batch][cap] the sequence's other active ids, ascending
  int32_t* rest_pos;      // [batch][cap] their columns
  int32_t* rest_n;        // [batch]
  int32_t shared_cap, min_share;
};

}  // namespace nanospec

struct nanospec_state {
  int32_t V, d, batch, window, topk_cap, m_cap, k_cap;
  int32_t device;
  nanospec_layout layout;
  nanospec::VocabPtrs vp;
  char* base;               // the one device allocation everything lives in
  float* partial;           // split-K partial logits
  char* topk_ws;            // two-pass top-k candidates
  int64_t partial_bytes, topk_ws_bytes;
  int32_t* h_err_pinned;    // pinned host word for reading the device flags
  int vocab_lds_bytes, unique_lds_bytes, unique_cap, fifo_lds_bytes;
  int32_t policy, policy_next;   // vocabulary reading in force / chosen for the next init
  nanospec::PackedPtrs pk;       // packed-buffer variant; pk.buf == nullptr until nanospec_packed_enable
  char* pk_base;                 // its one device allocation
  nanospec::UnionPtrs un;        // batch-union head; un_base == nullptr until nanospec_union_enable
  char* un_base;
  int32_t un_groups;             // groups of 64 hidden rows at M = m_cap
  hipStream_t un_side;           // the shared-row product runs here, beside the per-sequence product
  hipEvent_t un_fork, un_join;
};

namespace nanospec {

// vocab.hip
hipError_t launch_vocab_clear(const nanospec_state* st, hipStream_t s);
hipError_t launch_vocab_apply(const nanospec_state* st, const int32_t* d_new, const Offsets& noff,
                              const int32_t* d_topk, const Offsets& toff, int replace_T, hipStream_t s);
hipError_t vocab_configure(nanospec_state* st);
hipError_t vocab_configure_device();
hipError_t launch_vocab_append_unique(const nanospec_state* st, const int32_t* d_cand, int per_seq, int64_t stride,
                                      hipStream_t s);

// head.hip
hipError_t head_configure_device();
// logits[b][m][j] for j < n_b (n read on the device).  ids == nullptr: identity list of n_fixed rows.
// opos != nullptr (row stride ids_stride): row j's logits go to column opos[j] instead, nowhere if negative.
hipError_t launch_head(const void* W, const void* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed,
                       int32_t cap_rows, int32_t V, int32_t batch, int32_t M, int32_t d, int64_t ld_logits,
                       int64_t ids_stride, float* logits, float* partial, int64_t partial_bytes, const int32_t* opos,
                       hipStream_t s);

// every row of one list against rows_total hidden rows of several sequences (seq_rows each); columns per sequence
hipError_t launch_head_shared(const void* W, const void* H, const int32_t* ids, const int32_t* n_rep, int32_t cap_rows, int32_t V,
                              int32_t rows_total, int32_t seq_rows, int32_t d, int64_t ld_logits, float* logits, const int32_t* opos,
                              int64_t opos_stride, hipStream_t s);

// wide.hip: register-blocked product for more than 16 hidden rows of one sequence / the dense head
bool wide_supported(int32_t M, int32_t d, int32_t batch, int32_t cap_rows);
hipError_t wide_configure_device();
hipError_t launch_head_wide(const void* W, const void* H, const int32_t* ids, const int32_t* n_dev, int32_t n_fixed, int32_t cap_rows,
                            int32_t V, int32_t M, int32_t d, int64_t ld, float* logits, const int32_t* opos, hipStream_t s);

// union.hip
hipError_t union_configure_device();
hipError_t launch_union_reset(const nanospec_state* st, hipStream_t s);
hipError_t launch_union_build(const nanospec_state* st, hipStream_t s);

// topk.hip
int64_t topk_workspace_bytes(int32_t cap, int32_t rows, int32_t k);
hipError_t launch_topk(const float* logits, int64_t ld, const int32_t* ids, int64_t ids_stride, const int32_t* n_dev,
                       int32_t n_fixed, int32_t cap, int32_t batch, int32_t M, int32_t k, int32_t* out_ids,
                       float* out_vals, bool logprob, char* ws, int64_t ws_bytes, hipStream_t s);

// packed.hip
hipError_t launch_packed_reset(const nanospec_state* st, hipStream_t s);
hipError_t launch_packed_gather(const nanospec_state* st, const void* W, hipStream_t s);

// calib.hip
hipError_t launch_calib_stream(const void* buf, int64_t bytes, void* sink, hipStream_t s);
hipError_t launch_calib_valu_head(const void* W, const void* H, int32_t V, int32_t d, int32_t M, const int32_t* ids,
                                  const int32_t* n_dev, int32_t cap, float* logits, hipStream_t s);
hipError_t calib_configure_device();
hipError_t launch_calib_gather(const void* W, int32_t V, int32_t d, const int32_t* ids, const int32_t* n_dev, int32_t cap,
                               void* sink, hipStream_t s);

}  // namespace nanospec
