/*
 * nanospec.h -- C ABI of the NanoSpec draft-step hot path for AMD MI355X (gfx950).
 *
 * The library keeps a context-aware active vocabulary on the GPU, projects draft hidden states
 * onto the active rows of the bf16 LM-head matrix, and selects the top-k draft tokens.  It
 * follows the problem statement of the NanoSpec paper (arXiv 2605.26444):
 *
 *   Eq. 1   z = W_head h                       dense head (the comparison point)
 *   Sec 3.1 z' = W_head[I_t, :] h              sparse head on the active rows only
 *   Eq. 2-3 candidate stream S, appended to at prefill and after every verification
 *   Eq. 4   I_t = Unique(Suffix(S, W_max))     active index set, recency eviction
 *   Alg. 1  SelectDraftTokens(z', I)           top-k over z' mapped back to global ids
 *   Sec 3.3 / appendix                         the same state read as a first-in first-out queue of
 *                                              distinct ids (nanospec_set_stream_policy)
 *   Sec 4.2 softmax over the active set only   log-probabilities with the selection
 *                                              (nanospec_topk_logprob_remap)
 *
 * Conventions
 *   - Token ids are 0-based int32 in [0, V).
 *   - Pointers named d_* are DEVICE pointers, h_* are HOST pointers.  The caller owns every
 *     buffer it passes in; the library owns the state object and frees it in nanospec_destroy.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call
 *     documented as "asynchronous" only enqueues kernels on that stream: it never synchronises
 *     the host, never allocates and never frees, so it may be recorded into a HIP graph.
 *   - All functions return a nanospec_status; nothing aborts or throws.  Argument errors are
 *     found on the host before anything is launched, in which case nothing is enqueued.
 *   - A state object must not be used from two streams at once.
 *   - bf16 = upper 16 bits of an IEEE fp32.  Products are accumulated in fp32.
 */
#ifndef NANOSPEC_H_
#define NANOSPEC_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define NANOSPEC_API __attribute__((visibility("default")))
#else
#define NANOSPEC_API
#endif

typedef struct nanospec_state nanospec_state; /* opaque; owns all device-resident state */
typedef int32_t nanospec_status;

enum {
  NANOSPEC_OK = 0,
  NANOSPEC_EINVAL = -1,    /* null pointer, non-positive size, unsupported shape, bad offsets   */
  NANOSPEC_ENOMEM = -2,    /* device or host allocation failed (nanospec_create only)           */
  NANOSPEC_ECAPACITY = -3, /* an input exceeds a capacity fixed at nanospec_create              */
  NANOSPEC_EHIP = -4       /* a HIP runtime call failed                                         */
};

/* Bits reported by nanospec_last_device_error. */
enum {
  NANOSPEC_DEV_BAD_ID = 1 /* an appended or candidate id was outside [0, V); it was ignored     */
};

/* Largest batch (independent sequences per state) supported: per-sequence offsets travel as
 * kernel arguments so that no call needs a host-to-device copy. */
#define NANOSPEC_MAX_BATCH 256

/* Human-readable name of a status code (static storage). */
NANOSPEC_API const char* nanospec_status_string(nanospec_status s);

/* Byte sizes of the device buffers a state with these parameters owns.  Pure host arithmetic
 * (usable without a GPU); nanospec_create allocates exactly these.  For the paper's Llama-3.1-8B
 * setting (V=128256, W_max=3072) the bitmap is ceil(V/32)*4 = 16032 B and the stream ring
 * 3072*4 = 12288 B, the "16 KB" and "12 KB" rows of Table 6; `gathered_bytes_at_cap` is the size
 * the paper's repack buffer would have (window * d * 2; 24 MiB there), which this library never
 * allocates because the gather is fused into the projection. */
typedef struct nanospec_layout {
  int64_t ring_bytes;            /* per sequence: last `window` stream ids, int32                */
  int64_t counter_bytes;         /* per sequence: window multiplicity of every id, uint32[V]     */
  int64_t window_bitmap_bytes;   /* per sequence: 1 bit per id, set iff multiplicity > 0         */
  int64_t topk_bitmap_bytes;     /* per sequence: 1 bit per id, set iff id is in the set T       */
  int64_t ids_bytes;             /* per sequence: ascending active ids, int32[capacity]          */
  int64_t scalars_bytes;         /* per sequence: n, ring position, fill                         */
  int64_t workspace_bytes;       /* whole state: split-K partial logits + top-k candidates       */
  int64_t total_bytes;           /* everything, all sequences                                    */
  int64_t gathered_bytes_at_cap; /* window * d * 2: what a packed copy of the rows would take    */
  int32_t capacity;              /* row stride of ids / logits: max |I_t| rounded up to 64       */
} nanospec_layout;

NANOSPEC_API nanospec_status nanospec_state_layout(int32_t V, int32_t d, int32_t batch, int32_t window,
                                      int32_t topk_cap, int32_t m_cap, int32_t k_cap,
                                      nanospec_layout* out);

/* Create the device-resident state for `batch` independent sequences on the current device.
 *   V         vocabulary size (rows of W_head)            d        hidden size, multiple of 8
 *   window    W_max of Eq. 4                               topk_cap largest |T| per sequence
 *   m_cap     largest number of draft hidden rows per sequence and call
 *   k_cap     largest k of nanospec_topk_remap (<= 64)
 * Limits: batch <= NANOSPEC_MAX_BATCH; min(window + topk_cap, V) <= 262144 (16 top-k chunks); the vocabulary
 * kernels keep three V-bit bitmaps in one workgroup's LDS, which bounds V at about 420 000.
 * Errors: EINVAL (null, a size < 1, d % 8 != 0, a limit above exceeded), ENOMEM, EHIP.
 * Synchronous (allocates).  The state starts empty: stream length 0, T empty, I empty.  The state belongs to
 * the device that is current here; every later call on it returns EINVAL if another device is current. */
NANOSPEC_API nanospec_status nanospec_create(nanospec_state** out, int32_t V, int32_t d, int32_t batch,
                                int32_t window, int32_t topk_cap, int32_t m_cap, int32_t k_cap);
NANOSPEC_API nanospec_status nanospec_destroy(nanospec_state* st);

/* Which reading of the paper's vocabulary the state follows; takes effect at the next nanospec_vocab_init.
 *   NANOSPEC_POLICY_WINDOW (default): Eq. 4 -- the window covers the last W_max entries of the raw stream,
 *       repeats included; a token stays while any of its occurrences is inside the window.
 *   NANOSPEC_POLICY_FIFO: the state management of Sec. 3.3 as the appendix on vocabulary evolution describes
 *       it -- a first-in first-out queue of at most W_max distinct ids.  One call (init, update,
 *       append_unique) pushes, in the order of their first occurrence, the ids that are valid, not members
 *       when the call starts and not repeated inside the call; the oldest members leave first; a member
 *       that is appended again keeps its place.  Ids outside [0,V) are skipped and flagged.
 * Everything else (T, the ascending list, head, selection) is the same.  Errors: EINVAL. */
#define NANOSPEC_POLICY_WINDOW 0
#define NANOSPEC_POLICY_FIFO 1
NANOSPEC_API nanospec_status nanospec_set_stream_policy(nanospec_state* st, int32_t policy);

/* Stream initialisation, Eq. 2 and the first I of Alg. 1: for sequence b the stream becomes
 * ctx_ids[h_ctx_off[b] .. h_ctx_off[b+1]) (only its last `window` ids matter) and the candidate
 * set T becomes topk_ids[h_topk_off[b] .. h_topk_off[b+1]) (duplicates allowed, order
 * irrelevant).  The active set I = Unique(Suffix(S, window)) U T is left on the device as an
 * ascending id list with its count.  The paper appends top-K candidates to the stream itself;
 * that mode is T = empty with those ids appended through ctx/new ids.
 *   d_ctx_ids, d_topk_ids : device int32; may be NULL when every range is empty.
 *   h_ctx_off, h_topk_off : host int32[batch+1], non-decreasing, read before the call returns.
 * Errors: EINVAL (null state/offsets, decreasing offsets), ECAPACITY (a T range > topk_cap).
 * Asynchronous.  Ids outside [0,V) hold their stream position but never become members; they
 * raise NANOSPEC_DEV_BAD_ID. */
NANOSPEC_API nanospec_status nanospec_vocab_init(nanospec_state* st, const int32_t* d_ctx_ids, const int32_t* h_ctx_off,
                                    const int32_t* d_topk_ids, const int32_t* h_topk_off, void* hip_stream);

/* Stream update, Eq. 3 followed by Eq. 4: append new_ids[h_new_off[b] .. h_new_off[b+1]) to the
 * stream of sequence b (zero ids is legal), evict what leaves the window, and bring the
 * ascending active list and its count up to date -- one launch for the whole batch (appends of
 * at most 16 ids that leave T alone patch the list in place, anything else rebuilds it; the
 * result is the same list either way).  If d_topk_ids is not
 * NULL (or h_topk_off is not NULL with all-empty ranges) the set T of every sequence is replaced
 * wholesale; pass both NULL to keep T.  Same argument rules and errors as nanospec_vocab_init.
 * Asynchronous. */
NANOSPEC_API nanospec_status nanospec_vocab_update(nanospec_state* st, const int32_t* d_new_ids, const int32_t* h_new_off,
                                      const int32_t* d_topk_ids, const int32_t* h_topk_off, void* hip_stream);

/* Stream update with the candidate set built on the device, Eq. 3 for C_draft (Sec. 3.2: every distinct
 * token id that occurs in the step's draft tree, accepted or not): for sequence b the ids
 * d_cand_ids[b*cand_stride .. +cand_per_seq) -- typically the [M][k] output of nanospec_topk_remap of the
 * same state, passed without a host round trip -- are de-duplicated and appended to the stream in
 * ascending id order (the paper leaves the order of tuple(set) open), then Eq. 4 as in
 * nanospec_vocab_update.  The number of ids appended is known only on the device.  Entries equal to -1
 * (top-k padding) are skipped; other ids outside [0,V) are skipped and raise NANOSPEC_DEV_BAD_ID.  T is kept.
 * The same call finishes Eq. 2 on the device: after nanospec_vocab_init with the prompt, pass the [L][K_pre]
 * output of nanospec_dense_topk over the prefill logits (the tail of S^(0) is a de-duplicated union too).
 *   d_cand_ids : device int32 [batch][cand_stride]; cand_per_seq is bounded by the LDS of one workgroup:
 *                39776 - 12 * ceil(V/128) entries (27 752 at V = 128256); at least m_cap * k_cap.
 * Errors: EINVAL (null, negative, stride < count), ECAPACITY (cand_per_seq above that bound).  Asynchronous; takes no host integers that
 * change from step to step, so one recorded HIP graph of a whole draft step can be replayed indefinitely. */
NANOSPEC_API nanospec_status nanospec_vocab_append_unique(nanospec_state* st, const int32_t* d_cand_ids,
                                                          int32_t cand_per_seq, int64_t cand_stride, void* hip_stream);

/* Borrowed device views of the active vocabulary, valid until nanospec_destroy; contents are
 * valid in stream order after the last init/update.
 *   *d_ids : int32[batch][capacity], row b holds I of sequence b ascending in [0, n_b)
 *   *d_n   : int32[batch]            |I| per sequence
 *   *capacity : row stride (also the row stride of the logits of nanospec_sparse_head). */
NANOSPEC_API nanospec_status nanospec_vocab_view(const nanospec_state* st, const int32_t** d_ids, const int32_t** d_n,
                                    int32_t* capacity);

/* Sparse head, Eq. 1 restricted to the active rows (Sec. 3.1):
 *   logits[b][m][j] = sum_c W[ids_b[j]][c] * H[b][m][c]   for j < n_b, fp32 accumulation.
 *   d_W_bf16  : bf16 [V][d] row-major by token id          d_H_bf16 : bf16 [batch][M][d]
 *   d_logits  : fp32 [batch][M][capacity]; entries j >= n_b are unspecified.
 * The rows are gathered inside the projection; no packed copy of them is made.  The result for a
 * given (W row, H row) pair does not depend on j, on n or on the other active ids.
 * Errors: EINVAL (null, M < 1), ECAPACITY (M > m_cap).  Asynchronous. */
NANOSPEC_API nanospec_status nanospec_sparse_head(nanospec_state* st, const void* d_W_bf16, const void* d_H_bf16, int32_t M,
                                     float* d_logits, void* hip_stream);

/* The paper's own system design as a variant of the head (Sec. 3.3 "Avoiding sparse computation via asynchronous
 * gathering"; Alg. 1 Gather_Async; the weight-gather row of Table 4; the repacked-weights row of Table 6): a
 * pre-allocated packed buffer of `capacity` rows holds a copy of every active row of W_head; after a vocabulary
 * update only the rows of ids that entered the active set are copied in, and the head is a dense product on
 * the packed buffer.  Slots are stable (an id keeps its slot while it stays active; an entering id takes the
 * lowest free slot), and the logits still come out in the layout of nanospec_sparse_head (column j = j-th
 * active id ascending), so nanospec_topk_remap / nanospec_topk_logprob_remap apply unchanged, ties by lower id
 * included.  One sequence per state (batch == 1).
 *   nanospec_packed_bytes  : device bytes nanospec_packed_enable allocates (capacity*d*2 for the rows -- 24 MiB at
 *                            the paper's W_max = 3072, d = 4096 -- plus V*4 + 20*capacity bytes of slot tables).
 *   nanospec_packed_enable : allocate and clear them.  Synchronous; idempotent.  Errors: EINVAL (batch != 1), ENOMEM, EHIP.
 *   nanospec_packed_gather : bring the buffer in line with the current active list: free the slots of ids that
 *                            left, give every id without a slot one, copy those rows W[id] -> buffer[slot], refresh
 *                            the slot -> column map.  Two launches on `hip_stream`, which may be a second stream
 *                            running beside the draft backbone; the caller orders it after the vocabulary call
 *                            and before nanospec_packed_head with events (the paper's dual-stream pipeline).  The
 *                            first call after nanospec_vocab_init, a T replacement or a long append copies many
 *                            rows, a decoding step a handful.  Asynchronous.  Errors: EINVAL (not enabled), EHIP.
 *   nanospec_packed_head   : logits as nanospec_sparse_head, computed from the packed buffer (W_head is not
 *                            touched).  Asynchronous.  Errors: EINVAL, ECAPACITY (M > m_cap).
 *   nanospec_packed_view   : borrowed device views for inspection: the row buffer bf16 [capacity][d], the id
 *                            held by each slot (-1 free), each slot's logit column (-1 none), and two counters
 *                            {slots that may hold a row, rows copied by the last gather}. */
NANOSPEC_API int64_t nanospec_packed_bytes(const nanospec_state* st);
NANOSPEC_API nanospec_status nanospec_packed_enable(nanospec_state* st);
NANOSPEC_API nanospec_status nanospec_packed_gather(nanospec_state* st, const void* d_W_bf16, void* hip_stream);
NANOSPEC_API nanospec_status nanospec_packed_head(nanospec_state* st, const void* d_H_bf16, int32_t M, float* d_logits,
                                                  void* hip_stream);
NANOSPEC_API nanospec_status nanospec_packed_view(const nanospec_state* st, const void** d_buf, const int32_t** d_slot_id,
                                                  const int32_t** d_out_pos, const int32_t** d_counts);

/* Several sequences in one state (multi-sequence serving; Sec. 4.6 states only that the method's per-sequence cost
 * adds up over the batch): sequences drawing from one token distribution hold many of the same ids, and
 * nanospec_sparse_head fetches such a row once per sequence.  The batch-union head splits the active sets: an id
 * held by at least `min_share` of the sequences is a shared row -- listed once, fetched once, multiplied with the
 * hidden rows of all sequences --, every other id stays on a per-sequence list and is handled as before.  Every
 * (sequence, active id) pair is covered by exactly one part and its logit lands in the column the id has in that
 * sequence's ascending active list: the logits have the layout of nanospec_sparse_head (a sequence that lacks a
 * shared row has no column for it) and nanospec_topk_remap / nanospec_topk_logprob_remap apply unchanged.
 *   nanospec_union_bytes  : device bytes nanospec_union_enable allocates for the given shared_cap (-1: bad argument).
 *   nanospec_union_enable : allocate and clear the lists.  min_share: 0 = max(2, batch/8).  shared_cap: room on the
 *                           shared list, a multiple of 64 in [64, capacity], 0 = capacity; when more ids qualify the
 *                           lowest shared_cap are shared and the others stay per sequence.  Synchronous; once per
 *                           state.  Errors: EINVAL (bad arguments, already enabled), ENOMEM, EHIP.
 *   nanospec_union_build  : rebuild the lists from the current vocabulary state (two launches); call after every
 *                           vocabulary call and before nanospec_union_head; it needs no hidden states, so it may run
 *                           beside the draft backbone.  Asynchronous.  Errors: EINVAL (not enabled), EHIP.
 *   nanospec_union_head   : d_logits fp32 [batch][M][capacity] as nanospec_sparse_head (entries j >= n_b
 *                           unspecified), from d_W_bf16 [V][d] and d_H_bf16 [batch][M][d].  The shared-row product
 *                           runs on a stream the state owns (default priority), forked from `hip_stream` and joined
 *                           back into it by events before the call returns its work to `hip_stream`; a graph
 *                           capture of `hip_stream` records both branches.  Two calls on one state must not
 *                           overlap.  Asynchronous.  Errors: EINVAL, ECAPACITY (M > m_cap), EHIP.
 *   nanospec_union_view   : borrowed device views for inspection: shared ids [shared_cap] and their number
 *                           (first entry of d_shared_n), shared_pos [batch][shared_cap] (column or -1), rest ids
 *                           and columns [batch][capacity], rest_n [batch]; any pointer may be NULL. */
NANOSPEC_API int64_t nanospec_union_bytes(const nanospec_state* st, int32_t shared_cap);
NANOSPEC_API nanospec_status nanospec_union_enable(nanospec_state* st, int32_t min_share, int32_t shared_cap);
NANOSPEC_API nanospec_status nanospec_union_build(nanospec_state* st, void* hip_stream);
NANOSPEC_API nanospec_status nanospec_union_head(nanospec_state* st, const void* d_W_bf16, const void* d_H_bf16, int32_t M,
                                                 float* d_logits, void* hip_stream);
NANOSPEC_API nanospec_status nanospec_union_view(const nanospec_state* st, const int32_t** d_shared_ids, const int32_t** d_shared_n,
                                                 const int32_t** d_shared_pos, const int32_t** d_rest_ids,
                                                 const int32_t** d_rest_pos, const int32_t** d_rest_n, int32_t* shared_cap,
                                                 int32_t* min_share);

/* Draft-token selection, SelectDraftTokens(z', I) of Alg. 1 with the operator T_K of Sec. 3.2:
 * for every (b, m) the k largest of logits[b][m][0..n_b), ordered by value descending then global
 * id ascending (+0 and -0 tie), written as global ids and values.  Slots beyond n_b get id -1
 * and value -inf.  NaN logits are not supported.
 *   d_out_ids : int32 [batch][M][k]       d_out_vals : fp32 [batch][M][k] (may be NULL)
 * Errors: EINVAL, ECAPACITY (M > m_cap or k > k_cap).  Asynchronous. */
NANOSPEC_API nanospec_status nanospec_topk_remap(nanospec_state* st, const float* d_logits, int32_t M, int32_t k,
                                    int32_t* d_out_ids, float* d_out_vals, void* hip_stream);

/* Draft-token selection with the draft distribution renormalised over the active vocabulary (Sec. 4.2
 * attributes the acceptance gain on context-heavy tasks to exactly this renormalisation; tree-style
 * drafters rank their nodes by these log-probabilities): ids and order as nanospec_topk_remap, values
 *   logprob[b][m][r] = z_r - log(sum_{j < n_b} exp(logits[b][m][j])),
 * fp32, the sum taken after subtracting the row maximum, partial sums added in a fixed order (the
 * result is reproducible bit for bit).  Slots beyond n_b get id -1 and -inf.
 *   d_out_logprob : fp32 [batch][M][k], required.
 * Errors: EINVAL, ECAPACITY (M > m_cap or k > k_cap).  Asynchronous. */
NANOSPEC_API nanospec_status nanospec_topk_logprob_remap(nanospec_state* st, const float* d_logits, int32_t M, int32_t k,
                                                         int32_t* d_out_ids, float* d_out_logprob, void* hip_stream);

/* Dense full-vocabulary head, Eq. 1: logits[m][v] = sum_c W[v][c] * H[m][c] for all v < V.
 *   d_logits : fp32 [M_total][V].  Stateless.  Errors: EINVAL (null, sizes < 1, d % 8 != 0).
 * Asynchronous. */
NANOSPEC_API nanospec_status nanospec_dense_head(const void* d_W_bf16, const void* d_H_bf16, int32_t V, int32_t d,
                                    int32_t M_total, float* d_logits, void* hip_stream);

/* Top-k over dense logits (the selection step of the full-vocabulary comparison point):
 * rows [M_total][V], ids are the column indices; same ordering rule as nanospec_topk_remap.
 *   d_workspace : device scratch of at least nanospec_dense_topk_workspace(V, M_total, k) bytes.
 * Errors: EINVAL (null, sizes < 1, k > 64), ECAPACITY (workspace too small).  Asynchronous. */
NANOSPEC_API int64_t nanospec_dense_topk_workspace(int32_t V, int32_t M_total, int32_t k);
NANOSPEC_API nanospec_status nanospec_dense_topk(const float* d_logits, int32_t V, int32_t M_total, int32_t k,
                                    int32_t* d_out_ids, float* d_out_vals, void* d_workspace,
                                    int64_t workspace_bytes, void* hip_stream);

/* The same selection for callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: no workspace argument; the per-chunk candidates go to a
 * fixed 4 MiB device array inside the library (one per GPU, held until the process ends, its address looked
 * up on the first call on each device).  The call allocates and frees nothing.  Output as
 * nanospec_dense_topk, bit for bit.  Every call on a GPU shares that GPU's array: calls that overlap on one
 * GPU (two streams, two threads) race and must be serialised by the caller; calls in stream order need no
 * clearing in between.
 * Errors: EINVAL (as nanospec_dense_topk), ECAPACITY (nanospec_dense_topk_workspace(V, M_total, k) above
 * nanospec_dense_topk_static_limit() = 4 MiB, e.g. more than 5957 rows at V = 128256, k = 10), EHIP.
 * Asynchronous. */
NANOSPEC_API int64_t nanospec_dense_topk_static_limit(void);
NANOSPEC_API nanospec_status nanospec_dense_topk_static(const float* d_logits, int32_t V, int32_t M_total, int32_t k,
                                                        int32_t* d_out_ids, float* d_out_vals, void* hip_stream);

/* Measurement aids, not part of the method: read-only kernels that move the bytes the head moves and
 * compute nothing, to measure what one launch of that size and access pattern can reach on the chip.
 *   nanospec_calib_stream_read : reads d_buf[0, bytes) once, contiguously (bytes a multiple of 16).
 *   nanospec_calib_gather_read : reads the d bf16 of every row W[ids_b[j]], j < n_b, of sequence 0 of the
 *                                state's active list (the rows nanospec_sparse_head would gather).
 *   d_sink : device scratch of at least 1024 bytes (written practically never).
 *   nanospec_calib_valu_head   : the sparse head of one sequence (Eq. 1 on the active rows) computed on the
 *                                vector ALUs (unpack + fused multiply-add) instead of the matrix cores, with the
 *                                workgroup shape and loads of the product kernel for M <= 8: the measurement
 *                                behind the choice of the matrix cores below 16 hidden rows.  Logits as
 *                                nanospec_sparse_head (same layout and tolerance; the summation order differs).
 *                                batch == 1, M <= 8, d = 2048 or 4096, else EINVAL.
 * Errors: EINVAL (null, sizes < 1, bytes % 16 != 0).  Asynchronous. */
NANOSPEC_API nanospec_status nanospec_calib_valu_head(nanospec_state* st, const void* d_W_bf16, const void* d_H_bf16, int32_t M,
                                                      float* d_logits, void* hip_stream);
NANOSPEC_API nanospec_status nanospec_calib_stream_read(const void* d_buf, int64_t bytes, void* d_sink, void* hip_stream);
NANOSPEC_API nanospec_status nanospec_calib_gather_read(nanospec_state* st, const void* d_W_bf16, void* d_sink,
                                                        void* hip_stream);

/* Read and clear the sticky device error flags (NANOSPEC_DEV_* bits).  Synchronises `hip_stream`. */
NANOSPEC_API nanospec_status nanospec_last_device_error(nanospec_state* st, int32_t* flags, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* NANOSPEC_H_ */
