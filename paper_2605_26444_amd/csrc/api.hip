// C ABI of libnanospec: argument checking, state allocation, kernel dispatch.
#include <mutex>
#include <new>

#include "common.h"

using namespace nanospec;

namespace {

inline int64_t round_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

// split-K partial logits are only used while the row count is small; bound their footprint.
constexpr int kSplitRowsMax = 16384;
constexpr int kSplitMax = 16;

bool fill_layout(int32_t V, int32_t d, int32_t batch, int32_t window, int32_t topk_cap, int32_t m_cap, int32_t k_cap,
                 nanospec_layout* L) {
  if (V < 1 || d < 8 || d % 8 != 0 || batch < 1 || batch > NANOSPEC_MAX_BATCH || window < 1 || topk_cap < 0 ||
      m_cap < 1 || k_cap < 1 || k_cap > kMaxK)
    return false;
  const int64_t nwords = round_up((V + 31) / 32, 4);
  // three V-bit bitmaps, a 1024-entry chunk and m_cap*k_cap candidates share one workgroup's 160 KB of LDS
  if (3 * nwords + 32 + kVocabThreads + (int64_t)m_cap * k_cap > (160 * 1024 - 512) / 4) return false;
  int64_t maxn = (int64_t)window + topk_cap;
  if (maxn > V) maxn = V;
  const int64_t cap = round_up(maxn, 64);
  if (cap > (int64_t)kTopkChunk * 16) return false;
  L->capacity = (int32_t)cap;
  L->ring_bytes = (int64_t)window * 4;
  L->counter_bytes = (int64_t)V * 4;
  L->window_bitmap_bytes = nwords * 4;
  L->topk_bitmap_bytes = nwords * 4;
  L->ids_bytes = cap * 4;
  L->scalars_bytes = 3 * 4;
  const int64_t srows = cap < kSplitRowsMax ? cap : kSplitRowsMax;
  const int64_t partial = (int64_t)kSplitMax * batch * m_cap * srows * 4;
  const int64_t tws = topk_workspace_bytes((int32_t)cap, batch * m_cap, k_cap);
  L->workspace_bytes = round_up(partial, 256) + round_up(tws, 256);
  const int64_t per_seq = round_up(L->ring_bytes, 256) + round_up(L->counter_bytes, 256) +
                          2 * round_up(L->window_bitmap_bytes, 256) + round_up(L->ids_bytes, 256);
  L->total_bytes = per_seq * batch + round_up(3 * 4 * (int64_t)batch, 256) + 256 + L->workspace_bytes;
  L->gathered_bytes_at_cap = (int64_t)window * d * 2;
  return true;
}

nanospec_status offsets_to_arg(const int32_t* h_off, int batch, Offsets* out, int64_t per_seq_limit, bool* any) {
  *any = false;
  for (int i = 0; i <= NANOSPEC_MAX_BATCH; ++i) out->v[i] = 0;
  if (!h_off) return NANOSPEC_OK;
  for (int b = 0; b <= batch; ++b) out->v[b] = h_off[b];
  if (h_off[0] < 0) return NANOSPEC_EINVAL;
  for (int b = 0; b < batch; ++b) {
    const int64_t len = (int64_t)h_off[b + 1] - h_off[b];
    if (len < 0) return NANOSPEC_EINVAL;
    if (per_seq_limit >= 0 && len > per_seq_limit) return NANOSPEC_ECAPACITY;
    if (len > 0) *any = true;
  }
  return NANOSPEC_OK;
}

// Per-device, once: raise the dynamic-LDS limit of every kernel that needs it (a property of the function on a
// device, not of a state).  Done at nanospec_create and at the first stateless head call on a device.
std::mutex g_cfg_mu;
bool g_cfg_done[64] = {};

hipError_t ensure_device_configured() {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_cfg_mu);
  if (g_cfg_done[dev]) return hipSuccess;
  e = head_configure_device();
  if (e == hipSuccess) e = vocab_configure_device();
  if (e == hipSuccess) e = calib_configure_device();
  if (e == hipSuccess) e = union_configure_device();
  if (e == hipSuccess) e = wide_configure_device();
  if (e == hipSuccess) g_cfg_done[dev] = true;
  return e;
}

// The state's memory and its kernels belong to the device that was current at nanospec_create: a call made
// with another device current would launch there on foreign pointers, so it is refused instead.
bool wrong_device(const nanospec_state* st) {
  int dev = -1;
  return hipGetDevice(&dev) != hipSuccess || dev != st->device;
}

nanospec_status vocab_call(nanospec_state* st, const int32_t* d_new, const int32_t* h_noff, const int32_t* d_topk,
                           const int32_t* h_toff, bool is_init, void* stream) {
  if (!st || wrong_device(st)) return NANOSPEC_EINVAL;
  if (is_init && !h_noff) return NANOSPEC_EINVAL;
  Offsets noff, toff;
  bool any_new = false, any_t = false;
  nanospec_status rc = offsets_to_arg(h_noff, st->batch, &noff, -1, &any_new);
  if (rc != NANOSPEC_OK) return rc;
  rc = offsets_to_arg(h_toff, st->batch, &toff, st->topk_cap, &any_t);
  if (rc != NANOSPEC_OK) return rc;
  if (any_new && !d_new) return NANOSPEC_EINVAL;
  if (any_t && !d_topk) return NANOSPEC_EINVAL;
  if (d_topk && !h_toff) return NANOSPEC_EINVAL;
  const int replace_T = (is_init || h_toff != nullptr) ? 1 : 0;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (is_init) {
    st->policy = st->policy_next;
    if (launch_vocab_clear(st, s) != hipSuccess) return NANOSPEC_EHIP;
  }
  if (launch_vocab_apply(st, d_new, noff, d_topk, toff, replace_T, s) != hipSuccess) return NANOSPEC_EHIP;
  return NANOSPEC_OK;
}

}  // namespace

extern "C" {

const char* nanospec_status_string(nanospec_status s) {
  switch (s) {
    case NANOSPEC_OK: return "ok";
    case NANOSPEC_EINVAL: return "invalid argument";
    case NANOSPEC_ENOMEM: return "out of memory";
    case NANOSPEC_ECAPACITY: return "capacity exceeded";
    case NANOSPEC_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

nanospec_status nanospec_state_layout(int32_t V, int32_t d, int32_t batch, int32_t window, int32_t topk_cap,
                                      int32_t m_cap, int32_t k_cap, nanospec_layout* out) {
  if (!out) return NANOSPEC_EINVAL;
  return fill_layout(V, d, batch, window, topk_cap, m_cap, k_cap, out) ? NANOSPEC_OK : NANOSPEC_EINVAL;
}

nanospec_status nanospec_create(nanospec_state** out, int32_t V, int32_t d, int32_t batch, int32_t window,
                                int32_t topk_cap, int32_t m_cap, int32_t k_cap) {
  if (!out) return NANOSPEC_EINVAL;
  *out = nullptr;
  nanospec_layout L;
  if (!fill_layout(V, d, batch, window, topk_cap, m_cap, k_cap, &L)) return NANOSPEC_EINVAL;
  nanospec_state* st = new (std::nothrow) nanospec_state();
  if (!st) return NANOSPEC_ENOMEM;
  st->V = V; st->d = d; st->batch = batch; st->window = window;
  st->topk_cap = topk_cap; st->m_cap = m_cap; st->k_cap = k_cap;
  st->policy = st->policy_next = NANOSPEC_POLICY_WINDOW;
  st->layout = L;
  if (hipGetDevice(&st->device) != hipSuccess) { delete st; return NANOSPEC_EHIP; }
  if (hipMalloc(reinterpret_cast<void**>(&st->base), L.total_bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete st;
    return NANOSPEC_ENOMEM;
  }
  if (hipHostMalloc(reinterpret_cast<void**>(&st->h_err_pinned), 64, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(st->base);
    delete st;
    return NANOSPEC_ENOMEM;
  }
  char* p = st->base;
  auto take = [&](int64_t bytes) { char* r = p; p += round_up(bytes, 256); return r; };
  VocabPtrs& vp = st->vp;
  vp.V = V; vp.window = window; vp.nwords = (int32_t)(L.window_bitmap_bytes / 4); vp.cap = L.capacity;
  vp.ring = reinterpret_cast<int32_t*>(take(round_up(L.ring_bytes, 256) * batch));
  vp.cnt = reinterpret_cast<uint32_t*>(take(round_up(L.counter_bytes, 256) * batch));
  vp.wbit = reinterpret_cast<uint32_t*>(take(round_up(L.window_bitmap_bytes, 256) * batch));
  vp.tbit = reinterpret_cast<uint32_t*>(take(round_up(L.topk_bitmap_bytes, 256) * batch));
  vp.ids = reinterpret_cast<int32_t*>(take(round_up(L.ids_bytes, 256) * batch));
  int32_t* sc = reinterpret_cast<int32_t*>(take(3 * 4 * (int64_t)batch));
  vp.n = sc; vp.pos = sc + batch; vp.fill = sc + 2 * batch;
  vp.err = reinterpret_cast<int32_t*>(take(4));
  const int64_t srows = L.capacity < kSplitRowsMax ? L.capacity : kSplitRowsMax;
  st->partial_bytes = (int64_t)kSplitMax * batch * m_cap * srows * 4;
  st->partial = reinterpret_cast<float*>(take(st->partial_bytes));
  st->topk_ws_bytes = topk_workspace_bytes(L.capacity, batch * m_cap, k_cap);
  st->topk_ws = take(st->topk_ws_bytes);
  if (p - st->base > L.total_bytes || ensure_device_configured() != hipSuccess || vocab_configure(st) != hipSuccess || hipMemset(vp.err, 0, 4) != hipSuccess ||
      launch_vocab_clear(st, nullptr) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
    (void)hipGetLastError();
    (void)hipHostFree(st->h_err_pinned);
    (void)hipFree(st->base);
    delete st;
    return NANOSPEC_EHIP;
  }
  *out = st;
  return NANOSPEC_OK;
}

nanospec_status nanospec_destroy(nanospec_state* st) {
  if (!st) return NANOSPEC_EINVAL;
  if (st->pk_base) (void)hipFree(st->pk_base);
  if (st->un_base) {
    (void)hipStreamSynchronize(st->un_side);
    (void)hipEventDestroy(st->un_fork);
    (void)hipEventDestroy(st->un_join);
    (void)hipStreamDestroy(st->un_side);
    (void)hipFree(st->un_base);
  }
  hipError_t e1 = hipFree(st->base);
  hipError_t e2 = hipHostFree(st->h_err_pinned);
  delete st;
  return (e1 == hipSuccess && e2 == hipSuccess) ? NANOSPEC_OK : NANOSPEC_EHIP;
}

int64_t nanospec_packed_bytes(const nanospec_state* st) {
  if (!st) return -1;
  const int64_t cap = st->vp.cap;
  return round_up(cap * st->d * 2, 256) + round_up((int64_t)st->V * 4, 256) + 5 * round_up(cap * 4, 256) + 256;
}

nanospec_status nanospec_packed_enable(nanospec_state* st) {
  if (!st || wrong_device(st) || st->batch != 1) return NANOSPEC_EINVAL;
  if (st->pk_base) return NANOSPEC_OK;
  const int64_t cap = st->vp.cap;
  char* base = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&base), nanospec_packed_bytes(st)) != hipSuccess) {
    (void)hipGetLastError();
    return NANOSPEC_ENOMEM;
  }
  char* p = base;
  auto take = [&](int64_t bytes) { char* r = p; p += round_up(bytes, 256); return r; };
  PackedPtrs& k = st->pk;
  k.cap = (int32_t)cap;
  k.buf = reinterpret_cast<uint16_t*>(take(cap * st->d * 2));
  k.slot_of = reinterpret_cast<int32_t*>(take((int64_t)st->V * 4));
  k.slot_id = reinterpret_cast<int32_t*>(take(cap * 4));
  k.out_pos = reinterpret_cast<int32_t*>(take(cap * 4));
  k.free_list = reinterpret_cast<int32_t*>(take(cap * 4));
  k.copy_list = reinterpret_cast<int32_t*>(take(2 * cap * 4));
  k.scal = reinterpret_cast<int32_t*>(take(8));
  st->pk_base = base;
  if (launch_packed_reset(st, nullptr) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(base);
    st->pk_base = nullptr;
    k.buf = nullptr;
    return NANOSPEC_EHIP;
  }
  return NANOSPEC_OK;
}

nanospec_status nanospec_packed_gather(nanospec_state* st, const void* d_W_bf16, void* hip_stream) {
  if (!st || !d_W_bf16 || wrong_device(st) || !st->pk_base) return NANOSPEC_EINVAL;
  return launch_packed_gather(st, d_W_bf16, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_packed_head(nanospec_state* st, const void* d_H_bf16, int32_t M, float* d_logits, void* hip_stream) {
  if (!st || !d_H_bf16 || !d_logits || M < 1 || wrong_device(st) || !st->pk_base) return NANOSPEC_EINVAL;
  if (M > st->m_cap) return NANOSPEC_ECAPACITY;
  const int32_t cap = st->vp.cap;
  // a dense product over the slots that may hold a row (count on the device), logits to the columns of the ascending list
  hipError_t e = launch_head(st->pk.buf, d_H_bf16, nullptr, st->pk.scal, 0, cap, cap, 1, M, st->d, cap, cap, d_logits, st->partial,
                             st->partial_bytes, st->pk.out_pos, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_packed_view(const nanospec_state* st, const void** d_buf, const int32_t** d_slot_id, const int32_t** d_out_pos,
                                     const int32_t** d_counts) {
  if (!st || !st->pk_base) return NANOSPEC_EINVAL;
  if (d_buf) *d_buf = st->pk.buf;
  if (d_slot_id) *d_slot_id = st->pk.slot_id;
  if (d_out_pos) *d_out_pos = st->pk.out_pos;
  if (d_counts) *d_counts = st->pk.scal;
  return NANOSPEC_OK;
}

int64_t nanospec_union_bytes(const nanospec_state* st, int32_t shared_cap) {
  if (!st) return -1;
  const int64_t cap = st->vp.cap, nw = st->vp.nwords, B = st->batch;
  if (shared_cap == 0) shared_cap = (int32_t)cap;
  if (shared_cap < 64 || shared_cap % 64 != 0 || shared_cap > cap) return -1;
  const int64_t groups = (B * st->m_cap + 63) / 64;
  return 2 * round_up(nw * 4, 256) + round_up((int64_t)shared_cap * 4, 256) + round_up(groups * 4, 256) +
         round_up(B * shared_cap * 4, 256) + 2 * round_up(B * cap * 4, 256) + round_up(B * 4, 256);
}

nanospec_status nanospec_union_enable(nanospec_state* st, int32_t min_share, int32_t shared_cap) {
  if (!st || wrong_device(st) || min_share < 0) return NANOSPEC_EINVAL;
  if (st->un_base) return NANOSPEC_EINVAL;                 // thresholds are fixed once enabled
  const int64_t cap = st->vp.cap, nw = st->vp.nwords, B = st->batch;
  if (shared_cap == 0) shared_cap = (int32_t)cap;
  if (min_share == 0) min_share = B / 8 > 2 ? (int32_t)(B / 8) : 2;
  const int64_t bytes = nanospec_union_bytes(st, shared_cap);
  if (bytes < 0) return NANOSPEC_EINVAL;
  char* base = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&base), bytes) != hipSuccess) {
    (void)hipGetLastError();
    return NANOSPEC_ENOMEM;
  }
  char* p = base;
  auto take = [&](int64_t b) { char* r = p; p += round_up(b, 256); return r; };
  UnionPtrs& u = st->un;
  st->un_groups = (int32_t)((B * st->m_cap + 63) / 64);
  u.shared_cap = shared_cap;
  u.min_share = min_share;
  u.shared_bits = reinterpret_cast<uint32_t*>(take(nw * 4));
  u.shared_cnt = reinterpret_cast<int32_t*>(take(nw * 4));
  u.shared_ids = reinterpret_cast<int32_t*>(take((int64_t)shared_cap * 4));
  u.shared_n = reinterpret_cast<int32_t*>(take((int64_t)st->un_groups * 4));
  u.shared_pos = reinterpret_cast<int32_t*>(take(B * shared_cap * 4));
  u.rest_ids = reinterpret_cast<int32_t*>(take(B * cap * 4));
  u.rest_pos = reinterpret_cast<int32_t*>(take(B * cap * 4));
  u.rest_n = reinterpret_cast<int32_t*>(take(B * 4));
  st->un_base = base;
  bool ok = p - base <= bytes && hipStreamCreateWithFlags(&st->un_side, hipStreamNonBlocking) == hipSuccess;
  if (ok) {
    ok = hipEventCreateWithFlags(&st->un_fork, hipEventDisableTiming) == hipSuccess;
    if (ok) {
      ok = hipEventCreateWithFlags(&st->un_join, hipEventDisableTiming) == hipSuccess;
      if (!ok) (void)hipEventDestroy(st->un_fork);
    }
    if (!ok) (void)hipStreamDestroy(st->un_side);
  }
  if (ok && (launch_union_reset(st, nullptr) != hipSuccess || hipDeviceSynchronize() != hipSuccess)) {
    (void)hipEventDestroy(st->un_fork);
    (void)hipEventDestroy(st->un_join);
    (void)hipStreamDestroy(st->un_side);
    ok = false;
  }
  if (!ok) {
    (void)hipGetLastError();
    (void)hipFree(base);
    st->un_base = nullptr;
    return NANOSPEC_EHIP;
  }
  return NANOSPEC_OK;
}

nanospec_status nanospec_union_build(nanospec_state* st, void* hip_stream) {
  if (!st || wrong_device(st) || !st->un_base) return NANOSPEC_EINVAL;
  return launch_union_build(st, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_union_head(nanospec_state* st, const void* d_W_bf16, const void* d_H_bf16, int32_t M, float* d_logits,
                                    void* hip_stream) {
  if (!st || !d_W_bf16 || !d_H_bf16 || !d_logits || M < 1 || wrong_device(st) || !st->un_base) return NANOSPEC_EINVAL;
  if (M > st->m_cap) return NANOSPEC_ECAPACITY;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const UnionPtrs& u = st->un;
  const int32_t cap = st->vp.cap;
  // The two products are independent and write disjoint columns.  The shared one is few workgroups that each walk
  // all of K (latency-bound), the per-sequence one many short workgroups (throughput-bound): the first runs on the
  // state's side stream (default priority), forked from and joined back into the caller's stream by events, so a
  // graph capture of the caller's stream records both branches.
  if (hipEventRecord(st->un_fork, s) != hipSuccess || hipStreamWaitEvent(st->un_side, st->un_fork, 0) != hipSuccess) return NANOSPEC_EHIP;
  // shared rows: fetched once, multiplied with every sequence's hidden rows, scattered to each sequence's columns
  hipError_t e = launch_head_shared(d_W_bf16, d_H_bf16, u.shared_ids, u.shared_n, u.shared_cap, st->V, st->batch * M, M, st->d, cap,
                                    d_logits, u.shared_pos, u.shared_cap, st->un_side);
  if (hipEventRecord(st->un_join, st->un_side) != hipSuccess) return NANOSPEC_EHIP;   // joined even after a failed launch
  // the rest per sequence, exactly as nanospec_sparse_head but on the shorter lists
  hipError_t e2 = launch_head(d_W_bf16, d_H_bf16, u.rest_ids, u.rest_n, 0, cap, st->V, st->batch, M, st->d, cap, cap, d_logits,
                              st->partial, st->partial_bytes, u.rest_pos, s);
  if (hipStreamWaitEvent(s, st->un_join, 0) != hipSuccess) return NANOSPEC_EHIP;
  return e == hipSuccess && e2 == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_union_view(const nanospec_state* st, const int32_t** d_shared_ids, const int32_t** d_shared_n,
                                    const int32_t** d_shared_pos, const int32_t** d_rest_ids, const int32_t** d_rest_pos,
                                    const int32_t** d_rest_n, int32_t* shared_cap, int32_t* min_share) {
  if (!st || !st->un_base) return NANOSPEC_EINVAL;
  if (d_shared_ids) *d_shared_ids = st->un.shared_ids;
  if (d_shared_n) *d_shared_n = st->un.shared_n;
  if (d_shared_pos) *d_shared_pos = st->un.shared_pos;
  if (d_rest_ids) *d_rest_ids = st->un.rest_ids;
  if (d_rest_pos) *d_rest_pos = st->un.rest_pos;
  if (d_rest_n) *d_rest_n = st->un.rest_n;
  if (shared_cap) *shared_cap = st->un.shared_cap;
  if (min_share) *min_share = st->un.min_share;
  return NANOSPEC_OK;
}

nanospec_status nanospec_set_stream_policy(nanospec_state* st, int32_t policy) {
  if (!st || (policy != NANOSPEC_POLICY_WINDOW && policy != NANOSPEC_POLICY_FIFO)) return NANOSPEC_EINVAL;
  st->policy_next = policy;
  return NANOSPEC_OK;
}

nanospec_status nanospec_vocab_init(nanospec_state* st, const int32_t* d_ctx_ids, const int32_t* h_ctx_off,
                                    const int32_t* d_topk_ids, const int32_t* h_topk_off, void* hip_stream) {
  return vocab_call(st, d_ctx_ids, h_ctx_off, d_topk_ids, h_topk_off, true, hip_stream);
}

nanospec_status nanospec_vocab_update(nanospec_state* st, const int32_t* d_new_ids, const int32_t* h_new_off,
                                      const int32_t* d_topk_ids, const int32_t* h_topk_off, void* hip_stream) {
  return vocab_call(st, d_new_ids, h_new_off, d_topk_ids, h_topk_off, false, hip_stream);
}

nanospec_status nanospec_vocab_append_unique(nanospec_state* st, const int32_t* d_cand_ids, int32_t cand_per_seq,
                                             int64_t cand_stride, void* hip_stream) {
  if (!st || cand_per_seq < 0 || (cand_per_seq > 0 && !d_cand_ids) || cand_stride < cand_per_seq || wrong_device(st))
    return NANOSPEC_EINVAL;
  if (cand_per_seq > st->unique_cap) return NANOSPEC_ECAPACITY;
  hipError_t e = launch_vocab_append_unique(st, d_cand_ids, cand_per_seq, cand_stride, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_vocab_view(const nanospec_state* st, const int32_t** d_ids, const int32_t** d_n,
                                    int32_t* capacity) {
  if (!st) return NANOSPEC_EINVAL;
  if (d_ids) *d_ids = st->vp.ids;
  if (d_n) *d_n = st->vp.n;
  if (capacity) *capacity = st->vp.cap;
  return NANOSPEC_OK;
}

nanospec_status nanospec_sparse_head(nanospec_state* st, const void* d_W_bf16, const void* d_H_bf16, int32_t M,
                                     float* d_logits, void* hip_stream) {
  if (!st || !d_W_bf16 || !d_H_bf16 || !d_logits || M < 1 || wrong_device(st)) return NANOSPEC_EINVAL;
  if (M > st->m_cap) return NANOSPEC_ECAPACITY;
  hipError_t e = launch_head(d_W_bf16, d_H_bf16, st->vp.ids, st->vp.n, 0, st->vp.cap, st->V, st->batch, M, st->d, st->vp.cap,
                             st->vp.cap, d_logits, st->partial, st->partial_bytes, nullptr, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_topk_remap(nanospec_state* st, const float* d_logits, int32_t M, int32_t k, int32_t* d_out_ids,
                                    float* d_out_vals, void* hip_stream) {
  if (!st || !d_logits || !d_out_ids || M < 1 || k < 1 || wrong_device(st)) return NANOSPEC_EINVAL;
  if (M > st->m_cap || k > st->k_cap) return NANOSPEC_ECAPACITY;
  hipError_t e = launch_topk(d_logits, st->vp.cap, st->vp.ids, st->vp.cap, st->vp.n, 0, st->vp.cap, st->batch, M, k,
                             d_out_ids, d_out_vals, false, st->topk_ws, st->topk_ws_bytes,
                             static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_topk_logprob_remap(nanospec_state* st, const float* d_logits, int32_t M, int32_t k,
                                            int32_t* d_out_ids, float* d_out_logprob, void* hip_stream) {
  if (!st || !d_logits || !d_out_ids || !d_out_logprob || M < 1 || k < 1 || wrong_device(st)) return NANOSPEC_EINVAL;
  if (M > st->m_cap || k > st->k_cap) return NANOSPEC_ECAPACITY;
  hipError_t e = launch_topk(d_logits, st->vp.cap, st->vp.ids, st->vp.cap, st->vp.n, 0, st->vp.cap, st->batch, M, k,
                             d_out_ids, d_out_logprob, true, st->topk_ws, st->topk_ws_bytes,
                             static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_dense_head(const void* d_W_bf16, const void* d_H_bf16, int32_t V, int32_t d, int32_t M_total,
                                    float* d_logits, void* hip_stream) {
  if (!d_W_bf16 || !d_H_bf16 || !d_logits || V < 1 || d < 8 || d % 8 != 0 || M_total < 1) return NANOSPEC_EINVAL;
  if (ensure_device_configured() != hipSuccess) return NANOSPEC_EHIP;   // a flag test after the first call on the device
  hipError_t e = launch_head(d_W_bf16, d_H_bf16, nullptr, nullptr, V, V, V, 1, M_total, d, V, 0, d_logits, nullptr, 0, nullptr,
                             static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

int64_t nanospec_dense_topk_workspace(int32_t V, int32_t M_total, int32_t k) {
  if (V < 1 || M_total < 1 || k < 1 || k > kMaxK) return -1;
  const int64_t b = topk_workspace_bytes(V, M_total, k);
  return b > 256 ? b : 256;
}

nanospec_status nanospec_dense_topk(const float* d_logits, int32_t V, int32_t M_total, int32_t k, int32_t* d_out_ids,
                                    float* d_out_vals, void* d_workspace, int64_t workspace_bytes, void* hip_stream) {
  if (!d_logits || !d_out_ids || !d_workspace || V < 1 || M_total < 1 || k < 1 || k > kMaxK) return NANOSPEC_EINVAL;
  if ((int64_t)V > (int64_t)kTopkChunk * 16) return NANOSPEC_EINVAL;
  if (workspace_bytes < nanospec_dense_topk_workspace(V, M_total, k)) return NANOSPEC_ECAPACITY;
  hipError_t e = launch_topk(d_logits, V, nullptr, 0, nullptr, V, V, 1, M_total, k, d_out_ids, d_out_vals, false,
                             static_cast<char*>(d_workspace), workspace_bytes, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NANOSPEC_OK : NANOSPEC_EHIP;
}

nanospec_status nanospec_calib_stream_read(const void* d_buf, int64_t bytes, void* d_sink, void* hip_stream) {
  if (!d_buf || !d_sink || bytes < 16 || bytes % 16 != 0) return NANOSPEC_EINVAL;
  return launch_calib_stream(d_buf, bytes, d_sink, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? NANOSPEC_OK
                                                                                                        : NANOSPEC_EHIP;
}

nanospec_status nanospec_calib_gather_read(nanospec_state* st, const void* d_W_bf16, void* d_sink, void* hip_stream) {
  if (!st || !d_W_bf16 || !d_sink || wrong_device(st)) return NANOSPEC_EINVAL;
  return launch_calib_gather(d_W_bf16, st->V, st->d, st->vp.ids, st->vp.n, st->vp.cap, d_sink,
                             static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? NANOSPEC_OK
             : NANOSPEC_EHIP;
}

nanospec_status nanospec_calib_valu_head(nanospec_state* st, const void* d_W_bf16, const void* d_H_bf16, int32_t M, float* d_logits,
                                         void* hip_stream) {
  if (!st || !d_W_bf16 || !d_H_bf16 || !d_logits || M < 1 || M > 8 || st->batch != 1 || (st->d != 2048 && st->d != 4096) || wrong_device(st))
    return NANOSPEC_EINVAL;
  return launch_calib_valu_head(d_W_bf16, d_H_bf16, st->V, st->d, M, st->vp.ids, st->vp.n, st->vp.cap, d_logits,
                                static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? NANOSPEC_OK
             : NANOSPEC_EHIP;
}

nanospec_status nanospec_last_device_error(nanospec_state* st, int32_t* flags, void* hip_stream) {
  if (!st || !flags || wrong_device(st)) return NANOSPEC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (hipMemcpyAsync(st->h_err_pinned, st->vp.err, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return NANOSPEC_EHIP;
  if (hipMemsetAsync(st->vp.err, 0, 4, s) != hipSuccess) return NANOSPEC_EHIP;
  if (hipStreamSynchronize(s) != hipSuccess) return NANOSPEC_EHIP;
  *flags = *st->h_err_pinned;
  return NANOSPEC_OK;
}

}  // extern "C"
