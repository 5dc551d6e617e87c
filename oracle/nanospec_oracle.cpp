// CPU oracle for the NanoSpec draft-step hot path.  TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, obviously-correct statement of what the GPU library must compute, written from
// the paper's definitions.  It shares no code, header, table or helper with the HIP path, and the
// product never calls it: only tests, the smoke check and the benchmark's cpu_baseline leg do.
//
//   * Vocabulary  (Sec. 3.2, Eq. 2-4; Alg. 1 "Init/Update stream S and I"):
//       the candidate stream S is every id ever appended, in order; the active index set is
//       I = Unique(Suffix(S, W_max)) united with a caller-supplied candidate set T.  It is
//       recomputed from scratch from S and T each time it is asked for: std::vector + std::set.
//   * Vocabulary, second reading (Sec. 3.3 and the appendix on vocabulary evolution): a first-in
//       first-out queue of at most W_max distinct ids; ids already in the vocabulary are not pushed again.
//   * Sparse head (Sec. 3.1, Eq. 1 restricted to the rows I_t):  z'[m][j] = sum_c W[I_j][c]*H[m][c],
//       scalar accumulation in index order, once in fp32 (the precision the method computes in:
//       bf16 operands, fp32 accumulate) and once in fp64 (to bound the rounding error).
//   * Dense head  (Eq. 1): the same loop over all V rows.
//   * Top-k + remap (Alg. 1 "SelectDraftTokens(z', I)", operator T_K of Sec. 3.2): full sort of
//       (value, global id) by value descending then id ascending; the first k.
//   * Log-softmax over the active set (Sec. 4.2, the renormalised draft distribution): fp64.
//
// Readings where the paper is silent are listed in the repository's design notes; in short:
// ids are 0-based; the active list is in ascending id order; top-k ties go to the lower id;
// T is a set that is not windowed and is replaced wholesale; a stream shorter than the window is
// taken whole; an id outside [0,V) keeps its stream position but is never a member of I.
//
// Parity status: every function here is pinned by tests/test_oracle_*.py (brute force on tiny
// inputs, closed forms, invariants, independent float64 library matmul, hand-worked cases).
#include <algorithm>
#include <cmath>
#include <deque>
#include <cstdint>
#include <cstring>
#include <limits>
#include <set>
#include <utility>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

struct Vocab {
  int32_t V;
  int64_t window;
  std::vector<int32_t> S;   // candidate stream, oldest first
  std::set<int32_t> T;      // extra candidate set
};

// Second reading of the vocabulary (Sec. 3.3, GPU-resident state management: only candidates that are new
// to the vocabulary are pushed; App. on vocabulary evolution: the vocabulary grows monotonically up to
// the capacity W_max and is evicted first-in first-out): a queue of at most W_max *distinct* ids.
struct FifoVocab {
  int32_t V;
  int64_t window;
  std::deque<int32_t> Q;    // members in the order they were pushed, oldest first
  std::set<int32_t> T;
};

// One call = one batch: the ids that are valid, not members when the call starts and not seen earlier
// in the call, in the order of their first occurrence; of those at most the last W_max are pushed, after
// as many of the oldest members as needed have been dropped.
void fifo_push_batch(FifoVocab* v, const int32_t* ids, int64_t n) {
  std::set<int32_t> members(v->Q.begin(), v->Q.end());
  std::set<int32_t> seen;
  std::vector<int32_t> F;
  for (int64_t i = 0; i < n; ++i) {
    const int32_t a = ids[i];
    if (a < 0 || a >= v->V) continue;
    if (members.count(a) || seen.count(a)) continue;
    seen.insert(a);
    F.push_back(a);
  }
  const int64_t W = v->window;
  const int64_t nF = static_cast<int64_t>(F.size());
  const int64_t first = nF > W ? nF - W : 0;
  int64_t evict = static_cast<int64_t>(v->Q.size()) + (nF - first) - W;
  for (; evict > 0; --evict) v->Q.pop_front();
  for (int64_t i = first; i < nF; ++i) v->Q.push_back(F[i]);
}

inline float bf16_to_float(uint16_t b) {
  uint32_t u = static_cast<uint32_t>(b) << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return f;
}

}  // namespace

extern "C" {

void* oracle_vocab_new(int32_t V, int64_t window) {
  Vocab* v = new Vocab;
  v->V = V;
  v->window = window;
  return v;
}

void oracle_vocab_free(void* h) { delete static_cast<Vocab*>(h); }

// Eq. 2 / Alg. 1 stream initialisation: S <- ctx, T <- set(topk).
void oracle_vocab_init(void* h, const int32_t* ctx, int64_t n_ctx, const int32_t* topk, int64_t n_topk) {
  Vocab* v = static_cast<Vocab*>(h);
  v->S.assign(ctx, ctx + n_ctx);
  v->T.clear();
  v->T.insert(topk, topk + n_topk);
}

// Eq. 3 stream update: S <- S (+) new_ids; if replace_T, T <- set(topk).
void oracle_vocab_update(void* h, const int32_t* new_ids, int64_t n_new, int32_t replace_T,
                         const int32_t* topk, int64_t n_topk) {
  Vocab* v = static_cast<Vocab*>(h);
  v->S.insert(v->S.end(), new_ids, new_ids + n_new);
  if (replace_T) {
    v->T.clear();
    v->T.insert(topk, topk + n_topk);
  }
}

// Eq. 3 for a candidate *set* (C_draft: every distinct token id of the draft tree): the distinct
// valid ids are appended in ascending order (the paper leaves the order of tuple(set) open); -1 entries
// are padding.
void oracle_vocab_append_unique(void* h, const int32_t* cand, int64_t n_cand) {
  Vocab* v = static_cast<Vocab*>(h);
  std::set<int32_t> C;
  for (int64_t i = 0; i < n_cand; ++i)
    if (cand[i] >= 0 && cand[i] < v->V) C.insert(cand[i]);
  v->S.insert(v->S.end(), C.begin(), C.end());
}

void* oracle_fifo_new(int32_t V, int64_t window) {
  FifoVocab* v = new FifoVocab;
  v->V = V;
  v->window = window;
  return v;
}

void oracle_fifo_free(void* h) { delete static_cast<FifoVocab*>(h); }

void oracle_fifo_init(void* h, const int32_t* ctx, int64_t n_ctx, const int32_t* topk, int64_t n_topk) {
  FifoVocab* v = static_cast<FifoVocab*>(h);
  v->Q.clear();
  v->T.clear();
  v->T.insert(topk, topk + n_topk);
  fifo_push_batch(v, ctx, n_ctx);
}

void oracle_fifo_update(void* h, const int32_t* new_ids, int64_t n_new, int32_t replace_T, const int32_t* topk,
                        int64_t n_topk) {
  FifoVocab* v = static_cast<FifoVocab*>(h);
  fifo_push_batch(v, new_ids, n_new);
  if (replace_T) {
    v->T.clear();
    v->T.insert(topk, topk + n_topk);
  }
}

// a candidate set: its distinct valid ids in ascending order, then one batch
void oracle_fifo_append_unique(void* h, const int32_t* cand, int64_t n_cand) {
  FifoVocab* v = static_cast<FifoVocab*>(h);
  std::set<int32_t> C;
  for (int64_t i = 0; i < n_cand; ++i)
    if (cand[i] >= 0 && cand[i] < v->V) C.insert(cand[i]);
  std::vector<int32_t> sorted(C.begin(), C.end());
  fifo_push_batch(v, sorted.data(), static_cast<int64_t>(sorted.size()));
}

int64_t oracle_fifo_size(void* h) { return static_cast<int64_t>(static_cast<FifoVocab*>(h)->Q.size()); }

// members U T, ascending.  Returns the count; writes at most cap ids.
int64_t oracle_fifo_active(void* h, int32_t* out, int64_t cap) {
  FifoVocab* v = static_cast<FifoVocab*>(h);
  std::set<int32_t> I(v->Q.begin(), v->Q.end());
  for (int32_t t : v->T) I.insert(t);
  int64_t n = 0;
  for (int32_t id : I) {
    if (id < 0 || id >= v->V) continue;
    if (n < cap) out[n] = id;
    ++n;
  }
  return n;
}

int64_t oracle_vocab_stream_len(void* h) { return static_cast<int64_t>(static_cast<Vocab*>(h)->S.size()); }

// Eq. 4: I = Unique(Suffix(S, W_max)) U T, ascending.  Returns |I|; writes at most cap ids.
int64_t oracle_vocab_active(void* h, int32_t* out, int64_t cap) {
  Vocab* v = static_cast<Vocab*>(h);
  std::set<int32_t> I;
  int64_t len = static_cast<int64_t>(v->S.size());
  int64_t first = len > v->window ? len - v->window : 0;
  for (int64_t p = first; p < len; ++p) I.insert(v->S[p]);
  for (int32_t t : v->T) I.insert(t);
  int64_t n = 0;
  for (int32_t id : I) {
    if (id < 0 || id >= v->V) continue;
    if (n < cap) out[n] = id;
    ++n;
  }
  return n;
}

// Eq. 1 on the rows ids[0..n): out32/out64 are [M][ld] with entry (m, j) at m*ld + j.
// ids == nullptr means the identity list 0..n-1 (the dense head).  Either output may be null.
void oracle_head(const uint16_t* W, const uint16_t* H, const int32_t* ids, int64_t n, int32_t M, int32_t d,
                 int64_t ld, float* out32, double* out64) {
#pragma omp parallel for schedule(static)
  for (int64_t j = 0; j < n; ++j) {
    const uint16_t* w = W + static_cast<int64_t>(ids ? ids[j] : j) * d;
    for (int32_t m = 0; m < M; ++m) {
      const uint16_t* h = H + static_cast<int64_t>(m) * d;
      float acc32 = 0.0f;
      double acc64 = 0.0;
      for (int32_t c = 0; c < d; ++c) {
        float a = bf16_to_float(w[c]), b = bf16_to_float(h[c]);
        acc32 += a * b;
        acc64 += static_cast<double>(a) * static_cast<double>(b);
      }
      if (out32) out32[m * ld + j] = acc32;
      if (out64) out64[m * ld + j] = acc64;
    }
  }
}

// T_K followed by the local -> global id map: sorts all n (value, id) pairs.
// Slots beyond n get id -1 and value -infinity.
void oracle_topk(const float* vals, const int32_t* ids, int64_t n, int32_t k, int32_t* out_ids, float* out_vals) {
  std::vector<std::pair<float, int32_t>> p(static_cast<size_t>(n));
  for (int64_t j = 0; j < n; ++j) p[j] = {vals[j], ids ? ids[j] : static_cast<int32_t>(j)};
  std::sort(p.begin(), p.end(), [](const std::pair<float, int32_t>& a, const std::pair<float, int32_t>& b) {
    if (a.first != b.first) return a.first > b.first;
    return a.second < b.second;
  });
  for (int32_t r = 0; r < k; ++r) {
    if (r < n) {
      out_ids[r] = p[r].second;
      out_vals[r] = p[r].first;
    } else {
      out_ids[r] = -1;
      out_vals[r] = -std::numeric_limits<float>::infinity();
    }
  }
}

// Draft distribution on the pruned vocabulary (Sec. 4.2: with the irrelevant tokens gone, the softmax is
// renormalised over the active set only): logp[j] = z[j] - log(sum_i exp(z[i])), i over the n active
// entries, in fp64, the sum taken after subtracting the largest logit.  n == 0 leaves nothing to write.
void oracle_log_softmax(const float* vals, int64_t n, double* out_logp) {
  if (n <= 0) return;
  double zmax = vals[0];
  for (int64_t j = 1; j < n; ++j) zmax = std::max(zmax, static_cast<double>(vals[j]));
  double sum = 0.0;
  for (int64_t j = 0; j < n; ++j) sum += std::exp(static_cast<double>(vals[j]) - zmax);
  const double lse = zmax + std::log(sum);
  for (int64_t j = 0; j < n; ++j) out_logp[j] = static_cast<double>(vals[j]) - lse;
}

int32_t oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

}  // extern "C"
