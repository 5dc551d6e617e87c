"""Pins for the oracle's vocabulary (Sec. 3.2, Eq. 2-4): worked examples, brute force, invariants."""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(V, W, stream, T=(), split=None):
    """active set after feeding `stream` (init on the first `split` ids, the rest by updates)."""
    v = oracle.Vocab(V, W)
    split = len(stream) if split is None else split
    v.init(stream[:split], T)
    for x in stream[split:]:
        v.update([x])
    return v.active().tolist()


def brute(V, W, stream, T):
    """independent O(V*W) membership test: v is active iff it sits at one of the last W stream
    positions or is in T."""
    out = []
    L = len(stream)
    for v in range(V):
        hit = False
        for back in range(1, W + 1):
            p = L - back
            if p < 0:
                break
            if stream[p] == v:
                hit = True
        for t in T:
            if t == v:
                hit = True
        if hit:
            out.append(v)
    return out


def parse_examples():
    rows = []
    for line in open(os.path.join(GOLD, "vocab_worked_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        W, S, T, exp = [f.strip() for f in line.split("|")]
        ints = lambda s: [] if s == "-" else [int(x) for x in s.split()]
        rows.append((int(W), ints(S), ints(T), ints(exp)))
    return rows


@pytest.mark.parametrize("W,S,T,exp", parse_examples())
def test_worked_examples(W, S, T, exp):
    assert run_oracle(16, W, S, T) == exp
    # the same stream fed token by token after an empty init gives the same set
    assert run_oracle(16, W, S, T, split=0) == exp
    assert brute(16, W, S, T) == exp


def test_exhaustive_tiny():
    """all streams of length <= 6 over 3 ids, all windows 1..4, against brute force."""
    for L in range(0, 7):
        for S in itertools.product(range(3), repeat=L):
            for W in (1, 2, 3, 4):
                assert run_oracle(3, W, list(S)) == brute(3, W, S, ())


def test_fuzz_against_brute_force():
    rng = np.random.default_rng(7)
    for trial in range(300):
        V = int(rng.integers(2, 64))
        W = int(rng.integers(1, 9))
        v = oracle.Vocab(V, W)
        S = rng.integers(0, V, size=int(rng.integers(0, 20))).tolist()
        T = rng.integers(0, V, size=int(rng.integers(0, 6))).tolist()
        v.init(S, T)
        assert v.active().tolist() == brute(V, W, S, T)
        for step in range(12):
            new = rng.integers(0, V, size=int(rng.integers(0, 2 * W + 2))).tolist()
            if rng.random() < 0.4:
                T = rng.integers(0, V, size=int(rng.integers(0, 6))).tolist()
                v.update(new, T)
            else:
                v.update(new)
            S = S + new
            assert v.stream_len() == len(S)
            assert v.active().tolist() == brute(V, W, S, T), (trial, step)


def test_invariants():
    rng = np.random.default_rng(11)
    for trial in range(100):
        V, W = 200, int(rng.integers(1, 40))
        S = rng.integers(0, V, size=int(rng.integers(1, 120))).tolist()
        T = rng.integers(0, V, size=int(rng.integers(0, 10))).tolist()
        A = run_oracle(V, W, S, T)
        assert A == sorted(set(A))                                   # ascending, unique
        assert set(S[-W:]) <= set(A)                                 # every suffix token is active
        assert set(T) <= set(A)
        assert len(A) <= min(W, len(S)) + len(set(T))                # |I| <= W_max (+|T|)
        assert set(A) == set(S[-W:]) | set(T)
        if W >= len(S):
            assert set(A) == set(S) | set(T)                         # short stream: taken whole
        assert run_oracle(V, 1, S, T) == sorted({S[-1]} | set(T))    # W=1: last token only
        # incremental updates == init on the full stream, whatever the split point
        for split in (0, len(S) // 2, len(S)):
            assert run_oracle(V, W, S, T, split=split) == A
        # relabelling ids by a permutation maps the set through the permutation
        pi = rng.permutation(V)
        assert run_oracle(V, W, [int(pi[s]) for s in S], [int(pi[t]) for t in T]) == sorted(int(pi[a]) for a in A)
        # order and multiplicity of T's elements are irrelevant
        assert run_oracle(V, W, S, list(reversed(T)) + T) == A


def test_recency_eviction():
    """a token leaves exactly when its most recent occurrence leaves the window (text after Eq. 4)."""
    V, W = 50, 5
    v = oracle.Vocab(V, W)
    v.init([7])
    for i in range(1, W):                  # 7 is still among the last W ids
        v.update([10 + i])
        assert 7 in v.active()
    v.update([30])                         # now W newer ids follow it
    assert 7 not in v.active()
    v.update([7])                          # re-appended: back in
    assert 7 in v.active()


def test_update_replaces_T_wholesale_and_keeps_it_otherwise():
    v = oracle.Vocab(100, 2)
    v.init([1, 2], [50, 60])
    v.update([3])
    assert v.active().tolist() == [2, 3, 50, 60]
    v.update([], [70])
    assert v.active().tolist() == [2, 3, 70]
    v.update([4], [])
    assert v.active().tolist() == [3, 4]


def test_out_of_range_ids_hold_a_position_but_are_not_members():
    v = oracle.Vocab(10, 2)
    v.init([1, 2, 99])
    assert v.active().tolist() == [2]
    v.update([-5], [3, 10, -1])
    assert v.active().tolist() == [3]


def test_window_bound_paper_setting():
    """W_max = 3072 (Sec. 4.1): the active set never exceeds it however long the stream grows."""
    rng = np.random.default_rng(3)
    v = oracle.Vocab(128256, 3072)
    v.init(rng.integers(0, 128256, size=5000))
    for _ in range(5):
        v.update(rng.integers(0, 128256, size=2000))
        assert len(v.active()) <= 3072


def test_append_unique_is_a_sorted_set_append():
    """Eq. 3 with a candidate set: distinct valid ids, ascending, -1 padding and bad ids dropped."""
    v = oracle.Vocab(100, 4)
    v.init([50, 51])
    v.append_unique([7, 3, 7, -1, 3, 99, 100, 250])
    assert v.stream_len() == 5                          # 3, 7, 99 appended
    assert v.active().tolist() == [3, 7, 51, 99]        # window 4: 51, 3, 7, 99
    w = oracle.Vocab(100, 4)
    w.init([50, 51])
    w.update([3, 7, 99])                                # the same thing through the plain append
    assert w.active().tolist() == v.active().tolist()
    v.append_unique([])
    v.append_unique([-1, -1])
    assert v.stream_len() == 5


# ---- second reading: first-in first-out queue of distinct ids (Sec. 3.3 and the appendix on vocabulary evolution)

def _fifo_cases():
    for line in open(os.path.join(GOLD, "fifo_worked_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        W, calls, T, exp = [x.strip() for x in line.split("|")]
        calls = [[] if c.strip() == "-" else [int(x) for x in c.split()] for c in calls.split(";")]
        T = [] if T == "-" else [int(x) for x in T.split()]
        yield int(W), calls, T, [int(x) for x in exp.split()]


def test_fifo_worked_examples():
    n = 0
    for W, calls, T, exp in _fifo_cases():
        v = oracle.FifoVocab(100, W)
        v.init(calls[0], T)
        for c in calls[1:]:
            v.update(c)
        assert v.active().tolist() == exp, (W, calls, T)
        n += 1
    assert n >= 13


def _fifo_reference(V, W, calls):
    """an independent statement of the same queue: the members after the calls are the last W entries of the
    list of all pushes, where a call's pushes are its distinct valid ids that are not among the last W pushes
    made before the call (plain Python lists, recomputed from the whole history at every call)."""
    pushes = []
    for c in calls:
        members = pushes[-W:] if W > 0 else []
        new = []
        for a in c:
            if 0 <= a < V and a not in members and a not in new:
                new.append(a)
        pushes.extend(new)
    return sorted(set(pushes[-W:]))


def test_fifo_against_history_recomputation():
    rng = np.random.default_rng(11)
    for trial in range(300):
        V = int(rng.integers(4, 40))
        W = int(rng.integers(1, 12))
        calls = [rng.integers(-2, V + 2, size=int(rng.integers(0, 3 * W + 2))).tolist() for _ in range(int(rng.integers(1, 9)))]
        v = oracle.FifoVocab(V, W)
        v.init(calls[0])
        for i, c in enumerate(calls[1:], start=2):
            v.update(c)
            assert v.active().tolist() == _fifo_reference(V, W, calls[:i]), (V, W, calls[:i])
        assert v.size() <= W


def test_fifo_equals_window_when_nothing_repeats():
    """with no repeated id anywhere in the stream the two readings coincide (the Eq. 4 oracle is pinned on its own)."""
    rng = np.random.default_rng(12)
    for trial in range(100):
        V, W = 500, int(rng.integers(1, 60))
        stream = rng.permutation(V)[: int(rng.integers(1, 200))].astype(np.int32)
        cuts = np.sort(rng.integers(0, len(stream) + 1, size=4))
        parts = np.split(stream, cuts)
        T = rng.integers(0, V, size=5)
        f, w = oracle.FifoVocab(V, W), oracle.Vocab(V, W)
        f.init(parts[0], T)
        w.init(parts[0], T)
        for p in parts[1:]:
            f.update(p)
            w.update(p)
            assert np.array_equal(f.active(), w.active())


def test_fifo_invariants():
    rng = np.random.default_rng(13)
    V, W = 300, 40
    zipf_like = lambda n: np.minimum((rng.pareto(1.1, size=n) * 3).astype(np.int32), V - 1)
    f = oracle.FifoVocab(V, W)
    f.init(zipf_like(30))
    prev = set(f.active().tolist())
    grown = True
    for step in range(200):
        new = zipf_like(int(rng.integers(0, 9)))
        f.update(new)
        cur = set(f.active().tolist())
        assert len(cur) == f.size() <= W
        if len(prev) + len(set(new.tolist()) - prev) <= W:
            assert prev <= cur                                   # below capacity the vocabulary only grows
        assert set(new.tolist()) - prev <= cur or len(set(new.tolist()) - prev) > W   # every new id gets in
        f2_before = f.active().copy()
        f.update(np.array(sorted(cur), np.int32))                # re-appending members changes nothing
        assert np.array_equal(f.active(), f2_before)
        prev = cur
    # a candidate set is one call of its distinct valid ids in ascending order
    a, b = oracle.FifoVocab(V, 5), oracle.FifoVocab(V, 5)
    a.init([1, 2, 3])
    b.init([1, 2, 3])
    a.append_unique([9, 7, 7, -1, 2, 300, 8, 6])
    b.update([6, 7, 8, 9])
    assert np.array_equal(a.active(), b.active()) and a.active().tolist() == [3, 6, 7, 8, 9]


# ---- split of several sequences' active sets into shared rows and per-sequence rows -------------------------
def test_shared_rows_hand_worked():
    """Three sets over ids 0..9, worked by hand: 2 and 7 are in all three, 4 in two, the others in one."""
    A = [np.array([1, 2, 4, 7], np.int32), np.array([2, 4, 7, 9], np.int32), np.array([0, 2, 7], np.int32)]
    sh, pos, rest = oracle.shared_rows(A, 3, 10)
    assert sh.tolist() == [2, 7]
    assert pos.tolist() == [[1, 3], [0, 2], [1, 2]]
    assert [r[0].tolist() for r in rest] == [[1, 4], [4, 9], [0]]
    assert [r[1].tolist() for r in rest] == [[0, 2], [1, 3], [0]]
    sh, pos, rest = oracle.shared_rows(A, 2, 10)                      # 4 joins; sequence 2 does not hold it
    assert sh.tolist() == [2, 4, 7]
    assert pos.tolist() == [[1, 2, 3], [0, 1, 2], [1, -1, 2]]
    assert [r[0].tolist() for r in rest] == [[1], [9], [0]]
    sh, pos, rest = oracle.shared_rows(A, 2, 2)                       # room for two shared rows only: 7 stays per sequence
    assert sh.tolist() == [2, 4]
    assert [r[0].tolist() for r in rest] == [[1, 7], [7, 9], [0, 7]]
    assert [r[1].tolist() for r in rest] == [[0, 3], [2, 3], [0, 2]]
    sh, pos, rest = oracle.shared_rows(A, 1, 0)                       # no room at all: everything per sequence
    assert len(sh) == 0 and pos.shape == (3, 0) and [r[0].tolist() for r in rest] == [a.tolist() for a in A]


def test_shared_rows_partition_every_pair_exactly_once():
    """Property on random sets: every (sequence, active id) pair is covered by exactly one of the two parts, at the
    id's own position; shared ids meet the threshold (counted here with a dense 0/1 matrix, not the oracle's dict)."""
    rng = np.random.default_rng(11)
    for trial in range(40):
        V, B = int(rng.integers(5, 60)), int(rng.integers(1, 9))
        A = [np.flatnonzero(rng.random(V) < rng.uniform(0.1, 0.9)).astype(np.int32) for _ in range(B)]
        share, capP = int(rng.integers(1, B + 1)), int(rng.integers(0, V + 1))
        sh, pos, rest = oracle.shared_rows(A, share, capP)
        Mx = np.zeros((B, V), int)
        for b, a in enumerate(A):
            Mx[b, a] = 1
        want = np.flatnonzero(Mx.sum(0) >= share)[:capP]
        assert np.array_equal(sh, want)
        for b, a in enumerate(A):
            cover = np.zeros(len(a), int)
            for p, t in enumerate(sh):
                if pos[b, p] >= 0:
                    assert a[pos[b, p]] == t
                    cover[pos[b, p]] += 1
                else:
                    assert t not in a
            ids_r, pos_r = rest[b]
            assert np.array_equal(a[pos_r], ids_r) and np.all(np.diff(pos_r) > 0)
            cover[pos_r] += 1
            assert np.all(cover == 1)
