"""CPU oracle of the NanoSpec draft-step hot path -- test infrastructure, not the product.

Thin ctypes access to ``nanospec_oracle.cpp`` (plain C++17: std::set vocabulary, scalar
dot products, full-sort top-k).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP library and its
Python binding never do.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nanospec_oracle.cpp")
_LIBS = {False: os.path.join(_HERE, "liboracle.so"), True: os.path.join(_HERE, "liboracle_omp.so")}


def build(force: bool = False) -> None:
    """Compile the oracle twice: single-threaded, and with OpenMP over the active rows."""
    for omp, path in _LIBS.items():
        if not force and os.path.exists(path) and os.path.getmtime(path) >= os.path.getmtime(_SRC):
            continue
        cmd = ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math"]
        if omp:
            cmd.append("-fopenmp")
        subprocess.check_call(cmd + ["-o", path, _SRC])


_loaded: dict[bool, C.CDLL] = {}


def _lib(omp: bool = False) -> C.CDLL:
    if omp not in _loaded:
        build()
        L = C.CDLL(_LIBS[omp])
        i32p, u16p, f32p, f64p = (C.POINTER(t) for t in (C.c_int32, C.c_uint16, C.c_float, C.c_double))
        L.oracle_vocab_new.restype = C.c_void_p
        L.oracle_vocab_new.argtypes = [C.c_int32, C.c_int64]
        L.oracle_vocab_free.argtypes = [C.c_void_p]
        L.oracle_vocab_init.argtypes = [C.c_void_p, i32p, C.c_int64, i32p, C.c_int64]
        L.oracle_vocab_update.argtypes = [C.c_void_p, i32p, C.c_int64, C.c_int32, i32p, C.c_int64]
        L.oracle_vocab_append_unique.argtypes = [C.c_void_p, i32p, C.c_int64]
        L.oracle_fifo_new.restype = C.c_void_p
        L.oracle_fifo_new.argtypes = [C.c_int32, C.c_int64]
        L.oracle_fifo_free.argtypes = [C.c_void_p]
        L.oracle_fifo_init.argtypes = [C.c_void_p, i32p, C.c_int64, i32p, C.c_int64]
        L.oracle_fifo_update.argtypes = [C.c_void_p, i32p, C.c_int64, C.c_int32, i32p, C.c_int64]
        L.oracle_fifo_append_unique.argtypes = [C.c_void_p, i32p, C.c_int64]
        L.oracle_fifo_size.restype = C.c_int64
        L.oracle_fifo_size.argtypes = [C.c_void_p]
        L.oracle_fifo_active.restype = C.c_int64
        L.oracle_fifo_active.argtypes = [C.c_void_p, i32p, C.c_int64]
        L.oracle_vocab_stream_len.restype = C.c_int64
        L.oracle_vocab_stream_len.argtypes = [C.c_void_p]
        L.oracle_vocab_active.restype = C.c_int64
        L.oracle_vocab_active.argtypes = [C.c_void_p, i32p, C.c_int64]
        L.oracle_head.argtypes = [u16p, u16p, i32p, C.c_int64, C.c_int32, C.c_int32, C.c_int64, f32p, f64p]
        L.oracle_topk.argtypes = [f32p, i32p, C.c_int64, C.c_int32, i32p, f32p]
        L.oracle_log_softmax.argtypes = [f32p, C.c_int64, f64p]
        L.oracle_max_threads.restype = C.c_int32
        _loaded[omp] = L
    return _loaded[omp]


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct)) if a is not None else None


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class Vocab:
    """Candidate stream S plus candidate set T of one sequence (Sec. 3.2)."""

    def __init__(self, V: int, window: int):
        self._L = _lib()
        self._h = self._L.oracle_vocab_new(V, window)
        self.V, self.window = V, window

    def __del__(self):
        if getattr(self, "_h", None):
            self._L.oracle_vocab_free(self._h)
            self._h = None

    def init(self, ctx, topk=()):
        ctx, topk = _i32(ctx), _i32(topk)
        self._L.oracle_vocab_init(self._h, _p(ctx, C.c_int32), len(ctx), _p(topk, C.c_int32), len(topk))

    def update(self, new_ids, topk=None):
        new_ids = _i32(new_ids)
        t = _i32(topk) if topk is not None else np.zeros(0, np.int32)
        self._L.oracle_vocab_update(self._h, _p(new_ids, C.c_int32), len(new_ids), int(topk is not None),
                                    _p(t, C.c_int32), len(t))

    def append_unique(self, cand):
        cand = _i32(np.asarray(cand).ravel())
        self._L.oracle_vocab_append_unique(self._h, _p(cand, C.c_int32), len(cand))

    def stream_len(self) -> int:
        return int(self._L.oracle_vocab_stream_len(self._h))

    def active(self) -> np.ndarray:
        n = self._L.oracle_vocab_active(self._h, None, 0)
        out = np.empty(n, dtype=np.int32)
        self._L.oracle_vocab_active(self._h, _p(out, C.c_int32), n)
        return out


class FifoVocab:
    """Second reading of the vocabulary (Sec. 3.3 and the appendix on vocabulary evolution): a first-in first-out
    queue of at most ``window`` distinct ids, plus the candidate set T.  One call pushes, in order of first
    occurrence, the ids that are valid, not yet members when the call starts and not repeated inside the call."""

    def __init__(self, V: int, window: int):
        self._L = _lib()
        self._h = self._L.oracle_fifo_new(V, window)
        self.V, self.window = V, window

    def __del__(self):
        if getattr(self, "_h", None):
            self._L.oracle_fifo_free(self._h)
            self._h = None

    def init(self, ctx, topk=()):
        ctx, topk = _i32(ctx), _i32(topk)
        self._L.oracle_fifo_init(self._h, _p(ctx, C.c_int32), len(ctx), _p(topk, C.c_int32), len(topk))

    def update(self, new_ids, topk=None):
        new_ids = _i32(new_ids)
        t = _i32(topk) if topk is not None else np.zeros(0, np.int32)
        self._L.oracle_fifo_update(self._h, _p(new_ids, C.c_int32), len(new_ids), int(topk is not None),
                                   _p(t, C.c_int32), len(t))

    def append_unique(self, cand):
        cand = _i32(np.asarray(cand).ravel())
        self._L.oracle_fifo_append_unique(self._h, _p(cand, C.c_int32), len(cand))

    def size(self) -> int:
        return int(self._L.oracle_fifo_size(self._h))

    def active(self) -> np.ndarray:
        n = self._L.oracle_fifo_active(self._h, None, 0)
        out = np.empty(n, dtype=np.int32)
        self._L.oracle_fifo_active(self._h, _p(out, C.c_int32), n)
        return out


def head(W, H, ids=None, n=None, want32=True, want64=True, omp=False):
    """Eq. 1 on the rows ``ids`` (all V rows when ids is None).  W [V][d], H [M][d] as bf16 bits.

    Returns (logits_fp32 [M][n] or None, logits_fp64 [M][n] or None)."""
    W = np.ascontiguousarray(W, dtype=np.uint16)
    H = np.ascontiguousarray(H, dtype=np.uint16)
    V, d = W.shape
    M = H.shape[0]
    assert H.shape[1] == d
    if ids is not None:
        ids = _i32(ids)
        n = len(ids)
        assert n == 0 or (ids.min() >= 0 and ids.max() < V)
    else:
        n = V if n is None else n
    o32 = np.empty((M, n), dtype=np.float32) if want32 else None
    o64 = np.empty((M, n), dtype=np.float64) if want64 else None
    _lib(omp).oracle_head(_p(W, C.c_uint16), _p(H, C.c_uint16), _p(ids, C.c_int32), n, M, d, n,
                          _p(o32, C.c_float), _p(o64, C.c_double))
    return o32, o64


def topk(vals, ids, k: int):
    """Top-k of one logit row mapped to global ids: (ids int32[k], values float32[k])."""
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    n = len(vals)
    if ids is not None:
        ids = _i32(ids)
        assert len(ids) == n
    oi = np.empty(k, dtype=np.int32)
    ov = np.empty(k, dtype=np.float32)
    _lib().oracle_topk(_p(vals, C.c_float), _p(ids, C.c_int32), n, k, _p(oi, C.c_int32), _p(ov, C.c_float))
    return oi, ov


def log_softmax(vals):
    """Log-probabilities of one logit row renormalised over its own entries (Sec. 4.2): float64[n]."""
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    out = np.empty(len(vals), dtype=np.float64)
    _lib().oracle_log_softmax(_p(vals, C.c_float), len(vals), _p(out, C.c_double))
    return out


def topk_logprob(vals, ids, k: int):
    """Top-k of one row with the values replaced by log-probabilities over the active set:
    (ids int32[k], logp float64[k]); slots beyond the row length get id -1 and -inf."""
    oi, ov = topk(vals, ids, k)
    lp = log_softmax(vals)
    # the selected values are looked up by position: lowest position among equal (value, id) is irrelevant for logp
    out = np.full(k, -np.inf, dtype=np.float64)
    vals = np.asarray(vals, dtype=np.float32)
    for r in range(min(k, len(vals))):
        j = int(np.flatnonzero(vals == ov[r])[0])
        out[r] = lp[j]
    return oi, out


def shared_rows(actives, min_share: int, shared_cap: int):
    """Split of the active sets of several sequences into rows worth fetching once for the whole batch and rows
    handled per sequence (multi-sequence serving; Sec. 4.6 states only that the per-sequence cost adds up over the
    batch).  An id is *shared* when at least ``min_share`` of the sets hold it; only the ``shared_cap`` lowest such
    ids count.  Returns (shared ids ascending int32[P],
    pos int32[B][P] = position of shared id p in sequence b's ascending active list or -1 if b does not hold it,
    rest = per sequence (ids int32[], positions int32[]) of its active ids that are not shared, ascending).
    Written as the definition: a count per id over the sets, a threshold, list look-ups."""
    count: dict[int, int] = {}
    for a in actives:
        for t in a:
            count[int(t)] = count.get(int(t), 0) + 1
    shared = sorted(t for t, c in count.items() if c >= min_share)[:max(shared_cap, 0)]
    member = set(shared)
    pos = np.full((len(actives), len(shared)), -1, dtype=np.int32)
    rest = []
    for b, a in enumerate(actives):
        where = {int(t): j for j, t in enumerate(a)}
        for p, t in enumerate(shared):
            pos[b, p] = where.get(t, -1)
        keep = [j for j, t in enumerate(a) if int(t) not in member]
        rest.append((np.asarray([a[j] for j in keep], dtype=np.int32), np.asarray(keep, dtype=np.int32)))
    return np.asarray(shared, dtype=np.int32), pos, rest


def max_threads() -> int:
    return int(_lib(True).oracle_max_threads())
