"""Seeded synthetic inputs for the NanoSpec draft-step hot path.

This module only *makes inputs*: random bf16 matrices, Zipf token streams, id sets and
append schedules.  It contains none of the method's arithmetic (no vocabulary
construction, no projection, no top-k), so both the CPU oracle's tests and the HIP path's
tests may draw the same arrays from it.  Everything is numpy on the host, generated from
a counter-based generator written here, so values do not depend on the numpy, torch or
device version.

Workload shapes stand in for what the paper evaluates on (Sec. 4.1: Llama-3.1-8B /
Qwen-2-7B heads, SpecBench + HumanEval token streams): only the shapes and a Zipfian
token-frequency structure are imitated, no dataset item or trained weight is involved.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GOLD = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wraps modulo 2**64)."""
    z = z.copy() if isinstance(z, np.ndarray) else np.uint64(z)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def rand_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """count 64-bit words of the (seed, stream) sequence beginning at index start."""
    with np.errstate(over="ignore"):
        key = _mix(np.uint64(seed) * _GOLD + np.uint64(stream) * _M2 + np.uint64(0x1234567))
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix((idx + np.uint64(1)) * _GOLD + key)


def rand_unit(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """float64 uniforms in (0, 1]."""
    u = rand_u64(seed, stream, start, count)
    return ((u >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)


def rand_int(seed: int, stream: int, start: int, count: int, lo: int, hi: int) -> np.ndarray:
    """integers uniform in [lo, hi] (inclusive); modulo bias is irrelevant at these ranges."""
    u = rand_u64(seed, stream, start, count)
    return (lo + (u % np.uint64(hi - lo + 1)).astype(np.int64)).astype(np.int32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_block(seed: int, stream: int, start: int, count: int, sigma: float) -> np.ndarray:
    """count normals N(0, sigma^2) by Box-Muller; element i uses uniforms 2*(i//2), 2*(i//2)+1."""
    assert start % 2 == 0
    pairs = (count + 1) // 2
    u = rand_unit(seed, stream, start, 2 * pairs)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    t = (2.0 * np.pi) * u[1::2]
    out = np.empty(2 * pairs, dtype=np.float32)
    out[0::2] = (sigma * r * np.cos(t)).astype(np.float32)
    out[1::2] = (sigma * r * np.sin(t)).astype(np.float32)
    return out[:count]


def normal_bf16(seed: int, stream: int, shape, sigma: float, threads: int | None = None) -> np.ndarray:
    """bf16 (uint16 bits) array of N(0, sigma^2) samples, generated in parallel blocks."""
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.uint16)
    blk = 1 << 22
    nblk = (total + blk - 1) // blk

    def work(i):
        a = i * blk
        c = min(blk, total - a)
        out[a:a + c] = f32_to_bf16_bits(_normal_block(seed, stream, a, c, sigma))

    threads = threads or min(16, os.cpu_count() or 1)
    if nblk == 1 or threads == 1:
        for i in range(nblk):
            work(i)
    else:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(work, range(nblk)))
    return out.reshape(shape)


class ZipfVocab:
    """Zipf(s) over V ranks by inverse CDF, ranks mapped to token ids by a seeded permutation."""

    def __init__(self, V: int, s: float, seed: int):
        self.V, self.s, self.seed = V, s, seed
        w = 1.0 / np.power(np.arange(1, V + 1, dtype=np.float64), s)
        cdf = np.cumsum(w)
        self.cdf = cdf / cdf[-1]
        keys = rand_u64(seed, 2, 0, V)
        self.perm = np.argsort(keys, kind="stable").astype(np.int32)   # rank -> token id

    def ranks(self, stream: int, start: int, count: int) -> np.ndarray:
        u = rand_unit(self.seed, stream, start, count)
        return np.minimum(np.searchsorted(self.cdf, u, side="left"), self.V - 1)

    def tokens(self, stream: int, start: int, count: int) -> np.ndarray:
        return self.perm[self.ranks(stream, start, count)]

    def distinct_prefix(self, stream: int, K: int) -> np.ndarray:
        """the first K distinct token ids of the given stream, in order of first appearance."""
        got: list[np.ndarray] = []
        seen = np.zeros(self.V, dtype=bool)
        have, pos = 0, 0
        while have < K:
            chunk = self.tokens(stream, pos, max(4 * K, 4096))
            pos += len(chunk)
            _, first = np.unique(chunk, return_index=True)
            cand = chunk[np.sort(first)]
            cand = cand[~seen[cand]]
            seen[cand] = True
            got.append(cand)
            have += len(cand)
        return np.concatenate(got)[:K].astype(np.int32)


# --------------------------------------------------------------------------------------------------
# The five workloads.  `seed` = config number * 1000.  Streams: 0 weights, 1 hidden states,
# 2 id permutation, 3 TopK candidate stream, 4 accept counts, 16+b context/appended tokens of
# sequence b.
# --------------------------------------------------------------------------------------------------
CONFIGS = {
    "c1": dict(V=32000, d=512, zipf=1.1, ctx=512, window=256, topk=256, M=4, k=8, batch=1,
               steps=8, acc=(1, 4), seed=1000, replace_T="odd"),
    "c2": dict(V=128256, d=4096, zipf=1.1, ctx=2048, window=1024, topk="calibrate", active=3000, M=8,
               k=10, batch=1, steps=64, acc=(1, 4), seed=2000, replace_T="never"),
    "c3": dict(V=152064, d=3584, zipf=1.05, ctx=4096, window=2048, topk="calibrate", active=3000, M=64,
               k=10, batch=1, steps=64, acc=(1, 8), seed=3000, replace_T="never"),
    "c4": dict(V=128256, d=4096, zipf=1.1, ctx=8192, window=4096, topk=1024, M=8, k=10, batch=64,
               steps=128, acc=(1, 8), seed=4000, replace_T="always"),
    # c5: window = whole context, T empty, context length calibrated so that the unique count hits
    # the target; one entry per target size.
    "c5": dict(V=128256, d=8192, zipf=1.1, M=16, k=10, batch=1, steps=4, acc=(1, 4), seed=5000,
               targets=(1000, 3000, 8000, 32000), replace_T="never"),
}


def make_W(cfg) -> np.ndarray:
    """LM-head weights W[V][d], bf16 bits, N(0, 0.02^2)."""
    return normal_bf16(cfg["seed"], 0, (cfg["V"], cfg["d"]), 0.02)


def make_H(cfg, step: int, batch: int | None = None, M: int | None = None) -> np.ndarray:
    """draft hidden states H[batch][M][d] of one step, bf16 bits, N(0, 1)."""
    b = cfg["batch"] if batch is None else batch
    M = cfg["M"] if M is None else M
    return normal_bf16(cfg["seed"] + 1, 1000 + step, (b, M, cfg["d"]), 1.0, threads=1)


def context_len_for_unique(zv: ZipfVocab, stream: int, target: int) -> int:
    """smallest prefix length of the stream whose number of distinct tokens reaches target."""
    n = 4 * target
    while True:
        t = zv.tokens(stream, 0, n)
        _, first = np.unique(t, return_index=True)
        if len(first) >= target:
            return int(np.sort(first)[target - 1]) + 1
        n *= 2


def make_sequences(cfg, target: int | None = None):
    """Build everything the vocabulary calls consume for one config.

    Returns dict with: zv, window, topk_cap, ctx (list of int32 arrays per sequence),
    T0 (list of int32 arrays per sequence), appends[step][b] int32 arrays, T_step[step][b] or None.
    """
    zv = ZipfVocab(cfg["V"], cfg["zipf"], cfg["seed"])
    B = cfg["batch"]
    steps = cfg["steps"]
    lo, hi = cfg["acc"]
    if "targets" in cfg:                                   # c5
        L = context_len_for_unique(zv, 16, int(target))
        ctx = [zv.tokens(16, 0, L)]
        window = L + steps * hi
        T0 = [np.zeros(0, dtype=np.int32)]
        K = 0
    else:
        L = cfg["ctx"]
        ctx = [zv.tokens(16 + b, 0, L) for b in range(B)]
        window = cfg["window"]
        if cfg["topk"] == "calibrate":
            win_unique = np.unique(ctx[0][-window:])
            cand = zv.distinct_prefix(3, 2 * cfg["active"])
            extra = np.cumsum(~np.isin(cand, win_unique))
            K = int(np.searchsorted(extra, cfg["active"] - len(win_unique), side="left")) + 1
            T0 = [cand[:K]]
        else:
            K = cfg["topk"]
            T0 = [zv.distinct_prefix(100 + b, K) for b in range(B)]
    counts = rand_int(cfg["seed"], 4, 0, steps * B, lo, hi).reshape(steps, B)
    appends, T_step = [], []
    pos = [L] * B
    for s in range(steps):
        row = []
        for b in range(B):
            a = int(counts[s, b])
            row.append(zv.tokens(16 + b, pos[b], a))
            pos[b] += a
        appends.append(row)
        mode = cfg["replace_T"]
        if mode == "always" or (mode == "odd" and s % 2 == 1):
            T_step.append([zv.distinct_prefix(100 + b + 1000 * (s + 1), K) for b in range(B)])
        else:
            T_step.append(None)
    return dict(zv=zv, window=window, topk_cap=max(K, 1), ctx=ctx, T0=T0, appends=appends, T_step=T_step)
