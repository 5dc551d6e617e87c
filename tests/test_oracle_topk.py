"""Pins for the oracle's draft-token selection (operator T_K of Sec. 3.2; Alg. 1 SelectDraftTokens)."""
import numpy as np

import oracle


def brute_topk(vals, ids, k):
    order = np.lexsort((ids, -vals.astype(np.float64)))          # value desc, id asc
    order = order[:k]
    return ids[order], vals[order]


def test_against_lexsort():
    rng = np.random.default_rng(1)
    for trial in range(50):
        n = int(rng.integers(1, 400))
        vals = rng.normal(size=n).astype(np.float32)
        if trial % 3 == 0:
            vals = np.round(vals * 2) / 2                          # many exact ties
        ids = np.sort(rng.choice(5000, size=n, replace=False)).astype(np.int32)
        k = int(rng.integers(1, n + 1))
        oi, ov = oracle.topk(vals, ids, k)
        bi, bv = brute_topk(vals, ids, k)
        assert np.array_equal(oi, bi) and np.array_equal(ov, bv)


def test_hand_cases():
    ids = np.array([3, 10, 11, 40, 41], np.int32)
    vals = np.array([0.5, 2.0, 2.0, -1.0, 2.0], np.float32)
    oi, ov = oracle.topk(vals, ids, 4)
    assert oi.tolist() == [10, 11, 41, 3] and ov.tolist() == [2.0, 2.0, 2.0, 0.5]     # ties -> lower id
    oi, _ = oracle.topk(vals, ids, 1)
    assert oi.tolist() == [10]                                                         # k=1: argmax
    oi, _ = oracle.topk(vals, ids, 5)
    assert oi.tolist() == [10, 11, 41, 3, 40]                                          # k=n: full ranking
    oi, ov = oracle.topk(vals, ids, 7)                                                 # k>n: padding
    assert oi.tolist()[5:] == [-1, -1] and np.all(np.isneginf(ov[5:]))
    oi, _ = oracle.topk(np.full(6, 1.25, np.float32), np.array([9, 8, 7, 6, 5, 4], np.int32), 3)
    assert oi.tolist() == [4, 5, 6]                                                    # all equal: k lowest ids
    oi, _ = oracle.topk(np.array([-0.0, 0.0, -0.0], np.float32), np.array([2, 5, 1], np.int32), 2)
    assert oi.tolist() == [1, 2]                                                       # +0 == -0 is a tie
    oi, _ = oracle.topk(np.array([1.0, 3.0, 2.0], np.float32), None, 2)                # ids None: local index
    assert oi.tolist() == [1, 2]
