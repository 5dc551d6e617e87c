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


# ---- log-softmax over the active set (Sec. 4.2: the draft distribution renormalised on the pruned vocabulary)

def test_log_softmax_closed_forms():
    import math
    # n equal logits: every log-probability is -log n, whatever the common value
    for n, c in ((1, 3.5), (7, -2.0), (3000, 11.25)):
        lp = oracle.log_softmax(np.full(n, c, np.float32))
        assert np.allclose(lp, -math.log(n), rtol=0, atol=1e-12)
    # two entries a, b: logp(a) = -log(1 + e^(b-a))
    a, b = 0.75, -1.5
    lp = oracle.log_softmax(np.array([a, b], np.float32))
    assert abs(lp[0] + math.log1p(math.exp(b - a))) < 1e-12
    assert abs(lp[1] + math.log1p(math.exp(a - b))) < 1e-12
    # hand-worked: logits (0, ln 2, ln 5) -> probabilities 1/8, 2/8, 5/8
    z = np.array([0.0, math.log(2.0), math.log(5.0)], np.float32)
    p = np.exp(oracle.log_softmax(z))
    assert np.allclose(p, [0.125, 0.25, 0.625], atol=1e-7)      # float32 storage of ln 2, ln 5


def test_log_softmax_invariants():
    rng = np.random.default_rng(7)
    for n in (1, 2, 63, 64, 65, 1000, 3001):
        z = (rng.normal(size=n) * 6).astype(np.float32)
        lp = oracle.log_softmax(z)
        assert abs(np.exp(lp).sum() - 1.0) < 1e-12                # a distribution
        assert np.all(lp <= 1e-15)
        # differences of log-probabilities are differences of logits: nothing but one constant is subtracted
        assert np.allclose(lp - lp[0], z.astype(np.float64) - float(z[0]), rtol=0, atol=1e-12)
        # shifting every logit by a float32-exact constant leaves the result unchanged
        zs = (z.astype(np.float64) + 8.0).astype(np.float32)
        exact = zs.astype(np.float64) - 8.0 == z.astype(np.float64)
        if exact.all():
            assert np.allclose(oracle.log_softmax(zs), lp, rtol=0, atol=1e-12)
    # large magnitudes must not overflow: the maximum is subtracted first
    lp = oracle.log_softmax(np.array([1000.0, 999.0, -1000.0], np.float32))
    assert np.all(np.isfinite(lp)) and abs(np.exp(lp).sum() - 1.0) < 1e-12


def test_log_softmax_against_library():
    from scipy.special import log_softmax as sp_log_softmax
    rng = np.random.default_rng(8)
    for n in (5, 300, 4096):
        z = (rng.normal(size=n) * 4).astype(np.float32)
        assert np.allclose(oracle.log_softmax(z), sp_log_softmax(z.astype(np.float64)), rtol=0, atol=1e-11)


def test_topk_logprob():
    rng = np.random.default_rng(9)
    n = 500
    z = rng.normal(size=n).astype(np.float32)
    ids = np.sort(rng.choice(9000, size=n, replace=False)).astype(np.int32)
    oi, lp = oracle.topk_logprob(z, ids, 10)
    ti, tv = oracle.topk(z, ids, 10)
    assert np.array_equal(oi, ti)                                  # renormalising does not change the order
    lse = np.log(np.exp(z.astype(np.float64)).sum())
    assert np.allclose(lp, tv.astype(np.float64) - lse, rtol=0, atol=1e-12)
    assert np.all(np.diff(lp) <= 0)
    oi, lp = oracle.topk_logprob(z[:3], ids[:3], 5)                # padding past the row length
    assert oi.tolist()[3:] == [-1, -1] and np.all(np.isneginf(lp[3:]))
