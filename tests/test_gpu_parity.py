"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2605_26444_amd import binding as B
from paper_2605_26444_amd import synth

from harness import (ATOL, RTOL, assert_logits_close, check_topk, csr, dev, dev_bf16, dev_ids, host_W,
                     run_workload)

pytestmark = pytest.mark.gpu


def test_c1_tiny_every_step():
    st = run_workload(synth.CONFIGS["c1"])
    assert st["steps_checked"] == 9 and st.get("rows_checked_e2e", 0) > 0


def test_c2_llama8b_head_every_step():
    cfg = synth.CONFIGS["c2"]
    st = run_workload(cfg)
    n = np.array(st["n"])
    assert abs(n[0, 0] - 3000) <= 60                      # |active| ~ 3k as the workload states
    assert st["steps_checked"] == cfg["steps"] + 1
    print("c2", st["max_err"], st.get("rows_near_tie", 0))


def test_c3_qwen7b_head_wide_tree():
    cfg = synth.CONFIGS["c3"]
    st = run_workload(cfg)                                 # logits and selection on every step
    assert st["steps_checked"] == cfg["steps"] + 1
    print("c3", st["max_err"], st.get("rows_near_tie", 0))


def test_c4_batch64_vocab_stress():
    cfg = synth.CONFIGS["c4"]
    st = run_workload(cfg, check_steps={0, 1, 127} | set(range(16, 128, 16)))
    assert len(st["n"]) == cfg["steps"] + 1                # ids compared on every step
    print("c4", st["max_err"], np.mean(st["n"]))


@pytest.mark.parametrize("target", synth.CONFIGS["c5"]["targets"])
def test_c5_sparsity_sweep(target):
    cfg = synth.CONFIGS["c5"]
    st = run_workload(cfg, target=target)
    assert st["n"][0][0] == target
    print("c5", target, st["max_err"])


def test_dense_head_and_topk_small_full_check():
    cfg = synth.CONFIGS["c1"]
    W = host_W(cfg)
    V, d, M, k = cfg["V"], cfg["d"], 5, 8
    H = synth.make_H(cfg, 99, 1, M)[0]
    dW, dH = dev_bf16(W), dev_bf16(H)
    logits = torch.empty((M, V), dtype=torch.float32, device="cuda")
    B.nanospec_dense_head(dW, dH, V, d, M, logits)
    ws_bytes = B.nanospec_dense_topk_workspace(V, M, k)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    oi_d = torch.empty((M, k), dtype=torch.int32, device="cuda")
    ov_d = torch.empty((M, k), dtype=torch.float32, device="cuda")
    B.nanospec_dense_topk(logits, V, M, k, oi_d, ov_d, ws, ws_bytes)
    torch.cuda.synchronize()
    g = logits.cpu().numpy()
    o32, o64 = oracle.head(W, H, omp=True)
    assert_logits_close(g, o64, o32, "dense c1")
    stats = {}
    allids = np.arange(V, dtype=np.int32)
    for m in range(M):
        check_topk(oi_d.cpu().numpy()[m], ov_d.cpu().numpy()[m], g[m], o32[m], allids, k, stats, f"dense row {m}")


def test_dense_head_full_size_sampled():
    """V=128256, d=4096 dense head in the shape the benchmark times; oracle on sampled rows."""
    cfg = synth.CONFIGS["c2"]
    W = host_W(cfg)
    V, d, M, k = cfg["V"], cfg["d"], cfg["M"], cfg["k"]
    H = synth.make_H(cfg, 7, 1, M)[0]
    dW, dH = dev_bf16(W), dev_bf16(H)
    logits = torch.empty((M, V), dtype=torch.float32, device="cuda")
    B.nanospec_dense_head(dW, dH, V, d, M, logits)
    ws_bytes = B.nanospec_dense_topk_workspace(V, M, k)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    oi_d = torch.empty((M, k), dtype=torch.int32, device="cuda")
    ov_d = torch.empty((M, k), dtype=torch.float32, device="cuda")
    B.nanospec_dense_topk(logits, V, M, k, oi_d, ov_d, ws, ws_bytes)
    torch.cuda.synchronize()
    g = logits.cpu().numpy()
    rng = np.random.default_rng(0)
    sample = np.unique(np.concatenate([rng.choice(V, 4000, replace=False), [0, 1, V - 2, V - 1],
                                       oi_d.cpu().numpy().ravel()])).astype(np.int32)
    o32, o64 = oracle.head(W, H, ids=sample, omp=True)
    assert_logits_close(g[:, sample], o64, o32, "dense c2 sampled")
    allids = np.arange(V, dtype=np.int32)
    for m in range(M):                                       # selection checked exactly on the GPU's logits
        ei, ev = oracle.topk(g[m], allids, k)
        assert np.array_equal(oi_d.cpu().numpy()[m], ei) and np.array_equal(ov_d.cpu().numpy()[m], ev)


def _dense_entries_against_oracle(W, V, d, M_total, k, seed, n_sample=1500, full=False):
    """nanospec_dense_head + nanospec_dense_topk on M_total hidden rows: logits against the oracle on sampled
    columns (first and last included, plus every selected column) or on all of them, selection exact on the
    GPU's own logits for every hidden row."""
    H = synth.normal_bf16(seed, 1, (M_total, d), 1.0, threads=1)
    dW, dH = dev_bf16(W), dev_bf16(H)
    logits = torch.full((M_total, V), float("nan"), dtype=torch.float32, device="cuda")
    B.nanospec_dense_head(dW, dH, V, d, M_total, logits)
    wsb = B.nanospec_dense_topk_workspace(V, M_total, k)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    oi = torch.empty((M_total, k), dtype=torch.int32, device="cuda")
    ov = torch.empty((M_total, k), dtype=torch.float32, device="cuda")
    B.nanospec_dense_topk(logits, V, M_total, k, oi, ov, ws, wsb)
    torch.cuda.synchronize()
    g, gi, gv = logits.cpu().numpy(), oi.cpu().numpy(), ov.cpu().numpy()
    del logits, dW
    assert not np.isnan(g).any(), "a logit was never written"
    if full:
        o32, o64 = oracle.head(W, H, omp=True)
        assert_logits_close(g, o64, o32, f"dense V={V} d={d} M={M_total}")
    else:
        rng = np.random.default_rng(seed)
        edge = [0, 1, 2, 3, 63, 64, V - 65, V - 64, V - 4, V - 3, V - 2, V - 1]
        sample = np.unique(np.concatenate([rng.choice(V, n_sample, replace=False), edge, gi.ravel()])).astype(np.int32)
        o32, o64 = oracle.head(W, H, ids=sample, omp=True)
        assert_logits_close(g[:, sample], o64, o32, f"dense V={V} d={d} M={M_total} sampled")
    allids = np.arange(V, dtype=np.int32)
    for m in range(M_total):
        ei, ev = oracle.topk(g[m], allids, k)
        assert np.array_equal(gi[m], ei) and np.array_equal(gv[m], ev), f"dense selection row {m}"


def test_dense_entries_c5_comparator_m16_d8192():
    cfg = synth.CONFIGS["c5"]
    _dense_entries_against_oracle(host_W(cfg), cfg["V"], cfg["d"], 16, cfg["k"], 5100)


def test_dense_entries_c3_comparator_m64():
    cfg = synth.CONFIGS["c3"]
    _dense_entries_against_oracle(host_W(cfg), cfg["V"], cfg["d"], 64, cfg["k"], 3100)


@pytest.mark.parametrize("M_total", [70, 512])
def test_dense_entries_c4_comparator_many_hidden_rows(M_total):
    """more than 64 hidden rows through the dense entry (the batched comparator of the 64-sequence workload)."""
    cfg = synth.CONFIGS["c4"]
    _dense_entries_against_oracle(host_W(cfg), cfg["V"], cfg["d"], M_total, cfg["k"], 4100 + M_total, n_sample=600)


@pytest.mark.parametrize("d,M_total", [(512, 5), (512, 16), (1024, 40), (520, 40), (512, 70), (1032, 130), (8192, 16), (4096, 12),
                                        (1024, 130), (512, 300), (128, 257)])   # the register-blocked kernel's three block shapes, scalar stores
def test_dense_entries_row_stride_not_a_multiple_of_four(d, M_total):
    """V = 50001: logit rows start at odd addresses (the per-element store branch of the head kernels, the scalar
    load branch of the selection) and the last row tile is ragged."""
    V = 50001
    W = synth.normal_bf16(9100 + d, 0, (V, d), 0.02)
    _dense_entries_against_oracle(W, V, d, M_total, 10, 9200 + d + M_total, full=d <= 1032, n_sample=3000)


@pytest.mark.parametrize("V,W,nT,alphabet", [(3000, 150, 60, 400), (128256, 1024, 2000, 5000), (50000, 300, 0, 350), (700, 64, 700, 700),
                                            (200000, 6000, 100, 9000)])
def test_feedback_of_active_ids(V, W, nT, alphabet):
    """nanospec_vocab_append_unique with candidates drawn from the active set itself (what a closed draft loop
    feeds back), 1 to 128 per call (the sets small enough to be sorted without the scratch bitmap): windows small
    enough that every call evicts, rings full of repeats, ids held by T only, repeats and -1 padding among the
    candidates, an id that leaves and is appended in the same call; every few calls a candidate that is not
    active, and a plain update in between."""
    rng = np.random.default_rng(V + W)
    st = B.State(V, 64, 1, W, max(nT, 1), 8, 16)
    orc = oracle.Vocab(V, W)
    pool = rng.choice(V, alphabet, replace=False).astype(np.int32)
    ctx = rng.choice(pool, 3 * W).astype(np.int32)
    T = rng.choice(V, nT, replace=False).astype(np.int32)
    B.nanospec_vocab_init(st.h, dev(ctx), [0, len(ctx)], dev_ids(T), [0, len(T)])
    orc.init(ctx, T)
    for step in range(40):
        act = orc.active()
        assert np.array_equal(st.read_active()[0], act), step
        per = int(rng.choice([1, 7, 80, 128]))
        cand = rng.choice(act, per).astype(np.int32)                       # members, with repeats
        cand[rng.random(per) < 0.1] = -1                                   # padding
        if step % 3 == 1:                                                  # ids about to leave the window, appended again
            tail = ctx[-W:] if step == 1 else cand
            cand[: min(per, 5)] = tail[: min(per, 5)]
        if step % 7 == 6:
            cand[0] = int(rng.integers(0, V))                              # most likely not active: everything is rebuilt
        B.nanospec_vocab_append_unique(st.h, dev(cand), per, per)
        orc.append_unique(cand)
        if step % 5 == 4:
            new = rng.choice(pool, int(rng.integers(1, 9))).astype(np.int32)
            B.nanospec_vocab_update(st.h, dev(new), [0, len(new)])
            orc.update(new)
    assert np.array_equal(st.read_active()[0], orc.active())
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()


def _small_state(V=1000, d=64, batch=1, window=8, topk_cap=4, m_cap=3, k_cap=64):
    return B.State(V, d, batch, window, topk_cap, m_cap, k_cap)


def test_edge_cases_vocab():
    st = _small_state()
    o = oracle.Vocab(1000, 8)
    # empty init: n == 0
    B.nanospec_vocab_init(st.h, None, [0, 0], None, [0, 0])
    o.init([], [])
    assert len(st.read_active()[0]) == 0
    # zero-length update is legal; update with only a T replacement
    B.nanospec_vocab_update(st.h, None, [0, 0])
    B.nanospec_vocab_update(st.h, None, [0, 0], dev(np.array([5, 5, 7], np.int32)), [0, 3])
    o.update([], [5, 5, 7])
    assert np.array_equal(st.read_active()[0], o.active())
    # more new ids than the window holds; duplicates; id evicted and re-appended in one call
    new = np.array([1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 3, 3, 900], np.int32)
    B.nanospec_vocab_update(st.h, dev(new), [0, len(new)])
    o.update(new)
    assert np.array_equal(st.read_active()[0], o.active())
    new = np.array([7, 8, 9, 10, 11, 3, 3, 900], np.int32)       # evicts exactly what it re-appends
    B.nanospec_vocab_update(st.h, dev(new), [0, len(new)])
    o.update(new)
    assert np.array_equal(st.read_active()[0], o.active())
    new = np.array([42] * 8, np.int32)                              # all-duplicate append fills the window
    B.nanospec_vocab_update(st.h, dev(new), [0, 8], None, [0, 0])
    o.update(new, [])
    assert np.array_equal(st.read_active()[0], o.active()) and st.read_active()[0].tolist() == [42]
    assert B.nanospec_last_device_error(st.h) == 0
    # out-of-range ids: flagged, hold a stream position, never members
    new = np.array([1, 1000, -3, 2], np.int32)
    B.nanospec_vocab_update(st.h, dev(new), [0, 4], dev(np.array([2000, 6], np.int32)), [0, 2])
    o.update(new, [2000, 6])
    assert np.array_equal(st.read_active()[0], o.active())
    assert B.nanospec_last_device_error(st.h) == B.DEV_BAD_ID
    assert B.nanospec_last_device_error(st.h) == 0                  # reading clears the flags
    # re-init discards everything
    B.nanospec_vocab_init(st.h, dev(np.array([9, 9, 8], np.int32)), [0, 3], None, [0, 0])
    o.init([9, 9, 8], [])
    assert np.array_equal(st.read_active()[0], o.active())
    st.close()


@pytest.mark.parametrize("policy", [0, 1])
@pytest.mark.parametrize("V,W,distinct", [(60000, 20000, 13000), (5000, 4096, 5000), (300, 37, 300), (64, 64, 64)])
def test_short_appends_patch_the_list(V, W, distinct, policy):
    """Updates of at most 16 ids with T untouched take the list-patching route (both stream policies): ids below the first and
    above the last entry, ids that T holds, ids that leave and come back in one call, duplicates, ids out of
    range, lists of several passes, a list at its capacity (V = 64: the general route takes over) -- the
    active list equals the oracle's after every call, for three sequences with different streams."""
    Bn, tcap = 3, 64
    rng = np.random.default_rng(V + W)
    st = B.State(V, 64, Bn, W, tcap, 4, 8)
    B.nanospec_set_stream_policy(st.h, policy)
    orc = [oracle.FifoVocab(V, W) if policy else oracle.Vocab(V, W) for _ in range(Bn)]
    ctx = [rng.integers(V // 10, V // 10 + distinct * 8 // 10, size=W + 50).astype(np.int32) % V for _ in range(Bn)]
    T = [rng.integers(0, V, size=tcap).astype(np.int32) for _ in range(Bn)]
    f, off = csr(ctx)
    tf, toff = csr(T)
    B.nanospec_vocab_init(st.h, dev_ids(f), off, dev_ids(tf), toff)
    for b in range(Bn):
        orc[b].init(ctx[b], T[b])
    bad_expected = False
    for step in range(120):
        new = []
        for b in range(Bn):
            a = int(rng.integers(0, 17))
            kind = int(rng.integers(0, 6))
            if kind == 0:
                x = rng.integers(0, max(1, V // 10), size=a)              # below the context's range
            elif kind == 1:
                x = rng.integers(V - max(1, V // 20), V, size=a)          # above it
            elif kind == 2:
                x = rng.choice(T[b], size=a)                              # ids that T holds
            elif kind == 3:
                x = np.repeat(rng.integers(0, V, size=1), a)              # one id, many times
            elif kind == 4:
                x = orc[b].active()[:a] if len(orc[b].active()) else rng.integers(0, V, size=a)   # the lowest active ids
            else:
                x = rng.integers(0, V, size=a)
            x = np.asarray(x, np.int32).copy()
            if step % 37 == 5 and a:
                x[0] = V + 3                                              # out of range: flagged, holds a position
                bad_expected = True
            new.append(x)
        f, off = csr(new)
        B.nanospec_vocab_update(st.h, dev_ids(f), off)
        for b in range(Bn):
            orc[b].update(new[b], None)
        act = st.read_active()
        for b in range(Bn):
            assert np.array_equal(act[b], orc[b].active()), (step, b)
    assert (B.nanospec_last_device_error(st.h) == B.DEV_BAD_ID) == bad_expected
    # the general route afterwards sees a consistent state: a T replacement rebuilds the list from the bitmaps
    B.nanospec_vocab_update(st.h, None, [0] * (Bn + 1), dev_ids(tf), toff)
    for b in range(Bn):
        orc[b].update([], T[b])
    act = st.read_active()
    for b in range(Bn):
        assert np.array_equal(act[b], orc[b].active())
    st.close()


def test_vocab_fuzz_ragged_batch():
    rng = np.random.default_rng(5)
    V, W, Bn = 5000, 37, 7
    st = B.State(V, 64, Bn, W, 20, 2, 4)
    orc = [oracle.Vocab(V, W) for _ in range(Bn)]
    ctx = [rng.integers(0, 300, size=int(rng.integers(0, 120))).astype(np.int32) for _ in range(Bn)]
    T = [rng.integers(0, V, size=int(rng.integers(0, 21))).astype(np.int32) for _ in range(Bn)]
    f, off = csr(ctx)
    tf, toff = csr(T)
    B.nanospec_vocab_init(st.h, dev_ids(f), off, dev_ids(tf), toff)
    for b in range(Bn):
        orc[b].init(ctx[b], T[b])
    for step in range(60):
        new = [rng.integers(0, 300, size=int(rng.integers(0, 90 if step % 10 == 0 else 9))).astype(np.int32) for _ in range(Bn)]
        f, off = csr(new)
        if step % 3 == 0:
            T = [rng.integers(0, V, size=int(rng.integers(0, 21))).astype(np.int32) for _ in range(Bn)]
            tf, toff = csr(T)
            B.nanospec_vocab_update(st.h, dev_ids(f), off, dev_ids(tf), toff)
        else:
            B.nanospec_vocab_update(st.h, dev_ids(f), off)
        act = st.read_active()
        for b in range(Bn):
            orc[b].update(new[b], T[b] if step % 3 == 0 else None)
            assert np.array_equal(act[b], orc[b].active()), (step, b)
    st.close()


def test_head_and_topk_edge_cases():
    V, d, M = 1000, 64, 3
    W = synth.normal_bf16(77, 0, (V, d), 0.02, threads=1)
    W[10] = W[20]                                             # duplicate rows -> exact ties
    W[30] = W[20]
    H = synth.normal_bf16(77, 1, (M, d), 1.0, threads=1)
    dW, dH = dev_bf16(W), dev_bf16(H)
    st = B.State(V, d, 1, 16, 8, M, 64)
    cap = st.capacity
    logits = torch.full((1, M, cap), float("nan"), dtype=torch.float32, device="cuda")
    for k in (1, 5, 64):
        oi = torch.empty((1, M, k), dtype=torch.int32, device="cuda")
        ov = torch.empty((1, M, k), dtype=torch.float32, device="cuda")
        # n == 0: nothing active, all slots padded
        B.nanospec_vocab_init(st.h, None, [0, 0], None, [0, 0])
        B.nanospec_sparse_head(st.h, dW, dH, M, logits)
        B.nanospec_topk_remap(st.h, logits, M, k, oi, ov)
        torch.cuda.synchronize()
        assert (oi.cpu().numpy() == -1).all() and np.isneginf(ov.cpu().numpy()).all()
        # a handful of ids including the tied rows; k > n pads
        ctx = np.array([30, 20, 10, 500, 999, 0], np.int32)
        B.nanospec_vocab_init(st.h, dev(ctx), [0, len(ctx)], dev(np.array([7], np.int32)), [0, 1])
        B.nanospec_sparse_head(st.h, dW, dH, M, logits)
        B.nanospec_topk_remap(st.h, logits, M, k, oi, ov)
        torch.cuda.synchronize()
        act = st.read_active()[0]
        assert act.tolist() == [0, 7, 10, 20, 30, 500, 999]
        g = logits.cpu().numpy()[0]
        o32, o64 = oracle.head(W, H, ids=act)
        assert_logits_close(g[:, :7], o64, o32)
        assert np.array_equal(g[:, 2], g[:, 3]) and np.array_equal(g[:, 3], g[:, 4])   # duplicate rows: identical bits
        for m in range(M):
            ei, ev = oracle.topk(g[m, :7], act, k)
            assert np.array_equal(oi.cpu().numpy()[0, m], ei) and np.array_equal(ov.cpu().numpy()[0, m], ev)
    st.close()


@pytest.mark.parametrize("V", [4096, 7000, 12000])          # one per single-pass selection kernel
def test_topk_all_equal_and_signed_zero(V):
    d, M, k = 8, 2, 6
    st = B.State(V, d, 1, V, 0, M, 64)
    ctx = np.arange(0, V, 3 if V == 4096 else 1, dtype=np.int32)
    B.nanospec_vocab_init(st.h, dev(ctx), [0, len(ctx)], None, [0, 0])
    n, cap = len(ctx), st.capacity
    vals = np.zeros((1, M, cap), np.float32)
    vals[0, 0, :n] = 1.25                                     # all equal: the k lowest ids win
    vals[0, 1, :n] = np.where(np.arange(n) % 2 == 0, -0.0, 0.0)   # +0 and -0 tie
    lg = dev(vals)
    oi = torch.empty((1, M, k), dtype=torch.int32, device="cuda")
    B.nanospec_topk_remap(st.h, lg, M, k, oi, None)
    torch.cuda.synchronize()
    assert oi.cpu().numpy()[0, 0].tolist() == ctx[:k].tolist()
    assert oi.cpu().numpy()[0, 1].tolist() == ctx[:k].tolist()
    st.close()


@pytest.mark.parametrize("V,n_ctx", [(4096, 3017), (7000, 6500), (12000, 11111), (40000, 33000)])   # one per selection kernel + chunked
@pytest.mark.parametrize("k", [1, 10, 64])
def test_topk_winner_placement(V, n_ctx, k):
    """Winners crowded into one lane's run of 16 positions, exactly four / five of them in one run, a few
    dozen equal maxima spread over the row, winners only in the ragged last run, and a descending ramp:
    every route through the selection kernel gives the oracle's ids and values, with and without
    log-probabilities."""
    d, M = 8, 8
    st = B.State(V, d, 1, V, 0, M, 64)
    rng = np.random.default_rng(V + k)
    ctx = rng.choice(V, size=n_ctx, replace=False).astype(np.int32)
    B.nanospec_vocab_init(st.h, dev_ids(ctx), [0, n_ctx], None, [0, 0])
    act = st.read_active()[0]
    n, cap = len(act), st.capacity
    z = np.full((1, M, cap), np.nan, np.float32)
    base = rng.normal(size=(M, n)).astype(np.float32)
    at = 16 * (n // 32)                                           # start of a run somewhere in the middle
    base[0, at:at + 16] += 20.0 + rng.normal(size=16)             # 16 winners in one lane
    base[1, at + 3:at + 7] += 20.0                                # exactly four in one lane
    base[2, at + 3:at + 8] += 20.0                                # five in one lane
    base[3, rng.choice(n, size=40, replace=False)] = 9.0          # 40 equal maxima: ranked by position
    base[4, n - (n % 16 or 16):] += 30.0                          # winners in the ragged tail
    base[5] = np.linspace(5.0, -5.0, n, dtype=np.float32)         # descending ramp: the first k positions
    base[6] = np.linspace(-5.0, 5.0, n, dtype=np.float32)         # ascending ramp: the last k positions
    base[7, :] = np.float32(0.5)
    base[7, rng.choice(n, size=min(n, 300), replace=False)] = 0.75   # 300 equal maxima: more than the candidate list holds
    z[0, :, :n] = base
    lg = dev(z)
    oi = torch.empty((1, M, k), dtype=torch.int32, device="cuda")
    ov = torch.empty((1, M, k), dtype=torch.float32, device="cuda")
    ol = torch.empty((1, M, k), dtype=torch.float32, device="cuda")
    oi2 = torch.empty_like(oi)
    B.nanospec_topk_remap(st.h, lg, M, k, oi, ov)
    B.nanospec_topk_logprob_remap(st.h, lg, M, k, oi2, ol)
    torch.cuda.synchronize()
    gi, gv, gl = oi.cpu().numpy()[0], ov.cpu().numpy()[0], ol.cpu().numpy()[0]
    assert torch.equal(oi, oi2)
    for m in range(M):
        ei, ev = oracle.topk(z[0, m, :n], act, k)
        assert np.array_equal(gi[m], ei), f"row {m}"
        assert np.array_equal(gv[m], ev), f"row {m}"
        _, elp = oracle.topk_logprob(z[0, m, :n], act, k)
        assert np.all(np.abs(gl[m].astype(np.float64) - elp) <= 1e-4), f"row {m}"
    st.close()


def test_result_independent_of_position_and_run():
    """the logit of a (W row, H row) pair does not depend on where the row sits in the active list,
    and two runs give identical bits."""
    cfg = synth.CONFIGS["c1"]
    W = host_W(cfg)
    V, d, M = cfg["V"], cfg["d"], 4
    H = synth.make_H(cfg, 3, 1, M)[0]
    dW, dH = dev_bf16(W), dev_bf16(H)
    st = B.State(V, d, 1, 512, 0, M, 8)
    cap = st.capacity
    res = []
    for ctx in (np.arange(100, 400, dtype=np.int32), np.arange(0, 400, dtype=np.int32), np.arange(100, 400, dtype=np.int32)):
        B.nanospec_vocab_init(st.h, dev(ctx), [0, len(ctx)], None, [0, 0])
        lg = torch.empty((1, M, cap), dtype=torch.float32, device="cuda")
        B.nanospec_sparse_head(st.h, dW, dH, M, lg)
        torch.cuda.synchronize()
        res.append(lg.cpu().numpy()[0])
    assert np.array_equal(res[0][:, :300], res[2][:, :300])
    assert np.array_equal(res[0][:, :300], res[1][:, 100:400])
    st.close()


def test_argument_errors():
    L = B.lib()
    st = _small_state()
    import ctypes as C
    assert L.nanospec_create(None, 10, 8, 1, 1, 0, 1, 1) == B.EINVAL
    h = C.c_void_p()
    assert L.nanospec_create(C.byref(h), 10, 12, 1, 1, 0, 1, 1) == B.EINVAL        # d % 8 != 0
    assert L.nanospec_create(C.byref(h), 10, 8, 1, 1, 0, 1, 65) == B.EINVAL        # k_cap > 64
    assert L.nanospec_create(C.byref(h), 10, 8, 257, 1, 0, 1, 1) == B.EINVAL       # batch > max
    off_bad = (C.c_int32 * 2)(3, 1)
    off_ok = (C.c_int32 * 2)(0, 5)
    assert L.nanospec_vocab_update(st.h, None, off_bad, None, None, None) == B.EINVAL
    assert L.nanospec_vocab_update(st.h, None, off_ok, None, None, None) == B.EINVAL     # ids missing
    assert L.nanospec_vocab_init(st.h, None, None, None, None, None) == B.EINVAL
    buf = torch.zeros(64, dtype=torch.int32, device="cuda")
    assert L.nanospec_vocab_update(st.h, None, None, buf.data_ptr(), off_ok, None) == B.ECAPACITY  # |T| > topk_cap
    assert L.nanospec_sparse_head(st.h, buf.data_ptr(), buf.data_ptr(), 4, buf.data_ptr(), None) == B.ECAPACITY
    assert L.nanospec_sparse_head(st.h, None, buf.data_ptr(), 1, buf.data_ptr(), None) == B.EINVAL
    assert L.nanospec_topk_remap(st.h, buf.data_ptr(), 1, 65, buf.data_ptr(), None, None) == B.ECAPACITY
    assert L.nanospec_topk_logprob_remap(st.h, buf.data_ptr(), 1, 1, buf.data_ptr(), None, None) == B.EINVAL   # values required
    assert L.nanospec_topk_logprob_remap(st.h, buf.data_ptr(), 4, 1, buf.data_ptr(), buf.data_ptr(), None) == B.ECAPACITY
    assert L.nanospec_dense_head(buf.data_ptr(), buf.data_ptr(), 10, 12, 1, buf.data_ptr(), None) == B.EINVAL
    assert L.nanospec_calib_stream_read(buf.data_ptr(), 24, buf.data_ptr(), None) == B.EINVAL          # not a multiple of 16
    assert L.nanospec_calib_gather_read(st.h, None, buf.data_ptr(), None) == B.EINVAL
    assert L.nanospec_dense_topk(buf.data_ptr(), 100000, 1, 4, buf.data_ptr(), None, buf.data_ptr(), 8, None) == B.ECAPACITY
    torch.cuda.synchronize()
    assert np.array_equal(st.read_active()[0], np.zeros(0, np.int32))               # nothing was enqueued
    st.close()


def test_step_recorded_in_hip_graph_replays_correctly():
    """the three hot calls enqueue kernels only (no sync, no allocation, no memset node): a step captured
    in a HIP graph and replayed several times, with eager work and synchronisations in between, gives the
    oracle's vocabulary and the eager path's bits on every replay."""
    cfg = synth.CONFIGS["c1"]
    W = host_W(cfg)
    V, d, M, k = cfg["V"], cfg["d"], cfg["M"], cfg["k"]
    dW = dev_bf16(W)
    dH = dev_bf16(synth.make_H(cfg, 5, 1, M)[0])
    seqs = synth.make_sequences(cfg)
    st = B.State(V, d, 1, seqs["window"], seqs["topk_cap"], M, k)
    o = oracle.Vocab(V, seqs["window"])
    ctx, T0 = seqs["ctx"][0], seqs["T0"][0]
    B.nanospec_vocab_init(st.h, dev(ctx), [0, len(ctx)], dev(T0), [0, len(T0)])
    o.init(ctx, T0)
    new = np.array([17, 4242, 17, 31999, 5], np.int32)
    d_new = dev(new)
    cap = st.capacity
    lg_g = torch.empty((1, M, cap), dtype=torch.float32, device="cuda")
    lg_e = torch.empty((1, M, cap), dtype=torch.float32, device="cuda")
    oi_g = torch.empty((1, M, k), dtype=torch.int32, device="cuda")
    ov_g = torch.empty((1, M, k), dtype=torch.float32, device="cuda")
    oi_e, ov_e = torch.empty_like(oi_g), torch.empty_like(ov_g)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cs = torch.cuda.current_stream().cuda_stream
        B.nanospec_vocab_update(st.h, d_new, [0, len(new)], None, None, cs)
        B.nanospec_sparse_head(st.h, dW, dH, M, lg_g, cs)
        B.nanospec_topk_remap(st.h, lg_g, M, k, oi_g, ov_g, cs)
    torch.cuda.synchronize()
    assert np.array_equal(st.read_active()[0], o.active())            # capture itself ran nothing
    for rep in range(4):
        g.replay()
        torch.cuda.synchronize()
        o.update(new)
        act = st.read_active()[0]
        assert np.array_equal(act, o.active()), rep
        B.nanospec_sparse_head(st.h, dW, dH, M, lg_e)                  # eager work between replays
        B.nanospec_topk_remap(st.h, lg_e, M, k, oi_e, ov_e)
        torch.cuda.synchronize()
        n = len(act)
        assert np.array_equal(lg_g.cpu().numpy()[0, :, :n], lg_e.cpu().numpy()[0, :, :n]), rep
        assert np.array_equal(oi_g.cpu().numpy(), oi_e.cpu().numpy()) and np.array_equal(ov_g.cpu().numpy(), ov_e.cpu().numpy())
        o32, o64 = oracle.head(W, synth.make_H(cfg, 5, 1, M)[0], ids=act)
        assert_logits_close(lg_g.cpu().numpy()[0, :, :n], o64, o32, f"replay {rep}")
        extra = np.array([rep, 100 + rep], np.int32)                   # eager update between replays
        B.nanospec_vocab_update(st.h, dev(extra), [0, 2])
        o.update(extra)
    st.close()


@pytest.mark.parametrize("d,M,n_ctx,batch", [
    (520, 1, 37, 1), (520, 3, 300, 2), (1032, 5, 1500, 1), (3592, 8, 3001, 1), (4096, 9, 777, 1), (1032, 13, 2900, 3),
    (520, 16, 9000, 1), (1032, 17, 1000, 1), (3592, 33, 1234, 1), (1032, 64, 17000, 1), (520, 70, 500, 1), (520, 70, 200, 2),
    (4096, 16, 3000, 1), (3592, 12, 1500, 1), (8200, 16, 2000, 1), (8200, 8, 9000, 1), (1032, 8, 3100, 3), (4104, 6, 200, 1),
    # the variants without bounds tests (d a whole number of K-iterations / slices), with hidden rows that fill the
    # last tile and with hidden rows that do not; the last sequence's hidden rows end the H buffer
    (8192, 32, 70, 2), (1024, 17, 1000, 1), (2048, 48, 300, 2), (1024, 64, 2000, 1), (512, 64, 17000, 1), (512, 40, 17000, 1),
    (8192, 12, 1300, 1), (8192, 10, 500, 2), (6144, 16, 9000, 1), (4096, 3, 100, 1),
    # the register-blocked product on a gathered list (at least 16384 rows of capacity, d a multiple of 128): both block shapes
    (512, 70, 17000, 1), (1024, 130, 16500, 1), (128, 17, 19999, 1), (384, 64, 16400, 1),
    # ... and its 32 x 32 shape on a few thousand rows (d a multiple of 512; from 2560 rows of capacity, 4096 up to 32 hidden rows)
    (512, 64, 3000, 1), (1024, 40, 4000, 1), (512, 24, 5000, 1), (3584, 64, 2600, 1), (1024, 33, 2561, 1), (512, 17, 9000, 1),
])
def test_head_shapes_against_oracle(d, M, n_ctx, batch):
    """every head kernel and its ragged tails: row counts that are not multiples of the tile, hidden sizes that
    are not multiples of a K slice, hidden-row counts on both sides of each kernel boundary, several sequences."""
    V = 20000
    W = synth.normal_bf16(900 + d, 0, (V, d), 0.02)
    H = synth.normal_bf16(901 + d, M, (batch, M, d), 1.0, threads=1)
    dW, dH = dev_bf16(W), dev_bf16(H)
    st = B.State(V, d, batch, n_ctx, 0, M, 4)
    rng = np.random.default_rng(d * 1000 + M)
    ctx = [rng.choice(V, size=n_ctx - 3 * b, replace=False).astype(np.int32) for b in range(batch)]
    flat, off = csr(ctx)
    B.nanospec_vocab_init(st.h, dev(flat), off, None, np.zeros(batch + 1, np.int32))
    cap = st.capacity
    logits = torch.full((batch, M, cap), float("nan"), dtype=torch.float32, device="cuda")
    B.nanospec_sparse_head(st.h, dW, dH, M, logits)
    torch.cuda.synchronize()
    act = st.read_active()
    g = logits.cpu().numpy()
    for b in range(batch):
        assert np.array_equal(act[b], np.sort(ctx[b]))
        n = len(act[b])
        o32, o64 = oracle.head(W, H[b], ids=act[b], omp=True)
        assert_logits_close(g[b, :, :n], o64, o32, f"d={d} M={M} seq {b}")
    st.close()


def test_device_side_feedback_loop():
    """Eq. 3 closed on the device: the top-k ids of every draft node go straight from nanospec_topk_remap's
    output into the stream (de-duplicated, ascending) with no host integers; recorded once as a HIP graph and
    replayed.  Checked every step: the active set against the oracle fed with the GPU's own top-k ids, and the
    top-k ids against the oracle's selection on the GPU's logits."""
    cfg = synth.CONFIGS["c1"]
    W = host_W(cfg)
    V, d, M, k = cfg["V"], cfg["d"], cfg["M"], cfg["k"]
    dW = dev_bf16(W)
    seqs = synth.make_sequences(cfg)
    for batch, window in ((1, 64), (3, 300)):
        st = B.State(V, d, batch, window, seqs["topk_cap"], M, k)
        orc = [oracle.Vocab(V, window) for _ in range(batch)]
        ctx = [seqs["ctx"][0][37 * b: 37 * b + 200] for b in range(batch)]
        T0 = [seqs["T0"][0][: 100 + 50 * b] for b in range(batch)]
        f, off = csr(ctx)
        tf, toff = csr(T0)
        B.nanospec_vocab_init(st.h, dev(f), off, dev(tf), toff)
        for b in range(batch):
            orc[b].init(ctx[b], T0[b])
        cap = st.capacity
        H = synth.make_H(cfg, 11, batch, M)
        dH = dev_bf16(H)
        logits = torch.empty((batch, M, cap), dtype=torch.float32, device="cuda")
        oi = torch.full((batch, M, k), -1, dtype=torch.int32, device="cuda")
        ov = torch.empty((batch, M, k), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            cs = torch.cuda.current_stream().cuda_stream
            B.nanospec_vocab_append_unique(st.h, oi, M * k, M * k, cs)       # ids of the previous step
            B.nanospec_sparse_head(st.h, dW, dH, M, logits, cs)
            B.nanospec_topk_remap(st.h, logits, M, k, oi, ov, cs)
        prev = oi.cpu().numpy().copy()                                       # all -1: nothing appended in step 0
        for step in range(12):
            g.replay()
            torch.cuda.synchronize()
            act = st.read_active()
            gl, gi = logits.cpu().numpy(), oi.cpu().numpy()
            for b in range(batch):
                orc[b].append_unique(prev[b])
                exp = orc[b].active()
                assert np.array_equal(act[b], exp), (batch, step, b)
                for m in range(M):
                    ei, _ = oracle.topk(gl[b, m, :len(exp)], exp, k)
                    assert np.array_equal(gi[b, m], ei), (batch, step, b, m)
            prev = gi.copy()
            if step == 5:                                                     # eager call between replays: bad ids
                junk = dev(np.array([[V, -1, -7, 5] + [-1] * (M * k - 4)] * batch, np.int32))
                B.nanospec_vocab_append_unique(st.h, junk, M * k, M * k)
                for b in range(batch):
                    orc[b].append_unique([5])
                assert B.nanospec_last_device_error(st.h) == B.DEV_BAD_ID
        assert B.nanospec_last_device_error(st.h) == 0
        import ctypes as C
        assert B.lib().nanospec_vocab_append_unique(st.h, oi.data_ptr(), 41000, 41000, None) == B.ECAPACITY   # beyond the LDS bound
        assert B.lib().nanospec_vocab_append_unique(st.h, None, 4, 4, None) == B.EINVAL
        assert B.lib().nanospec_vocab_append_unique(st.h, oi.data_ptr(), 4, 2, None) == B.EINVAL
        st.close()


@pytest.mark.parametrize("window,n_ctx", [(64, 0), (64, 7), (3500, 3000), (6000, 5000), (12000, 9000), (40000, 33000), (40000, 9000),
                                          (40000, 0)])
def test_topk_logprob_against_oracle(window, n_ctx):
    """Selection with log-probabilities renormalised over the active set (Sec. 4.2): ids bit-exact against
    the oracle's selection; values within 1e-4 of the fp64 log-softmax (fp32 exp and a sum of at most 4e4
    positive terms: relative error of the sum below 1e-5, so below 1e-5 absolute in its logarithm; the
    final subtraction rounds at 1e-6 for |z - lse| < 16)."""
    V, d, M, k = 50000, 8, 4, 10
    st = B.State(V, d, 1, window, 0, M, 64)
    rng = np.random.default_rng(window + n_ctx)
    ctx = rng.choice(V, size=n_ctx, replace=False).astype(np.int32)
    B.nanospec_vocab_init(st.h, dev_ids(ctx), [0, n_ctx], None, [0, 0])
    act = st.read_active()[0]
    n, cap = len(act), st.capacity
    assert n == n_ctx
    z = np.full((1, M, cap), np.nan, np.float32)
    z[0, 0, :n] = rng.normal(size=n) * 3.0
    z[0, 1, :n] = np.round(rng.normal(size=n) * 2.0) / 2.0         # many ties
    z[0, 2, :n] = -7.5                                            # all equal: the general path, logp = -log n
    z[0, 3, :n] = rng.normal(size=n) * 0.01 + 80.0                # large offset: the maximum must be subtracted
    lg = dev(z)
    oi = torch.empty((1, M, k), dtype=torch.int32, device="cuda")
    ov = torch.empty((1, M, k), dtype=torch.float32, device="cuda")
    B.nanospec_topk_logprob_remap(st.h, lg, M, k, oi, ov)
    torch.cuda.synchronize()
    gi, gv = oi.cpu().numpy()[0], ov.cpu().numpy()[0]
    for m in range(M):
        ei, elp = oracle.topk_logprob(z[0, m, :n], act, k)
        assert np.array_equal(gi[m], ei), f"row {m}"
        fin = np.isfinite(elp)
        assert np.array_equal(np.isneginf(gv[m]), ~fin)
        assert np.all(np.abs(gv[m][fin].astype(np.float64) - elp[fin]) <= 1e-4), f"row {m}"
    if n:
        assert abs(float(gv[2, 0]) + np.log(n)) <= 1e-4
    # plain selection on the same logits: same ids; and a second run gives the same bits
    oi2 = torch.empty_like(oi)
    ov2 = torch.empty_like(ov)
    B.nanospec_topk_remap(st.h, lg, M, k, oi2, None)
    assert torch.equal(oi, oi2)
    B.nanospec_topk_logprob_remap(st.h, lg, M, k, oi2, ov2)
    torch.cuda.synchronize()
    assert torch.equal(oi, oi2) and torch.equal(ov.view(torch.int32), ov2.view(torch.int32))
    st.close()


@pytest.mark.parametrize("window", [64, 700, 4096])
def test_prefill_stream_initialisation_on_device(window):
    """Eq. 2 composed on the device: S(0) = prompt, then the de-duplicated union of the top-K_pre ids of every
    prompt position.  The prefill logits are synthetic (the target model is outside the path); the top-K_pre
    ids come from nanospec_dense_topk over the L x V matrix and go into the stream without a host copy.
    Windows shorter than the appended union exercise ids that enter and leave within one call."""
    V, d, L, Kpre = 32000, 8, 300, 3
    rng = np.random.default_rng(window)
    zipf = synth.ZipfVocab(V, 1.1, seed=5)
    prompt = zipf.tokens(6, 0, L).astype(np.int32)
    Z = rng.normal(size=(L, V)).astype(np.float32)
    hot = zipf.tokens(7, 0, 40).astype(np.int64)                    # a few tokens are likely at many positions
    Z[:, hot] += rng.normal(size=(L, len(hot))).astype(np.float32) * 2.0 + 2.0
    dZ = dev(Z)
    ws_bytes = B.nanospec_dense_topk_workspace(V, L, Kpre)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    pre_ids = torch.empty((L, Kpre), dtype=torch.int32, device="cuda")
    B.nanospec_dense_topk(dZ, V, L, Kpre, pre_ids, None, ws, ws_bytes)
    st = B.State(V, d, 1, window, 16, 4, 8)
    T = np.array([3, 31999, 17], np.int32)
    B.nanospec_vocab_init(st.h, dev(prompt), [0, L], dev(T), [0, len(T)])
    B.nanospec_vocab_append_unique(st.h, pre_ids, L * Kpre, L * Kpre)
    torch.cuda.synchronize()
    gi = pre_ids.cpu().numpy()
    allids = np.arange(V, dtype=np.int32)
    union = set()
    for i in range(L):
        ei, _ = oracle.topk(Z[i], allids, Kpre)
        assert np.array_equal(gi[i], ei), i
        union.update(int(x) for x in ei)
    assert len(union) < L * Kpre                                    # the synthetic logits do produce repeats
    orc = oracle.Vocab(V, window)
    orc.init(prompt, T)
    orc.append_unique(np.array(sorted(union), np.int32)[::-1])      # any order: the oracle takes the set
    assert np.array_equal(st.read_active()[0], orc.active())
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()


@pytest.mark.parametrize("d,M,n_ctx", [(4096, 8, 3001), (4096, 5, 777), (2048, 8, 1500), (2048, 1, 40)])
def test_vector_alu_head_against_oracle(d, M, n_ctx):
    """the measurement-aid form of the head on the vector ALUs computes Eq. 1 on the active rows too"""
    V = 20000
    W = synth.normal_bf16(990 + d, 0, (V, d), 0.02)
    H = synth.normal_bf16(991 + d, M, (1, M, d), 1.0, threads=1)
    st = B.State(V, d, 1, n_ctx, 0, 8, 4)
    rng = np.random.default_rng(d + M)
    ctx = rng.choice(V, size=n_ctx, replace=False).astype(np.int32)
    B.nanospec_vocab_init(st.h, dev(ctx), [0, n_ctx], None, [0, 0])
    logits = torch.full((1, M, st.capacity), float("nan"), dtype=torch.float32, device="cuda")
    B.nanospec_calib_valu_head(st.h, dev_bf16(W), dev_bf16(H), M, logits)
    torch.cuda.synchronize()
    act = st.read_active()[0]
    o32, o64 = oracle.head(W, H[0], ids=act, omp=True)
    assert_logits_close(logits.cpu().numpy()[0, :, :len(act)], o64, o32, f"vector-ALU head d={d} M={M}")
    st.close()


def test_calibration_reads_run_and_touch_nothing():
    """the measurement aids only read: they return OK, leave the state and their inputs unchanged."""
    V, d = 2000, 512
    W = synth.normal_bf16(5, 0, (V, d), 0.02, threads=1)
    dW = dev_bf16(W)
    st = B.State(V, d, 1, 300, 0, 1, 1)
    ctx = np.arange(0, 1800, 7, dtype=np.int32)
    B.nanospec_vocab_init(st.h, dev(ctx), [0, len(ctx)], None, [0, 0])
    before = st.read_active()[0].copy()
    sink = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    B.nanospec_calib_gather_read(st.h, dW, sink)
    B.nanospec_calib_stream_read(dW, V * d * 2, sink)
    B.nanospec_calib_stream_read(dW, 16, sink)
    torch.cuda.synchronize()
    assert np.array_equal(st.read_active()[0], before)
    assert np.array_equal(dW.view(torch.int16).cpu().numpy().view(np.uint16), W)
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()


# ---- second reading of the vocabulary: first-in first-out queue of distinct ids (NANOSPEC_POLICY_FIFO)

def test_fifo_policy_worked_and_edge_cases():
    V = 1000
    st = B.State(V, 64, 1, 4, 4, 2, 4)
    B.nanospec_set_stream_policy(st.h, B.POLICY_FIFO)
    orc = oracle.FifoVocab(V, 4)
    B.nanospec_vocab_init(st.h, dev(np.array([5, 6, 5, 7], np.int32)), [0, 4], dev(np.array([90], np.int32)), [0, 1])
    orc.init([5, 6, 5, 7], [90])
    assert st.read_active()[0].tolist() == [5, 6, 7, 90]
    for new in ([6, 8, 9], [5], [], [5, 5, 5], [1, 2, 3, 4, 10, 11], [999, 1000, -1, 0]):
        B.nanospec_vocab_update(st.h, dev_ids(np.array(new, np.int32)), [0, len(new)])
        orc.update(new)
        assert np.array_equal(st.read_active()[0], orc.active()), new
    assert B.nanospec_last_device_error(st.h) == B.DEV_BAD_ID       # 1000 and -1 were skipped and flagged
    assert st.read_active()[0].tolist() == [0, 10, 11, 90, 999]
    # switching back takes effect at the next init
    B.nanospec_set_stream_policy(st.h, B.POLICY_WINDOW)
    B.nanospec_vocab_init(st.h, dev(np.array([1, 4, 4, 4, 4, 4], np.int32)), [0, 6], None, [0, 0])
    assert st.read_active()[0].tolist() == [4]                      # raw-stream window of 4: (4 4 4 4)
    B.nanospec_set_stream_policy(st.h, B.POLICY_FIFO)
    B.nanospec_vocab_init(st.h, dev(np.array([1, 4, 4, 4, 4, 4], np.int32)), [0, 6], None, [0, 0])
    assert st.read_active()[0].tolist() == [1, 4]
    assert B.lib().nanospec_set_stream_policy(st.h, 7) == B.EINVAL
    st.close()


@pytest.mark.parametrize("W,vals,big", [(37, 300, 90), (3000, 6000, 5000), (64, 100000, 2500)])
def test_fifo_policy_fuzz_ragged_batch(W, vals, big):
    """windows smaller and larger than one workgroup's chunk, appends longer than the queue and longer than a
    chunk (several passes, wrap of the staging list), T replaced every third step."""
    rng = np.random.default_rng(W)
    V, Bn = 100000, 5
    st = B.State(V, 64, Bn, W, 20, 2, 4)
    B.nanospec_set_stream_policy(st.h, B.POLICY_FIFO)
    orc = [oracle.FifoVocab(V, W) for _ in range(Bn)]
    ctx = [rng.integers(0, vals, size=int(rng.integers(0, big))).astype(np.int32) for _ in range(Bn)]
    T = [rng.integers(0, V, size=int(rng.integers(0, 21))).astype(np.int32) for _ in range(Bn)]
    f, off = csr(ctx)
    tf, toff = csr(T)
    B.nanospec_vocab_init(st.h, dev_ids(f), off, dev_ids(tf), toff)
    for b in range(Bn):
        orc[b].init(ctx[b], T[b])
    act = st.read_active()
    for b in range(Bn):
        assert np.array_equal(act[b], orc[b].active()), ("init", b)
    for step in range(40):
        new = [rng.integers(0, vals, size=int(rng.integers(0, big if step % 10 == 0 else 9))).astype(np.int32) for _ in range(Bn)]
        f, off = csr(new)
        if step % 3 == 0:
            T = [rng.integers(0, V, size=int(rng.integers(0, 21))).astype(np.int32) for _ in range(Bn)]
            tf, toff = csr(T)
            B.nanospec_vocab_update(st.h, dev_ids(f), off, dev_ids(tf), toff)
        else:
            B.nanospec_vocab_update(st.h, dev_ids(f), off)
        act = st.read_active()
        for b in range(Bn):
            orc[b].update(new[b], T[b] if step % 3 == 0 else None)
            assert np.array_equal(act[b], orc[b].active()), (step, b)
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()


def test_fifo_policy_device_side_feedback():
    """append_unique under the queue reading: a candidate set is one batch of its distinct valid ids, ascending."""
    rng = np.random.default_rng(77)
    V, W, Bn, per = 3000, 50, 3, 24
    st = B.State(V, 64, Bn, W, 0, 4, 6)
    B.nanospec_set_stream_policy(st.h, B.POLICY_FIFO)
    orc = [oracle.FifoVocab(V, W) for _ in range(Bn)]
    ctx = [rng.integers(0, 200, size=30).astype(np.int32) for _ in range(Bn)]
    f, off = csr(ctx)
    B.nanospec_vocab_init(st.h, dev(f), off, None, np.zeros(Bn + 1, np.int32))
    for b in range(Bn):
        orc[b].init(ctx[b])
    for step in range(30):
        cand = rng.integers(-1, 260, size=(Bn, per)).astype(np.int32)      # -1 = padding
        B.nanospec_vocab_append_unique(st.h, dev(cand), per, per)
        act = st.read_active()
        for b in range(Bn):
            orc[b].append_unique(cand[b])
            assert np.array_equal(act[b], orc[b].active()), (step, b)
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()


@pytest.mark.parametrize("policy", [0, 1])
def test_limits_odd_vocabulary_full_membership_and_widest_k(policy):
    """V not a multiple of 32, window larger than V (capacity clamps to V), every id active, k = 64, d = 8."""
    V, d, M, k = 1001, 8, 3, 64
    W = synth.normal_bf16(31, 0, (V, d), 0.02, threads=1)
    H = synth.normal_bf16(31, 1, (M, d), 1.0, threads=1)
    st = B.State(V, d, 1, 5000, 0, M, k)
    B.nanospec_set_stream_policy(st.h, policy)
    assert st.capacity == 1024
    rng = np.random.default_rng(policy)
    ctx = np.concatenate([rng.permutation(V), rng.integers(0, V, size=700)]).astype(np.int32)
    B.nanospec_vocab_init(st.h, dev(ctx), [0, len(ctx)], None, [0, 0])
    act = st.read_active()[0]
    assert np.array_equal(act, np.arange(V, dtype=np.int32))
    logits = torch.empty((1, M, st.capacity), dtype=torch.float32, device="cuda")
    oi = torch.empty((1, M, k), dtype=torch.int32, device="cuda")
    ov = torch.empty((1, M, k), dtype=torch.float32, device="cuda")
    B.nanospec_sparse_head(st.h, dev_bf16(W), dev_bf16(H), M, logits)
    B.nanospec_topk_remap(st.h, logits, M, k, oi, ov)
    torch.cuda.synchronize()
    g = logits.cpu().numpy()[0]
    o32, o64 = oracle.head(W, H, ids=act)
    assert_logits_close(g[:, :V], o64, o32)
    for m in range(M):
        ei, ev = oracle.topk(g[m, :V], act, k)
        assert np.array_equal(oi.cpu().numpy()[0, m], ei) and np.array_equal(ov.cpu().numpy()[0, m], ev)
    st.close()


def test_limits_largest_batch():
    """NANOSPEC_MAX_BATCH sequences in one state: ragged contexts, one update, head and selection for all."""
    V, d, M, k, Bn, Wn = 3000, 64, 2, 5, 256, 20
    W = synth.normal_bf16(41, 0, (V, d), 0.02, threads=1)
    H = synth.normal_bf16(41, 1, (Bn, M, d), 1.0, threads=1)
    st = B.State(V, d, Bn, Wn, 3, M, k)
    rng = np.random.default_rng(41)
    ctx = [rng.integers(0, V, size=int(rng.integers(0, 40))).astype(np.int32) for _ in range(Bn)]
    T = [rng.integers(0, V, size=int(rng.integers(0, 4))).astype(np.int32) for _ in range(Bn)]
    new = [rng.integers(0, V, size=int(rng.integers(0, 6))).astype(np.int32) for _ in range(Bn)]
    f, off = csr(ctx)
    tf, toff = csr(T)
    nf, noff = csr(new)
    B.nanospec_vocab_init(st.h, dev_ids(f), off, dev_ids(tf), toff)
    B.nanospec_vocab_update(st.h, dev_ids(nf), noff)
    logits = torch.empty((Bn, M, st.capacity), dtype=torch.float32, device="cuda")
    oi = torch.empty((Bn, M, k), dtype=torch.int32, device="cuda")
    B.nanospec_sparse_head(st.h, dev_bf16(W), dev_bf16(H), M, logits)
    B.nanospec_topk_remap(st.h, logits, M, k, oi, None)
    torch.cuda.synchronize()
    act = st.read_active()
    g, gi = logits.cpu().numpy(), oi.cpu().numpy()
    for b in range(Bn):
        o = oracle.Vocab(V, Wn)
        o.init(ctx[b], T[b])
        o.update(new[b])
        exp = o.active()
        assert np.array_equal(act[b], exp), b
        if len(exp):
            o32, o64 = oracle.head(W, H[b], ids=exp)
            assert_logits_close(g[b][:, :len(exp)], o64, o32, what=f"seq {b}")
        for m in range(M):
            ei, _ = oracle.topk(g[b, m, :len(exp)], exp, k)
            assert np.array_equal(gi[b, m], ei), (b, m)
    st.close()


# ---- randomised sweeps (fixed seeds): many small states / shapes that no hand-written case names

def test_randomised_vocabulary_calls():
    """200 random states: both policies, V 200..200k, window 1..5000, mixed update / T replacement / append_unique,
    appends up to twice the window plus a chunk; the active set is compared after every call."""
    for seed in range(200):
        rng = np.random.default_rng(1000 + seed)
        V = int(rng.choice([200, 5000, 70000, 140000, 200000]))
        W = int(rng.choice([1, 3, 37, 300, 1024, 2500, 5000]))
        Bn = int(rng.choice([1, 2, 5, 9]))
        tcap = int(rng.choice([0, 5, 64]))
        pol = int(rng.integers(0, 2))
        vals = int(rng.choice([min(V, 50), min(V, 400), V]))
        st = B.State(V, 64, Bn, W, tcap, 4, 8)
        B.nanospec_set_stream_policy(st.h, pol)
        orc = [oracle.FifoVocab(V, W) if pol else oracle.Vocab(V, W) for _ in range(Bn)]
        ctx = [rng.integers(0, vals, size=int(rng.integers(0, 3 * W + 50))).astype(np.int32) for _ in range(Bn)]
        T = [rng.integers(0, V, size=int(rng.integers(0, tcap + 1))).astype(np.int32) for _ in range(Bn)]
        f, off = csr(ctx)
        tf, toff = csr(T)
        B.nanospec_vocab_init(st.h, dev_ids(f), off, dev_ids(tf), toff)
        for b in range(Bn):
            orc[b].init(ctx[b], T[b])
        for step in range(12):
            kind = int(rng.integers(0, 4))
            if kind == 3:
                per = int(rng.integers(1, 40))
                cand = rng.integers(-1, vals, size=(Bn, per)).astype(np.int32)
                B.nanospec_vocab_append_unique(st.h, dev(cand), per, per)
                for b in range(Bn):
                    orc[b].append_unique(cand[b])
            else:
                big = step % 9 == 0
                new = [rng.integers(0, vals, size=int(rng.integers(0, (2 * W + 1100) if big else 9))).astype(np.int32)
                       for _ in range(Bn)]
                f, off = csr(new)
                if kind == 2:
                    T = [rng.integers(0, V, size=int(rng.integers(0, tcap + 1))).astype(np.int32) for _ in range(Bn)]
                    tf, toff = csr(T)
                    B.nanospec_vocab_update(st.h, dev_ids(f), off, dev_ids(tf), toff)
                else:
                    B.nanospec_vocab_update(st.h, dev_ids(f), off)
                for b in range(Bn):
                    orc[b].update(new[b], T[b] if kind == 2 else None)
            act = st.read_active()
            for b in range(Bn):
                assert np.array_equal(act[b], orc[b].active()), (seed, step, b, V, W, pol)
        st.close()


def test_randomised_head_shapes():
    """40 random (d, M, rows, sequences, k): logits within tolerance, plain and log-probability selection exact on
    the GPU's own logits."""
    for case in range(40):
        rng = np.random.default_rng(5000 + case)
        d = int(rng.choice([8, 64, 520, 1032, 2048, 3592, 4096, 4104, 8192]))
        M = int(rng.choice([1, 2, 4, 5, 8, 9, 12, 16, 17, 32, 33, 64, 65, 70]))
        batch = int(rng.choice([1, 1, 1, 2, 3]))
        nmax = int(rng.choice([5, 70, 700, 3000]))
        V = max(nmax + 10, int(rng.choice([1000, 20000])))
        k = int(rng.choice([1, 5, 10, 64]))
        W = synth.normal_bf16(7000 + case, 0, (V, d), 0.02, threads=4)
        H = synth.normal_bf16(7000 + case, 1, (batch, M, d), 1.0, threads=1)
        st = B.State(V, d, batch, nmax, 0, M, k)
        ctx = [rng.choice(V, size=int(rng.integers(0, nmax + 1)), replace=False).astype(np.int32) for _ in range(batch)]
        f, off = csr(ctx)
        B.nanospec_vocab_init(st.h, dev_ids(f), off, None, np.zeros(batch + 1, np.int32))
        logits = torch.full((batch, M, st.capacity), float("nan"), dtype=torch.float32, device="cuda")
        oi = torch.empty((batch, M, k), dtype=torch.int32, device="cuda")
        ov = torch.empty((batch, M, k), dtype=torch.float32, device="cuda")
        li, lv = torch.empty_like(oi), torch.empty_like(ov)
        B.nanospec_sparse_head(st.h, dev_bf16(W), dev_bf16(H), M, logits)
        B.nanospec_topk_remap(st.h, logits, M, k, oi, ov)
        B.nanospec_topk_logprob_remap(st.h, logits, M, k, li, lv)
        torch.cuda.synchronize()
        act, g = st.read_active(), logits.cpu().numpy()
        gi, gv, gli, glv = oi.cpu().numpy(), ov.cpu().numpy(), li.cpu().numpy(), lv.cpu().numpy()
        for b in range(batch):
            a = act[b]
            n = len(a)
            assert np.array_equal(a, np.sort(ctx[b])), case
            if n:
                o32, o64 = oracle.head(W, H[b], ids=a, omp=True)
                assert_logits_close(g[b][:, :n], o64, o32, what=f"case {case} (d={d} M={M} n={n}) seq {b}")
            for m in range(M):
                ei, ev = oracle.topk(g[b, m, :n], a, k)
                assert np.array_equal(gi[b, m], ei) and np.array_equal(gv[b, m], ev), (case, b, m)
                _, elp = oracle.topk_logprob(g[b, m, :n], a, k)
                fin = np.isfinite(elp)
                assert np.array_equal(gli[b, m], ei), (case, b, m)
                assert np.all(np.abs(glv[b, m][fin].astype(np.float64) - elp[fin]) <= 1e-4), (case, b, m)
        st.close()


@pytest.mark.parametrize("cap,M,d", [(3000, 64, 512), (5000, 24, 1024), (17000, 64, 256), (17000, 130, 128)])
def test_wide_tree_head_on_nearly_empty_lists(cap, M, d):
    """the register-blocked shapes are chosen by the capacity; the list may hold no row, one row, or one row more than a block"""
    V = 20000
    W = synth.normal_bf16(7700 + d, 0, (V, d), 0.02)
    H = synth.normal_bf16(7701 + d, M, (1, M, d), 1.0, threads=1)
    dW, dH = dev_bf16(W), dev_bf16(H)
    for n in (0, 1, 33, 257):
        st = B.State(V, d, 1, cap, 0, M, 4)
        ids = np.sort(np.random.default_rng(n + d).choice(V, size=n, replace=False)).astype(np.int32)
        ctx = np.concatenate([ids, ids[:1].repeat(7)]) if n else ids
        B.nanospec_vocab_init(st.h, dev_ids(ctx), [0, len(ctx)], None, [0, 0])
        logits = torch.full((1, M, st.capacity), float("nan"), dtype=torch.float32, device="cuda")
        B.nanospec_sparse_head(st.h, dW, dH, M, logits)
        torch.cuda.synchronize()
        assert np.array_equal(st.read_active()[0], ids)
        g = logits.cpu().numpy()[0]
        assert np.isnan(g[:, n:]).all(), "a column past the row count was written"
        if n:
            o32, o64 = oracle.head(W, H[0], ids=ids, omp=True)
            assert_logits_close(g[:, :n], o64, o32, f"cap={cap} M={M} d={d} n={n}")
        assert B.nanospec_last_device_error(st.h) == 0
        st.close()
