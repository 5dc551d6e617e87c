"""GPU parity of the batch-union head for several sequences (multi-sequence serving, Sec. 4.6):
nanospec_union_build + nanospec_union_head + the unchanged selection against the CPU oracle -- the shared / per-sequence
lists against oracle.shared_rows on the oracle's own active sets, the logits against oracle.head per sequence -- through
the C ABI."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2605_26444_amd import binding as B
from paper_2605_26444_amd import synth

from harness import assert_logits_close, check_topk, csr, dev_bf16, dev_ids, host_W

pytestmark = pytest.mark.gpu


def _run(V, d, M, k, window, ctx, T0, steps, W, seed, min_share, shared_cap=0, m_cap=None, sample_seqs=None, fifo=False):
    """ctx, T0: per-sequence lists; steps: list of (per-sequence appended ids, per-sequence new T or None)."""
    nb = len(ctx)
    dW = dev_bf16(W)
    topk_cap = max([1] + [len(t) for t in T0] + [len(t) for _, Ts in steps if Ts is not None for t in Ts])
    st = B.State(V, d, nb, window, topk_cap, m_cap or M, k)
    assert B.nanospec_union_bytes(st.h, shared_cap) > 0
    B.nanospec_union_enable(st.h, min_share, shared_cap)
    if fifo:
        B.nanospec_set_stream_policy(st.h, B.POLICY_FIFO)
    cap = st.capacity
    logits = torch.empty((nb, M, cap), dtype=torch.float32, device="cuda")
    oi = torch.empty((nb, M, k), dtype=torch.int32, device="cuda")
    ov = torch.empty((nb, M, k), dtype=torch.float32, device="cuda")
    orc = [(oracle.FifoVocab if fifo else oracle.Vocab)(V, window) for _ in range(nb)]
    flat, off = csr(ctx)
    tflat, toff = csr(T0)
    B.nanospec_vocab_init(st.h, dev_ids(flat), off, dev_ids(tflat), toff)
    for b in range(nb):
        orc[b].init(ctx[b], T0[b])
    stats = {"shared": [], "pairs_shared": 0, "pairs": 0}
    for step in range(-1, len(steps)):
        if step >= 0:
            new, Ts = steps[step]
            flat, off = csr([np.asarray(a, np.int32) for a in new])
            if Ts is None:
                B.nanospec_vocab_update(st.h, dev_ids(flat), off)
            else:
                tflat, toff = csr([np.asarray(t, np.int32) for t in Ts])
                B.nanospec_vocab_update(st.h, dev_ids(flat), off, dev_ids(tflat), toff)
            for b in range(nb):
                orc[b].update(new[b], None if Ts is None else Ts[b])
        B.nanospec_union_build(st.h)
        H = synth.normal_bf16(seed, 100 + step, (nb, M, d), 1.0, threads=1)
        dH = dev_bf16(H)
        logits.fill_(float("nan"))
        B.nanospec_union_head(st.h, dW, dH, M, logits)
        B.nanospec_topk_remap(st.h, logits, M, k, oi, ov)
        torch.cuda.synchronize()
        actives = [o.active() for o in orc]
        got = st.read_active()
        for b in range(nb):
            assert np.array_equal(got[b], actives[b])
        # the lists against the definition applied to the oracle's active sets
        sid, spos, rest, share, scap = st.read_union()
        e_sid, e_pos, e_rest = oracle.shared_rows(actives, share, scap)
        assert np.array_equal(sid, e_sid), f"step {step}: shared ids differ ({len(sid)} vs {len(e_sid)})"
        assert np.array_equal(spos, e_pos), f"step {step}: columns of the shared rows differ"
        for b in range(nb):
            assert np.array_equal(rest[b][0], e_rest[b][0]), f"step {step} seq {b}: per-sequence ids differ"
            assert np.array_equal(rest[b][1], e_rest[b][1]), f"step {step} seq {b}: per-sequence columns differ"
        stats["shared"].append(len(sid))
        stats["pairs_shared"] += int((e_pos >= 0).sum())
        stats["pairs"] += sum(len(a) for a in actives)
        # logits and selection against the oracle
        g, gi, gv = logits.cpu().numpy(), oi.cpu().numpy(), ov.cpu().numpy()
        for b in (range(nb) if sample_seqs is None else sample_seqs):
            a = actives[b]
            n = len(a)
            assert not np.isnan(g[b, :, :n]).any(), f"step {step} seq {b}: a logit column of an active id was never written"
            if n == 0:
                continue
            o32, o64 = oracle.head(W, H[b], ids=a, omp=True)
            assert_logits_close(g[b, :, :n], o64, o32, f"union step {step} seq {b}")
            for m in range(M):
                check_topk(gi[b, m], gv[b, m], g[b, m, :n], o32[m], a, k, stats, f"union step {step} seq {b} row {m}", o64_row=o64[m])
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()
    return stats


def _random_case(rng, V, nb, ctx_len, nT, hot, nsteps, replace_T=True):
    """sequences that draw most ids from a common hot range (shared) and the others from all of V"""
    def draw(nn):
        pick = rng.random(nn) < 0.7
        return np.where(pick, rng.integers(0, hot, nn), rng.integers(0, V, nn)).astype(np.int32)
    ctx = [draw(ctx_len) for _ in range(nb)]
    T0 = [np.unique(draw(nT)).astype(np.int32) for _ in range(nb)]
    steps = []
    for s in range(nsteps):
        new = [draw(int(rng.integers(0, 6))) for _ in range(nb)]
        Ts = [np.unique(draw(nT)).astype(np.int32) for _ in range(nb)] if (replace_T and s % 2 == 1) else None
        steps.append((new, Ts))
    return ctx, T0, steps


def test_union_small_tail_group_only():
    """6 sequences x 5 hidden rows: 30 hidden rows, one short group; shared rows held by at least 3 sequences"""
    rng = np.random.default_rng(21)
    V, d, M, k, window = 5000, 512, 5, 8, 96
    W = synth.normal_bf16(9100, 0, (V, d), 0.02)
    ctx, T0, steps = _random_case(rng, V, 6, 300, 40, 150, 6)
    st = _run(V, d, M, k, window, ctx, T0, steps, W, 9200, min_share=3)
    assert min(st["shared"]) > 0 and 0 < st["pairs_shared"] < st["pairs"]


def test_union_under_the_queue_reading_of_the_vocabulary():
    """the lists are built from the membership bitmaps, which both readings of the vocabulary maintain"""
    rng = np.random.default_rng(27)
    V, d, M, k, window = 6000, 512, 4, 6, 80
    W = synth.normal_bf16(9150, 0, (V, d), 0.02)
    ctx, T0, steps = _random_case(rng, V, 9, 300, 40, 150, 5)
    st = _run(V, d, M, k, window, ctx, T0, steps, W, 9250, min_share=3, fifo=True)
    assert min(st["shared"]) > 0


def test_union_more_sequences_than_a_wavefront_has_lanes():
    """130 sequences: the per-id count walks the batch in chunks of 64 lanes; 130 x 2 hidden rows = 4 groups and a tail of 4"""
    rng = np.random.default_rng(28)
    V, d, M, k, window = 2000, 256, 2, 3, 48
    W = synth.normal_bf16(9160, 0, (V, d), 0.02)
    ctx, T0, steps = _random_case(rng, V, 130, 120, 10, 60, 2)
    st = _run(V, d, M, k, window, ctx, T0, steps, W, 9260, min_share=70)
    assert min(st["shared"]) > 0 and st["pairs_shared"] < st["pairs"]


def test_union_groups_and_tail_hidden_size_not_a_whole_slice():
    """20 sequences x 8 hidden rows = two groups of 64 and a tail of 32; d = 1032 takes the bounds-tested loads"""
    rng = np.random.default_rng(22)
    V, d, M, k, window = 20000, 1032, 8, 10, 256
    W = synth.normal_bf16(9300, 0, (V, d), 0.02)
    ctx, T0, steps = _random_case(rng, V, 20, 700, 100, 400, 3)
    st = _run(V, d, M, k, window, ctx, T0, steps, W, 9400, min_share=0)          # default threshold: max(2, 20/8) = 2
    assert min(st["shared"]) > 64


def test_union_shared_list_overflows_and_sequences_of_three_rows():
    """room for 64 shared rows only (the others stay per sequence); 3 hidden rows per sequence cross group borders"""
    rng = np.random.default_rng(23)
    V, d, M, k, window = 9000, 1024, 3, 5, 128
    W = synth.normal_bf16(9500, 0, (V, d), 0.02)
    ctx, T0, steps = _random_case(rng, V, 30, 400, 60, 300, 3)
    st = _run(V, d, M, k, window, ctx, T0, steps, W, 9600, min_share=4, shared_cap=64)
    assert max(st["shared"]) == 64


def test_union_nothing_shared_and_everything_shared():
    rng = np.random.default_rng(24)
    V, d, M, k, window = 3000, 512, 8, 6, 64
    W = synth.normal_bf16(9700, 0, (V, d), 0.02)
    ctx, T0, steps = _random_case(rng, V, 8, 200, 30, 100, 2)
    st = _run(V, d, M, k, window, ctx, T0, steps, W, 9800, min_share=9)          # more than the batch: nothing is shared
    assert max(st["shared"]) == 0
    st = _run(V, d, M, k, window, ctx, T0, steps, W, 9800, min_share=1)          # every active id qualifies; the list is full
    assert min(st["shared"]) == 128 and st["pairs_shared"] < st["pairs"]
    same = [ctx[0]] * 8, [T0[0]] * 8, [([a[0]] * 8, None if t is None else [t[0]] * 8) for a, t in steps]
    st = _run(V, d, M, k, window, same[0], same[1], same[2], W, 9800, min_share=8)   # identical sequences: one list serves all
    assert st["pairs_shared"] == st["pairs"]


def test_union_one_sequence_and_empty_sets():
    V, d, M, k, window = 700, 64, 4, 4, 16
    W = synth.normal_bf16(9900, 0, (V, d), 0.02)
    empty = np.zeros(0, np.int32)
    _run(V, d, M, k, window, [np.array([5, 6, 5], np.int32)], [empty], [([np.array([9])], None)], W, 9950, min_share=1)
    steps = [([np.array([1, 2]), empty, np.array([2])], None), ([empty, empty, empty], [np.array([2, 699]), np.array([699]), empty])]
    _run(V, d, M, k, window, [empty, empty, empty], [empty, empty, empty], steps, W, 9960, min_share=2)


def test_union_wide_rows_per_sequence():
    """40 hidden rows per sequence: the per-sequence part takes the split-K kernels with a column map"""
    rng = np.random.default_rng(25)
    V, d, M, k, window = 12000, 1024, 40, 10, 512
    W = synth.normal_bf16(9970, 0, (V, d), 0.02)
    ctx, T0, steps = _random_case(rng, V, 3, 900, 80, 500, 2, replace_T=False)
    _run(V, d, M, k, window, ctx, T0, steps, W, 9980, min_share=2)


def test_union_c4_shape():
    """the 64-sequence workload at full size, two steps; oracle logits on a sample of the sequences"""
    cfg = dict(synth.CONFIGS["c4"])
    cfg["steps"] = 2
    seqs = synth.make_sequences(cfg)
    W = host_W(cfg)
    steps = [(seqs["appends"][s], seqs["T_step"][s]) for s in range(cfg["steps"])]
    st = _run(cfg["V"], cfg["d"], cfg["M"], cfg["k"], seqs["window"], seqs["ctx"], seqs["T0"], steps, W, 9990, min_share=0,
              sample_seqs=(0, 31, 63))
    assert min(st["shared"]) > 1000


def test_union_step_recorded_in_hip_graph_replays_correctly():
    """update + list build + union head (whose shared-row product forks onto the state's side stream and joins back) +
    selection captured in one HIP graph: every replay, with eager work and synchronisations in between, gives the
    oracle's vocabulary, the eager union head's bits and the oracle's logits."""
    rng = np.random.default_rng(26)
    V, d, M, k, window, nb = 8000, 512, 8, 6, 128, 12
    W = synth.normal_bf16(9991, 0, (V, d), 0.02)
    ctx, T0, _ = _random_case(rng, V, nb, 400, 50, 250, 0)
    dW = dev_bf16(W)
    H = synth.normal_bf16(9992, 0, (nb, M, d), 1.0, threads=1)
    dH = dev_bf16(H)
    st = B.State(V, d, nb, window, 64, M, k)
    B.nanospec_union_enable(st.h, 3, 0)
    orc = [oracle.Vocab(V, window) for _ in range(nb)]
    flat, off = csr(ctx)
    tflat, toff = csr(T0)
    B.nanospec_vocab_init(st.h, dev_ids(flat), off, dev_ids(tflat), toff)
    for b in range(nb):
        orc[b].init(ctx[b], T0[b])
    new = [rng.integers(0, 250, 3).astype(np.int32) for _ in range(nb)]
    nflat, noff = csr(new)
    d_new = dev_ids(nflat)
    cap = st.capacity
    lg_g = torch.empty((nb, M, cap), dtype=torch.float32, device="cuda")
    lg_e = torch.empty_like(lg_g)
    oi_g = torch.empty((nb, M, k), dtype=torch.int32, device="cuda")
    ov_g = torch.empty((nb, M, k), dtype=torch.float32, device="cuda")
    oi_e, ov_e = torch.empty_like(oi_g), torch.empty_like(ov_g)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cs = torch.cuda.current_stream().cuda_stream
        B.nanospec_vocab_update(st.h, d_new, noff, None, None, cs)
        B.nanospec_union_build(st.h, cs)
        B.nanospec_union_head(st.h, dW, dH, M, lg_g, cs)
        B.nanospec_topk_remap(st.h, lg_g, M, k, oi_g, ov_g, cs)
    torch.cuda.synchronize()
    for rep in range(4):
        lg_g.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        for b in range(nb):
            orc[b].update(new[b])
        act = st.read_active()
        for b in range(nb):
            assert np.array_equal(act[b], orc[b].active()), (rep, b)
        lg_e.fill_(float("nan"))
        B.nanospec_union_head(st.h, dW, dH, M, lg_e)                   # eager work between replays
        B.nanospec_topk_remap(st.h, lg_e, M, k, oi_e, ov_e)
        torch.cuda.synchronize()
        gg, ge = lg_g.cpu().numpy(), lg_e.cpu().numpy()
        for b in range(nb):
            n = len(act[b])
            assert not np.isnan(gg[b, :, :n]).any(), (rep, b)
            assert np.array_equal(gg[b, :, :n], ge[b, :, :n]), (rep, b)
            o32, o64 = oracle.head(W, H[b], ids=act[b], omp=True)
            assert_logits_close(gg[b, :, :n], o64, o32, f"replay {rep} seq {b}")
        assert np.array_equal(oi_g.cpu().numpy(), oi_e.cpu().numpy()) and np.array_equal(ov_g.cpu().numpy(), ov_e.cpu().numpy())
        extra = [np.array([rep, 7000 + rep], np.int32) for _ in range(nb)]   # eager update between replays
        ef, eo = csr(extra)
        B.nanospec_vocab_update(st.h, dev_ids(ef), eo)
        for b in range(nb):
            orc[b].update(extra[b])
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()
