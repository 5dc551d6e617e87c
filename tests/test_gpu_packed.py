"""GPU parity of the packed-buffer variant of the head (Sec. 3.3 asynchronous gathering; Table 4 gather row):
nanospec_packed_gather + nanospec_packed_head + the unchanged selection against the CPU oracle, the slot tables
against the oracle's active sets (only rows that entered are copied, slots are stable), through the C ABI."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle
from paper_2605_26444_amd import binding as B
from paper_2605_26444_amd import synth

from harness import assert_logits_close, check_topk, dev, dev_bf16, dev_ids, host_W

pytestmark = pytest.mark.gpu


def _run(V, d, M, k, window, ctx, T0, steps, W, seed, second_stream=False):
    """steps: list of (appended ids, new T or None).  Checks every step."""
    dW = dev_bf16(W)
    topk_cap = max([len(T0), 1] + [len(t) for _, t in steps if t is not None])
    st = B.State(V, d, 1, window, topk_cap, M, k)
    B.nanospec_packed_enable(st.h)
    assert B.nanospec_packed_bytes(st.h) >= st.capacity * d * 2
    cap = st.capacity
    logits = torch.full((1, M, cap), float("nan"), dtype=torch.float32, device="cuda")
    fused = torch.empty_like(logits)
    oi = torch.empty((1, M, k), dtype=torch.int32, device="cuda")
    ov = torch.empty((1, M, k), dtype=torch.float32, device="cuda")
    orc = oracle.Vocab(V, window)
    B.nanospec_vocab_init(st.h, dev_ids(ctx), [0, len(ctx)], dev_ids(T0), [0, len(T0)])
    orc.init(ctx, T0)
    side = torch.cuda.Stream() if second_stream else None
    prev_active, prev_slot = np.zeros(0, np.int32), {}
    stats = {}
    for step in range(-1, len(steps)):
        if step >= 0:
            new, T = steps[step]
            new = np.asarray(new, np.int32)
            if T is None:
                B.nanospec_vocab_update(st.h, dev_ids(new), [0, len(new)])
            else:
                B.nanospec_vocab_update(st.h, dev_ids(new), [0, len(new)], dev_ids(np.asarray(T, np.int32)), [0, len(T)])
            orc.update(new, T)
        if side is not None:                                  # the paper's dual-stream form: gather on a second stream
            ev = torch.cuda.Event()
            ev.record()
            side.wait_event(ev)
            B.nanospec_packed_gather(st.h, dW, side.cuda_stream)
            done = torch.cuda.Event()
            done.record(side)
            torch.cuda.current_stream().wait_event(done)
        else:
            B.nanospec_packed_gather(st.h, dW)
        H = synth.normal_bf16(seed, 100 + step, (M, d), 1.0, threads=1)
        dH = dev_bf16(H)
        logits.fill_(float("nan"))
        B.nanospec_packed_head(st.h, dH, M, logits)
        B.nanospec_topk_remap(st.h, logits, M, k, oi, ov)
        B.nanospec_sparse_head(st.h, dW, dH, M, fused)
        torch.cuda.synchronize()
        active = orc.active()
        n = len(active)
        assert np.array_equal(st.read_active()[0], active)
        # slot tables against the oracle's active set
        slot_id, out_pos, hi, ncopy, buf = st.read_packed()
        used = np.flatnonzero(slot_id >= 0)
        assert np.array_equal(np.sort(slot_id[used]), active), f"step {step}: slots do not hold exactly the active ids"
        assert hi == (used.max() + 1 if len(used) else 0) and hi <= cap
        where = {int(t): j for j, t in enumerate(active)}
        assert all(out_pos[s] == where[int(slot_id[s])] for s in used) and np.all(out_pos[slot_id < 0] == -1)
        entered = np.setdiff1d(active, prev_active)
        assert ncopy == len(entered), f"step {step}: {ncopy} rows copied, {len(entered)} ids entered"
        slot_now = {int(slot_id[s]): int(s) for s in used}
        assert all(slot_now[t] == s for t, s in prev_slot.items() if t in slot_now), "an id that stayed active changed its slot"
        assert np.array_equal(buf[used], W[slot_id[used]]), f"step {step}: a packed row differs from its W_head row"
        prev_active, prev_slot = active, slot_now
        # logits and selection against the oracle
        g = logits.cpu().numpy()[0]
        assert not np.isnan(g[:, :n]).any(), "a logit column of an active id was never written"
        if n:
            o32, o64 = oracle.head(W, H, ids=active, omp=True)
            assert_logits_close(g[:, :n], o64, o32, f"packed step {step}")
            assert np.array_equal(g[:, :n], fused.cpu().numpy()[0][:, :n]), "packed and fused heads differ in some bit"
            for m in range(M):
                check_topk(oi.cpu().numpy()[0, m], ov.cpu().numpy()[0, m], g[m, :n], o32[m], active, k, stats, f"packed step {step} row {m}",
                           o64_row=o64[m])
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()
    return stats


def test_packed_small_every_kind_of_update():
    V, d, M, k, window = 5000, 512, 5, 8, 96
    rng = np.random.default_rng(7)
    W = synth.normal_bf16(8100, 0, (V, d), 0.02)
    ctx = rng.integers(0, V, 300).astype(np.int32)
    T0 = rng.choice(V, 40, replace=False).astype(np.int32)
    steps = []
    for s in range(30):
        a = int(rng.integers(0, 5))
        new = rng.integers(0, 400, a) if s % 3 else rng.integers(0, V, a)      # repeats of earlier ids and fresh ones
        T = None
        if s == 9:
            T = rng.choice(V, 25, replace=False)                               # T replaced: many slots change hands
        if s == 14:
            new = rng.integers(0, V, 150)                                      # longer than the window: the rebuild route
        if s == 20:
            T = np.zeros(0, np.int64)                                          # T emptied: many ids leave
        steps.append((new, T))
    _run(V, d, M, k, window, ctx, T0, steps, W, 8200)


def test_packed_empty_and_refill():
    V, d, M, k, window = 700, 64, 3, 4, 16
    W = synth.normal_bf16(8300, 0, (V, d), 0.02)
    steps = [(np.array([5, 5, 6]), None), (np.zeros(0, np.int64), None), (np.arange(100, 140), None), (np.array([1]), np.array([3, 4, 699]))]
    _run(V, d, M, k, window, np.zeros(0, np.int32), np.zeros(0, np.int32), steps, W, 8400)


def test_packed_c2_shape_decoding_steps_on_a_second_stream():
    cfg = dict(synth.CONFIGS["c2"])
    cfg["steps"] = 10
    seqs = synth.make_sequences(cfg)
    W = host_W(cfg)
    steps = [(seqs["appends"][s][0], None) for s in range(cfg["steps"])]
    st = _run(cfg["V"], cfg["d"], cfg["M"], cfg["k"], seqs["window"], seqs["ctx"][0], seqs["T0"][0], steps, W, 8500, second_stream=True)
    assert st.get("rows_checked_e2e", 0) > 0


@pytest.mark.parametrize("name,M", [("c3", 64), ("c3", 40), ("c5", 16)])
def test_packed_wide_tree_and_long_rows(name, M):
    """the split-K kernels (16 < M <= 64) and the K-loop kernel (d = 8192) writing through the slot -> column map"""
    cfg = dict(synth.CONFIGS[name])
    cfg["steps"] = 3
    seqs = synth.make_sequences(cfg, 1000 if name == "c5" else None)
    W = host_W(cfg)
    steps = [(seqs["appends"][s][0], None) for s in range(cfg["steps"])]
    _run(cfg["V"], cfg["d"], M, cfg["k"], seqs["window"], seqs["ctx"][0], seqs["T0"][0], steps, W, 8600)
