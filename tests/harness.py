"""Shared driver of the GPU parity tests: runs one synthetic workload through the C ABI (via the
ctypes binding) and through the CPU oracle, and compares them.  Not collected by pytest."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2605_26444_amd import binding as B
from paper_2605_26444_amd import synth

ATOL, RTOL = 2e-3, 1e-3          # logit tolerance fixed by the benchmark spec (fp32 accumulation)
# two fp32 sums of the same d exact products differ by at most ~2*d*2^-24*sum|w h| (~5e-6 at d = 8192, |logit| ~ 2);
# only ranks whose exact logits are closer than this can come out in the other order
SWAP_TOL = 2e-5

_W_CACHE: dict = {}


def host_W(cfg):
    key = (cfg["seed"], cfg["V"], cfg["d"])
    if key not in _W_CACHE:
        _W_CACHE.clear()                                  # keep at most one matrix on the host
        _W_CACHE[key] = synth.make_W(cfg)
    return _W_CACHE[key]


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype)
    return t.cuda()


def dev_bf16(bits):
    return dev(bits.view(np.int16)).view(torch.bfloat16)


def csr(arrays):
    off = np.zeros(len(arrays) + 1, np.int32)
    off[1:] = np.cumsum([len(a) for a in arrays])
    flat = np.concatenate(arrays).astype(np.int32) if off[-1] > 0 else np.zeros(0, np.int32)
    return flat, off


def dev_ids(flat):
    return dev(flat) if len(flat) else None


def assert_logits_close(g, o64, o32=None, what=""):
    err = np.abs(g.astype(np.float64) - o64)
    tol = ATOL + RTOL * np.abs(o64)
    assert np.all(err <= tol), f"{what}: max err {err.max():.3e} (tol {ATOL}+{RTOL}|x|)"
    if o32 is not None:
        assert np.all(np.abs(g - o32) <= ATOL + RTOL * np.abs(o32)), what
    return float(err.max())


def check_topk(g_ids, g_vals, g_logits_row, o32_row, active, k, stats, what="", o64_row=None):
    """two-level check of one (sequence, hidden row)."""
    # level 1 (strict): the oracle's selection applied to the GPU's own logits, ties included
    oi, ov = oracle.topk(g_logits_row, active, k)
    assert np.array_equal(g_ids, oi), f"{what}: top-k ids differ from oracle selection on the same logits"
    assert np.array_equal(g_vals, ov), f"{what}: top-k values differ"
    # level 2 (end to end): oracle ids from oracle logits.  Rank r must agree wherever the oracle's
    # gaps to both neighbouring ranks exceed twice the logit tolerance; rows with a closer pair are
    # counted as near ties (their other ranks are still compared).
    kk = min(k + 1, len(active))
    ei, ev = oracle.topk(o32_row, active, kk)
    m = min(k, len(active))
    if m == 0:
        return
    tol = 2 * (ATOL + RTOL * float(np.abs(ev).max()))
    gaps = np.concatenate([[np.inf], ev[:-1] - ev[1:], [np.inf]])      # gaps[r] = gap above rank r
    safe = (gaps[:m] > tol) & (gaps[1:m + 1] > tol)
    assert np.array_equal(g_ids[:m][safe], ei[:m][safe]), f"{what}: end-to-end top-k ids differ"
    stats["ranks_checked_e2e"] = stats.get("ranks_checked_e2e", 0) + int(safe.sum())
    if safe.all():
        stats["rows_checked_e2e"] = stats.get("rows_checked_e2e", 0) + 1
    else:
        stats["rows_near_tie"] = stats.get("rows_near_tie", 0) + 1
        # a near tie may legitimately come out in the other order: the two sides add the same exact products in a
        # different order (observed |difference| <= 2e-6).  Where the ids differ the GPU's choice must still be a
        # valid one: at every rank its id's exact (fp64) logit lies within SWAP_TOL of the oracle's id's.
        if not np.array_equal(g_ids[:m], ei[:m]):
            stats["rows_near_tie_differ"] = stats.get("rows_near_tie_differ", 0) + 1
            if o64_row is not None:
                where = {int(t): j for j, t in enumerate(active)}
                ge = np.array([o64_row[where[int(t)]] for t in g_ids[:m]])
                oe = np.array([o64_row[where[int(t)]] for t in ei[:m]])
                assert np.all(np.abs(ge - oe) <= SWAP_TOL), f"{what}: ids differ beyond a near tie ({np.abs(ge - oe).max():.3e})"


def run_workload(cfg, target=None, check_steps=None, M=None, k=None, W_bits=None, dW=None):
    """init + every step of one config on the GPU and in the oracle; returns statistics."""
    seqs = synth.make_sequences(cfg, target)
    B_, V, d = cfg["batch"], cfg["V"], cfg["d"]
    M = M or cfg["M"]
    k = k or cfg["k"]
    steps = cfg["steps"]
    if check_steps is None:
        check_steps = set(range(steps))
    if W_bits is None:
        W_bits = host_W(cfg)
    if dW is None:
        dW = dev_bf16(W_bits)
    st = B.State(V, d, B_, seqs["window"], seqs["topk_cap"], M, k)
    cap = st.capacity
    logits = torch.empty((B_, M, cap), dtype=torch.float32, device="cuda")
    out_ids = torch.empty((B_, M, k), dtype=torch.int32, device="cuda")
    out_vals = torch.empty((B_, M, k), dtype=torch.float32, device="cuda")
    orc = [oracle.Vocab(V, seqs["window"]) for _ in range(B_)]
    stats = {"n": [], "max_err": 0.0, "steps_checked": 0}

    ctx, coff = csr(seqs["ctx"])
    T0, toff = csr(seqs["T0"])
    B.nanospec_vocab_init(st.h, dev_ids(ctx), coff, dev_ids(T0), toff)
    for b in range(B_):
        orc[b].init(seqs["ctx"][b], seqs["T0"][b])

    def compare(step, full):
        act = st.read_active()
        for b in range(B_):
            exp = orc[b].active()
            assert np.array_equal(act[b], exp), f"step {step} seq {b}: active ids differ (n={len(act[b])} vs {len(exp)})"
        stats["n"].append([len(a) for a in act])
        if not full:
            return
        H_bits = synth.make_H(cfg, step, B_, M)
        dH = dev_bf16(H_bits)
        B.nanospec_sparse_head(st.h, dW, dH, M, logits)
        B.nanospec_topk_remap(st.h, logits, M, k, out_ids, out_vals)
        torch.cuda.synchronize()
        gl, gi, gv = logits.cpu().numpy(), out_ids.cpu().numpy(), out_vals.cpu().numpy()
        for b in range(B_):
            n = len(act[b])
            o32, o64 = oracle.head(W_bits, H_bits[b], ids=act[b], omp=True)
            e = assert_logits_close(gl[b, :, :n], o64, o32, f"step {step} seq {b}")
            stats["max_err"] = max(stats["max_err"], e)
            for m in range(M):
                check_topk(gi[b, m], gv[b, m], gl[b, m, :n], o32[m], act[b], k, stats, f"step {step} seq {b} row {m}",
                           o64_row=o64[m])
        stats["steps_checked"] += 1

    compare(-1, -1 in check_steps or 0 in check_steps)
    for s in range(steps):
        new, noff = csr(seqs["appends"][s])
        Ts = seqs["T_step"][s]
        if Ts is not None:
            tf, tof = csr(Ts)
            B.nanospec_vocab_update(st.h, dev_ids(new), noff, dev_ids(tf), tof)
        else:
            B.nanospec_vocab_update(st.h, dev_ids(new), noff)
        for b in range(B_):
            orc[b].update(seqs["appends"][s][b], Ts[b] if Ts is not None else None)
        compare(s, s in check_steps)
    assert B.nanospec_last_device_error(st.h) == 0
    st.close()
    # rows whose near ties came out in the other order (each was checked to be a valid order above): a handful
    # at most -- more would point at a real difference
    assert stats.get("rows_near_tie_differ", 0) <= max(1, stats.get("rows_near_tie", 0) // 500), stats
    return stats
