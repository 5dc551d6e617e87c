#!/usr/bin/env python3
"""Benchmark of the NanoSpec draft-step hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input, with everything
already resident in HBM:  nanospec_vocab_update (append the accepted tokens, rebuild I)
-> nanospec_sparse_head (project the draft hidden rows onto W_head[I, :]) -> nanospec_topk_remap.
The default workload is the Llama-3-8B-shaped head the headline metric is quoted on
(V=128256, d=4096, |active| ~ 3k, M=8 draft rows, top-10, 1-4 accepted tokens per step).

Cold weights: consecutive draft steps touch almost the same ~24.6 MB of LM-head rows, which would
sit in the 256 MB Infinity Cache if nothing else ran.  In real decoding the draft backbone and the
target model stream gigabytes between two head calls, so the benchmark rotates through
`--replicas` (default 32) copies of W_head (distinct addresses, same values): every head launch then reads rows
that have been evicted, and `roofline.achieved` is an HBM number.  `--replicas 1` gives the warm
figure.

Prints ONE JSON line: metric / value / unit and the run parameters, `roofline` (the sparse-head kernel's
gathered bytes per launch over its event-timed launch time, against the 8 TB/s peak, with the counter-measured
traffic), `ceilings` (read-only kernels over the same bytes), `kernels_us`, `closed_loop` (device-side feedback
of the selected ids), `packed_buffer_variant`, `dense` (full-vocabulary head + top-k) and `cpu_baseline` (the
CPU oracle timed on the host cores).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak
# Bytes per sparse-head launch that leave L2 towards HBM, from the rocprofv3 --pmc runs summarised under
# profiles/ (FETCH_SIZE x 2.0 +
# WRITE_SIZE x 1.0, factors from copy / stream kernels of known size), as bytes per active row so that it
# follows the realised |active|.  c3: the split-K kernel without its reduce kernel; c5: measured at 32k rows.
PMC_TRAFFIC_PER_ROW = {"c2": 25313690 / 3004, "c3": 25943859 / 2998, "c4": 767895347 / 144911,
                       "c5@32000": 533476454 / 32007}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--target", type=int, default=3000, help="c5 only: number of distinct active ids")
    ap.add_argument("--replicas", type=int, default=32, help="copies of W_head rotated through (1 = warm caches)")
    ap.add_argument("--hidden-buffers", type=int, default=16, help="distinct hidden-state tensors rotated through")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly from Python instead of replaying HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-packed", action="store_true", help="skip the packed-buffer variant (the paper's own design)")
    ap.add_argument("--no-cold-check", action="store_true", help="skip timing the head over rotations of 16 / 32 / 48 weight copies")
    ap.add_argument("--no-union", action="store_true", help="skip the batch-union head (several sequences only)")
    ap.add_argument("--union-shares", default="2,4,8,16,32", help="min_share thresholds the batch-union leg sweeps")
    ap.add_argument("--only-union", type=int, default=0, metavar="MIN_SHARE",
                    help="run nothing but a train of nanospec_union_head launches at this threshold (for counter runs)")
    ap.add_argument("--traffic", default=None, help="HBM bytes per head launch from rocprofv3 --pmc runs (or omit)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 (the path has no collectives; "
              "sequences shard by sequence, one sequence by vocabulary range with one exchange of M x k pairs)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_26444_amd import binding as B
    from paper_2605_26444_amd import synth

    torch.cuda.set_device(0)

    def log(msg):
        """one line per finished leg on stderr (under a profiler a leg can take minutes)"""
        print(f"bench: {msg} [{time.time() - t_start:.1f} s]", file=sys.stderr, flush=True)
    t_start = time.time()
    cfg = dict(synth.CONFIGS[args.config])
    K, Wm = args.steps, args.warmup
    if K < 1 or Wm < 0:
        ap.error("--steps must be at least 1, --warmup at least 0")
    total_steps = K + Wm
    cfg["steps"] = total_steps
    V, d, M, k, Bn = cfg["V"], cfg["d"], cfg["M"], cfg["k"], cfg["batch"]
    seqs = synth.make_sequences(cfg, args.target if args.config == "c5" else None)

    t0 = time.time()
    W_host = synth.make_W(cfg)
    to_dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    R = max(1, args.replicas)
    Wd = [to_dev(W_host.view(np.int16)).view(torch.bfloat16)]
    for _ in range(R - 1):
        Wd.append(Wd[0].clone())
    NH = max(1, args.hidden_buffers)
    Hd = [to_dev(synth.make_H(cfg, s).view(np.int16)).view(torch.bfloat16) for s in range(NH)]

    st = B.State(V, d, Bn, seqs["window"], seqs["topk_cap"], M, k)
    cap = st.capacity
    logits = torch.empty((Bn, M, cap), dtype=torch.float32, device="cuda")
    out_ids = torch.empty((Bn, M, k), dtype=torch.int32, device="cuda")
    out_vals = torch.empty((Bn, M, k), dtype=torch.float32, device="cuda")

    def csr(arrays):
        off = np.zeros(len(arrays) + 1, np.int32)
        off[1:] = np.cumsum([len(a) for a in arrays])
        return np.concatenate(arrays).astype(np.int32), off

    ctx, coff = csr(seqs["ctx"])
    T0, toff = csr(seqs["T0"])
    d_ctx, d_T0 = to_dev(ctx), (to_dev(T0) if len(T0) else None)
    # all appended ids of all steps in one device buffer; per-step host offsets
    flat, offs, toffs, tflat = [], [], [], []
    base = 0
    for s in range(total_steps):
        f, o = csr(seqs["appends"][s])
        flat.append(f)
        offs.append(o + base)
        base += len(f)
    d_new = to_dev(np.concatenate(flat))
    d_T_steps = None
    if seqs["T_step"][0] is not None:                         # c4: T replaced every step; rotate 8 sets
        tf = [csr(seqs["T_step"][s]) for s in range(8)]
        d_T_steps = [(to_dev(f), o) for f, o in tf]
    use_graph = not args.no_graph

    def step(i, r, stream):
        if d_T_steps is not None:
            tfl, tof = d_T_steps[i % 8]
            B.nanospec_vocab_update(st.h, d_new, offs[i], tfl, tof, stream)
        else:
            B.nanospec_vocab_update(st.h, d_new, offs[i], None, None, stream)
        B.nanospec_sparse_head(st.h, Wd[r % R], Hd[r % NH], M, logits, stream)
        B.nanospec_topk_remap(st.h, logits, M, k, out_ids, out_vals, stream)

    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    REPS = 11                                              # timed repetitions per figure; the median is reported
    ROT = R * NH // math.gcd(R, NH)                        # period of the weight / hidden-state rotation

    def timed(fn, first, count, reset=None, reps=REPS):
        """Median time (ms) of `count` consecutive calls fn(i, r, stream), i = first .. first+count-1 the data
        index and r a counter that keeps running from one repetition to the next (it drives the rotation of
        weight copies, so that a copy is never met again sooner than after R-1 others, also across
        repetitions).  The launches are recorded into HIP graphs (the hot calls never synchronise or allocate,
        so they can be): as many graphs as the rotation needs to come round, each replayed once untimed and then
        timed between two events on the launch stream, `reps` times over all.  `reset` (untimed, eager) restores
        whatever state fn advances before every repetition.  With --no-graph the calls are issued eagerly."""
        cur = torch.cuda.current_stream()
        ngraph = ROT // math.gcd(count, ROT)
        graphs = []
        if use_graph:
            for gi in range(ngraph):
                if reset:
                    reset()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    cs = torch.cuda.current_stream().cuda_stream
                    for j in range(count):
                        fn(first + j, gi * count + j, cs)
                torch.cuda.synchronize()
                graphs.append(g)
            for g in graphs:                               # one untimed replay each: first-launch costs stay out
                if reset:
                    reset()
                g.replay()
            torch.cuda.synchronize()
        else:
            if reset:
                reset()
            for j in range(count):
                fn(first + j, j, cur.cuda_stream)
            torch.cuda.synchronize()
        times = []
        for rep in range(reps):
            if reset:
                reset()
            torch.cuda.synchronize()
            e0.record(cur)
            if use_graph:
                graphs[rep % ngraph].replay()
            else:
                for j in range(count):
                    fn(first + j, rep * count + j, cur.cuda_stream)
            e1.record(cur)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1))
        del graphs
        return float(np.median(times)), times

    stream = torch.cuda.current_stream().cuda_stream

    def reset_main():
        """the state as the W warm-up steps leave it: stream = context + their appended ids"""
        B.nanospec_vocab_init(st.h, d_ctx, coff, d_T0, toff, stream)
        for s_ in range(Wm):
            step(s_, s_, stream)
    if args.only_union:
        # counter runs: only the two head kernels of the batch-union head appear in the trace besides the set-up
        su = B.State(V, d, Bn, seqs["window"], seqs["topk_cap"], M, k)
        B.nanospec_union_enable(su.h, args.only_union, 0)
        B.nanospec_vocab_init(su.h, d_ctx, coff, d_T0, toff, stream)
        B.nanospec_union_build(su.h, stream)
        for i in range(Wm + K):
            B.nanospec_union_head(su.h, Wd[i % R], Hd[i % NH], M, logits, stream)
        torch.cuda.synchronize()
        sid, spos, rest, share, scap = su.read_union()
        print(json.dumps({"only_union": True, "min_share": share, "launches": Wm + K, "shared_rows": len(sid),
                          "pairs_shared": int((spos >= 0).sum()), "pairs_rest": int(sum(len(r[0]) for r in rest))}))
        su.close()
        return
    ms, ms_all = timed(step, Wm, K, reset=reset_main)
    n_active = [len(a) for a in st.read_active()]
    n_sum = int(np.sum(n_active))
    log("step loop timed")

    # roofline leg: the sparse-head kernel alone, same launch configuration, cold rotation, HIP events
    # on the launch stream around a back-to-back train of launches (no host work in between).
    NL = 15 * ROT
    head = lambda i, r, cs: B.nanospec_sparse_head(st.h, Wd[r % R], Hd[r % NH], M, logits, cs)
    head_us = timed(head, 0, NL)[0] * 1e3 / NL
    alg_bytes = n_sum * d * 2                                  # gathered weight bytes per launch
    # Several sequences hold many of the same rows; those are served by the caches, so the gathered bytes can exceed
    # what HBM delivers.  The roofline of a batch is quoted on the distinct rows (what must come from HBM at least
    # once per launch); the gathered rate is reported beside it.
    distinct_rows = int(len(np.unique(np.concatenate(st.read_active())))) if Bn > 1 else n_sum
    roof_bytes = distinct_rows * d * 2
    log("head alone timed")
    achieved = roof_bytes / (head_us * 1e-6) / 1e9
    gathered = alg_bytes / (head_us * 1e-6) / 1e9

    def train(fn, n=200, reset=None):
        """median us per call of a back-to-back train of n calls"""
        return timed(fn, 0, n, reset=reset)[0] * 1e3 / n

    # Is the rotation wide enough to be cold?  The same head launch timed over rotations of 16 / 32 / 48 weight
    # copies (0.4 / 0.8 / 1.2 GB of active rows against the 256 MB Infinity Cache): flat means no launch finds
    # its rows in a cache.
    cold_check = None
    if not args.no_cold_check and Bn == 1:
        cold_check = {}
        extra = []
        for Rx in (16, 32, 48):
            while len(Wd) + len(extra) < Rx:
                extra.append(Wd[0].clone())
            pool = Wd + extra
            us = timed(lambda i, r, cs: B.nanospec_sparse_head(st.h, pool[r % Rx], Hd[r % NH], M, logits, cs), 0, 15 * Rx,
                       reps=5)[0] * 1e3 / (15 * Rx)
            cold_check[f"head_us_{Rx}_copies"] = round(us, 3)
        cold_check["head_us_1_copy_warm"] = round(timed(lambda i, r, cs: B.nanospec_sparse_head(st.h, Wd[0], Hd[r % NH], M, logits, cs),
                                                        0, 240, reps=5)[0] * 1e3 / 240, 3)
        del extra, pool

    # per-call times of the other two steps (informational).  The update alone: the steps' own calls (same appended
    # ids, same T replacement) on a scratch state that is put back before every repetition.
    st_u = B.State(V, d, Bn, seqs["window"], seqs["topk_cap"], M, k)

    def upd_only(i, r, cs):
        if d_T_steps is not None:
            tfl, tof = d_T_steps[i % 8]
            B.nanospec_vocab_update(st_u.h, d_new, offs[i], tfl, tof, cs)
        else:
            B.nanospec_vocab_update(st_u.h, d_new, offs[i], None, None, cs)
    upd_us = timed(upd_only, 0, total_steps, reset=lambda: B.nanospec_vocab_init(st_u.h, d_ctx, coff, d_T0, toff, stream))[0] * 1e3 / total_steps
    st_u.close()
    topk_us = train(lambda i, r, cs: B.nanospec_topk_remap(st.h, logits, M, k, out_ids, out_vals, cs))
    log("cold check, update and selection timed")

    # What one launch of this size can reach on this chip: read-only kernels that move the head's bytes and
    # compute nothing -- the same rows through the same id list, the same number of bytes contiguously, and the
    # whole matrix as one long stream -- with the same cold rotation and the same timing as the head.
    ceilings = None
    if Bn == 1:
        sink = torch.zeros(1024, dtype=torch.uint8, device="cuda")
        nb = alg_bytes // 16 * 16
        g_us = train(lambda i, r, cs: B.nanospec_calib_gather_read(st.h, Wd[r % R], sink, cs), 240)
        s_us = train(lambda i, r, cs: B.nanospec_calib_stream_read(Wd[r % R], nb, sink, cs), 240)
        full = V * d * 2
        f_us = train(lambda i, r, cs: B.nanospec_calib_stream_read(Wd[r % R], full, sink, cs), 32)
        v_us = None
        if M <= 8 and d in (2048, 4096):            # the same head on the vector ALUs (unpack + FMA), for comparison
            vl = torch.empty((1, M, cap), dtype=torch.float32, device="cuda")
            v_us = round(train(lambda i, r, cs: B.nanospec_calib_valu_head(st.h, Wd[r % R], Hd[r % NH], M, vl, cs), 240), 2)
        ceilings = {"vector_alu_head_us": v_us, "gather_same_rows_us": round(g_us, 2), "gather_same_rows_GBps": round(alg_bytes / g_us / 1e3, 1),
                    "stream_same_bytes_us": round(s_us, 2), "stream_same_bytes_GBps": round(nb / s_us / 1e3, 1),
                    "stream_whole_matrix_GBps": round(full / f_us / 1e3, 1),
                    "head_over_gather": round(head_us / g_us, 3)}

    # The paper's own system design (Sec. 3.3 asynchronous gathering; Table 4's gather row; Table 5's Indexed GEMM
    # against async gather) through the library's packed-buffer variant: a slot-stable packed copy of the active
    # rows, nanospec_packed_gather copying only the rows of ids that entered, nanospec_packed_head as a dense
    # product on the buffer.  Cold like the fused head: NP states with their own packed buffers are rotated (NP x
    # ~30 MB of packed rows against the 256 MB Infinity Cache).  The dual-stream form: a stand-in backbone (a
    # read of 1 GB, what a draft layer stack streams) on the main stream, update + gather on a second stream of
    # equal priority, one event wait in front of the head -- against the same work on one stream.
    packed_variant = None
    if Bn == 1 and d_T_steps is None and not args.no_packed:
        NP = 12
        pst = [B.State(V, d, 1, seqs["window"], seqs["topk_cap"], M, k) for _ in range(NP)]
        for q in pst:
            B.nanospec_packed_enable(q.h)

        def reset_packed():
            for q in pst:
                B.nanospec_vocab_init(q.h, d_ctx, coff, d_T0, toff, stream)
                B.nanospec_packed_gather(q.h, Wd[0], stream)
        reset_packed()
        packed_us = train(lambda i, r, cs: B.nanospec_packed_head(pst[r % NP].h, Hd[r % NH], M, logits, cs), 20 * NP)
        # the per-step gather: update + gather against update alone, the steps' own appended ids, one state
        q0 = pst[0]
        nsteps = min(total_steps, 200)
        init_q0 = lambda: (B.nanospec_vocab_init(q0.h, d_ctx, coff, d_T0, toff, stream), B.nanospec_packed_gather(q0.h, Wd[0], stream))

        def upd_gather(i, r, cs):
            B.nanospec_vocab_update(q0.h, d_new, offs[i], None, None, cs)
            B.nanospec_packed_gather(q0.h, Wd[r % R], cs)
        ug_us = timed(upd_gather, 0, nsteps, reset=init_q0)[0] * 1e3 / nsteps
        u_us = timed(lambda i, r, cs: B.nanospec_vocab_update(q0.h, d_new, offs[i], None, None, cs), 0, nsteps, reset=init_q0)[0] * 1e3 / nsteps
        init_q0()
        copied = 0
        for i in range(nsteps):                                # rows copied per step (read back, untimed)
            upd_gather(i, i, stream)
            copied += q0.read_packed()[3]
        # dual-stream overlap, issued eagerly (two streams of equal priority, events between them)
        side = torch.cuda.Stream()
        main = torch.cuda.current_stream()
        sink2 = torch.zeros(1024, dtype=torch.uint8, device="cuda")
        back_bytes = min(1 << 30, V * d * 2) // 16 * 16        # never past the end of a weight copy

        def draft_step(i, overlap):
            if overlap:
                side.wait_stream(main)
                B.nanospec_vocab_update(q0.h, d_new, offs[i % nsteps], None, None, side.cuda_stream)
                B.nanospec_packed_gather(q0.h, Wd[i % R], side.cuda_stream)
                B.nanospec_calib_stream_read(Wd[(i + 7) % R], back_bytes, sink2, main.cuda_stream)      # the stand-in backbone
                main.wait_stream(side)
            else:
                B.nanospec_calib_stream_read(Wd[(i + 7) % R], back_bytes, sink2, main.cuda_stream)
                B.nanospec_vocab_update(q0.h, d_new, offs[i % nsteps], None, None, main.cuda_stream)
                B.nanospec_packed_gather(q0.h, Wd[i % R], main.cuda_stream)
            B.nanospec_packed_head(q0.h, Hd[i % NH], M, logits, main.cuda_stream)
            B.nanospec_topk_remap(q0.h, logits, M, k, out_ids, out_vals, main.cuda_stream)

        def eager(overlap, count=100):
            ts = []
            for rep in range(5):
                init_q0()
                for i in range(8):
                    draft_step(i, overlap)
                torch.cuda.synchronize()
                e0.record(main)
                for i in range(8, 8 + count):
                    draft_step(i, overlap)
                e1.record(main)
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3 / count)
            return float(np.median(ts))
        back_us = train(lambda i, r, cs: B.nanospec_calib_stream_read(Wd[r % R], back_bytes, sink2, cs), 2 * ROT)
        seq_us, ovl_us = eager(False), eager(True)
        packed_variant = {"packed_head_us": round(packed_us, 2), "fused_gather_head_us": round(head_us, 2),
                          "update_plus_gather_us": round(ug_us, 2), "update_alone_us": round(u_us, 2),
                          "gather_us_per_step": round(ug_us - u_us, 2), "rows_copied_per_step": round(copied / nsteps, 2),
                          "standin_backbone_us": round(back_us, 1),
                          "draft_step_one_stream_us": round(seq_us, 1), "draft_step_gather_on_second_stream_us": round(ovl_us, 1),
                          "note": "draft step = stand-in backbone + update + gather + packed head + top-k, issued eagerly"}
        for q in pst:
            q.close()

    # Several sequences: the batch-union head (ids held by at least min_share sequences are fetched once and meet all
    # hidden rows, the others stay per sequence) against the per-sequence head, on the state the context leaves;
    # same cold rotation and timing.  build = the two list kernels, which need no hidden states.
    union_variant = None
    if Bn > 1 and not args.no_union:
        sweep = {}
        best = None
        for share in [int(x) for x in args.union_shares.split(",") if 0 < int(x) <= Bn]:
            su = B.State(V, d, Bn, seqs["window"], seqs["topk_cap"], M, k)
            B.nanospec_union_enable(su.h, share, 0)
            B.nanospec_vocab_init(su.h, d_ctx, coff, d_T0, toff, stream)
            B.nanospec_union_build(su.h, stream)
            sid, spos, rest, _, _ = su.read_union()
            uh = train(lambda i, r, cs: B.nanospec_union_head(su.h, Wd[r % R], Hd[r % NH], M, logits, cs), 2 * ROT)
            ub = train(lambda i, r, cs: B.nanospec_union_build(su.h, cs), 64)
            sweep[str(share)] = {"shared_rows": len(sid), "pairs_shared": int((spos >= 0).sum()),
                                 "pairs_per_sequence": int(sum(len(r[0]) for r in rest)), "head_us": round(uh, 2), "build_us": round(ub, 2)}
            if best is None or uh < best[1]:
                best = (share, uh, ub)
            su.close()
        s0 = B.State(V, d, Bn, seqs["window"], seqs["topk_cap"], M, k)
        B.nanospec_vocab_init(s0.h, d_ctx, coff, d_T0, toff, stream)
        base_us = train(lambda i, r, cs: B.nanospec_sparse_head(s0.h, Wd[r % R], Hd[r % NH], M, logits, cs), 2 * ROT)
        s0.close()
        union_variant = {"per_sequence_head_us": round(base_us, 2), "by_min_share": sweep, "best_min_share": best[0],
                         "best_head_us": round(best[1], 2), "best_head_plus_build_us": round(best[1] + best[2], 2),
                         "speedup_head": round(base_us / best[1], 3), "speedup_head_plus_build": round(base_us / (best[1] + best[2]), 3)}
        log("batch-union head timed")

    log("ceilings and packed-buffer variant timed")
    # the one-off stream initialisation (S(0) = context, T = T0; clear + apply kernels), on a scratch state
    st_i = B.State(V, d, Bn, seqs["window"], seqs["topk_cap"], M, k)
    init_us = train(lambda i, r, cs: B.nanospec_vocab_init(st_i.h, d_ctx, coff, d_T0, toff, cs), 16)
    st_i.close()

    # closed loop on the device (Eq. 3 for C_draft): every step feeds the previous step's top-k ids of all M
    # nodes back into the stream with nanospec_vocab_append_unique -- no host integers at all -- and the
    # selection returns log-probabilities renormalised over the active set (Sec. 4.2)
    def loop_step(i, r, cs):
        B.nanospec_vocab_append_unique(st.h, out_ids, M * k, M * k, cs)
        B.nanospec_sparse_head(st.h, Wd[r % R], Hd[r % NH], M, logits, cs)
        B.nanospec_topk_logprob_remap(st.h, logits, M, k, out_ids, out_vals, cs)

    def reset_loop():
        reset_main()
        for s_ in range(16):
            loop_step(s_, s_, stream)
    KL = 240
    loop_ms = timed(loop_step, 0, KL, reset=reset_loop)[0]
    app_us = train(lambda i, r, cs: B.nanospec_vocab_append_unique(st.h, out_ids, M * k, M * k, cs), reset=reset_loop)
    lp_us = train(lambda i, r, cs: B.nanospec_topk_logprob_remap(st.h, logits, M, k, out_ids, out_vals, cs))
    n_loop = [len(a) for a in st.read_active()]
    closed = {"steps_per_s": round(KL / (loop_ms * 1e-3), 1), "us_per_step": round(loop_ms * 1e3 / KL, 2),
              "append_unique_us": round(app_us, 2), "topk_logprob_us": round(lp_us, 2), "active_after": n_loop[0]}

    log("closed loop timed")
    # The two readings of the vocabulary side by side (Eq. 4 window over the raw stream against the first-in
    # first-out queue of distinct ids of Sec. 3.3 / the appendix): the same context and the same appended ids on
    # two fresh states, |active| afterwards and the time per update over a graph of the real updates.
    policy_compare = {}
    for name, pol in (("window", B.POLICY_WINDOW), ("fifo", B.POLICY_FIFO)):
        st2 = B.State(V, d, Bn, seqs["window"], seqs["topk_cap"], M, k)
        B.nanospec_set_stream_policy(st2.h, pol)
        B.nanospec_vocab_init(st2.h, d_ctx, coff, d_T0, toff, stream)
        n_init = [len(a) for a in st2.read_active()]
        upd = lambda i, r, cs: B.nanospec_vocab_update(st2.h, d_new, offs[i], None, None, cs)
        us = timed(upd, 0, total_steps, reset=lambda: B.nanospec_vocab_init(st2.h, d_ctx, coff, d_T0, toff, stream))[0] * 1e3 / total_steps
        n_end = [len(a) for a in st2.read_active()]
        policy_compare[name] = {"active_after_init": int(np.mean(n_init)), "active_after_updates": int(np.mean(n_end)),
                                "update_us": round(us, 2)}
        st2.close()

    log("vocabulary policies timed")
    # dense comparison point: full-vocabulary head + top-k over V.  The ratio that is reported takes the faster
    # of this library's dense head and the vendor GEMM library on the same product (bf16 out, through
    # torch.matmul, timed eagerly) as the dense head.
    dense = None
    if not args.no_dense:
        Mt = Bn * M
        dl = torch.empty((Mt, V), dtype=torch.float32, device="cuda")
        wsb = B.nanospec_dense_topk_workspace(V, Mt, k)
        ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
        di = torch.empty((Mt, k), dtype=torch.int32, device="cuda")
        dv = torch.empty((Mt, k), dtype=torch.float32, device="cuda")

        def dstep(i, r, cs):
            B.nanospec_dense_head(Wd[r % R], Hd[r % NH], V, d, Mt, dl, cs)
            B.nanospec_dense_topk(dl, V, Mt, k, di, dv, ws, wsb, cs)
        dense_us = train(dstep, 2 * ROT)
        dense_head_us = train(lambda i, r, cs: B.nanospec_dense_head(Wd[r % R], Hd[r % NH], V, d, Mt, dl, cs), 2 * ROT)
        Hflat = [h.reshape(Mt, d) for h in Hd]
        lib = []
        for rep in range(4):
            torch.cuda.synchronize()
            e0.record()
            for i in range(ROT):
                torch.matmul(Hflat[i % NH], Wd[i % R].t())
            e1.record()
            torch.cuda.synchronize()
            lib.append(e0.elapsed_time(e1) * 1e3 / ROT)
        lib_us = float(np.median(lib[1:]))
        step_us = ms * 1e3 / K
        best_dense_step = dense_us - dense_head_us + min(dense_head_us, lib_us)
        dense = {"step_us": round(dense_us, 2), "head_us": round(dense_head_us, 2), "library_gemm_us": round(lib_us, 2),
                 "head_GBps": round(V * d * 2 / (dense_head_us * 1e-6) / 1e9, 1),
                 "speedup_step": round(best_dense_step / step_us, 2),
                 "speedup_step_note": "dense step with the faster of this library's dense head and the vendor GEMM, over the sparse step",
                 "speedup_step_own_dense_kernels": round(dense_us / step_us, 2),
                 "speedup_head": round(min(dense_head_us, lib_us) / head_us, 2)}

    log("dense comparison timed")
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, seqs, W_host, synth)

    pmc_key = f"c5@{args.target}" if args.config == "c5" else args.config
    out = {
        "metric": "sparse-head draft steps/s + gathered HBM GB/s (V=128256,d=4096,|active|~3k)" if args.config == "c2"
                  else f"sparse-head draft steps/s + gathered HBM GB/s ({args.config})",
        "value": round(K / (ms * 1e-3), 1), "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms / K, 6), "timing": f"median of {REPS} timed repetitions of the K steps (min {min(ms_all) / K * 1e3:.2f}, max {max(ms_all) / K * 1e3:.2f} us/step), state restored before each", "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: V={V} d={d} batch={Bn} M={M} k={k} |active|={n_active[0]} "
                               f"window={seqs['window']} |T|={len(seqs['T0'][0])} accept={cfg['acc']}",
                   "replicas_of_W": R, "weights": "cold (rotated)" if R > 1 else "warm",
                   "launch": "hip graph replay" if use_graph else "eager"},
        "gathered_GBps": round(gathered, 1),
        "roofline": {"bound": "hbm", "kernel": "nanospec_sparse_head", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": float(args.traffic) if args.traffic else (
                         round(PMC_TRAFFIC_PER_ROW[pmc_key] * n_sum) if pmc_key in PMC_TRAFFIC_PER_ROW else None),
                     "traffic_source": "quoted, not measured by this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this "
                                       "command summarised under profiles/, scaled per active row",
                     "bytes_per_launch": roof_bytes, "us_per_launch": round(head_us, 3),
                     "bytes_note": None if Bn == 1 else f"distinct rows of the batch ({distinct_rows} of {n_sum} gathered): rows that "
                                                         "several sequences hold come from HBM once and from the caches afterwards"},
        "ceilings": ceilings, "cold_check": cold_check,
        "kernels_us": {"vocab_update": round(upd_us, 2), "sparse_head": round(head_us, 2), "topk_remap": round(topk_us, 2)},
        "vocab_init_us": round(init_us, 2),
        "closed_loop": closed,
        "packed_buffer_variant": packed_variant,
        "batch_union_head": union_variant,
        "vocabulary_policies": policy_compare,
        "dense": dense,
        "cpu_baseline": cpu,
        "setup_s": round(time.time() - t0, 1),
    }
    print(json.dumps(out))
    st.close()


def cpu_baseline(cfg, seqs, W_host, synth):
    """The oracle as it stands, timed on this host's cores over a bounded run of the same steps."""
    import oracle
    M, k, Bn = cfg["M"], cfg["k"], cfg["batch"]
    threads = oracle.max_threads()
    voc = [oracle.Vocab(cfg["V"], seqs["window"]) for _ in range(Bn)]
    for b in range(Bn):
        voc[b].init(seqs["ctx"][b], seqs["T0"][b])

    def one(s, omp=True):
        Hs = synth.make_H(cfg, s % 16)
        for b in range(Bn):
            Ts = seqs["T_step"][s % len(seqs["T_step"])]
            voc[b].update(seqs["appends"][s % len(seqs["appends"])][b], Ts[b] if Ts is not None else None)
            act = voc[b].active()
            z32, _ = oracle.head(W_host, Hs[b], ids=act, want64=False, omp=omp)
            for m in range(M):
                oracle.topk(z32[m], act, k)
    t = time.time()
    one(0)
    t1 = time.time() - t
    n = int(min(max(15.0 / max(t1, 1e-3), 3), 5000))
    t = time.time()
    for s in range(1, 1 + n):
        one(s)
    el = time.time() - t
    # the same steps on one thread (about 2 s of them), and the dense full-vocabulary head of one step once
    n1 = int(min(max(2.0 / max(t1 * threads, 1e-3), 1), 200))
    t = time.time()
    for s in range(1 + n, 1 + n + n1):
        one(s, omp=False)
    el1 = time.time() - t
    t = time.time()
    Hs = synth.make_H(cfg, 0)
    oracle.head(W_host, Hs[0], ids=None, want64=False, omp=True)
    dense_s = (time.time() - t) * Bn
    return {"value": round(n / el, 3), "unit": "steps/s", "cores": threads, "kind": "oracle",
            "sample": f"{n} consecutive steps of the same workload (vocabulary rebuild + fp32 head + full-sort "
                      f"top-k), OpenMP over active rows, {el:.1f} s",
            "single_thread_steps_per_s": round(n1 / el1, 3), "single_thread_sample_steps": n1,
            "dense_head_s_per_step": round(dense_s, 4)}


if __name__ == "__main__":
    main()
