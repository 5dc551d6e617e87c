"""CPU model of the address arithmetic of the head kernels' variants that load without bounds tests.

The sparse/dense head has kernel variants whose loads are unconditional: instead of testing every address they
clamp rows and columns into range and mask by arithmetic (csrc/head.hip: head_quad_kernel with row groups of four,
head_quad_private_kernel<FAST>, head_tile64_kernel<FAST 1 / 2>).  Whether that is safe depends on which variant the
launcher picks for which shape.  This file restates, in plain Python, (1) the launcher's selection and (2) every
element index each variant's lanes form for H [batch][M][d], W [V][d], the id list [batch][cap], the row counts
[batch] and the logits [batch][M][ld] (or the split-K planes), and asserts that all of them lie inside their
buffers over an enumeration of shapes.  A variant choice that once faulted on the GPU (constant hidden-row strides
taken with M = 32: wavefronts 2-3 addressed hidden rows 32..63 past the end of H) must be rejected by the model.
New unconditional-load variants go through this model before they go to the GPU."""
import itertools

import numpy as np
import pytest


class OutOfBounds(AssertionError):
    pass


def need(cond, *what):
    if not cond:
        raise OutOfBounds(what)


def ceil_div(a, b):
    return (a + b - 1) // b


# ---- the launcher's choice (mirror of launch_head_64 / run_quad_auto / run_quad_private / run_splitk) ----------
def plan(M, d, batch, cap, dense, partial_bytes=1 << 62):
    """list of (variant, params) one launch_head_64 call uses; M <= 64."""
    rows = cap * batch
    if M <= 16:
        if M <= 4:
            MT, KS = 1, 8
        elif M <= 8:
            MT, KS = 2, 8
        elif M <= 12:
            MT, KS = (3, 8) if 2048 < d <= 4096 else (3, 4)
        else:
            MT, KS = (4, 8) if 2048 < d <= 4096 else (4, 4)
        if d > 512 * KS:
            RT = 1 if rows <= 5 * 256 else (2 if (MT <= 2 or rows < 8192) else 4)
            return [("private", dict(RT=RT, MT=MT, KS=KS, NW=4, fast=d % (4 * 128 * KS) == 0))]
        if batch > 1 and rows >= 8192:
            NRG, RT = 2, 2
        elif rows > 8 * 256:
            NRG, RT = 4, 1
        elif rows > 4 * 256:
            NRG, RT = 2, 1
        else:
            NRG, RT = 1, 1
        return [("quad", dict(NRG=NRG, RT=RT, MT=MT, KS=KS))]
    S = ceil_div(d, 512)
    MT = 2 if M <= 32 else 4
    fast = 0 if d % 512 != 0 else (2 if M == 64 else 1)
    split = (not dense) and S >= 2 and S * batch * M * cap * 4 <= partial_bytes and rows <= 16384 and cap % 64 == 0
    return [("tile64", dict(MT=MT, fast=fast, split=split, S=S))]


# ---- the variants' index arithmetic ---------------------------------------------------------------------------
LANES = np.arange(64)
OROW, PART, Q = (LANES & 15) >> 2, LANES & 3, LANES >> 4


def check_quad(M, d, batch, cap, V, n, dense, NRG, RT, MT, KS, ld=None):
    ld = ld or (V if dense else cap)
    ROWS, RPG = 4 * RT * NRG, 4 * RT
    need(d <= 512 * KS, "quad needs one K-iteration")
    tiles = ceil_div(cap, ROWS)
    uncond = RT == 1
    HI = MT * KS
    HPW = ceil_div(HI, NRG)
    for b in (0, batch - 1):
        for tile in (0, tiles - 1):
            for w in range(4 * NRG):
                kq, rg = w & 3, w >> 2
                j0 = (tile * NRG + rg) * RPG
                if not dense:                                   # int4 loads of the ids, not waiting for n
                    need(j0 + 4 * RT <= cap, "ids", j0, cap)
                coff = kq * 128 * KS + Q * 32 + PART * 8
                for ii in range(HPW):
                    i = rg * HPW + ii
                    if uncond:
                        ic = min(i, HI - 1)
                        mt, t = ic // KS, ic % KS
                        m = np.minimum(mt * 4 + OROW, M - 1)
                        c = coff + t * 128
                        c = np.where(c < d, c, 0)
                        need(np.all((m >= 0) & (m < M)) and np.all(c + 8 <= d), "H", M, d, i)
                    # the predicated form tests i < HI, m < M, c < d before it loads
                live = j0 < n
                for t in range(KS):
                    c = coff + t * 128
                    if uncond:
                        c = np.where(live & (c < d), c, 0)
                        need(np.all(c + 8 <= d), "W col", d, t)  # rows are clamped into [0, V) or replaced by row 0
                # stores: j < n and m < M
                need(n <= cap <= ld or dense, "logit row stride")


def check_private(M, d, batch, cap, V, n, dense, RT, MT, KS, NW, fast):
    ROWS = 4 * RT
    tiles = ceil_div(cap, ROWS)
    if not dense:
        need(tiles * ROWS <= cap, "ids", cap, ROWS)             # int4 loads j0 .. j0 + 4*RT
    if not fast:
        return                                                  # the generic form tests c < d and m < M per load
    need(d % (NW * 128 * KS) == 0, "FAST needs whole K-iterations")
    for kb in range(0, d, NW * 128 * KS):
        for w in range(NW):
            coff = w * 128 * KS + Q * 32 + PART * 8
            for t in range(KS):
                need(np.all(kb + coff + t * 128 + 8 <= d), "col", d, kb, w, t)
    for mt in range(MT):
        m = np.minimum(mt * 4 + OROW, M - 1)
        need(np.all((m >= 0) & (m < M)), "H row")


def check_tile64(M, d, batch, cap, V, n, dense, MT, fast, split, S, partial_elems=None):
    if not dense:
        need(ceil_div(cap, 64) * 64 <= cap, "ids: one per lane up to the tile's end", cap)
    if fast:
        need(d % 512 == 0, "FAST needs whole slices")
        for sl in range(S):
            need(np.all(sl * 512 + LANES * 8 + 8 <= d), "col")
        for b in range(batch):
            for w in range(4):
                for r in range(16):
                    m = w * 16 + r
                    if fast == 1:
                        m = min(m, M - 1)
                    need(0 <= b * M + m < batch * M if fast == 1 else b * M + m < (b + 1) * M, "H row", M, w, r)
    if split:
        need(cap % 64 == 0 and cap % 4 == 0, "plane rows")
        # every live tile stores four consecutive logits per lane without looking at n: j0 + 15 < cap
        need(ceil_div(cap, 64) * 64 <= cap, "plane store")
        if partial_elems is not None:
            need(S * batch * M * cap <= partial_elems, "planes", S, batch, M, cap)


def check_shared(rows_total, seq_rows, d, cap_rows, opos_stride, nseq=None):
    """launch_head_shared: one id list for all sequences; hidden rows [rows_total][d] walked in groups of 64 (the last
    one shorter), column tables [nseq][opos_stride] looked up per hidden row at the end."""
    nseq = nseq if nseq is not None else ceil_div(rows_total, seq_rows)
    need(cap_rows >= 64 and cap_rows % 64 == 0 and opos_stride % 4 == 0, "list capacity", cap_rows, opos_stride)
    groups, tail = rows_total // 64, rows_total % 64
    launches = ([(0, groups, 64)] if groups else []) + ([(groups * 64, 1, tail)] if tail else [])
    for row0, nb, M in launches:
        fast = 0 if d % 512 != 0 else (2 if M == 64 else 1)
        check_tile64(M, d, nb, cap_rows, 1 << 30, cap_rows, False, MT=2 if M <= 32 else 4, fast=fast, split=False, S=ceil_div(d, 512))
        for b in (0, nb - 1):
            for m in range(M):                                 # rows the kernel stores for: m < M
                r = row0 + b * M + m
                need(r < rows_total, "hidden row", r, rows_total)
                q = r // seq_rows
                need(q < nseq, "sequence of a hidden row", q, nseq)
                for j in range(0, cap_rows, 4):
                    if j + 3 < opos_stride:                    # the kernel's own guard
                        need(q * opos_stride + j + 3 < nseq * opos_stride, "column table", q, j)


def wide_supported(M, d, batch, cap_rows):
    """mirror of the launcher's choice of the register-blocked product (csrc/wide.hip)"""
    if batch != 1 or M <= 16:
        return False
    if cap_rows >= 16384:
        return d % 128 == 0
    return M <= 64 and d % 512 == 0 and cap_rows >= (4096 if M <= 32 else 2560)


def check_wide(M, d, V, n, cap_rows, ld, ids_len=None):
    """head_wide_kernel (csrc/wide.hip): BM x BN blocks of logits, K in steps of BK, both operand blocks through LDS."""
    need(wide_supported(M, d, 1, cap_rows), "launcher's condition")
    if cap_rows < 16384:
        WR, WH, FR, FH, BK = 2, 2, 1, 1, 256
    else:
        WR, WH, FR, FH, BK = (4, 1, 2, 4, 64) if M <= 64 else ((4, 2, 4, 4, 64) if M <= 128 else (2, 4, 8, 4, 64))
    NT = 64 * WR * WH
    BM, BN = WR * FR * 16, WH * FH * 16
    CPR = BK // 8
    RPP = NT // CPR
    NA, NB = BM // RPP, BN // RPP
    STR = BK * 2 + 32
    STAGE = (BM + BN) * STR
    lds = 2 * STAGE
    need(lds <= 160 * 1024 and BM % RPP == 0 and BN % RPP == 0 and d % (2 * BK) == 0, "tile shape, an even number of steps")
    row_blocks, hid_blocks = ceil_div(cap_rows, BM), ceil_div(M, BN)
    grid = ceil_div(row_blocks, 8) * hid_blocks * 8
    seen = set()
    tid = np.arange(NT)
    pc, pr = tid % CPR, tid // CPR
    lane, w = tid & 63, tid >> 6
    wr, wh = w // WH, w % WH
    for blk in range(grid):
        xq, xr = blk & 7, blk >> 3
        hb, rb = xr % hid_blocks, (xr // hid_blocks) * 8 + xq
        if rb >= row_blocks:
            continue
        seen.add((rb, hb))
        if rb not in (0, row_blocks - 1, (n - 1) // BM if n else 0) or hb not in (0, hid_blocks - 1):
            continue
        j0, m0 = rb * BM, hb * BN
        if j0 >= n:
            continue
        for i in range(NA):
            j = j0 + pr + i * RPP
            if ids_len is not None:
                need(np.all(j[j < n] < ids_len), "ids", j.max(), ids_len)
            # rows are clamped into [0, V) or replaced by row 0; the column bytes:
            need(np.all(pc * 16 + (d // BK - 1) * BK * 2 + 16 <= d * 2), "W column")
            need(np.all((pr + i * RPP) * STR + pc * 16 + 16 <= BM * STR), "LDS park A")
        for i in range(NB):
            m = np.minimum(m0 + pr + i * RPP, M - 1)
            need(np.all((m >= 0) & (m < M)), "H row")
            need(np.all((pr + i * RPP) * STR + pc * 16 + 16 <= BN * STR), "LDS park B")
        frag = (lane & 15) * STR + (lane >> 4) * 16
        for kk in range(BK // 32):
            need(np.all((wr * FR * 16 + (FR - 1) * 16) * STR + frag + kk * 64 + 16 <= BM * STR), "LDS read A")
            need(np.all(BM * STR + (wh * FH * 16 + (FH - 1) * 16) * STR + frag + kk * 64 + 16 <= STAGE), "LDS read B")
        for a in range(FR):
            j = j0 + (wr * FR + a) * 16 + 4 * (lane >> 4)
            for b_ in range(FH):
                m = m0 + (wh * FH + b_) * 16 + (lane & 15)
                ok = (m < M) & (j < n)
                vec = ok & (ld % 4 == 0) & (j + 3 < n)
                need(np.all((m * ld + j + 3)[vec] < M * ld), "vector store")
                need(np.all((j + 3)[vec] < ld), "row end")
    need(seen == {(r, h) for r in range(row_blocks) for h in range(hid_blocks)}, "every block is visited once", len(seen))


def check(M, d, batch, cap, V, n, dense):
    if wide_supported(M, d, batch, cap):
        check_wide(M, d, V, n, cap, V if dense else cap, ids_len=None if dense else cap)
        return
    for variant, prm in plan(M, d, batch, cap, dense):
        if variant == "quad":
            check_quad(M, d, batch, cap, V, n, dense, **prm)
        elif variant == "private":
            check_private(M, d, batch, cap, V, n, dense, **prm)
        else:
            check_tile64(M, d, batch, cap, V, n, dense, **prm)


# ---- tests ----------------------------------------------------------------------------------------------------
def caps():
    return [64, 1472, 3776, 4352, 32064]


@pytest.mark.parametrize("d", [8, 64, 512, 520, 1024, 1032, 2048, 3584, 3592, 4096, 4104, 6144, 8192, 8200])
def test_every_selected_variant_stays_inside_its_buffers_sparse(d):
    for M, batch, cap in itertools.product((1, 3, 4, 5, 8, 9, 12, 13, 16, 17, 31, 32, 33, 48, 63, 64), (1, 2, 64), caps()):
        for n in (0, cap // 2 + 1, cap):
            check(M, d, batch, cap, 128256, n, dense=False)


@pytest.mark.parametrize("V", [50001, 128256, 152064])
def test_every_selected_variant_stays_inside_its_buffers_dense(V):
    for M, d in itertools.product((1, 4, 5, 8, 12, 16, 17, 32, 40, 64), (512, 520, 3584, 4096, 8192)):
        check(M, d, 1, V, V, V, dense=True)


def test_shared_list_launches_stay_inside_their_buffers():
    for nseq, seq_rows, d, cap_rows in itertools.product((1, 3, 6, 20, 30, 64), (1, 3, 5, 8, 16, 40), (64, 512, 1032, 4096), (64, 1472)):
        check_shared(nseq * seq_rows, seq_rows, d, cap_rows, cap_rows)
        check_shared(nseq * seq_rows, seq_rows, d, cap_rows, 64)          # a column table narrower than the list
    with pytest.raises(OutOfBounds):                                       # hidden rows counted per launch, not over the whole batch
        check_shared(160, 8, 4096, 64, 64, nseq=19)
    with pytest.raises(OutOfBounds):
        check_shared(160, 8, 4096, 96, 96)


@pytest.mark.parametrize("V", [16384, 50001, 128256, 152064])
def test_register_blocked_product_stays_inside_its_buffers(V):
    for M, d in itertools.product((17, 32, 64, 65, 70, 128, 129, 130, 256, 257, 512), (128, 3584, 4096, 8192)):
        check_wide(M, d, V, V, V, V)                                   # the dense head
        for n in (1, 127, 128, 129, 16384, V - 1):                     # a long id list of capacity V
            check_wide(M, d, V, n, V, V, ids_len=V)
    for M, d, cap in itertools.product((17, 32, 33, 48, 64), (512, 3584, 4096, 8192), (2560, 4096, 4352, 16320)):
        if wide_supported(M, d, 1, cap):
            for n in (0, 1, 31, 32, 33, cap // 2 + 1, cap):            # the 32 x 32 shape on a few thousand gathered rows
                check_wide(M, d, 152064, n, cap, cap, ids_len=cap)
    assert wide_supported(64, 3584, 1, 4352) and not wide_supported(64, 3584, 1, 2048) and not wide_supported(32, 3584, 1, 2560)
    assert not wide_supported(64, 3592, 1, 4352) and not wide_supported(64, 3584, 2, 4352) and not wide_supported(16, 4096, 1, 152064)
    with pytest.raises(OutOfBounds):
        check_wide(64, 3592, 152064, 152064, 152064, 152064)           # d not a whole number of steps
    with pytest.raises(OutOfBounds):
        check_wide(64, 4096, 20000, 20000, 20000, 19996)               # logits rows shorter than the row count


def test_the_selection_that_once_faulted_is_rejected():
    """constant hidden-row strides (the M == 64 form) taken with M = 32 and two sequences: the last sequence's
    wavefronts 2-3 would address hidden rows 32..63, past the end of H."""
    with pytest.raises(OutOfBounds):
        check_tile64(32, 8192, 2, 128, 20000, 70, False, MT=2, fast=2, split=True, S=16)
    check_tile64(32, 8192, 2, 128, 20000, 70, False, MT=2, fast=1, split=True, S=16)      # the clamped form is fine
    assert plan(32, 8192, 2, 128, False)[0][1]["fast"] == 1                               # and is what the launcher takes
    assert plan(64, 8192, 2, 128, False)[0][1]["fast"] == 2


def test_the_model_rejects_other_planted_mistakes():
    with pytest.raises(OutOfBounds):       # a K-loop kernel's FAST form on a hidden size that is not a whole K-iteration
        check_private(16, 8200, 1, 1472, 128256, 1000, False, RT=1, MT=4, KS=4, NW=4, fast=True)
    with pytest.raises(OutOfBounds):       # whole-slice loads on d % 512 != 0
        check_tile64(64, 3592, 1, 4352, 152064, 3000, False, MT=4, fast=2, split=True, S=8)
    with pytest.raises(OutOfBounds):       # an id list whose capacity is not a whole number of row groups
        check_private(8, 8192, 1, 1470, 128256, 1000, False, RT=2, MT=2, KS=8, NW=4, fast=True)
    with pytest.raises(OutOfBounds):       # split-K planes larger than the workspace
        check_tile64(64, 3584, 1, 4352, 152064, 3000, False, MT=4, fast=2, split=True, S=7, partial_elems=1000)
