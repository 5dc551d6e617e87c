"""The allocation-free selection entry point against the workspace-taking one it is a variant of."""
import ctypes as C

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2605_26444_amd import binding as B
from paper_2605_26444_amd import synth

pytestmark = pytest.mark.gpu


def _logits(seed, M, V):
    # distinct values with some exact ties: quantised uniforms
    u = synth.rand_unit(seed, 7, 0, M * V).reshape(M, V)
    return np.round(u * 50000.0).astype(np.float32) / 64.0


def _both(seed, M, V, k):
    z = torch.from_numpy(_logits(seed, M, V)).cuda()
    wsb = B.nanospec_dense_topk_workspace(V, M, k)
    ws = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    ri = torch.empty((M, k), dtype=torch.int32, device="cuda")
    rv = torch.empty((M, k), dtype=torch.float32, device="cuda")
    B.nanospec_dense_topk(z, V, M, k, ri, rv, ws, wsb)
    si = torch.full((M, k), -7, dtype=torch.int32, device="cuda")
    sv = torch.full((M, k), float("nan"), dtype=torch.float32, device="cuda")
    # straight through the C ABI
    rc = B.lib().nanospec_dense_topk_static(C.c_void_p(z.data_ptr()), V, M, k, C.c_void_p(si.data_ptr()),
                                           C.c_void_p(sv.data_ptr()), C.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == B.OK
    torch.cuda.synchronize()
    assert np.array_equal(si.cpu().numpy(), ri.cpu().numpy()), (M, V, k)
    assert np.array_equal(sv.cpu().numpy(), rv.cpu().numpy()), (M, V, k)
    # and the ids are the k largest by (value descending, index ascending)
    zz = z.cpu().numpy()
    for m in range(M):
        order = np.lexsort((np.arange(V), -zz[m]))[:k]
        assert np.array_equal(si.cpu().numpy()[m], order.astype(np.int32))


def test_static_selection_matches_workspace_selection_two_calls_in_a_row():
    _both(11, 9, 100000, 10)          # 7 chunks per row through the library's own array
    _both(12, 3, 40000, 5)            # a smaller call right after: older candidates stay in the array, unread
    _both(13, 2, 9000, 64)            # single-pass shape (the array is not touched)


def test_static_selection_rejects_what_does_not_fit():
    lim = B.nanospec_dense_topk_static_limit()
    assert lim == 4 << 20
    V, k = 128256, 10
    rows = 1
    while B.nanospec_dense_topk_workspace(V, rows, k) <= lim:
        rows *= 2
    z = torch.zeros(8, dtype=torch.float32, device="cuda")     # never read: the call is refused on the host
    o = torch.zeros(8, dtype=torch.int32, device="cuda")
    with pytest.raises(B.NanoSpecError) as e:
        B.nanospec_dense_topk_static(z, V, rows, k, o, None)
    assert e.value.status == B.ECAPACITY
