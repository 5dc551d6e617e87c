"""CPU-side checks: the C-ABI library loads, exports what include/nanospec.h declares, and its
host-only layout arithmetic reproduces the buffer sizes the paper prints (Table 6)."""
import ctypes as C
import os
import re

import pytest

from paper_2605_26444_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2605_26444_amd import build
        build.build()
    return B.lib()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "nanospec.h")).read()
    declared = set(re.findall(r"NANOSPEC_API[^;(]*?\b(nanospec_\w+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    assert B.status_string(B.OK) == "ok"
    assert "capacity" in B.status_string(B.ECAPACITY)


def test_layout_matches_paper_table6(lib):
    """Table 6 (Llama-3.1-8B, d=4096, W_max=3072): token set index 16 KB, token buffer 12 KB,
    repacked weights 24.00 MB."""
    L = B.nanospec_state_layout(128256, 4096, 1, 3072, 0, 8, 10)
    assert L.window_bitmap_bytes == (128256 + 31) // 32 * 4 == 16032           # "16 KB"
    assert round(L.window_bitmap_bytes / 1024) == 16
    assert L.ring_bytes == 3072 * 4 == 12 * 1024                               # "12 KB"
    assert L.gathered_bytes_at_cap == 3072 * 4096 * 2 == 24 * 1024 * 1024      # "24.00 MB"
    assert L.capacity == 3072
    assert L.counter_bytes == 128256 * 4
    # the state is O(1) in the sequence length and linear in the batch (Sec. 4.6)
    L2 = B.nanospec_state_layout(128256, 4096, 2, 3072, 0, 8, 10)
    assert L2.ring_bytes == L.ring_bytes and L2.total_bytes > L.total_bytes


def test_layout_rejects_bad_shapes(lib):
    for args in [(0, 8, 1, 1, 0, 1, 1), (10, 12, 1, 1, 0, 1, 1), (10, 8, 0, 1, 0, 1, 1), (10, 8, 1, 0, 0, 1, 1),
                 (10, 8, 1, 1, -1, 1, 1), (10, 8, 1, 1, 0, 0, 1), (10, 8, 1, 1, 0, 1, 65), (10, 8, 257, 1, 0, 1, 1)]:
        out = B.Layout()
        assert lib.nanospec_state_layout(*args, C.byref(out)) == B.EINVAL
    assert lib.nanospec_state_layout(10, 8, 1, 1, 0, 1, 1, None) == B.EINVAL
    assert lib.nanospec_dense_topk_workspace(0, 1, 1) == -1


def test_capacity_is_bounded_by_vocabulary(lib):
    L = B.nanospec_state_layout(100, 8, 1, 5000, 300, 1, 1)
    assert L.capacity == 128                                                   # min(window+topk_cap, V) -> 64-multiple


def test_layout_rejects_vocabularies_beyond_the_lds_limit():
    import ctypes as C
    L = B.lib()
    lay = B.Layout()
    assert L.nanospec_state_layout(420000, 4096, 1, 1024, 2727, 8, 10, C.byref(lay)) == B.OK
    assert L.nanospec_state_layout(430000, 4096, 1, 1024, 2727, 8, 10, C.byref(lay)) == B.EINVAL
    assert L.nanospec_state_layout(128256, 4096, 1, 300000, 0, 8, 10, C.byref(lay)) == B.OK         # capacity clamps to V
    assert L.nanospec_state_layout(400000, 4096, 1, 300000, 0, 8, 10, C.byref(lay)) == B.EINVAL     # > 16 top-k chunks
