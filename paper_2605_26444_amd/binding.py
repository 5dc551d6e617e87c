"""ctypes binding of libnanospec.so -- argument marshalling only.

Function names mirror the C ABI declared in include/nanospec.h.  Tensors are torch CUDA(HIP)
tensors used purely as device memory; every step of the hot path runs inside the library's HIP
kernels.  There is no CPU fallback: if the shared library is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libnanospec.so")

OK, EINVAL, ENOMEM, ECAPACITY, EHIP = 0, -1, -2, -3, -4
POLICY_WINDOW, POLICY_FIFO = 0, 1
DEV_BAD_ID = 1
MAX_BATCH = 256

EXPORTS = [
    "nanospec_status_string", "nanospec_state_layout", "nanospec_create", "nanospec_destroy",
    "nanospec_set_stream_policy", "nanospec_vocab_init", "nanospec_vocab_update", "nanospec_vocab_append_unique", "nanospec_vocab_view", "nanospec_sparse_head",
    "nanospec_topk_remap", "nanospec_topk_logprob_remap", "nanospec_dense_head", "nanospec_dense_topk_workspace", "nanospec_dense_topk",
    "nanospec_dense_topk_static_limit", "nanospec_dense_topk_static",
    "nanospec_packed_bytes", "nanospec_packed_enable", "nanospec_packed_gather", "nanospec_packed_head", "nanospec_packed_view",
    "nanospec_union_bytes", "nanospec_union_enable", "nanospec_union_build", "nanospec_union_head", "nanospec_union_view",
    "nanospec_calib_stream_read", "nanospec_calib_gather_read", "nanospec_calib_valu_head", "nanospec_last_device_error",
]


class Layout(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "ring_bytes", "counter_bytes", "window_bitmap_bytes", "topk_bitmap_bytes", "ids_bytes", "scalars_bytes",
        "workspace_bytes", "total_bytes", "gathered_bytes_at_cap")] + [("capacity", C.c_int32)]


class NanoSpecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib() -> C.CDLL:
    """Load libnanospec.so (built in-tree by paper_2605_26444_amd.build); fail loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2605_26444_amd.build` (no fallback exists)")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        i32p = C.POINTER(C.c_int32)
        L.nanospec_status_string.restype = C.c_char_p
        L.nanospec_status_string.argtypes = [i32]
        L.nanospec_state_layout.argtypes = [i32] * 7 + [C.POINTER(Layout)]
        L.nanospec_create.argtypes = [C.POINTER(vp)] + [i32] * 7
        L.nanospec_destroy.argtypes = [vp]
        L.nanospec_set_stream_policy.argtypes = [vp, i32]
        L.nanospec_vocab_init.argtypes = [vp, vp, i32p, vp, i32p, vp]
        L.nanospec_vocab_update.argtypes = [vp, vp, i32p, vp, i32p, vp]
        L.nanospec_vocab_append_unique.argtypes = [vp, vp, i32, i64, vp]
        L.nanospec_vocab_view.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), i32p]
        L.nanospec_sparse_head.argtypes = [vp, vp, vp, i32, vp, vp]
        L.nanospec_topk_remap.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.nanospec_topk_logprob_remap.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        L.nanospec_calib_stream_read.argtypes = [vp, i64, vp, vp]
        L.nanospec_calib_gather_read.argtypes = [vp, vp, vp, vp]
        L.nanospec_calib_valu_head.argtypes = [vp, vp, vp, i32, vp, vp]
        L.nanospec_dense_head.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        L.nanospec_dense_topk_workspace.restype = i64
        L.nanospec_dense_topk_workspace.argtypes = [i32, i32, i32]
        L.nanospec_dense_topk.argtypes = [vp, i32, i32, i32, vp, vp, vp, i64, vp]
        L.nanospec_dense_topk_static_limit.restype = i64
        L.nanospec_dense_topk_static_limit.argtypes = []
        L.nanospec_dense_topk_static.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.nanospec_packed_bytes.restype = i64
        L.nanospec_packed_bytes.argtypes = [vp]
        L.nanospec_packed_enable.argtypes = [vp]
        L.nanospec_packed_gather.argtypes = [vp, vp, vp]
        L.nanospec_packed_head.argtypes = [vp, vp, i32, vp, vp]
        L.nanospec_packed_view.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
        L.nanospec_union_bytes.restype = i64
        L.nanospec_union_bytes.argtypes = [vp, i32]
        L.nanospec_union_enable.argtypes = [vp, i32, i32]
        L.nanospec_union_build.argtypes = [vp, vp]
        L.nanospec_union_head.argtypes = [vp, vp, vp, i32, vp, vp]
        L.nanospec_union_view.argtypes = [vp] + [C.POINTER(vp)] * 6 + [i32p, i32p]
        L.nanospec_last_device_error.argtypes = [vp, i32p, vp]
        for name in EXPORTS:
            if name not in ("nanospec_status_string", "nanospec_dense_topk_workspace", "nanospec_dense_topk_static_limit",
                            "nanospec_packed_bytes", "nanospec_union_bytes"):
                getattr(L, name).restype = i32
        _lib = L
    return _lib


def status_string(s: int) -> str:
    return lib().nanospec_status_string(s).decode()


def _check(rc: int, where: str):
    if rc != OK:
        raise NanoSpecError(rc, where)


def _ptr(t):
    """device pointer of a torch tensor (or None / int passthrough)."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA/HIP tensors"
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream if isinstance(stream, int) else stream.cuda_stream


def _off(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int32))


def nanospec_state_layout(V, d, batch, window, topk_cap, m_cap, k_cap) -> Layout:
    out = Layout()
    _check(lib().nanospec_state_layout(V, d, batch, window, topk_cap, m_cap, k_cap, C.byref(out)), "nanospec_state_layout")
    return out


def nanospec_create(V, d, batch, window, topk_cap, m_cap, k_cap) -> int:
    h = C.c_void_p()
    _check(lib().nanospec_create(C.byref(h), V, d, batch, window, topk_cap, m_cap, k_cap), "nanospec_create")
    return h.value


def nanospec_destroy(st: int):
    _check(lib().nanospec_destroy(st), "nanospec_destroy")


def nanospec_set_stream_policy(st, policy):
    _check(lib().nanospec_set_stream_policy(st, policy), "nanospec_set_stream_policy")


def nanospec_vocab_init(st, d_ctx_ids, h_ctx_off, d_topk_ids, h_topk_off, stream=None):
    a, ap = _off(h_ctx_off)
    b, bp = _off(h_topk_off)
    _check(lib().nanospec_vocab_init(st, _ptr(d_ctx_ids), ap, _ptr(d_topk_ids), bp, _stream(stream)), "nanospec_vocab_init")


def nanospec_vocab_update(st, d_new_ids, h_new_off, d_topk_ids=None, h_topk_off=None, stream=None):
    a, ap = _off(h_new_off)
    b, bp = _off(h_topk_off)
    _check(lib().nanospec_vocab_update(st, _ptr(d_new_ids), ap, _ptr(d_topk_ids), bp, _stream(stream)), "nanospec_vocab_update")


def nanospec_vocab_append_unique(st, d_cand_ids, cand_per_seq, cand_stride=None, stream=None):
    stride = cand_per_seq if cand_stride is None else cand_stride
    _check(lib().nanospec_vocab_append_unique(st, _ptr(d_cand_ids), cand_per_seq, stride, _stream(stream)),
           "nanospec_vocab_append_unique")


def nanospec_vocab_view(st):
    """(ids_ptr, n_ptr, capacity): raw device addresses borrowed from the state."""
    ids, n, cap = C.c_void_p(), C.c_void_p(), C.c_int32()
    _check(lib().nanospec_vocab_view(st, C.byref(ids), C.byref(n), C.byref(cap)), "nanospec_vocab_view")
    return ids.value, n.value, cap.value


def nanospec_sparse_head(st, d_W, d_H, M, d_logits, stream=None):
    _check(lib().nanospec_sparse_head(st, _ptr(d_W), _ptr(d_H), M, _ptr(d_logits), _stream(stream)), "nanospec_sparse_head")


def nanospec_topk_remap(st, d_logits, M, k, d_out_ids, d_out_vals=None, stream=None):
    _check(lib().nanospec_topk_remap(st, _ptr(d_logits), M, k, _ptr(d_out_ids), _ptr(d_out_vals), _stream(stream)),
           "nanospec_topk_remap")


def nanospec_topk_logprob_remap(st, d_logits, M, k, d_out_ids, d_out_logprob, stream=None):
    _check(lib().nanospec_topk_logprob_remap(st, _ptr(d_logits), M, k, _ptr(d_out_ids), _ptr(d_out_logprob),
                                             _stream(stream)), "nanospec_topk_logprob_remap")


def nanospec_calib_stream_read(d_buf, nbytes, d_sink, stream=None):
    if not isinstance(d_buf, int) and nbytes > d_buf.numel() * d_buf.element_size():      # the library cannot know the buffer's size
        raise ValueError(f"nanospec_calib_stream_read: {nbytes} bytes asked of a buffer of {d_buf.numel() * d_buf.element_size()}")
    _check(lib().nanospec_calib_stream_read(_ptr(d_buf), nbytes, _ptr(d_sink), _stream(stream)), "nanospec_calib_stream_read")


def nanospec_calib_gather_read(st, d_W, d_sink, stream=None):
    _check(lib().nanospec_calib_gather_read(st, _ptr(d_W), _ptr(d_sink), _stream(stream)), "nanospec_calib_gather_read")


def nanospec_calib_valu_head(st, d_W, d_H, M, d_logits, stream=None):
    _check(lib().nanospec_calib_valu_head(st, _ptr(d_W), _ptr(d_H), M, _ptr(d_logits), _stream(stream)), "nanospec_calib_valu_head")


def nanospec_dense_head(d_W, d_H, V, d, M_total, d_logits, stream=None):
    _check(lib().nanospec_dense_head(_ptr(d_W), _ptr(d_H), V, d, M_total, _ptr(d_logits), _stream(stream)),
           "nanospec_dense_head")


def nanospec_dense_topk_workspace(V, M_total, k) -> int:
    return int(lib().nanospec_dense_topk_workspace(V, M_total, k))


def nanospec_dense_topk(d_logits, V, M_total, k, d_out_ids, d_out_vals, d_workspace, workspace_bytes, stream=None):
    _check(lib().nanospec_dense_topk(_ptr(d_logits), V, M_total, k, _ptr(d_out_ids), _ptr(d_out_vals), _ptr(d_workspace),
                                     workspace_bytes, _stream(stream)), "nanospec_dense_topk")


def nanospec_dense_topk_static_limit() -> int:
    return int(lib().nanospec_dense_topk_static_limit())


def nanospec_dense_topk_static(d_logits, V, M_total, k, d_out_ids, d_out_vals, stream=None):
    _check(lib().nanospec_dense_topk_static(_ptr(d_logits), V, M_total, k, _ptr(d_out_ids), _ptr(d_out_vals),
                                            _stream(stream)), "nanospec_dense_topk_static")


def nanospec_packed_bytes(st) -> int:
    return int(lib().nanospec_packed_bytes(st))


def nanospec_packed_enable(st):
    _check(lib().nanospec_packed_enable(st), "nanospec_packed_enable")


def nanospec_packed_gather(st, d_W, stream=None):
    _check(lib().nanospec_packed_gather(st, _ptr(d_W), _stream(stream)), "nanospec_packed_gather")


def nanospec_packed_head(st, d_H, M, d_logits, stream=None):
    _check(lib().nanospec_packed_head(st, _ptr(d_H), M, _ptr(d_logits), _stream(stream)), "nanospec_packed_head")


def nanospec_packed_view(st):
    """(buf_ptr, slot_id_ptr, out_pos_ptr, counts_ptr): raw device addresses borrowed from the state."""
    a, b, c, d = C.c_void_p(), C.c_void_p(), C.c_void_p(), C.c_void_p()
    _check(lib().nanospec_packed_view(st, C.byref(a), C.byref(b), C.byref(c), C.byref(d)), "nanospec_packed_view")
    return a.value, b.value, c.value, d.value


def nanospec_union_bytes(st, shared_cap=0) -> int:
    return int(lib().nanospec_union_bytes(st, shared_cap))


def nanospec_union_enable(st, min_share=0, shared_cap=0):
    _check(lib().nanospec_union_enable(st, min_share, shared_cap), "nanospec_union_enable")


def nanospec_union_build(st, stream=None):
    _check(lib().nanospec_union_build(st, _stream(stream)), "nanospec_union_build")


def nanospec_union_head(st, d_W, d_H, M, d_logits, stream=None):
    _check(lib().nanospec_union_head(st, _ptr(d_W), _ptr(d_H), M, _ptr(d_logits), _stream(stream)), "nanospec_union_head")


def nanospec_union_view(st):
    """(shared_ids, shared_n, shared_pos, rest_ids, rest_pos, rest_n: raw device addresses; shared_cap, min_share)."""
    ptrs = [C.c_void_p() for _ in range(6)]
    cap, share = C.c_int32(), C.c_int32()
    _check(lib().nanospec_union_view(st, *[C.byref(x) for x in ptrs], C.byref(cap), C.byref(share)), "nanospec_union_view")
    return tuple(x.value for x in ptrs) + (cap.value, share.value)


def nanospec_last_device_error(st, stream=None) -> int:
    f = C.c_int32()
    _check(lib().nanospec_last_device_error(st, C.byref(f), _stream(stream)), "nanospec_last_device_error")
    return f.value


class State:
    """Owns one nanospec_state; convenience for tests and the benchmark (still marshalling only)."""

    def __init__(self, V, d, batch, window, topk_cap, m_cap, k_cap):
        self.V, self.d, self.batch, self.window, self.topk_cap, self.m_cap, self.k_cap = V, d, batch, window, topk_cap, m_cap, k_cap
        self.h = nanospec_create(V, d, batch, window, topk_cap, m_cap, k_cap)
        self.ids_ptr, self.n_ptr, self.capacity = nanospec_vocab_view(self.h)

    def close(self):
        if getattr(self, "h", None):
            nanospec_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def read_packed(self):
        """host copies of the packed-buffer tables: (slot ids int32[capacity], logit columns int32[capacity],
        slots that may hold a row, rows copied by the last gather, row buffer as uint16 [capacity][d])."""
        import torch
        torch.cuda.synchronize()
        buf, sid, pos, cnt = nanospec_packed_view(self.h)
        c = _copy_from_device(cnt, 2, np.int32)
        return (_copy_from_device(sid, self.capacity, np.int32), _copy_from_device(pos, self.capacity, np.int32), int(c[0]), int(c[1]),
                _copy_from_device(buf, self.capacity * self.d, np.uint16).reshape(self.capacity, self.d))

    def read_union(self):
        """host copies of the batch-union lists: (shared ids int32[P], shared_pos int32[batch][P],
        [(rest ids, rest columns) per sequence], min_share, shared_cap)."""
        import torch
        torch.cuda.synchronize()
        sid, sn, spos, rid, rpos, rn, cap, share = nanospec_union_view(self.h)
        P = int(_copy_from_device(sn, 1, np.int32)[0])
        ids = _copy_from_device(sid, cap, np.int32)[:P]
        pos = _copy_from_device(spos, self.batch * cap, np.int32).reshape(self.batch, cap)[:, :P]
        n = _copy_from_device(rn, self.batch, np.int32)
        ri = _copy_from_device(rid, self.batch * self.capacity, np.int32).reshape(self.batch, self.capacity)
        rp = _copy_from_device(rpos, self.batch * self.capacity, np.int32).reshape(self.batch, self.capacity)
        return ids, pos, [(ri[b, :n[b]].copy(), rp[b, :n[b]].copy()) for b in range(self.batch)], share, cap

    def read_active(self):
        """copy the active id lists back to the host: list of int32 arrays (one per sequence)."""
        import torch
        torch.cuda.synchronize()
        n = _copy_from_device(self.n_ptr, self.batch, np.int32)
        ids = _copy_from_device(self.ids_ptr, self.batch * self.capacity, np.int32).reshape(self.batch, self.capacity)
        return [ids[b, :n[b]].copy() for b in range(self.batch)]


def _copy_from_device(ptr: int, count: int, dtype):
    """host copy of `count` items at raw device address ptr (through hipMemcpy of the HIP runtime)."""
    hip = C.CDLL("libamdhip64.so")
    out = np.empty(count, dtype=dtype)
    hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
    rc = hip.hipMemcpy(out.ctypes.data, ptr, out.nbytes, 2)
    if rc != 0:
        raise RuntimeError(f"hipMemcpy failed: {rc}")
    return out
