"""Python binding of libhop.so, the MI355X chunked N-way reduce library.

Argument marshalling only: every function here turns tensors and lists into
the pointers and sizes of the C ABI declared in include/hop.h and calls it.
PyTorch provides device memory and streams, nothing else. There is no CPU
fallback: if the library has not been built, importing its symbols fails.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch  # imported before libhop.so so that both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libhop.so")

HOP_SUM, HOP_MIN, HOP_MAX = 0, 1, 2
HOP_F32, HOP_BF16, HOP_I32 = 0, 1, 2
HOP_OK, HOP_PARTIAL = 0, 1
HOP_ERR_INVALID, HOP_ERR_ALIGN, HOP_ERR_NO_SURVIVOR = -1, -2, -3
HOP_ERR_DEVICE, HOP_ERR_NOMEM, HOP_ERR_DEPTH, HOP_ERR_TOO_LARGE, HOP_ERR_CAPTURE = -4, -5, -6, -7, -8
HOP_MAX_DEPTH = 16

OPS = {"sum": HOP_SUM, "min": HOP_MIN, "max": HOP_MAX}
DTYPES = {"f32": HOP_F32, "bf16": HOP_BF16, "i32": HOP_I32,
          torch.float32: HOP_F32, torch.bfloat16: HOP_BF16, torch.int32: HOP_I32}

EXPORTS = ["hop_reduce", "hop_reduce_noalloc", "hop_noalloc_scratch_bytes", "hop_broadcast", "hop_allreduce", "hop_bcast_begin", "hop_bcast_source_ready",
           "hop_bcast_join", "hop_bcast_fail", "hop_bcast_step", "hop_bcast_sender", "hop_bcast_finish", "hop_session_begin", "hop_session_ready", "hop_session_ready_after",
           "hop_session_fail", "hop_session_finish", "hop_session_set_eager", "hop_session_set_adaptive", "hop_session_set_retention", "hop_session_set_workspace", "hop_session_chunks_final",
           "hop_plan_session_begin", "hop_plan_session_finish", "hop_plan_reduce", "hop_plan_split", "hop_plan_chains", "hop_plan_slots",
           "hop_pick_degree", "hop_calibrate", "hop_workspace_bytes", "hop_shutdown", "hop_strerror", "hop_kernel_config"]


class HopInfo(ctypes.Structure):
    _fields_ = [("k_eff", ctypes.c_int32), ("n_failed_seen", ctypes.c_int32),
                ("n_replaced", ctypes.c_int32), ("degree_used", ctypes.c_int32),
                ("chunks_redone", ctypes.c_int64), ("n_launches", ctypes.c_int32),
                ("stack_depth", ctypes.c_int32), ("chunk_steps", ctypes.c_int64), ("chunk_stores", ctypes.c_int64),
                ("partial_loads", ctypes.c_int64), ("partial_stores", ctypes.c_int64)]

    def as_dict(self):
        return {"k_eff": self.k_eff, "n_failed_seen": self.n_failed_seen, "n_replaced": self.n_replaced,
                "degree_used": self.degree_used, "chunks_redone": self.chunks_redone, "n_launches": self.n_launches,
                "stack_depth": self.stack_depth, "chunk_steps": self.chunk_steps, "chunk_stores": self.chunk_stores,
                "partial_loads": self.partial_loads, "partial_stores": self.partial_stores}


class BcastCopy(ctypes.Structure):
    _fields_ = [("from_", ctypes.c_int32), ("to", ctypes.c_int32), ("chunk_begin", ctypes.c_int64),
                ("chunk_end", ctypes.c_int64)]


class BcastInfo(ctypes.Structure):
    _fields_ = [("n_receivers", ctypes.c_int32), ("n_failed", ctypes.c_int32), ("n_resumed", ctypes.c_int32),
                ("n_complete", ctypes.c_int32), ("chunks_copied", ctypes.c_int64)]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_}


class PlanEntry(ctypes.Structure):
    _fields_ = [("obj", ctypes.c_int32), ("level", ctypes.c_uint8), ("set", ctypes.c_uint8),
                ("n_fold", ctypes.c_uint16), ("save", ctypes.c_int16), ("save_level", ctypes.c_uint8),
                ("reserved", ctypes.c_uint8)]

    def __init__(self, obj=0, level=0, set=0, n_fold=0, save=-1, save_level=0):
        super().__init__(obj, level, set, n_fold, save, save_level, 0)


class PlanLaunch(ctypes.Structure):
    _fields_ = [("chunk_begin", ctypes.c_int64), ("chunk_end", ctypes.c_int64),
                ("entry_begin", ctypes.c_int32), ("entry_end", ctypes.c_int32),
                ("step_begin", ctypes.c_int32), ("step_end", ctypes.c_int32),
                ("final", ctypes.c_int32), ("live_before", ctypes.c_int32), ("live_after", ctypes.c_int32),
                ("reserved", ctypes.c_int32)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C library. Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libhop.so is missing: build it with "
                               "`python -m paper_2002_05814_amd.build` (hipcc, gfx950)")
        L = ctypes.CDLL(LIB_PATH)
        vp, vpp = ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)
        i32p, i64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        infop = ctypes.POINTER(HopInfo)
        L.hop_reduce.argtypes = [vp, vpp, ctypes.c_int, ctypes.c_size_t, i32p, ctypes.c_int, ctypes.c_int,
                                 ctypes.c_int, ctypes.c_size_t, ctypes.c_int, i64p, vp, infop]
        L.hop_reduce_noalloc.argtypes = L.hop_reduce.argtypes
        L.hop_noalloc_scratch_bytes.argtypes = []
        L.hop_noalloc_scratch_bytes.restype = ctypes.c_size_t
        L.hop_broadcast.argtypes = [vpp, ctypes.c_int, vp, ctypes.c_size_t, ctypes.c_size_t, vp]
        L.hop_allreduce.argtypes = [vpp, ctypes.c_int, vpp, ctypes.c_int, ctypes.c_size_t, i32p, ctypes.c_int,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, i64p, vp, infop]
        L.hop_bcast_begin.argtypes = [ctypes.POINTER(vp), vp, ctypes.c_size_t, ctypes.c_size_t, vp]
        L.hop_bcast_source_ready.argtypes = [vp, ctypes.c_int64]
        L.hop_bcast_join.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int)]
        L.hop_bcast_fail.argtypes = [vp, ctypes.c_int]
        L.hop_bcast_step.argtypes = [vp, ctypes.c_int64]
        L.hop_bcast_sender.argtypes = [vp, ctypes.c_int]
        L.hop_bcast_finish.argtypes = [vp, ctypes.POINTER(BcastInfo), ctypes.POINTER(BcastCopy), ctypes.c_int,
                                       ctypes.POINTER(ctypes.c_int)]
        L.hop_session_begin.argtypes = [ctypes.POINTER(vp), vp, vpp, ctypes.c_int, ctypes.c_size_t, ctypes.c_int,
                                        ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_int, vp]
        L.hop_session_ready.argtypes = [vp, ctypes.c_int, ctypes.c_int64]
        L.hop_session_ready_after.argtypes = [vp, ctypes.c_int, ctypes.c_int64, vp]
        L.hop_session_fail.argtypes = [vp, ctypes.c_int]
        L.hop_session_finish.argtypes = [vp, infop]
        L.hop_session_set_eager.argtypes = [vp, ctypes.c_int]
        L.hop_session_set_adaptive.argtypes = [vp, ctypes.c_int]
        L.hop_session_set_retention.argtypes = [vp, ctypes.c_int]
        L.hop_session_set_workspace.argtypes = [vp, vp, ctypes.c_size_t]
        L.hop_session_chunks_final.argtypes = [vp]
        L.hop_session_chunks_final.restype = ctypes.c_int64
        L.hop_plan_session_begin.argtypes = [ctypes.POINTER(vp), ctypes.c_int, ctypes.c_size_t, ctypes.c_int,
                                             ctypes.c_int, ctypes.c_size_t, ctypes.c_int]
        L.hop_plan_session_finish.argtypes = [vp, infop, ctypes.POINTER(PlanLaunch), ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_int), ctypes.POINTER(PlanEntry), ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_int)]
        L.hop_plan_reduce.argtypes = [ctypes.c_int, ctypes.c_size_t, i32p, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_size_t, ctypes.c_int, i64p, infop,
                                      ctypes.POINTER(PlanLaunch), ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                      ctypes.POINTER(PlanEntry), ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
        L.hop_plan_split.argtypes = [ctypes.POINTER(PlanEntry), ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.POINTER(PlanEntry), ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                     ctypes.POINTER(PlanEntry), ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                     i32p, i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_int),
                                     ctypes.POINTER(ctypes.c_int)]
        L.hop_plan_chains.argtypes = [ctypes.POINTER(PlanEntry), ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_int), i32p, i32p, ctypes.c_int,
                                      ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.hop_plan_slots.argtypes = [ctypes.c_int, ctypes.c_int, i32p]
        L.hop_pick_degree.argtypes = [ctypes.c_int, ctypes.c_size_t, ctypes.c_double, ctypes.c_double]
        L.hop_calibrate.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        L.hop_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_size_t, ctypes.c_size_t, ctypes.c_int,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.hop_workspace_bytes.restype = ctypes.c_size_t
        L.hop_shutdown.argtypes = []
        L.hop_strerror.argtypes = [ctypes.c_int]
        L.hop_strerror.restype = ctypes.c_char_p
        L.hop_kernel_config.argtypes = []
        L.hop_kernel_config.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("hop_workspace_bytes", "hop_noalloc_scratch_bytes", "hop_strerror", "hop_kernel_config", "hop_session_chunks_final"):
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def hop_strerror(status: int) -> str:
    return lib().hop_strerror(int(status)).decode()


# ------------------------------------------------------------------ marshalling helpers

class PtrTable:
    """A host array of device pointers built once from tensors (or raw addresses), for callers that
    pass the same buffers again and again and do not want to re-marshal them on every call."""

    def __init__(self, items: Sequence):
        self.items = list(items)                     # keeps the tensors alive
        self.array, self.n = _ptr_table(self.items)
        self.object_bytes = (self.items[0].numel() * self.items[0].element_size()
                             if self.n and isinstance(self.items[0], torch.Tensor) else None)

    def __len__(self):
        return self.n

    def __getitem__(self, i):
        return self.items[i]


def _ptr_table(items) -> Tuple[ctypes.Array, int]:
    """Host array of device pointers from tensors or raw integer addresses."""
    if isinstance(items, PtrTable):
        return items.array, items.n
    ptrs = [int(t.data_ptr()) if isinstance(t, torch.Tensor) else int(t) for t in items]
    return (ctypes.c_void_p * max(len(ptrs), 1))(*ptrs), len(ptrs)


_I32P = ctypes.POINTER(ctypes.c_int32)
_i32_recent = {}        # id(array) -> (array, pointer): callers repeat calls with the same order array


def _i32(a):
    if a is None:
        return None, None
    hit = _i32_recent.get(id(a))
    if hit is not None and hit[0] is a:
        return hit
    arr = np.ascontiguousarray(a, dtype=np.int32)
    out = (arr, arr.ctypes.data_as(_I32P))
    if arr is a:                       # the pointer is into the caller's own array: later contents are seen too
        if len(_i32_recent) >= 16:
            _i32_recent.clear()
        _i32_recent[id(a)] = out
    return out


def _i64(a):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=np.int64)
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, torch.cuda.Stream):
        return ctypes.c_void_p(stream.cuda_stream)
    return ctypes.c_void_p(int(stream))


def _bytes_of(t, object_bytes):
    if object_bytes is not None:
        return int(object_bytes)
    return t.numel() * t.element_size()


def _table_bytes(objs, n, fallback, object_bytes):
    """Size of one object: given, or known to the pointer table, or taken from the first tensor."""
    if object_bytes is not None:
        return int(object_bytes)
    if isinstance(objs, PtrTable) and objs.object_bytes is not None:
        return objs.object_bytes
    return _bytes_of(objs[0] if n else fallback, None)


def _code(table, v):
    return table[v] if v in table else int(v)


# ------------------------------------------------------------------ the C ABI, same names

def hop_reduce(dst, objs, k, op, dtype, chunk_bytes, tree_degree, ready_order=None, fail_mask=None,
               stream=None, object_bytes=None):
    """hop_reduce of include/hop.h. dst/objs: CUDA tensors (or raw addresses with object_bytes).

    Returns (status, info dict).
    """
    tab, n = _ptr_table(objs)
    _ro, ro = _i32(ready_order)
    _fm, fm = _i64(fail_mask)
    info = HopInfo()
    dptr = ctypes.c_void_p(int(dst.data_ptr()) if isinstance(dst, torch.Tensor) else int(dst))
    rc = lib().hop_reduce(dptr, tab, n, _table_bytes(objs, n, dst, object_bytes), ro, int(k),
                          _code(OPS, op), _code(DTYPES, dtype), int(chunk_bytes), int(tree_degree), fm,
                          _stream(stream), ctypes.byref(info))
    return rc, info.as_dict()


def hop_reduce_noalloc(dst, objs, k, op, dtype, chunk_bytes, tree_degree, ready_order=None, fail_mask=None,
                       stream=None, object_bytes=None):
    """hop_reduce_noalloc of include/hop.h: hop_reduce with the library's static device scratch."""
    tab, n = _ptr_table(objs)
    _ro, ro = _i32(ready_order)
    _fm, fm = _i64(fail_mask)
    info = HopInfo()
    dptr = ctypes.c_void_p(int(dst.data_ptr()) if isinstance(dst, torch.Tensor) else int(dst))
    rc = lib().hop_reduce_noalloc(dptr, tab, n, _bytes_of(objs[0] if n else dst, object_bytes), ro, int(k),
                                  _code(OPS, op), _code(DTYPES, dtype), int(chunk_bytes), int(tree_degree), fm,
                                  _stream(stream), ctypes.byref(info))
    return rc, info.as_dict()


def hop_noalloc_scratch_bytes() -> int:
    return int(lib().hop_noalloc_scratch_bytes())


def hop_broadcast(dsts, src, chunk_bytes, stream=None, object_bytes=None):
    tab, n_dst = _ptr_table(dsts)
    sptr = ctypes.c_void_p(int(src.data_ptr()) if isinstance(src, torch.Tensor) else int(src))
    return lib().hop_broadcast(tab, n_dst, sptr, _bytes_of(src, object_bytes), int(chunk_bytes), _stream(stream))


def hop_bcast_begin(src, object_bytes, chunk_bytes, stream=None):
    """src: CUDA tensor / address, or None for a host-only session. Returns (status, handle)."""
    h = ctypes.c_void_p()
    if src is None:
        rc = lib().hop_bcast_begin(ctypes.byref(h), None, int(object_bytes), int(chunk_bytes), None)
    else:
        sptr = ctypes.c_void_p(int(src.data_ptr()) if isinstance(src, torch.Tensor) else int(src))
        rc = lib().hop_bcast_begin(ctypes.byref(h), sptr, int(object_bytes), int(chunk_bytes), _stream(stream))
    return rc, h


def hop_bcast_source_ready(b, chunks_ready_total):
    return lib().hop_bcast_source_ready(b, int(chunks_ready_total))


def hop_bcast_join(b, dst=None):
    """Returns (copy id or negative status, sender)."""
    sender = ctypes.c_int(-1)
    dptr = None if dst is None else ctypes.c_void_p(int(dst.data_ptr()) if isinstance(dst, torch.Tensor) else int(dst))
    rc = lib().hop_bcast_join(b, dptr, ctypes.byref(sender))
    return rc, sender.value


def hop_bcast_fail(b, copy):
    return lib().hop_bcast_fail(b, int(copy))


def hop_bcast_step(b, max_chunks=0):
    return lib().hop_bcast_step(b, int(max_chunks))


def hop_bcast_sender(b, copy):
    return lib().hop_bcast_sender(b, int(copy))


def hop_bcast_finish(b, capacity=1 << 14):
    """Returns (status, info dict, [(from, to, chunk_begin, chunk_end), ...])."""
    info = BcastInfo()
    log = (BcastCopy * capacity)()
    n = ctypes.c_int(0)
    rc = lib().hop_bcast_finish(b, ctypes.byref(info), log, capacity, ctypes.byref(n))
    m = min(n.value, capacity)
    return rc, info.as_dict(), [(log[i].from_, log[i].to, log[i].chunk_begin, log[i].chunk_end) for i in range(m)]


def hop_allreduce(dsts, objs, k, op, dtype, chunk_bytes, tree_degree, ready_order=None, fail_mask=None,
                  stream=None, object_bytes=None):
    dtab, n_dst = _ptr_table(dsts)
    tab, n = _ptr_table(objs)
    _ro, ro = _i32(ready_order)
    _fm, fm = _i64(fail_mask)
    info = HopInfo()
    rc = lib().hop_allreduce(dtab, n_dst, tab, n, _bytes_of(objs[0] if n else dsts[0], object_bytes), ro, int(k),
                             _code(OPS, op), _code(DTYPES, dtype), int(chunk_bytes), int(tree_degree), fm,
                             _stream(stream), ctypes.byref(info))
    return rc, info.as_dict()


def hop_session_begin(dst, objs, k, op, dtype, chunk_bytes, tree_degree, stream=None, object_bytes=None):
    """Returns (status, session handle)."""
    tab, n = _ptr_table(objs)
    h = ctypes.c_void_p()
    dptr = ctypes.c_void_p(int(dst.data_ptr()) if isinstance(dst, torch.Tensor) else int(dst))
    rc = lib().hop_session_begin(ctypes.byref(h), dptr, tab, n, _bytes_of(objs[0] if n else dst, object_bytes),
                                 int(k), _code(OPS, op), _code(DTYPES, dtype), int(chunk_bytes),
                                 int(tree_degree), _stream(stream))
    return rc, h


def hop_session_ready(session, obj, chunks_ready_total):
    return lib().hop_session_ready(session, int(obj), int(chunks_ready_total))


def hop_session_ready_after(session, obj, chunks_ready_total, event=None):
    """event: a recorded torch.cuda.Event (or a raw hipEvent_t address) after which the chunks are valid."""
    ev = None
    if event is not None:
        ev = ctypes.c_void_p(int(event.cuda_event) if isinstance(event, torch.cuda.Event) else int(event))
    return lib().hop_session_ready_after(session, int(obj), int(chunks_ready_total), ev)


def hop_session_fail(session, obj):
    return lib().hop_session_fail(session, int(obj))


def hop_session_set_adaptive(session, on):
    return lib().hop_session_set_adaptive(session, int(bool(on)))


def hop_session_set_workspace(session, buf, nbytes=None):
    """buf: a CUDA tensor (or raw address with nbytes) the session takes all its device scratch from."""
    if isinstance(buf, torch.Tensor):
        return lib().hop_session_set_workspace(session, ctypes.c_void_p(int(buf.data_ptr())),
                                               buf.numel() * buf.element_size() if nbytes is None else int(nbytes))
    return lib().hop_session_set_workspace(session, ctypes.c_void_p(int(buf)), int(nbytes))


def hop_session_set_retention(session, on):
    return lib().hop_session_set_retention(session, int(bool(on)))


def hop_session_set_eager(session, min_steps):
    return lib().hop_session_set_eager(session, int(min_steps))


def hop_session_chunks_final(session):
    return int(lib().hop_session_chunks_final(session))


def hop_plan_session_begin(n, object_bytes, k, dtype, chunk_bytes, tree_degree):
    """Host-only session (enqueues nothing). Returns (status, handle)."""
    h = ctypes.c_void_p()
    rc = lib().hop_plan_session_begin(ctypes.byref(h), int(n), int(object_bytes), int(k), _code(DTYPES, dtype),
                                      int(chunk_bytes), int(tree_degree))
    return rc, h


def hop_plan_session_finish(session, capacity=1 << 16):
    """Returns (status, info, launches, entries) like hop_plan_reduce; the handle is dead afterwards."""
    info = HopInfo()
    nl, ne = ctypes.c_int(0), ctypes.c_int(0)
    L = (PlanLaunch * capacity)()
    E = (PlanEntry * capacity)()
    rc = lib().hop_plan_session_finish(session, ctypes.byref(info), L, capacity, ctypes.byref(nl), E, capacity,
                                       ctypes.byref(ne))
    return rc, info.as_dict(), _launch_tuples(L, min(nl.value, capacity)), _entry_tuples(E, min(ne.value, capacity))


def _launch_tuples(L, n):
    return [(L[i].chunk_begin, L[i].chunk_end, L[i].entry_begin, L[i].entry_end, L[i].step_begin, L[i].step_end,
             L[i].final, L[i].live_before, L[i].live_after) for i in range(n)]


def _entry_tuples(E, n):
    """(obj, level, set, n_fold) per step; a step that stores a kept partial result carries two more
    fields, (..., save, save_level). obj = -(1 + q) reads kept partial q."""
    return [(E[i].obj, E[i].level, E[i].set, E[i].n_fold) if E[i].save < 0 else
            (E[i].obj, E[i].level, E[i].set, E[i].n_fold, E[i].save, E[i].save_level) for i in range(n)]


def hop_session_finish(session):
    """Returns (status, info dict); the session handle is dead afterwards."""
    info = HopInfo()
    rc = lib().hop_session_finish(session, ctypes.byref(info))
    return rc, info.as_dict()


def hop_plan_reduce(n, object_bytes, k, dtype, chunk_bytes, tree_degree, ready_order=None, fail_mask=None):
    """Host-only schedule: (status, info, launches, entries) with launches as
    (chunk_begin, chunk_end, entry_begin, entry_end, step_begin, step_end, final, live_before, live_after)
    and entries as (obj, level, set, n_fold)."""
    _ro, ro = _i32(ready_order)
    _fm, fm = _i64(fail_mask)
    info = HopInfo()
    nl, ne = ctypes.c_int(0), ctypes.c_int(0)
    args = (int(n), int(object_bytes), ro, int(k), _code(DTYPES, dtype), int(chunk_bytes), int(tree_degree), fm)
    rc = lib().hop_plan_reduce(*args, ctypes.byref(info), None, 0, ctypes.byref(nl), None, 0, ctypes.byref(ne))
    if rc < 0:
        return rc, info.as_dict(), [], []
    L = (PlanLaunch * max(nl.value, 1))()
    E = (PlanEntry * max(ne.value, 1))()
    rc = lib().hop_plan_reduce(*args, ctypes.byref(info), L, nl.value, ctypes.byref(nl), E, ne.value,
                               ctypes.byref(ne))
    return rc, info.as_dict(), _launch_tuples(L, nl.value), _entry_tuples(E, ne.value)


def hop_plan_split(entries, want_steps, min_run, max_run):
    """(status, top entries, [(pass, sub-program entries), ...]) for a program of (obj, level, set, n_fold) tuples."""
    n = len(entries)
    E = (PlanEntry * max(n, 1))(*[PlanEntry(*e) for e in entries])
    top = (PlanEntry * max(n, 1))()
    sub = (PlanEntry * (2 * n + 1))()
    begins = np.zeros(n + 2, np.int32)
    passes = np.zeros(n + 2, np.int32)
    nt, ns, nsub, npass = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    i32 = ctypes.POINTER(ctypes.c_int32)
    rc = lib().hop_plan_split(E, n, int(want_steps), int(min_run), int(max_run), top, n, ctypes.byref(nt), sub, 2 * n + 1,
                              ctypes.byref(ns), begins.ctypes.data_as(i32), passes.ctypes.data_as(i32), n + 2,
                              ctypes.byref(nsub), ctypes.byref(npass))
    as_t = lambda a, i: (a[i].obj, a[i].level, a[i].set, a[i].n_fold)
    tops = [as_t(top, i) for i in range(nt.value)]
    subs = [(int(passes[s]), [as_t(sub, i) for i in range(begins[s], begins[s + 1])]) for s in range(nsub.value)]
    return rc, tops, subs


def hop_plan_chains(entries, min_cut=4, max_items=23):
    """(status, [(pass, [item, ...]), ...]) for a program of (obj, level, set, n_fold[, save, save_level]) tuples:
    item >= 0 is an object, item = -(1 + g) the value of chain g; the last chain's value is the result."""
    n = len(entries)
    E = (PlanEntry * max(n, 1))(*[PlanEntry(e[0], e[1], e[2], e[3], e[4] if len(e) > 4 else -1, e[5] if len(e) > 4 else 0)
                                  for e in entries])
    items = np.zeros(2 * n + 2, np.int32)
    begins = np.zeros(n + 2, np.int32)
    passes = np.zeros(n + 2, np.int32)
    ni, nc, npass = ctypes.c_int(0), ctypes.c_int(0), ctypes.c_int(0)
    i32 = ctypes.POINTER(ctypes.c_int32)
    rc = lib().hop_plan_chains(E, n, int(min_cut), int(max_items), items.ctypes.data_as(i32), 2 * n + 2, ctypes.byref(ni),
                               begins.ctypes.data_as(i32), passes.ctypes.data_as(i32), n + 2, ctypes.byref(nc),
                               ctypes.byref(npass))
    chains = [(int(passes[g]), [int(x) for x in items[begins[g]:begins[g + 1]]]) for g in range(nc.value)]
    assert rc != HOP_OK or (ni.value <= 2 * n + 2 and npass.value == 1 + max(p for p, _ in chains))
    return rc, chains


def hop_plan_slots(k, tree_degree):
    out = np.empty(max(k, 1), np.int32)
    rc = lib().hop_plan_slots(int(k), int(tree_degree), out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    return rc, out


def hop_pick_degree(k, object_bytes, latency_s=0.0, bytes_per_s=0.0):
    return lib().hop_pick_degree(int(k), int(object_bytes), float(latency_s), float(bytes_per_s))


def hop_calibrate():
    """Measures Eq. 1's constants on the current device. Returns (status, latency_s, bytes_per_s)."""
    lat, bw = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = lib().hop_calibrate(ctypes.byref(lat), ctypes.byref(bw))
    return rc, lat.value, bw.value


HOP_WS_EAGER, HOP_WS_FAILURES = 1, 2


def hop_workspace_bytes(n, k, object_bytes, chunk_bytes, tree_degree, dtype, n_dst=1, policy=0):
    return lib().hop_workspace_bytes(int(n), int(k), int(object_bytes), int(chunk_bytes), int(tree_degree),
                                     _code(DTYPES, dtype), int(n_dst), int(policy))


def hop_kernel_config() -> str:
    return lib().hop_kernel_config().decode()


def hop_shutdown():
    return lib().hop_shutdown()
