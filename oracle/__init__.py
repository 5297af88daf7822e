"""CPU oracle for the tree-ordered N-way reduce of Hoplite (arXiv 2002.05814).

TEST INFRASTRUCTURE ONLY.  This package wraps ``hoplite_oracle.c`` (plain C,
compiled with gcc) through ctypes so that tests, the smoke check and the
CPU-baseline leg of the benchmark can ask "what should the result be?".
It imports nothing from the GPU package and the GPU package imports nothing
from here.

Functions mirror the C file one to one; see its header for the passages of the
paper each one follows (Table 1, sections 3.4.1, 3.4.2 and 3.5.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

SUM, MIN, MAX = 0, 1, 2
F32, BF16, I32 = 0, 1, 2
OK, PARTIAL, ERR_INVALID, ERR_NO_SURVIVOR = 0, 1, -1, -3

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hoplite_oracle.c")
_LIB = os.path.join(_HERE, "libhoplite_oracle.so")

# Plain scalar code: no fast-math, no contraction, so float adds are single
# IEEE binary32 operations in source order.
CFLAGS = ["-O2", "-std=c99", "-fPIC", "-shared", "-fno-fast-math", "-ffp-contract=off",
          "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the C oracle next to its source and return the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", *CFLAGS, _SRC, "-o", tmp], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, i32p, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        L.oracle_tree_slots.argtypes = [ctypes.c_int, ctypes.c_int, i32p, i32p]
        L.oracle_occupants.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, i32p, i64p, i32p, i32p, i32p]
        L.oracle_reduce.argtypes = [vp, ctypes.POINTER(vp), ctypes.c_int, ctypes.c_size_t, i32p,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_size_t,
                                    ctypes.c_int, i64p, i32p, i32p]
        L.oracle_reduce_set.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.c_size_t, i32p,
                                        ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.oracle_broadcast.argtypes = [ctypes.POINTER(vp), ctypes.c_int, vp, ctypes.c_size_t]
        L.oracle_f32_to_bf16.argtypes = [vp, vp, ctypes.c_size_t]
        L.oracle_bf16_to_f32.argtypes = [vp, vp, ctypes.c_size_t]
        for f in (L.oracle_tree_slots, L.oracle_occupants, L.oracle_reduce, L.oracle_reduce_set,
                  L.oracle_broadcast):
            f.restype = ctypes.c_int
        L.oracle_f32_to_bf16.restype = None
        L.oracle_bf16_to_f32.restype = None
        _lib = L
    return _lib


_NP_OF = {F32: np.float32, BF16: np.uint16, I32: np.int32}


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int64)


def _ptr(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def tree_slots(k: int, d: int):
    """(node_of_slot, parent_of_node) of the complete d-ary tree on k nodes."""
    nos = np.empty(k, np.int32)
    par = np.empty(k, np.int32)
    rc = lib().oracle_tree_slots(k, d, _ptr(nos, ctypes.c_int32), _ptr(par, ctypes.c_int32))
    if rc != OK:
        raise ValueError("oracle_tree_slots: status %d" % rc)
    return nos, par


def occupants(n, k, n_chunks, ready_order=None, fail_mask=None):
    """(status, occupant[k] with -1 for holes, k_eff, n_replaced)."""
    ro, fm = _i32(ready_order), _i64(fail_mask)
    occ = np.full(k, -1, np.int32)
    ke, nr = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().oracle_occupants(n, k, n_chunks, _ptr(ro, ctypes.c_int32), _ptr(fm, ctypes.c_int64),
                                _ptr(occ, ctypes.c_int32), ctypes.byref(ke), ctypes.byref(nr))
    return rc, occ, ke.value, nr.value


def _obj_table(objs, dtype):
    arrs = [np.ascontiguousarray(o, dtype=_NP_OF[dtype]) for o in objs]
    n_elems = arrs[0].size
    for a in arrs:
        if a.size != n_elems:
            raise ValueError("objects differ in size")
    tab = (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
    return arrs, tab, n_elems


def reduce(objs, k, op, dtype, chunk_elems, d, ready_order=None, fail_mask=None):
    """Tree-ordered reduce. objs: list of 1-D arrays (bf16 as uint16 bit patterns).

    Returns (status, dst, k_eff, n_replaced); dst is None on error.
    """
    arrs, tab, n_elems = _obj_table(objs, dtype)
    ro, fm = _i32(ready_order), _i64(fail_mask)
    dst = np.zeros(n_elems, _NP_OF[dtype])
    ke, nr = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().oracle_reduce(dst.ctypes.data, tab, len(arrs), n_elems, _ptr(ro, ctypes.c_int32),
                             k, op, dtype, chunk_elems, d, _ptr(fm, ctypes.c_int64),
                             ctypes.byref(ke), ctypes.byref(nr))
    if rc < 0:
        return rc, None, ke.value, nr.value
    return rc, dst, ke.value, nr.value


def reduce_set(objs, occupant, op, dtype):
    """Order-free result over the occupants: float64 (floats) or int64 (int32, unwrapped)."""
    arrs, tab, n_elems = _obj_table(objs, dtype)
    occ = _i32(occupant)
    if dtype == I32:
        out = np.zeros(n_elems, np.int64)
        rc = lib().oracle_reduce_set(None, out.ctypes.data, tab, n_elems, _ptr(occ, ctypes.c_int32),
                                     len(occ), op, dtype)
    else:
        out = np.zeros(n_elems, np.float64)
        rc = lib().oracle_reduce_set(out.ctypes.data, None, tab, n_elems, _ptr(occ, ctypes.c_int32),
                                     len(occ), op, dtype)
    if rc != OK:
        raise ValueError("oracle_reduce_set: status %d" % rc)
    return out


def broadcast(src, n_dst):
    """n_dst byte-identical copies of src."""
    s = np.ascontiguousarray(src)
    outs = [np.zeros_like(s) for _ in range(n_dst)]
    tab = (ctypes.c_void_p * max(n_dst, 1))(*[o.ctypes.data for o in outs])
    rc = lib().oracle_broadcast(tab, n_dst, s.ctypes.data, s.nbytes)
    if rc != OK:
        raise ValueError("oracle_broadcast: status %d" % rc)
    return outs


def allreduce(objs, n_dst, k, op, dtype, chunk_elems, d, ready_order=None, fail_mask=None):
    """Reduce, then broadcast of the result (section 3.4.3)."""
    rc, dst, ke, nr = reduce(objs, k, op, dtype, chunk_elems, d, ready_order, fail_mask)
    if rc < 0:
        return rc, None, ke, nr
    return rc, broadcast(dst, n_dst), ke, nr


def f32_to_bf16(x):
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().oracle_f32_to_bf16(x.ctypes.data, out.ctypes.data, x.size)
    return out


def bf16_to_f32(h):
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().oracle_bf16_to_f32(h.ctypes.data, out.ctypes.data, h.size)
    return out
