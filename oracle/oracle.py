"""ctypes wrapper around the plain-C fp64 oracle (test infrastructure only).

All tensors are numpy arrays: bf16 data travels as uint16 bit patterns, ids as
int32, results as float64 / int32.  The wrapper only marshals arguments; every
arithmetic step is in `evospec_oracle.c`.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "evospec_oracle.c")
_LIB = os.path.join(_HERE, "libevospec_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP, no fast-math). Returns the .so path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build()
    lib = ctypes.CDLL(_LIB)
    c_u16p = ctypes.POINTER(ctypes.c_uint16)
    c_i32p = ctypes.POINTER(ctypes.c_int32)
    c_f64p = ctypes.POINTER(ctypes.c_double)
    ci = ctypes.c_int
    lib.oracle_num_threads.restype = ci
    lib.oracle_set_num_threads.argtypes = [ci]
    lib.oracle_active_gather.restype = ci
    lib.oracle_active_gather.argtypes = [c_u16p, ci, ci, c_i32p, c_i32p, ci, c_u16p, c_i32p, ci]
    lib.oracle_logits.restype = None
    lib.oracle_logits.argtypes = [c_u16p, ci, ci, c_u16p, ci, c_f64p]
    lib.oracle_logz.restype = None
    lib.oracle_logz.argtypes = [c_f64p, ci, ci, c_f64p]
    lib.oracle_topk.restype = ci
    lib.oracle_topk.argtypes = [c_f64p, c_i32p, ci, ci, ci, c_f64p, c_i32p]
    lib.oracle_active_lmhead_topk.restype = ci
    lib.oracle_active_lmhead_topk.argtypes = [c_u16p, ci, ci, c_u16p, c_i32p, ci, ci,
                                              c_f64p, c_i32p, c_f64p, c_f64p]
    lib.oracle_active_lmhead_topk_segmented.restype = ci
    lib.oracle_active_lmhead_topk_segmented.argtypes = [
        c_u16p, ci, ci, c_u16p, c_i32p, ci, c_u16p, c_i32p, ci, c_i32p, ci, ci,
        c_f64p, c_i32p, c_f64p]
    _lib = lib
    return lib


def _u16(a, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 data must be passed as uint16 bit patterns")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"shape {a.shape} != {shape}")
    return a


def _i32(a):
    a = np.ascontiguousarray(a)
    if a.dtype != np.int32:
        raise TypeError("ids must be int32")
    return a


def _p(a, ctype):
    return a.ctypes.data_as(ctypes.POINTER(ctype)) if a is not None else None


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def active_gather(W_lm, src_ids, slots, W_act, act_ids):
    """In place: W_act[slot_i] = W_lm[src_ids[i]], act_ids[slot_i] = src_ids[i]."""
    lib = _load()
    W_lm = _u16(W_lm)
    V, d = W_lm.shape
    src_ids = _i32(src_ids)
    n = src_ids.shape[0]
    if slots is not None:
        slots = _i32(slots)
        if slots.shape[0] != n:
            raise ValueError("slots and src_ids differ in length")
    if W_act.dtype != np.uint16 or not W_act.flags.c_contiguous or W_act.shape[1] != d:
        raise ValueError("W_act must be contiguous uint16 [V_act, d]")
    if act_ids.dtype != np.int32 or not act_ids.flags.c_contiguous:
        raise ValueError("act_ids must be contiguous int32")
    V_act = W_act.shape[0]
    rc = lib.oracle_active_gather(_p(W_lm, ctypes.c_uint16), V, d, _p(src_ids, ctypes.c_int32),
                                  _p(slots, ctypes.c_int32), n, _p(W_act, ctypes.c_uint16),
                                  _p(act_ids, ctypes.c_int32), V_act)
    if rc:
        raise ValueError("id or slot out of range")


def logits(h, W):
    """z[m,i] = sum_j h[m,j] W[i,j] in fp64 (Eq. 1 before the softmax)."""
    lib = _load()
    h = _u16(h)
    W = _u16(W)
    M, d = h.shape
    Vn, d2 = W.shape
    if d != d2:
        raise ValueError("hidden sizes differ")
    z = np.empty((M, Vn), dtype=np.float64)
    lib.oracle_logits(_p(h, ctypes.c_uint16), M, d, _p(W, ctypes.c_uint16), Vn, _p(z, ctypes.c_double))
    return z


def logz(z):
    lib = _load()
    z = np.ascontiguousarray(z, dtype=np.float64)
    M, Vn = z.shape
    out = np.empty((M,), dtype=np.float64)
    lib.oracle_logz(_p(z, ctypes.c_double), M, Vn, _p(out, ctypes.c_double))
    return out


def topk(z, ids, kk):
    lib = _load()
    z = np.ascontiguousarray(z, dtype=np.float64)
    M, Vn = z.shape
    if ids is not None:
        ids = _i32(ids)
        if ids.shape[0] != Vn:
            raise ValueError("ids length")
    vals = np.empty((M, kk), dtype=np.float64)
    oid = np.empty((M, kk), dtype=np.int32)
    rc = lib.oracle_topk(_p(z, ctypes.c_double), _p(ids, ctypes.c_int32), M, Vn, kk,
                         _p(vals, ctypes.c_double), _p(oid, ctypes.c_int32))
    if rc:
        raise ValueError(f"oracle_topk failed ({rc})")
    return vals, oid


def active_lmhead_topk(h, W_act, ids, kk, return_logits=False):
    """Restricted head: returns (vals[M,kk], ids[M,kk], logz[M]) (+ z[M,V_act])."""
    lib = _load()
    h = _u16(h)
    W_act = _u16(W_act)
    M, d = h.shape
    V_act, d2 = W_act.shape
    if d != d2:
        raise ValueError("hidden sizes differ")
    if ids is not None:
        ids = _i32(ids)
        if ids.shape[0] != V_act:
            raise ValueError("ids length")
    vals = np.empty((M, kk), dtype=np.float64)
    oid = np.empty((M, kk), dtype=np.int32)
    lz = np.empty((M,), dtype=np.float64)
    z = np.empty((M, V_act), dtype=np.float64) if return_logits else None
    rc = lib.oracle_active_lmhead_topk(_p(h, ctypes.c_uint16), M, d, _p(W_act, ctypes.c_uint16),
                                       _p(ids, ctypes.c_int32), V_act, kk,
                                       _p(vals, ctypes.c_double), _p(oid, ctypes.c_int32),
                                       _p(lz, ctypes.c_double), _p(z, ctypes.c_double))
    if rc:
        raise ValueError(f"oracle_active_lmhead_topk failed ({rc})")
    if return_logits:
        return vals, oid, lz, z
    return vals, oid, lz


def active_lmhead_topk_segmented(h, W_core, ids_core, W_arc, ids_arc, row_off, kk):
    """Segmented variant: rows of sequence s see core || arc[s]."""
    lib = _load()
    h = _u16(h)
    M, d = h.shape
    W_core = _u16(W_core)
    V_core = W_core.shape[0]
    W_arc = _u16(W_arc)
    S, V_arc, d3 = W_arc.shape
    if W_core.shape[1] != d or d3 != d:
        raise ValueError("hidden sizes differ")
    if ids_core is not None:
        ids_core = _i32(ids_core)
    ids_arc = _i32(ids_arc)
    if ids_arc.shape != (S, V_arc):
        raise ValueError("ids_arc shape")
    row_off = _i32(row_off)
    if row_off.shape[0] != S + 1:
        raise ValueError("row_off length")
    vals = np.empty((M, kk), dtype=np.float64)
    oid = np.empty((M, kk), dtype=np.int32)
    lz = np.empty((M,), dtype=np.float64)
    rc = lib.oracle_active_lmhead_topk_segmented(
        _p(h, ctypes.c_uint16), M, d, _p(W_core, ctypes.c_uint16), _p(ids_core, ctypes.c_int32), V_core,
        _p(W_arc, ctypes.c_uint16), _p(ids_arc, ctypes.c_int32), V_arc,
        _p(row_off, ctypes.c_int32), S, kk,
        _p(vals, ctypes.c_double), _p(oid, ctypes.c_int32), _p(lz, ctypes.c_double))
    if rc:
        raise ValueError(f"oracle segmented failed ({rc})")
    return vals, oid, lz
