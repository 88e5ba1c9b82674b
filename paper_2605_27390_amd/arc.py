"""ctypes binding of the dynamic-buffer manager declared in include/evospec_arc.h (host only):
argument marshalling, nothing else.  The manager itself is C++ inside libevospec.so."""
from __future__ import annotations

import ctypes

import numpy as np

from .binding import EvospecError, _matrix, lib


class _Config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("capacity", "p0", "ghost_capacity", "max_insert",
                                            "min_residency", "warmup_events", "slot_base")]


_i32p = ctypes.POINTER(ctypes.c_int32)
lib.evospec_arc_default_config.restype = None
lib.evospec_arc_default_config.argtypes = [ctypes.POINTER(_Config)]
lib.evospec_arc_create.restype = ctypes.c_int
lib.evospec_arc_create.argtypes = [ctypes.POINTER(_Config), _i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_void_p)]
lib.evospec_arc_destroy.restype = None
lib.evospec_arc_destroy.argtypes = [ctypes.c_void_p]
lib.evospec_arc_get_config.restype = ctypes.c_int
lib.evospec_arc_get_config.argtypes = [ctypes.c_void_p, ctypes.POINTER(_Config)]
lib.evospec_arc_advance.restype = ctypes.c_int
lib.evospec_arc_advance.argtypes = [ctypes.c_void_p, ctypes.c_int]
lib.evospec_arc_touch.restype = ctypes.c_int
lib.evospec_arc_touch.argtypes = [ctypes.c_void_p, _i32p, ctypes.c_int]
lib.evospec_arc_event.restype = ctypes.c_int
lib.evospec_arc_event.argtypes = [ctypes.c_void_p, _i32p, ctypes.c_int, _i32p, _i32p, ctypes.POINTER(ctypes.c_int)]
lib.evospec_arc_sizes.restype = ctypes.c_int
lib.evospec_arc_sizes.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_int64)]
lib.evospec_arc_list.restype = ctypes.c_int
lib.evospec_arc_list.argtypes = [ctypes.c_void_p, ctypes.c_int, _i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
lib.evospec_arc_resident.restype = ctypes.c_int
lib.evospec_arc_resident.argtypes = [ctypes.c_void_p, _i32p, _i32p, ctypes.POINTER(ctypes.c_int)]


_i64p = ctypes.POINTER(ctypes.c_int64)
lib.evospec_form_candidates.restype = ctypes.c_int
lib.evospec_form_candidates.argtypes = [_i32p, ctypes.c_int, _i32p, ctypes.c_int, _i64p, _i32p, ctypes.c_int,
                                        ctypes.c_int, _i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
lib.evospec_path_a_workspace_bytes.restype = ctypes.c_int
lib.evospec_path_a_workspace_bytes.argtypes = [ctypes.c_int] * 4 + [ctypes.POINTER(ctypes.c_size_t)]
lib.evospec_path_a_event.restype = ctypes.c_int
lib.evospec_path_a_event.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_int,
                                     _i32p, ctypes.c_int, ctypes.c_int, _i64p, _i32p, ctypes.c_int,
                                     ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                     _i32p, _i32p, ctypes.POINTER(ctypes.c_int)]


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(_i32p)


def _check(status: int, where: str) -> None:
    if status != 0:
        raise EvospecError(status, where)


class ArcManager:
    """The dynamic buffer V_dyn of Eq. 3 under the ARC policy of the appendix.  Defaults are the
    paper's: capacity 256, p0 128, ghosts 256, 32 insertions per event, 8 steps, 50 warm-up events."""

    def __init__(self, capacity=256, p0=128, ghost_cap=256, max_insert=32, min_residency=8,
                 warmup_events=50, slot_base=0, core=()):
        cfg = _Config(capacity, p0, ghost_cap, max_insert, min_residency, warmup_events, slot_base)
        core = np.ascontiguousarray(np.asarray(list(core) if not isinstance(core, np.ndarray) else core, dtype=np.int32))
        h = ctypes.c_void_p()
        _check(lib.evospec_arc_create(ctypes.byref(cfg), _ptr(core) if core.size else None, int(core.size),
                                      ctypes.byref(h)), "evospec_arc_create")
        self._h = h
        self.capacity, self.max_insert, self.ghost_cap = capacity, max_insert, ghost_cap
        self._slots = np.empty(max(1, max_insert), dtype=np.int32)
        self._ids = np.empty(max(1, max_insert), dtype=np.int32)

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            lib.evospec_arc_destroy(h)

    def advance(self, steps=1):
        _check(lib.evospec_arc_advance(self._h, int(steps)), "evospec_arc_advance")

    def touch(self, ids):
        a = np.ascontiguousarray(np.asarray(ids, dtype=np.int32))
        _check(lib.evospec_arc_touch(self._h, _ptr(a) if a.size else None, int(a.size)), "evospec_arc_touch")

    def event_arrays(self, candidates):
        """(slots, ids) int32 arrays of this event's writes (views valid until the next event)."""
        a = np.ascontiguousarray(np.asarray(candidates, dtype=np.int32))
        n = ctypes.c_int(0)
        _check(lib.evospec_arc_event(self._h, _ptr(a) if a.size else None, int(a.size), _ptr(self._slots),
                                     _ptr(self._ids), ctypes.byref(n)), "evospec_arc_event")
        return self._slots[:n.value], self._ids[:n.value]

    def event(self, candidates):
        s, i = self.event_arrays(candidates)
        return list(zip(s.tolist(), i.tolist()))

    def _list(self, which, cap):
        out = np.empty(max(1, cap), dtype=np.int32)
        n = ctypes.c_int(0)
        _check(lib.evospec_arc_list(self._h, which, _ptr(out), int(out.size), ctypes.byref(n)), "evospec_arc_list")
        return out[:n.value].tolist()

    def resident(self):
        s = np.empty(self.capacity, dtype=np.int32)
        i = np.empty(self.capacity, dtype=np.int32)
        n = ctypes.c_int(0)
        _check(lib.evospec_arc_resident(self._h, _ptr(s), _ptr(i), ctypes.byref(n)), "evospec_arc_resident")
        return list(zip(s[:n.value].tolist(), i[:n.value].tolist()))

    def state(self):
        z = (ctypes.c_int64 * 7)()
        _check(lib.evospec_arc_sizes(self._h, z), "evospec_arc_sizes")
        return {"p": int(z[0]), "T1": self._list(0, self.capacity), "T2": self._list(1, self.capacity),
                "B1": self._list(2, self.ghost_cap), "B2": self._list(3, self.ghost_cap),
                "slots": {t: s for s, t in self.resident()}, "step": int(z[5]), "events": int(z[6])}


def form_candidates(target_top, mips_top, row_ptr, col_idx, V, max_successors=8, cap=4096):
    """Ordered, de-duplicated candidate ids of one failure event (host arrays in, list out)."""
    t = np.ascontiguousarray(np.asarray(target_top, dtype=np.int32))
    m = np.ascontiguousarray(np.asarray(mips_top, dtype=np.int32))
    rp = None if row_ptr is None else np.ascontiguousarray(np.asarray(row_ptr, dtype=np.int64))
    ci = None if col_idx is None else np.ascontiguousarray(np.asarray(col_idx, dtype=np.int32))
    out = np.empty(max(1, cap), dtype=np.int32)
    n = ctypes.c_int(0)
    _check(lib.evospec_form_candidates(_ptr(t) if t.size else None, int(t.size), _ptr(m) if m.size else None, int(m.size),
                                       None if rp is None else rp.ctypes.data_as(_i64p),
                                       _ptr(ci) if ci is not None and ci.size else None, int(V), int(max_successors),
                                       _ptr(out), int(cap), ctypes.byref(n)), "evospec_form_candidates")
    return out[:n.value].tolist()


def path_a_workspace_bytes(V, d, n_mips, max_insert):
    out = ctypes.c_size_t(0)
    _check(lib.evospec_path_a_workspace_bytes(int(V), int(d), int(n_mips), int(max_insert), ctypes.byref(out)),
           "evospec_path_a_workspace_bytes")
    return int(out.value)


def path_a_event(arc, h_target, W_lm, target_top, n_mips, row_ptr, col_idx, max_successors, W_act, act_ids, workspace):
    """One failure event (search, candidates, admission, gather) on torch's current stream; returns
    the admitted (slot, id) pairs.  Tensors are CUDA tensors; row_ptr / col_idx / target_top host arrays."""
    import torch
    t = np.ascontiguousarray(np.asarray(target_top, dtype=np.int32))
    rp = np.ascontiguousarray(np.asarray(row_ptr, dtype=np.int64))
    ci = np.ascontiguousarray(np.asarray(col_idx, dtype=np.int32))
    V, d = W_lm.shape
    V_act, _, layout = _matrix(W_act, "W_act")
    cap = max(1, arc.max_insert)
    slots, ids = np.empty(cap, dtype=np.int32), np.empty(cap, dtype=np.int32)
    n = ctypes.c_int(0)
    _check(lib.evospec_path_a_event(arc._h, h_target.data_ptr(), int(d), W_lm.data_ptr(), int(V),
                                    _ptr(t) if t.size else None, int(t.size), int(n_mips),
                                    rp.ctypes.data_as(_i64p), _ptr(ci) if ci.size else None, int(max_successors),
                                    W_act.data_ptr(), act_ids.data_ptr(), int(V_act), int(layout),
                                    workspace.data_ptr(), int(workspace.numel()),
                                    torch.cuda.current_stream().cuda_stream, _ptr(slots), _ptr(ids), ctypes.byref(n)),
           "evospec_path_a_event")
    return list(zip(slots[:n.value].tolist(), ids[:n.value].tolist()))
