"""ctypes binding of the C ABI in include/evospec.h: argument marshalling only.

Tensors are torch tensors on the GPU (bf16 matrices, int32 ids, fp32/int32 outputs); the
binding passes their device pointers and torch's current HIP stream.  Every step of the path
runs inside the library's kernels.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libevospec.so")

K_MAX = 64
M_TILE = 64
STATUS = {
    0: "OK", 1: "NULL_POINTER", 2: "BAD_SHAPE", 3: "BAD_K", 4: "MISALIGNED",
    5: "WORKSPACE_TOO_SMALL", 6: "BAD_SEGMENTS", 7: "INVALID_IDS", 8: "HIP_ERROR", 9: "BAD_LAYOUT",
    10: "STATIC_SCRATCH_EXCEEDED",
}
STATIC_SCRATCH_BYTES = 8 << 20
ROW_MAJOR = 0
PACKED = 1


class EvospecError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib.evospec_status_string(status).decode()
        if status == 8:
            msg += ": " + lib.evospec_last_hip_error().decode()
        super().__init__(f"{where}: {STATUS.get(status, status)} ({msg})")


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2605_27390_amd.build` "
            "(hipcc, gfx950).  There is no CPU fallback.")
    # PyTorch ships its own copy of the HIP runtime.  Streams and device pointers cross between it
    # and this library, so both must resolve to one runtime: load PyTorch's first (the order in
    # which the two were loaded decided, on the MI355X boxes, whether the library saw a device).
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.evospec_version.restype = ci
    L.evospec_status_string.restype = ctypes.c_char_p
    L.evospec_status_string.argtypes = [ci]
    L.evospec_last_hip_error.restype = ctypes.c_char_p
    L.evospec_workspace_bytes.restype = ci
    L.evospec_workspace_bytes.argtypes = [ci, ci, ci, ci, ctypes.POINTER(sz)]
    L.evospec_workspace_bytes_segmented.restype = ci
    L.evospec_workspace_bytes_segmented.argtypes = [ci, ci, ci, ci, ci, ci, ctypes.POINTER(sz)]
    L.evospec_active_gather.restype = ci
    L.evospec_matrix_bytes.restype = ci
    L.evospec_matrix_bytes.argtypes = [ci, ci, ci, ctypes.POINTER(sz)]
    L.evospec_active_gather.argtypes = [vp, ci, ci, vp, vp, ci, vp, vp, ci, ci, vp]
    L.evospec_active_lmhead_topk.restype = ci
    L.evospec_active_lmhead_topk.argtypes = [vp, ci, ci, vp, vp, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    L.evospec_active_lmhead_topk_static.restype = ci
    L.evospec_active_lmhead_topk_static.argtypes = [vp, ci, ci, vp, vp, ci, ci, ci, vp, vp, vp, vp]
    L.evospec_active_lmhead_topk_then_update.restype = ci
    L.evospec_active_lmhead_topk_then_update.argtypes = [vp, ci, ci, vp, vp, ci, ci, ci, vp, vp, vp, vp, sz,
                                                         vp, ci, vp, vp, ci, vp]
    L.evospec_active_lmhead_partials.restype = ci
    L.evospec_active_lmhead_partials.argtypes = [vp, ci, ci, vp, vp, ci, ci, ci, vp, sz, vp]
    L.evospec_active_lmhead_merge.restype = ci
    L.evospec_active_lmhead_merge.argtypes = [ci, ci, ci, ci, vp, vp, vp, vp, sz, vp]
    L.evospec_active_lmhead_topk_segmented.restype = ci
    L.evospec_active_lmhead_topk_segmented.argtypes = [vp, ci, ci, vp, vp, ci, vp, vp, ci, ci,
                                                       ctypes.POINTER(ctypes.c_int32), ci, ci,
                                                       vp, vp, vp, vp, sz, vp]
    L.evospec_kl_gate.restype = ci
    L.evospec_kl_gate.argtypes = [vp, ci, ci, vp, ci, vp, ci, ctypes.c_float, vp, vp, vp, vp, vp, sz, vp]
    L.evospec_kl_gate_workspace_bytes.restype = ci
    L.evospec_kl_gate_workspace_bytes.argtypes = [ci, ci, ctypes.POINTER(sz)]
    L.evospec_validate_ids.restype = ci
    L.evospec_validate_ids.argtypes = [vp, ci, ci, vp]
    return L


lib = _load()


def lib_path() -> str:
    return _LIB_PATH


def version() -> int:
    return int(lib.evospec_version())


def status_string(status: int) -> str:
    return lib.evospec_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != 0:
        raise EvospecError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _expect(t, dtype, name, ndim=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU torch tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if ndim is not None and t.dim() != ndim:
        raise ValueError(f"{name} must have {ndim} dims")


def matrix_bytes(rows: int, d: int, layout: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib.evospec_matrix_bytes(int(rows), int(d), int(layout), ctypes.byref(out)), "evospec_matrix_bytes")
    return int(out.value)


class PackedMatrix:
    """A compact active matrix in the packed layout of include/evospec.h (EVOSPEC_PACKED): `rows` rows
    of `d` bf16 elements (`batch` such matrices back to back when batch is given).  `data` is the 1-D
    bf16 device buffer; only the library's gather writes it.  Wherever a call takes a W_act, a 2-D bf16
    tensor means row-major and a PackedMatrix means packed."""

    def __init__(self, rows: int, d: int, device="cuda", batch=None, data=None):
        import torch
        self.rows, self.d, self.batch = int(rows), int(d), batch
        self.matrix_elems = matrix_bytes(rows, d, PACKED) // 2
        n = self.matrix_elems * (1 if batch is None else int(batch))
        if data is None:
            data = torch.empty(max(n, 8), dtype=torch.bfloat16, device=device)
        _expect(data, torch.bfloat16, "data", 1)
        if data.numel() < n:
            raise ValueError("data is smaller than evospec_matrix_bytes reports")
        self.data = data

    def data_ptr(self):
        return self.data.data_ptr()

    def sub(self, s: int):
        """Matrix s of a batch, sharing the buffer."""
        return PackedMatrix(self.rows, self.d, data=self.data[s * self.matrix_elems:(s + 1) * self.matrix_elems])


def _matrix(W, name, ndim=2):
    """(rows, d, layout) of a W_act argument."""
    import torch
    if isinstance(W, PackedMatrix):
        return W.rows, W.d, PACKED
    _expect(W, torch.bfloat16, name, ndim)
    return W.shape[-2], W.shape[-1], ROW_MAJOR


def workspace_bytes(M: int, V_act: int, d: int, k: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib.evospec_workspace_bytes(M, V_act, d, k, ctypes.byref(out)), "evospec_workspace_bytes")
    return int(out.value)


def workspace_bytes_segmented(M: int, V_core: int, V_arc: int, S: int, d: int, k: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib.evospec_workspace_bytes_segmented(M, V_core, V_arc, S, d, k, ctypes.byref(out)),
           "evospec_workspace_bytes_segmented")
    return int(out.value)


def active_gather(W_lm, src_ids, slots, W_act, act_ids) -> None:
    """W_act[slot_i] = W_lm[src_ids[i]], act_ids[slot_i] = src_ids[i] (slots=None: slot_i = i)."""
    import torch
    _expect(W_lm, torch.bfloat16, "W_lm", 2)
    V_act, d_act, layout = _matrix(W_act, "W_act")
    _expect(src_ids, torch.int32, "src_ids", 1)
    _expect(act_ids, torch.int32, "act_ids", 1)
    if slots is not None:
        _expect(slots, torch.int32, "slots", 1)
        if slots.shape[0] != src_ids.shape[0]:
            raise ValueError("slots and src_ids differ in length")
    V, d = W_lm.shape
    if d_act != d or act_ids.shape[0] != V_act:
        raise ValueError("W_act / act_ids shapes do not match")
    _check(lib.evospec_active_gather(_ptr(W_lm), V, d, _ptr(src_ids), _ptr(slots), src_ids.shape[0],
                                     _ptr(W_act), _ptr(act_ids), V_act, layout, _stream()), "evospec_active_gather")


def _head_shapes(h, W_act, ids):
    import torch
    _expect(h, torch.bfloat16, "h", 2)
    V_act, d_act, layout = _matrix(W_act, "W_act")
    M, d = h.shape
    if d_act != d:
        raise ValueError("hidden sizes of h and W_act differ")
    if ids is not None:
        _expect(ids, torch.int32, "ids", 1)
        if ids.shape[0] != V_act:
            raise ValueError("ids length != V_act")
    return M, d, V_act, layout


def _workspace(workspace, need, device):
    import torch
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=device)
    return workspace


def active_lmhead_topk(h, W_act, ids, k, out_vals=None, out_ids=None, out_logz=None, workspace=None):
    """Restricted head: returns (vals[M,k] f32, ids[M,k] i32, logz[M] f32)."""
    import torch
    M, d, V_act, layout = _head_shapes(h, W_act, ids)
    dev = h.device
    out_vals = torch.empty((M, k), dtype=torch.float32, device=dev) if out_vals is None else out_vals
    out_ids = torch.empty((M, k), dtype=torch.int32, device=dev) if out_ids is None else out_ids
    out_logz = torch.empty((M,), dtype=torch.float32, device=dev) if out_logz is None else out_logz
    if workspace is None:
        workspace = _workspace(None, workspace_bytes(M, V_act, d, k), dev)
    _check(lib.evospec_active_lmhead_topk(_ptr(h), M, d, _ptr(W_act), _ptr(ids), V_act, layout, k,
                                          _ptr(out_vals), _ptr(out_ids), _ptr(out_logz),
                                          _ptr(workspace), workspace.numel(), _stream()),
           "evospec_active_lmhead_topk")
    return out_vals, out_ids, out_logz


def active_lmhead_topk_static(h, W_act, ids, k, out_vals, out_ids, out_logz):
    """The restricted head on the library's own fixed scratch (no workspace, nothing allocated here
    either: the caller passes the outputs)."""
    M, d, V_act, layout = _head_shapes(h, W_act, ids)
    _check(lib.evospec_active_lmhead_topk_static(_ptr(h), M, d, _ptr(W_act), _ptr(ids), V_act, layout, k,
                                                 _ptr(out_vals), _ptr(out_ids), _ptr(out_logz), _stream()),
           "evospec_active_lmhead_topk_static")
    return out_vals, out_ids, out_logz


def active_lmhead_topk_then_update(h, W_act, act_ids, k, W_lm, src_ids, slots, out_vals=None, out_ids=None,
                                   out_logz=None, workspace=None):
    """The head on W_act / act_ids as they are, then the update W_act[slots] <- W_lm[src_ids] (one launch
    fewer than the two calls).  Returns (vals, ids, logz) of the head."""
    import torch
    M, d, V_act, layout = _head_shapes(h, W_act, act_ids)
    dev = h.device
    out_vals = torch.empty((M, k), dtype=torch.float32, device=dev) if out_vals is None else out_vals
    out_ids = torch.empty((M, k), dtype=torch.int32, device=dev) if out_ids is None else out_ids
    out_logz = torch.empty((M,), dtype=torch.float32, device=dev) if out_logz is None else out_logz
    if workspace is None:
        workspace = _workspace(None, workspace_bytes(M, V_act, d, k), dev)
    n = int(src_ids.numel())
    _check(lib.evospec_active_lmhead_topk_then_update(
        _ptr(h), M, d, _ptr(W_act), _ptr(act_ids), V_act, layout, k, _ptr(out_vals), _ptr(out_ids), _ptr(out_logz),
        _ptr(workspace), workspace.numel(), _ptr(W_lm), int(W_lm.shape[0]), _ptr(src_ids),
        _ptr(slots) if slots is not None else None, n, _stream()), "evospec_active_lmhead_topk_then_update")
    return out_vals, out_ids, out_logz


def active_lmhead_partials(h, W_act, ids, k, workspace) -> None:
    M, d, V_act, layout = _head_shapes(h, W_act, ids)
    _check(lib.evospec_active_lmhead_partials(_ptr(h), M, d, _ptr(W_act), _ptr(ids), V_act, layout, k,
                                              _ptr(workspace), workspace.numel(), _stream()),
           "evospec_active_lmhead_partials")


def active_lmhead_merge(M, V_act, d, k, out_vals, out_ids, out_logz, workspace) -> None:
    _check(lib.evospec_active_lmhead_merge(M, V_act, d, k, _ptr(out_vals), _ptr(out_ids), _ptr(out_logz),
                                           _ptr(workspace), workspace.numel(), _stream()),
           "evospec_active_lmhead_merge")


def active_lmhead_topk_segmented(h, W_core, ids_core, W_arc, ids_arc, row_off, k, workspace=None):
    """Batched variant: rows [row_off[s], row_off[s+1]) see core u arc[s]. row_off: host ints."""
    import torch
    _expect(h, torch.bfloat16, "h", 2)
    V_core, d1, layout = _matrix(W_core, "W_core")
    V_arc, d2, layout_arc = _matrix(W_arc, "W_arc", 3)
    if layout != layout_arc:
        raise ValueError("W_core and W_arc must share a layout")
    _expect(ids_arc, torch.int32, "ids_arc", 2)
    if ids_core is not None:
        _expect(ids_core, torch.int32, "ids_core", 1)
    M, d = h.shape
    S = W_arc.batch if layout == PACKED else W_arc.shape[0]
    if S is None or d1 != d or d2 != d or tuple(ids_arc.shape) != (S, V_arc):
        raise ValueError("shape mismatch")
    ro = (ctypes.c_int32 * (S + 1))(*[int(x) for x in row_off])
    dev = h.device
    out_vals = torch.empty((M, k), dtype=torch.float32, device=dev)
    out_ids = torch.empty((M, k), dtype=torch.int32, device=dev)
    out_logz = torch.empty((M,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = _workspace(None, workspace_bytes_segmented(M, V_core, V_arc, S, d, k), dev)
    _check(lib.evospec_active_lmhead_topk_segmented(
        _ptr(h), M, d, _ptr(W_core), _ptr(ids_core), V_core, _ptr(W_arc), _ptr(ids_arc), V_arc, layout,
        ro, S, k, _ptr(out_vals), _ptr(out_ids), _ptr(out_logz), _ptr(workspace), workspace.numel(),
        _stream()), "evospec_active_lmhead_topk_segmented")
    return out_vals, out_ids, out_logz


def validate_ids(ids, V: int) -> bool:
    """True when every id is in [0, V) and no id repeats (synchronises)."""
    import torch
    _expect(ids, torch.int32, "ids", 1)
    st = lib.evospec_validate_ids(_ptr(ids), ids.shape[0], V, _stream())
    if st == 7:
        return False
    _check(st, "evospec_validate_ids")
    return True


def kl_gate_workspace_bytes(E, V):
    out = ctypes.c_size_t(0)
    _check(lib.evospec_kl_gate_workspace_bytes(int(E), int(V), ctypes.byref(out)), "evospec_kl_gate_workspace_bytes")
    return int(out.value)


def kl_gate(z_target, h_draft, W_lm, K=256, T=1.0, out_support=None, out_zt=None, out_zq=None, out_kl=None,
            workspace=None):
    """Retained-support KL gate (Path B): returns (support int32 [E,K], target logits, draft logits
    fp32 [E,K], kl fp32 [E]).  z_target fp32 [E,V], h_draft bf16 [E,d], W_lm bf16 [V,d], all on the GPU."""
    import torch
    E, V = z_target.shape
    d = W_lm.shape[1]
    dev = z_target.device
    assert z_target.dtype == torch.float32 and z_target.is_contiguous() and h_draft.is_contiguous() and W_lm.is_contiguous()
    if out_support is None:
        out_support = torch.empty((E, K), dtype=torch.int32, device=dev)
        out_zt = torch.empty((E, K), dtype=torch.float32, device=dev)
        out_zq = torch.empty((E, K), dtype=torch.float32, device=dev)
        out_kl = torch.empty((E,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = torch.empty(kl_gate_workspace_bytes(E, V), dtype=torch.uint8, device=dev)
    _check(lib.evospec_kl_gate(z_target.data_ptr(), int(E), int(V), h_draft.data_ptr(), int(d), W_lm.data_ptr(),
                               int(K), float(T), out_support.data_ptr(), out_zt.data_ptr(), out_zq.data_ptr(),
                               out_kl.data_ptr(), workspace.data_ptr(), int(workspace.numel()),
                               torch.cuda.current_stream().cuda_stream), "evospec_kl_gate")
    return out_support, out_zt, out_zq, out_kl
