"""Shared helpers for the GPU parity tests: device upload and the acceptance rule.

Acceptance (from the benchmark spec): gathered rows and id remaps bit-exact; logits and
log-normaliser within 1e-3 relative error; top-k id sets identical wherever the oracle's k-th and
(k+1)-th logits differ by more than 1e-3 relative.  Where that gap is smaller several answers are
correct: then every returned id must still be an active id whose oracle logit is within the
tolerance of the oracle's k-th logit.
"""
import numpy as np

REL_TOL = 1e-3


def to_dev_bf16(bits):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def to_dev_i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def bf16_dev_to_bits(t):
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def check_head(gv, gi_, gl, z, ids, k, where=""):
    """Compare GPU outputs (vals [M,k], ids [M,k], logz [M]) with the oracle's full logits
    z [M, V_act] (fp64) over the active ids (None = identity).  Returns stats."""
    from scipy.special import logsumexp
    M, V_act = z.shape
    ids = np.arange(V_act, dtype=np.int32) if ids is None else np.asarray(ids)
    gv = np.asarray(gv, dtype=np.float64)
    gi_ = np.asarray(gi_)
    gl = np.asarray(gl, dtype=np.float64)
    assert gv.shape == (M, k) and gi_.shape == (M, k) and gl.shape == (M,), where
    pos = {int(t): i for i, t in enumerate(ids)}
    lz = logsumexp(z, axis=1)
    rel_lz = np.abs(gl - lz) / np.maximum(np.abs(lz), 1e-30)
    assert np.all(rel_lz <= REL_TOL), f"{where}: logZ rel err {rel_lz.max():.3e}"
    exempt = 0
    max_err = 0.0
    for m in range(M):
        order = np.lexsort((ids, -z[m]))
        top = order[:k]
        zk = z[m][top[-1]]
        row_ids = gi_[m].tolist()
        assert len(set(row_ids)) == k, f"{where}: row {m} repeats an id {row_ids}"
        for j, t in enumerate(row_ids):
            assert t in pos, f"{where}: row {m} returned id {t} that is not active"
            ref = z[m][pos[t]]
            err = abs(gv[m, j] - ref)
            max_err = max(max_err, err)
            assert err <= REL_TOL * max(abs(ref), 1.0), f"{where}: row {m} logit of id {t}: {gv[m, j]} vs {ref}"
            assert ref >= zk - REL_TOL * max(abs(zk), 1.0), f"{where}: row {m} id {t} is not a top-{k} entry"
        assert np.all(np.diff(gv[m]) <= 0), f"{where}: row {m} values not descending"
        if k < V_act:
            zk1 = z[m][order[k]]
            gap = abs(zk - zk1) / max(abs(zk), abs(zk1), 1e-30)
        else:
            gap = np.inf
        if gap > REL_TOL:
            assert set(row_ids) == set(ids[top].tolist()), f"{where}: row {m} top-{k} id set differs (gap {gap:.2e})"
        else:
            exempt += 1
    return dict(max_abs_err=max_err, max_rel_logz=float(rel_lz.max()), exempt_rows=exempt)


NAN_BITS = 0x7FC1        # a bf16 NaN: what never-written rows and pad pieces of a packed matrix must not leak


def unpack_bits(bits, rows, d, batch=None):
    """Row-major uint16 [rows, d] (or [batch, rows, d]) from the bits of a packed buffer, and the
    padded matrix itself: piece (r, c) of the packed layout sits at piece index
    (r // 16) * (2 * dp) + (c // 4) * 64 + (c % 4) * 16 + r % 16, dp = d rounded up to 256."""
    dp = (d + 255) // 256 * 256
    rp = (rows + 15) // 16 * 16
    n = rp * dp
    B = 1 if batch is None else batch
    a = np.asarray(bits[:B * n]).reshape(B, rp // 16, dp // 32, 4, 16, 8)      # [tile][k-step][g][n16][8]
    full = a.transpose(0, 1, 4, 2, 3, 5).reshape(B, rp, dp)                     # [tile][n16][k-step][g][8]
    out = full[:, :rows, :d]
    return (out[0] if batch is None else out), full


def new_matrix(ev, rows, d, layout, batch=None):
    """An uninitialised compact matrix on the GPU: a PackedMatrix pre-filled with NaNs, or a
    row-major tensor."""
    import torch
    if layout == "packed":
        P = ev.PackedMatrix(rows, d, batch=batch)
        P.data.view(torch.int16).fill_(NAN_BITS)
        return P
    shape = (rows, d) if batch is None else (batch, rows, d)
    return torch.empty(shape, dtype=torch.bfloat16, device="cuda")


def matrix_bits(Wm, batch=None):
    """Row-major bits (host) of a compact matrix in either layout."""
    if hasattr(Wm, "rows"):
        return unpack_bits(bf16_dev_to_bits(Wm.data), Wm.rows, Wm.d, batch=batch)[0]
    return bf16_dev_to_bits(Wm)
