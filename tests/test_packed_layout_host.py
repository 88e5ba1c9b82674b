"""Host-only pin of the packed layout's bookkeeping: the helper that the GPU tests use to undo the
packed order (reshapes and transposes) against the piece-index formula of include/evospec.h written
out piece by piece, and the buffer sizes the library reports."""
import numpy as np
import pytest

from helpers import unpack_bits


def pack_by_formula(W, fill):
    """Packed copy of a row-major uint16 matrix, one 16-byte piece at a time:
    piece (r, c) -> piece index (r // 16) * (2 * dp) + (c // 4) * 64 + (c % 4) * 16 + r % 16."""
    rows, d = W.shape
    dp = (d + 255) // 256 * 256
    rp = (rows + 15) // 16 * 16
    out = np.full(rp * dp, fill, dtype=np.uint16)
    for r in range(rows):
        for c in range(dp // 8):
            piece = (r // 16) * (2 * dp) + (c // 4) * 64 + (c % 4) * 16 + r % 16
            src = W[r, 8 * c:8 * c + 8] if 8 * c < d else np.zeros(8, np.uint16)
            out[8 * piece:8 * piece + 8] = src
    return out


@pytest.mark.parametrize("rows,d", [(1, 8), (16, 256), (17, 264), (37, 72), (50, 520)])
def test_unpack_inverts_the_documented_formula(rows, d):
    rng = np.random.default_rng(rows * 1000 + d)
    W = rng.integers(1, 65535, size=(rows, d)).astype(np.uint16)
    P = pack_by_formula(W, fill=0xABCD)
    got, full = unpack_bits(P, rows, d)
    assert np.array_equal(got, W)
    assert np.all(full[0, :rows, d:] == 0)                  # pad elements of real rows
    assert np.all(full[0, rows:, :] == 0xABCD)              # rows past the end: untouched


def test_every_piece_index_is_used_once():
    rows, d = 48, 512
    dp = 512
    seen = set()
    for r in range(rows):
        for c in range(dp // 8):
            seen.add((r // 16) * (2 * dp) + (c // 4) * 64 + (c % 4) * 16 + r % 16)
    assert seen == set(range(rows * dp // 8))


def test_batch_of_matrices():
    rng = np.random.default_rng(3)
    Ws = rng.integers(1, 65535, size=(3, 20, 40)).astype(np.uint16)
    P = np.concatenate([pack_by_formula(Ws[s], fill=7) for s in range(3)])
    got, _ = unpack_bits(P, 20, 40, batch=3)
    assert np.array_equal(got, Ws)


def test_library_sizes_match_the_layout():
    import paper_2605_27390_amd as ev
    for rows, d in [(1, 8), (16, 256), (17, 264), (36864, 4096), (2048, 4096), (151936, 4096)]:
        dp = (d + 255) // 256 * 256
        rp = (rows + 15) // 16 * 16
        assert ev.matrix_bytes(rows, d, ev.PACKED) == rp * dp * 2
        assert ev.matrix_bytes(rows, d, ev.ROW_MAJOR) == rows * d * 2
