"""GPU parity on seeded random shapes: draft rows, active-set size, hidden size and k drawn so that
tile, slab, pass and path boundaries (64 / 128 / 129 draft rows, 16-row tiles, 256-element chunks)
are hit from both sides; every shape on a row-major and on a packed matrix, against the fp64 oracle
and against each other.  Needs an MI355X: run with `-m gpu`."""
import numpy as np
import pytest

from helpers import check_head
from test_gpu_packed import run_head_packed, run_head_rows
from test_gpu_parity import ev, problem  # noqa: F401  (fixture and helper)

pytestmark = pytest.mark.gpu


def shapes():
    rng = np.random.default_rng(20260527)
    out = []
    Ms = [1, 2, 15, 16, 17, 31, 63, 64, 65, 100, 127, 128, 129, 130, 200, 255, 256, 257, 300]
    for i in range(28):
        M = int(rng.choice(Ms))
        V_act = int(rng.choice([1, 7, 15, 16, 17, 31, 33, 63, 64, 65, 127, 129, 143, 144, 145, 255, 257, 500, 1000, 1537, 3001]))
        if M >= 129:
            d = int(rng.choice([64, 128, 192, 320, 72, 200]))          # multiples of 64 take the large-M path, the rest passes
        else:
            d = int(rng.choice([8, 16, 24, 40, 64, 72, 248, 256, 264, 512, 520, 1000]))
        k = int(min(V_act, rng.choice([1, 2, 5, 10, 16, 17, 33, 64])))
        out.append((M, V_act, d, k))
    return out


@pytest.mark.parametrize("M,V_act,d,k", shapes())
def test_random_shape(ev, oracle_mod, M, V_act, d, k):
    W, h, ids = problem(7000 + M * 31 + V_act * 7 + d + k, V_act, d, M)
    z = oracle_mod.logits(h, W)
    v0, i0, l0 = run_head_rows(ev, h, W, ids, k)
    check_head(v0, i0, l0, z, ids, k, f"row-major M={M} V_act={V_act} d={d} k={k}")
    v1, i1, l1 = run_head_packed(ev, h, W, ids, k)
    assert np.array_equal(v0, v1) and np.array_equal(i0, i1) and np.array_equal(l0, l1)
