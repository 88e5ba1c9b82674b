"""Pins of the candidate-formation oracle (no GPU): a case worked by hand, agreement of the
exact inner-product search with a brute-force scan, and properties of the result."""
import numpy as np

import evospec_inputs as gi
from oracle import exact_mips, form_candidates


def test_hand_worked_case():
    # graph: 0 -> 5 6 7 | 1 -> (none) | 2 -> 6 0 9 8 | 3 -> 1 | 4.. -> none
    row_ptr = np.array([0, 3, 3, 7, 8, 8, 8, 8, 8, 8, 8], dtype=np.int64)
    col = np.array([5, 6, 7, 6, 0, 9, 8, 1], dtype=np.int32)
    # target candidates 2, 0; retrieved neighbours 0 (again), 3.  Seeds: 2 0 3.
    # successors, two per seed: of 2: 6 0 -> 6 (0 is a seed); of 0: 5 6 -> 5; of 3: 1 -> 1.
    assert form_candidates([2, 0], [0, 3], row_ptr, col, max_successors=2) == [2, 0, 3, 6, 5, 1]
    assert form_candidates([2, 0], [0, 3], row_ptr, col, max_successors=8) == [2, 0, 3, 6, 9, 8, 5, 7, 1]
    assert form_candidates([2, 0], [0, 3], row_ptr, col, max_successors=8, cap=4) == [2, 0, 3, 6]
    assert form_candidates([], [], row_ptr, col) == []
    assert form_candidates([4], [4], row_ptr, col) == [4]


def test_exact_mips_is_the_brute_force_argmax():
    W = gi.gen_normal_bf16(700, 48, 5, 0.05)
    h = gi.gen_h(1, 48, 6)
    Wf, hf = gi.bf16_bits_to_f32(W).astype(np.float64), gi.bf16_bits_to_f32(h).astype(np.float64)[0]
    scores = [sum(Wf[i, j] * hf[j] for j in range(48)) for i in range(700)]      # plain loops
    want = sorted(range(700), key=lambda i: (-scores[i], i))[:10]
    assert exact_mips(h, W, 10).tolist() == want
    # ties go to the smaller id: duplicate a row
    W2 = W.copy(); W2[want[0] + 1 if want[0] + 1 < 700 else 0] = W2[want[0]]
    top = exact_mips(h, W2, 2).tolist()
    assert top == sorted(top) and want[0] in top


def test_properties_on_a_synthetic_graph():
    V = 5000
    row_ptr, col = gi.bigram_graph(V, 3)
    deg = np.diff(row_ptr)
    assert deg.max() <= 64 and row_ptr[0] == 0 and row_ptr[-1] == col.shape[0]
    for u in (0, 17, V - 1):
        succ = col[row_ptr[u]:row_ptr[u + 1]]
        assert len(set(succ.tolist())) == len(succ) and u not in succ
    rng = np.random.default_rng(1)
    for _ in range(50):
        t, m = rng.integers(0, V, 10), rng.integers(0, V, 10)
        out = form_candidates(t, m, row_ptr, col, 8)
        assert len(out) == len(set(out)) <= 20 + 20 * 8
        seeds = list(dict.fromkeys(t.tolist() + m.tolist()))
        assert out[:len(seeds)] == seeds
        allowed = set(seeds)
        for s in seeds:
            allowed |= set(col[row_ptr[s]:min(row_ptr[s + 1], row_ptr[s] + 8)].tolist())
        assert set(out) == allowed
