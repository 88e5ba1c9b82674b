"""Structure of the seeded synthetic inputs (host only)."""
import numpy as np

import evospec_inputs as gi


def test_bf16_round_to_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625], dtype=np.float32)
    b = gi.f32_to_bf16_bits(x)
    back = gi.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6 -> even mantissa (1+2^-6)
    assert back.tolist() == [1.0, 1.0, 1.015625, -2.5, 0.0, 3.140625]
    import torch
    y = torch.randn(4096, generator=torch.Generator().manual_seed(0))
    ref = y.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(gi.f32_to_bf16_bits(y.numpy()), ref)


def test_generators_are_reproducible_and_blockwise():
    a = gi.gen_normal_bf16(100, 16, 5, 0.02, block_rows=32)
    b = gi.gen_normal_bf16(100, 16, 5, 0.02, block_rows=32)
    assert np.array_equal(a, b)
    c = gi.gen_normal_bf16(64, 16, 5, 0.02, block_rows=32)
    assert np.array_equal(a[:64], c)
    assert gi.checksum(a) == gi.checksum(b) != gi.checksum(c)
    f = gi.bf16_bits_to_f32(gi.gen_normal_bf16(2048, 64, 1, 0.02)).astype(np.float64)
    assert abs(f.std() - 0.02) < 5e-4 and abs(f.mean()) < 2e-4


def test_core_plus_arc_is_a_set_within_budget():
    V, n_core, n_arc = 5000, 1000, 200
    core, arc = gi.core_arc_ids(V, n_core, n_arc, seed=3)
    ids = np.concatenate([core, arc])
    assert ids.dtype == np.int32 and ids.shape[0] <= n_core + n_arc       # |V_t| <= |V_static| + N_dyn
    assert np.unique(ids).shape[0] == ids.shape[0]                        # union of disjoint sets
    assert ids.min() >= 0 and ids.max() < V
    rank = gi.zipf_ranking(V, 3)
    assert np.array_equal(core, rank[:n_core])
    # ARC ids come from the tail and favour its frequent end
    pos = np.empty(V, dtype=np.int64)
    pos[rank] = np.arange(V)
    assert pos[arc].min() >= n_core
    assert np.median(pos[arc]) < (n_core + V) / 2


def test_named_configs():
    ids = gi.active_ids("tiny")
    assert ids.shape == (1024,) and np.all(np.diff(ids) > 0) and ids.max() < 8192
    assert gi.CONFIGS["draft60"]["n_core"] + gi.CONFIGS["draft60"]["n_arc"] == 36864
    small = gi.active_ids("draft60", V=4000, n_core=512, n_arc=64)
    assert small.shape == (576,) and np.unique(small).shape[0] == 576
    assert np.array_equal(gi.active_ids("fullvocab", V=100), np.arange(100))


def test_batched_and_update_recipes():
    core, arcs = gi.batched_ids(3000, 500, 40, 4)
    assert arcs.shape == (4, 40)
    for s in range(4):
        assert np.intersect1d(core, arcs[s]).size == 0 and np.unique(arcs[s]).size == 40
    ids = np.concatenate(gi.core_arc_ids(3000, 500, 100, seed=1))
    slots, new = gi.arc_update(3000, ids, 500, 32, seed=2)
    assert np.unique(slots).size == 32 and slots.min() >= 500 and slots.max() < 600
    assert np.intersect1d(new, ids).size == 0 and np.unique(new).size == 32
