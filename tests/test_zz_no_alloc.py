"""evospec_active_lmhead_topk_static (the entry point that allocates nothing) against
evospec_active_lmhead_topk on the same inputs: two calls in a row through the C ABI, the second
on a smaller problem, so that what the first call left in the library's fixed scratch array is
still there when the second runs."""
import numpy as np
import pytest

import evospec_inputs as gen
from helpers import to_dev_bf16, to_dev_i32, check_head

pytestmark = pytest.mark.gpu


def _problem(ev, torch, seed, V, d, V_act, M, layout):
    rng = np.random.default_rng(seed)
    W = gen.gen_normal_bf16(V, d, seed, 0.05, block_rows=256)
    h = gen.gen_h(M, d, seed + 1)
    ids = np.sort(rng.choice(V, size=V_act, replace=False)).astype(np.int32)
    dW, dh, dids = to_dev_bf16(W), to_dev_bf16(h), to_dev_i32(ids)
    if layout == "packed":
        Wa = ev.PackedMatrix(V_act, d)
    else:
        Wa = torch.empty((V_act, d), dtype=torch.bfloat16, device="cuda")
    act = torch.empty(V_act, dtype=torch.int32, device="cuda")
    ev.active_gather(dW, dids, None, Wa, act)
    return W, h, ids, dh, Wa, act


@pytest.mark.parametrize("layout", ["row_major", "packed"])
def test_static_scratch_head_equals_workspace_head(oracle_mod, layout):
    import torch
    import paper_2605_27390_amd as ev
    # first a problem that spans several slabs and a ragged tail, then a smaller one
    cases = [(11, 6000, 512, 4133, 37, 10), (12, 3000, 264, 1000, 5, 7)]
    for seed, V, d, V_act, M, k in cases:
        W, h, ids, dh, Wa, act = _problem(ev, torch, seed, V, d, V_act, M, layout)
        ref = ev.active_lmhead_topk(dh, Wa, act, k)
        ov = torch.full((M, k), float("nan"), dtype=torch.float32, device="cuda")
        oi = torch.full((M, k), -7, dtype=torch.int32, device="cuda")
        ol = torch.full((M,), float("nan"), dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        ev.active_lmhead_topk_static(dh, Wa, act, k, ov, oi, ol)
        assert torch.cuda.memory_allocated() == before          # nothing went through torch's allocator either
        torch.cuda.synchronize()
        # same kernels, same plan: bit-identical to the workspace variant
        assert torch.equal(ov, ref[0]) and torch.equal(oi, ref[1]) and torch.equal(ol, ref[2]), (layout, seed)
        # and both agree with the oracle
        z = oracle_mod.logits(h, W[ids])
        check_head(ov.cpu().numpy(), oi.cpu().numpy(), ol.cpu().numpy(), z, ids, k, where=f"static {layout} {seed}")


def test_static_scratch_limit_is_enforced():
    import torch
    import paper_2605_27390_amd as ev
    h = torch.zeros((4, 64), dtype=torch.bfloat16, device="cuda")
    V_act = ev.STATIC_SCRATCH_BYTES // (8 * 11) + 64          # one slab past what fits at k = 10
    W = torch.zeros((V_act, 64), dtype=torch.bfloat16, device="cuda")
    ov = torch.zeros((4, 10), dtype=torch.float32, device="cuda")
    oi = torch.zeros((4, 10), dtype=torch.int32, device="cuda")
    ol = torch.zeros((4,), dtype=torch.float32, device="cuda")
    with pytest.raises(ev.EvospecError) as e:
        ev.active_lmhead_topk_static(h, W, None, 10, ov, oi, ol)
    assert e.value.status == 10
