"""GPU parity of the retained-support KL gate against its fp64 oracle.  Needs an MI355X."""
import numpy as np
import pytest

import evospec_inputs as gi
from helpers import to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ev():
    import torch
    assert torch.cuda.is_available()
    import paper_2605_27390_amd as ev
    return ev


def run(ev, z, h, W, K, T):
    import torch
    s, zt, zq, kl = ev.kl_gate(torch.from_numpy(z).cuda(), to_dev_bf16(h), to_dev_bf16(W), K, T)
    torch.cuda.synchronize()
    return s.cpu().numpy(), zt.cpu().numpy(), zq.cpu().numpy(), kl.cpu().numpy()


def check(got, want, where):
    s, zt, zq, kl = got
    os_, ozt, ozq, okl = want
    assert np.array_equal(s, os_), where                          # exact: keys are compared in fp32 on both sides
    assert np.array_equal(zt.astype(np.float64), ozt), where
    np.testing.assert_allclose(zq, ozq, rtol=1e-3, atol=1e-4, err_msg=where)
    np.testing.assert_allclose(kl, okl, rtol=1e-3, atol=1e-5, err_msg=where)


@pytest.mark.parametrize("E,V,d,K,T", [
    (3, 5000, 64, 256, 1.0),
    (1, 300, 8, 256, 1.0),          # K close to V
    (2, 70000, 264, 100, 2.0),      # ragged sizes, another temperature
    (4, 1000, 4096, 1, 1.0),        # K = 1: divergence is zero
    (2, 256, 128, 256, 0.5),        # K = V
    (2, 30000, 64, 256, 1.0),       # one slice, eight 16-byte loads per thread
    (2, 32770, 64, 256, 1.0),       # eight slices, rows not 16-byte aligned: the looping sweep
])
def test_shapes(ev, E, V, d, K, T):
    from oracle import kl_gate
    rng = np.random.default_rng(E + V + K)
    W = gi.gen_normal_bf16(V, d, 11, 0.05)
    h = gi.gen_h(E, d, 12)
    z = (rng.standard_normal((E, V)) * 2.5).astype(np.float32)
    got, want = run(ev, z, h, W, K, T), kl_gate(z, h, W, K, T)
    check(got, want, f"E={E} V={V} d={d} K={K}")
    if K == 1:
        assert np.all(np.abs(got[3]) < 1e-5)


def test_ties_and_degenerate_logits(ev):
    from oracle import kl_gate
    V, d = 4000, 32
    W = gi.gen_normal_bf16(V, d, 13, 0.05)
    h = gi.gen_h(3, d, 14)
    z = np.zeros((3, V), dtype=np.float32)                        # all equal: the 256 smallest ids
    z[1, 100:900] = 1.0                                           # 800 tied at the top: ids 100..355
    z[2] = -0.0
    z[2, ::7] = 0.0                                               # +0 and -0 tie
    got, want = run(ev, z, h, W, 256, 1.0), kl_gate(z, h, W, 256, 1.0)
    check(got, want, "ties")
    assert got[0][0].tolist() == list(range(256)) and got[0][1].tolist() == list(range(100, 356))


def test_many_equal_logits_across_slices(ev):
    """1,500 logits per eighth of the vocabulary tie at the top: every slice hands all of them on
    (fewer than its list holds), 12,000 keys reach the bound on the logits alone, more than the
    last stage's list holds, so it has to fall back to the bound on the whole (logit, id) key.
    The support is then the 256 smallest ids among the tied ones."""
    from oracle import kl_gate
    V, d, E = 151936, 64, 2
    rng = np.random.default_rng(77)
    W = gi.gen_normal_bf16(V, d, 15, 0.05)
    h = gi.gen_h(E, d, 16)
    z = (rng.standard_normal((E, V)) * 0.5).astype(np.float32).clip(-4.0, 4.0)
    tied = []
    for e in range(E):
        ids = np.concatenate([g * 18992 + rng.choice(18992, 1500, replace=False) for g in range(8)])
        z[e, ids] = 5.0
        tied.append(np.sort(ids))
    got, want = run(ev, z, h, W, 256, 1.0), kl_gate(z, h, W, 256, 1.0)
    check(got, want, "ties across slices")
    for e in range(E):
        assert got[0][e].tolist() == tied[e][:256].tolist()


def test_full_size(ev):
    """60 verification events over the 151,936-token vocabulary, K = 256, d = 4096."""
    from oracle import kl_gate
    c = gi.CONFIGS["draft60"]
    W = gi.gen_W_lm(c["V"], c["d"])
    E = 60
    h = gi.gen_h(E, c["d"], gi.SEED_H + 70)
    rng = np.random.default_rng(5)
    # target logits = the draft's own logits plus noise, so that the divergence is of order 0.1
    hf = gi.bf16_bits_to_f32(h)
    z = np.empty((E, c["V"]), dtype=np.float32)
    for r0 in range(0, c["V"], 16384):
        z[:, r0:r0 + 16384] = hf @ gi.bf16_bits_to_f32(W[r0:r0 + 16384]).T
    z += (rng.standard_normal(z.shape) * 0.5).astype(np.float32)
    got = run(ev, z, h, W, 256, 1.0)
    want = kl_gate(z, h, W, 256, 1.0)                             # the oracle on every event
    check(got, want, "full size")
    assert np.all(got[3] > 0) and np.all(np.isfinite(got[3]))
    for e in range(E):                                            # properties on all events
        assert len(set(got[0][e].tolist())) == 256 and np.all(np.diff(got[1][e]) <= 0)
        assert got[1][e][-1] >= np.partition(z[e], -256)[-256]
