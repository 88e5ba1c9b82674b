"""Pins of the KL-gate oracle (no GPU): closed forms, library cross-checks, invariances."""
import math

import numpy as np
import pytest
import scipy.special
import torch

import evospec_inputs as gi
from oracle import kl_gate


def bits(x):
    return gi.f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_two_point_closed_form():
    # V = 4, d = 2, K = 2.  Target logits 0, ln 3, -5, -7 -> support ids 1, 0 with p = (3/4, 1/4).
    # W rows (bf16-exact): id0 = (1, 0), id1 = (0, 1); h = (ln-free) (0.5, 1.5) -> draft logits
    # on the support (id1, id0) = (1.5, 0.5) -> q = (e/(1+e), 1/(1+e)).
    z = np.array([[0.0, math.log(3.0), -5.0, -7.0]], dtype=np.float32)
    W = bits([[1, 0], [0, 1], [2, 2], [3, 3]])
    h = bits([[0.5, 1.5]])
    s, zt, zq, kl = kl_gate(z, h, W, 2, 1.0)
    assert s.tolist() == [[1, 0]] and zq.tolist() == [[1.5, 0.5]]
    p = np.array([np.exp(np.float64(z[0, 1])), 1.0]); p /= p.sum()
    q = np.array([math.e, 1.0]) / (1.0 + math.e)
    want = float(np.sum(p * np.log(p / q)))
    assert abs(kl[0] - want) < 1e-12
    # temperature 2 halves both logit vectors
    _, _, _, kl2 = kl_gate(z, h, W, 2, 2.0)
    p2 = np.array([np.exp(np.float64(z[0, 1]) / 2), 1.0]); p2 /= p2.sum()
    q2 = np.array([math.exp(0.5), 1.0]) / (1.0 + math.exp(0.5))
    assert abs(kl2[0] - float(np.sum(p2 * np.log(p2 / q2)))) < 1e-12


def test_against_library_routines_and_properties():
    rng = np.random.default_rng(0)
    E, V, d, K = 5, 3000, 64, 256
    W = gi.gen_normal_bf16(V, d, 3, 0.05)
    h = gi.gen_h(E, d, 4)
    z = (rng.standard_normal((E, V)) * 2).astype(np.float32)
    s, zt, zq, kl = kl_gate(z, h, W, K, 1.0)
    Wf, hf = gi.bf16_bits_to_f32(W).astype(np.float64), gi.bf16_bits_to_f32(h).astype(np.float64)
    for e in range(E):
        top = torch.topk(torch.from_numpy(z[e].astype(np.float64)), K)
        assert set(top.indices.tolist()) == set(s[e].tolist())
        assert np.all(np.diff(zt[e]) <= 0)
        np.testing.assert_allclose(zq[e], (hf[e] @ Wf.T)[s[e]], rtol=1e-12)
        p = scipy.special.softmax(zt[e]); q = scipy.special.softmax(zq[e])
        assert abs(kl[e] - scipy.special.rel_entr(p, q).sum()) < 1e-10
        t = torch.nn.functional.kl_div(torch.log_softmax(torch.from_numpy(zq[e]), 0),
                                       torch.softmax(torch.from_numpy(zt[e]), 0), reduction="sum")
        assert abs(kl[e] - float(t)) < 1e-10
        assert kl[e] > 0
    # a draft that reproduces the target up to a constant has zero divergence: put the target
    # logits (plus 3) where the draft's would be, via W = I-like rows (d = V here)
    V2 = 40
    W2 = bits(np.eye(V2))
    zt2 = np.round(rng.standard_normal((1, V2)) * 4) / 4                  # bf16-exact values
    _, _, zq2, kl2 = kl_gate(zt2.astype(np.float32), bits(zt2 + 3.0), W2, 8, 1.5)
    np.testing.assert_allclose(zq2[0], np.sort(zt2[0])[::-1][:8] + 3.0)
    assert abs(kl2[0]) < 1e-14


def test_ties_go_to_the_smaller_id_and_support_is_ordered():
    z = np.zeros((1, 50), dtype=np.float32)
    z[0, 40] = 1.0
    W = gi.gen_normal_bf16(50, 8, 1, 0.1)
    s, zt, _, _ = kl_gate(z, gi.gen_h(1, 8, 2), W, 5)
    assert s.tolist() == [[40, 0, 1, 2, 3]] and zt.tolist() == [[1.0, 0.0, 0.0, 0.0, 0.0]]
