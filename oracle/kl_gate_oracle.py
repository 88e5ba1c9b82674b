"""Plain reference of the retained-support KL gate of Path B (test infrastructure).

What it follows: the EvoSpec paper, Sec. "Online parameter update" (Eq. 5 and the text around
it) and Algorithm 1, Path B: the target model's K_logit = 256 largest logits are retained; they
and the draft model's logits on the same ids are turned into distributions with the distillation
temperature T_KD,  p = Softmax(z_target[S] / T),  q = Softmax(z_draft[S] / T),  and the sample is
admitted to the replay buffer when  D_KL(p || q) > eps_align = 0.1  (or the draft was rejected).
Draft logits come from Eq. 1: z_draft[i] = h_draft . W_LM[i].

fp64 throughout, on the bf16 bit patterns of h and W and the fp32 target logits.  Readings where
the paper is silent: ties among target logits go to the smaller id (as everywhere in this build);
the support is reported by decreasing target logit; T_KD^2 of Eq. 5 belongs to the training loss,
not to the gate.

Only tests, the smoke check and the benchmark's CPU leg may import this module.
"""
from __future__ import annotations

import numpy as np


def _bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def kl_gate(z_target: np.ndarray, h_bits: np.ndarray, W_bits: np.ndarray, K: int, T: float = 1.0):
    """z_target fp32 [E, V]; h_bits uint16 [E, d]; W_bits uint16 [V, d].
    Returns (support int32 [E, K], z_t float64 [E, K], z_q float64 [E, K], kl float64 [E])."""
    E, V = z_target.shape
    support = np.empty((E, K), dtype=np.int32)
    zt = np.empty((E, K), dtype=np.float64)
    zq = np.empty((E, K), dtype=np.float64)
    kl = np.empty((E,), dtype=np.float64)
    for e in range(E):
        z = z_target[e].astype(np.float64)
        order = np.lexsort((np.arange(V), -z))[:K]              # by decreasing logit, then increasing id
        support[e] = order
        zt[e] = z[order]
        h = _bf16_to_f64(h_bits[e])
        zq[e] = _bf16_to_f64(W_bits[order]) @ h
        a, b = zt[e] / T, zq[e] / T
        log_p = a - (a.max() + np.log(np.exp(a - a.max()).sum()))
        log_q = b - (b.max() + np.log(np.exp(b - b.max()).sum()))
        kl[e] = float(np.sum(np.exp(log_p) * (log_p - log_q)))
    return support, zt, zq, kl
