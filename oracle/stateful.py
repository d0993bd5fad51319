"""Oracle: the stateful variant of the step - Algorithm 2 ("Mobile MP-LoRA module"), where the perturbed pair is
kept between steps and the noise of the last step is read back from it instead of being regenerated.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

Algorithm 2 is printed for q = 1 and for the factor B only, and keeps no master: the pair (B[0], B[1]) is the
state.  Its steps, in the paper's notation:  diff = (B[0] - B[1]) / 2  (= eps z of the last step);
update = eta g diff / eps;  z = eps randn;  B[0] <- B[0] - diff - update + z;  B[1] <- B[1] + diff - update - z.
`mobile_pair_step` is that recurrence as printed.  `stateful_update` is the reading used for q queries and an
explicit binary32 master theta (every pair is centred on it, so B[0] - diff and B[1] + diff are both theta up to
rounding):  diff_k = (theta_k(+) - theta_k(-)) / 2,  theta <- theta - sum_k (eta g_k / q) diff_k / eps,  and the
new pairs are theta +- eps z'_k with fresh noise - exactly Algorithm 1's update with z_k replaced by what the
stored pair says it was.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from .precision import Precision
from .zo import draw_z, perturb


def mobile_pair_step(B0: np.ndarray, B1: np.ndarray, g: float, eta: float, eps: float, z_scaled: np.ndarray):
    """Algorithm 2 as printed (q = 1, no master), in binary64.  `z_scaled` is the algorithm's z = eps * randn.
    Returns the new pair."""
    B0 = np.asarray(B0, np.float64)
    B1 = np.asarray(B1, np.float64)
    diff = (B0 - B1) / 2.0
    update = eta * g * (diff / eps)
    return B0 - diff - update + z_scaled, B1 + diff - update - z_scaled


def recovered_noise(plus: np.ndarray, minus: np.ndarray, eps: float, prec: Precision) -> np.ndarray:
    """diff / eps of Algorithm 2: the direction the stored pair was actually perturbed along."""
    if prec.exact:
        return (np.asarray(plus, np.float64) - np.asarray(minus, np.float64)) / 2.0 / float(np.float32(eps))
    d = (plus.astype(np.float32) - minus.astype(np.float32)) * np.float32(0.5)     # binary32 subtract, exact halving
    return d / np.float32(eps)                                                     # binary32 divide


def stateful_update(masters: np.ndarray, pairs: Sequence[Tuple[np.ndarray, np.ndarray]], g: np.ndarray,
                    eps: float, lr: float, prec: Precision) -> np.ndarray:
    """theta <- theta - sum_k (lr g_k / q) (diff_k / eps)  (Algorithm 2's diff and update, q queries)."""
    q = len(g)
    if prec.exact:
        acc = np.zeros(masters.size, dtype=np.float64)
        for k in range(q):
            acc += g[k] * recovered_noise(pairs[k][0], pairs[k][1], eps, prec)
        return masters.astype(np.float64) - float(np.float32(lr)) * acc / q
    acc = np.zeros(masters.size, dtype=np.float32)
    for k in range(q):
        c = np.float32(float(np.float32(lr)) * float(np.float32(g[k])) / q)       # same coefficient as Algorithm 1's update
        acc = acc + c * recovered_noise(pairs[k][0], pairs[k][1], eps, prec)
    return (masters - acc).astype(np.float32)


def make_pairs(masters: np.ndarray, layout, seed: int, step: int, q: int, eps: float, perturb_A: bool,
               prec: Precision) -> List[Tuple[np.ndarray, np.ndarray]]:
    """The 2q perturbed copies of a step, pair k = (theta + eps z_k, theta - eps z_k)."""
    out = []
    for k in range(q):
        z = draw_z(layout, seed, step, k, masters.size, perturb_A)
        out.append((perturb(masters, z, +1, eps, prec), perturb(masters, z, -1, eps, prec)))
    return out


def stateful_update_and_reperturb(masters, pairs, g, layout, seed: int, next_step: int, eps: float, lr: float,
                                  perturb_A: bool, prec: Precision):
    """One pass of Algorithm 2 over the state: update from the stored pairs, then re-perturb with the noise of
    `next_step`.  Returns (new masters, new pairs)."""
    new = stateful_update(masters, pairs, g, eps, lr, prec)
    return new, make_pairs(new, layout, seed, next_step, len(g), eps, perturb_A, prec)
