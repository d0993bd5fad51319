"""Oracle: one step of Algorithm 1 - perturb, 2q losses, two-point estimates, update.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

Follows Algorithm 1 step by step with n = 2q *separate* single-copy evaluations (the batched
MP-LoRA pass of Section 3 must give the same numbers, since the copies are independent).  Copy
order: c = 2k + s, s = 0 for +eps z_k and s = 1 for -eps z_k.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np

from .noise import noise_tensor
from .model import copy_loss
from .precision import Precision


def draw_z(layout, seed: int, step: int, k: int, total: int, perturb_A: bool) -> np.ndarray:
    """z_k over the flat LoRA vector (zero on A when only B is perturbed, as in LoRA-FA)."""
    z = np.zeros(total, dtype=np.float32)
    for t in layout:
        if t.factor == 0 and not perturb_A:
            continue
        n = t.rows * t.cols
        z[t.offset:t.offset + n] = noise_tensor(seed, step, k, t.tensor_id, n)
    return z


def perturb(masters: np.ndarray, z: np.ndarray, sign: int, eps: float, prec: Precision) -> np.ndarray:
    """theta_l + sign * eps * z  (Algorithm 1, the perturbation step of the inner loop)."""
    e32 = np.float32(eps)
    if prec.exact:
        return masters.astype(np.float64) + sign * float(e32) * z.astype(np.float64)
    p = e32 * z                                   # binary32 product, then binary32 add/subtract
    return masters + p if sign > 0 else masters - p


def split_factors(layout, flat) -> Dict[Tuple[int, int], Tuple[np.ndarray, np.ndarray]]:
    out: Dict[Tuple[int, int], List] = {}
    for t in layout:
        out.setdefault((t.layer, t.target), [None, None])[t.factor] = \
            flat[t.offset:t.offset + t.rows * t.cols].reshape(t.rows, t.cols)
    return {k: (v[0], v[1]) for k, v in out.items()}


def perturbed_losses(w, layout, frozen, masters, tokens, labels, seed: int, step: int,
                     prec: Precision, q=None, eps=None, lengths=None) -> np.ndarray:
    """l_c for c = 0..2q-1 (Algorithm 1, outer and inner loops)."""
    q = w.q if q is None else q
    eps = w.eps if eps is None else eps
    losses = np.zeros(2 * q, dtype=np.float64)
    for k in range(q):
        z = draw_z(layout, seed, step, k, masters.size, w.perturb_A)
        for s, sign in enumerate((+1, -1)):
            theta = perturb(masters, z, sign, eps, prec)
            losses[2 * k + s] = copy_loss(w, frozen, split_factors(layout, theta), tokens, labels, prec, lengths=lengths)
    return losses


def projected_grads(losses: np.ndarray, eps: float) -> np.ndarray:
    """g_k = (l_k(+) - l_k(-)) / (2 eps)  (Algorithm 1, the two-point estimate), in binary64."""
    losses = np.asarray(losses, dtype=np.float64)
    return (losses[0::2] - losses[1::2]) / (2.0 * float(np.float32(eps)))


def zo_update(masters: np.ndarray, g: np.ndarray, layout, seed: int, step: int, lr: float,
              perturb_A: bool, prec: Precision) -> np.ndarray:
    """theta_l <- theta_l - lr * (1/q) sum_k g_k z_k with z_k regenerated (Algorithm 1, the parameter update)."""
    q = len(g)
    if prec.exact:
        acc = np.zeros(masters.size, dtype=np.float64)
        for k in range(q):
            acc += g[k] * draw_z(layout, seed, step, k, masters.size, perturb_A).astype(np.float64)
        return masters.astype(np.float64) - float(np.float32(lr)) * acc / q
    # binary32 masters: coefficient c_k = fl32(lr * fl32(g_k) / q), sum over k in order, one subtract
    acc = np.zeros(masters.size, dtype=np.float32)
    for k in range(q):
        c = np.float32(float(np.float32(lr)) * float(np.float32(g[k])) / q)
        acc = acc + c * draw_z(layout, seed, step, k, masters.size, perturb_A)
    return (masters - acc).astype(np.float32)


def zo_step(w, layout, frozen, masters, tokens, labels, seed: int, step: int, prec: Precision):
    """One full step; returns (losses[2q], g[q], new masters)."""
    losses = perturbed_losses(w, layout, frozen, masters, tokens, labels, seed, step, prec)
    if not prec.exact:
        losses = losses.astype(np.float32).astype(np.float64)
    g = projected_grads(losses, w.eps)
    new = zo_update(masters, g, layout, seed, step, w.lr, w.perturb_A, prec)
    return losses, g, new
