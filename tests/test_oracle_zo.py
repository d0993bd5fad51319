"""Pins for the oracle's estimator and update (CPU only): the four checks the method's
definition fixes - eps = 0 identity, sign-flip swap, g_k against brute-force central finite
differences, and convergence of the averaged estimate to the per-parameter gradient.
"""
import numpy as np
import pytest
import torch

from oracle import zo
from oracle.model import copy_loss
from oracle.precision import Precision

from small_workloads import C1, MINI_LLAMA, MICRO, bundle
from torch_reference import torch_loss

EXACT = Precision("exact")
SEED = 3456


def _losses(b, prec, **kw):
    return zo.perturbed_losses(b["w"], b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"],
                               SEED, kw.pop("step", 0), prec, **kw)


def _torch(b, flat):
    return float(torch_loss(b["w"], b["frozen"], b["layout"], torch.as_tensor(flat, dtype=torch.float64),
                            b["tokens"], b["labels"]))


@pytest.mark.parametrize("mode", ["exact", "f32", "bf16"])
def test_eps_zero_gives_identical_losses_equal_to_unperturbed(mode):
    b = bundle(C1, b_std=0.02)
    prec = Precision(mode)
    l = _losses(b, prec, eps=0.0)
    base = copy_loss(C1, b["frozen"], zo.split_factors(b["layout"], b["masters"]), b["tokens"], b["labels"], prec)
    assert l.shape == (2 * C1.q,)
    assert np.all(l == base)
    if mode == "exact":
        assert base == pytest.approx(_torch(b, b["masters"]), rel=1e-12)


@pytest.mark.parametrize("mode", ["exact", "f32", "bf16"])
def test_negating_noise_swaps_plus_and_minus(mode):
    b = bundle(C1, b_std=0.02)
    prec = Precision(mode)
    lp = _losses(b, prec, eps=1e-3)
    lm = _losses(b, prec, eps=-1e-3)
    assert np.array_equal(lp[0::2], lm[1::2]) and np.array_equal(lp[1::2], lm[0::2])
    assert np.array_equal(zo.projected_grads(lp, 1e-3), -zo.projected_grads(lm, 1e-3))
    assert np.all(lp[0::2] != lp[1::2])


def test_copies_use_distinct_noise_per_query_and_shared_noise_per_sign():
    b = bundle(C1, b_std=0.02)
    z0 = zo.draw_z(b["layout"], SEED, 0, 0, b["masters"].size, True)
    z1 = zo.draw_z(b["layout"], SEED, 0, 1, b["masters"].size, True)
    assert not np.array_equal(z0, z1)
    plus = zo.perturb(b["masters"], z0, +1, 1e-3, EXACT)
    minus = zo.perturb(b["masters"], z0, -1, 1e-3, EXACT)
    assert np.allclose((plus - minus) / (2 * float(np.float32(1e-3))), z0, rtol=0, atol=1e-9)
    assert np.allclose((plus + minus) / 2, b["masters"], rtol=0, atol=1e-12)
    zfa = zo.draw_z(b["layout"], SEED, 0, 0, b["masters"].size, False)     # LoRA-FA: A untouched
    for t in b["layout"]:
        sl = slice(t.offset, t.offset + t.rows * t.cols)
        assert np.all(zfa[sl] == 0) if t.factor == 0 else np.array_equal(zfa[sl], z0[sl])


@pytest.mark.parametrize("wl", [C1, MINI_LLAMA], ids=lambda w: w.name)
def test_projected_gradient_matches_brute_force_central_difference(wl):
    """g_k vs (L(theta + h z) - L(theta - h z)) / 2h evaluated by the independent torch loss."""
    b = bundle(wl, b_std=0.02)
    eps = float(np.float32(1e-3))
    g = zo.projected_grads(_losses(b, EXACT, eps=eps), eps)
    flat = b["masters"].astype(np.float64)
    t = torch.tensor(flat, requires_grad=True)
    torch_loss(wl, b["frozen"], b["layout"], t, b["tokens"], b["labels"]).backward()
    grad = t.grad.numpy()
    for k in range(wl.q):
        z = zo.draw_z(b["layout"], SEED, 0, k, flat.size, True).astype(np.float64)
        fd = {h: (_torch(b, flat + h * z) - _torch(b, flat - h * z)) / (2 * h) for h in (1e-2, 1e-3, 1e-4)}
        assert g[k] == pytest.approx(fd[eps if eps in fd else 1e-3], rel=1e-4)
        # brute force at the same step agrees to rounding; smaller steps converge quadratically
        same = (_torch(b, flat + eps * z) - _torch(b, flat - eps * z)) / (2 * eps)
        assert g[k] == pytest.approx(same, rel=1e-8)
        exact = float(grad @ z)
        e2, e3 = abs(fd[1e-2] - exact), abs(fd[1e-3] - exact)
        # O(eps^2) truncation of the two-point formula; a directional derivative can be small by chance,
        # so the bound is relative to its typical size |grad|
        assert abs(g[k] - exact) <= 2e-3 * np.linalg.norm(grad)
        assert e3 < e2 * 0.05 or e2 < 1e-9 * abs(exact)


def test_average_of_g_z_converges_to_per_parameter_finite_difference_gradient():
    b = bundle(MICRO, b_std=0.05, scale_weights=4.0)
    w, flat = MICRO, b["masters"].astype(np.float64)
    n = flat.size
    assert n == 256
    h = 1e-5
    fd = np.zeros(n)
    lora_loss = lambda v: copy_loss(w, b["frozen"], zo.split_factors(b["layout"], v), b["tokens"], b["labels"], EXACT)
    for i in range(n):                                # backprop-free brute-force gradient
        e = np.zeros(n)
        e[i] = h
        fd[i] = (lora_loss(flat + e) - lora_loss(flat - e)) / (2 * h)
    t = torch.tensor(flat, requires_grad=True)
    torch_loss(w, b["frozen"], b["layout"], t, b["tokens"], b["labels"]).backward()
    assert np.allclose(fd, t.grad.numpy(), rtol=1e-5, atol=1e-9 * np.abs(fd).max() + 1e-12)

    eps = 1e-3
    acc = np.zeros(n)
    errs = {}
    N = 6000
    for i in range(N):
        z = zo.draw_z(b["layout"], SEED + i // 4, i % 4, 0, n, True).astype(np.float64)
        g = (lora_loss(flat + eps * z) - lora_loss(flat - eps * z)) / (2 * eps)
        acc += g * z
        if i + 1 in (375, 1500, 6000):
            errs[i + 1] = np.linalg.norm(acc / (i + 1) - fd) / np.linalg.norm(fd)
    # relative error ~ sqrt((d+1)/N): 0.83, 0.41, 0.21; must fall by about 2x per 4x samples
    assert errs[6000] < 0.30
    assert errs[6000] < 0.7 * errs[1500] < 0.7 * 0.7 * errs[375] * 1.2
    est = acc / N
    assert est @ fd / (np.linalg.norm(est) * np.linalg.norm(fd)) > 0.95


def test_with_zero_B_the_A_block_of_the_gradient_vanishes():
    b = bundle(MICRO, scale_weights=4.0)              # B = 0
    flat = b["masters"].astype(np.float64)
    t = torch.tensor(flat, requires_grad=True)
    torch_loss(MICRO, b["frozen"], b["layout"], t, b["tokens"], b["labels"]).backward()
    g = t.grad.numpy()
    for tn in b["layout"]:
        blk = g[tn.offset:tn.offset + tn.rows * tn.cols]
        assert np.all(blk == 0) if tn.factor == 0 else np.any(blk != 0)
    # the estimator sees this too: perturbing only A gives l(+) == l(-) exactly
    z = zo.draw_z(b["layout"], SEED, 0, 0, flat.size, True).astype(np.float64)
    for tn in b["layout"]:
        if tn.factor == 1:
            z[tn.offset:tn.offset + tn.rows * tn.cols] = 0
    lp = copy_loss(MICRO, b["frozen"], zo.split_factors(b["layout"], flat + 1e-3 * z), b["tokens"], b["labels"], EXACT)
    lm = copy_loss(MICRO, b["frozen"], zo.split_factors(b["layout"], flat - 1e-3 * z), b["tokens"], b["labels"], EXACT)
    assert lp == lm


@pytest.mark.parametrize("mode", ["exact", "f32"])
def test_update_is_minus_lr_over_q_times_sum_g_z(mode):
    b = bundle(C1, b_std=0.02)
    g = np.array([0.37, -1.25])
    new = zo.zo_update(b["masters"], g, b["layout"], SEED, 4, 1e-2, True, Precision(mode))
    z = [zo.draw_z(b["layout"], SEED, 4, k, b["masters"].size, True).astype(np.float64) for k in range(2)]
    want = b["masters"].astype(np.float64) - float(np.float32(1e-2)) * (g[0] * z[0] + g[1] * z[1]) / 2
    tol = 1e-15 if mode == "exact" else 2e-7 * np.abs(want).max()
    assert np.abs(new - want).max() <= tol
    assert new.dtype == (np.float64 if mode == "exact" else np.float32)


def test_lora_fa_update_leaves_A_bit_unchanged():
    b = bundle(C1.with_(perturb_A=False), b_std=0.02)
    new = zo.zo_update(b["masters"], np.array([0.5, 0.25]), b["layout"], SEED, 0, 1e-2, False, Precision("f32"))
    for t in b["layout"]:
        sl = slice(t.offset, t.offset + t.rows * t.cols)
        assert np.array_equal(new[sl], b["masters"][sl]) == (t.factor == 0)


def test_steps_chain_and_decrease_a_learnable_loss():
    """Several steps in a row: state is only (masters, seed, step); the loss goes down on average."""
    wl = MICRO.with_(q=8, lr=2e-2, eps=1e-3)
    b = bundle(wl, scale_weights=4.0)
    prec = Precision("exact")
    m = b["masters"].astype(np.float64)
    first = copy_loss(wl, b["frozen"], zo.split_factors(b["layout"], m), b["tokens"], b["labels"], prec)
    for step in range(30):
        _, g, m = zo.zo_step(wl, b["layout"], b["frozen"], m, b["tokens"], b["labels"], SEED, step, prec)
        assert g.shape == (8,)
    last = copy_loss(wl, b["frozen"], zo.split_factors(b["layout"], m), b["tokens"], b["labels"], prec)
    assert last < first
    # replaying steps 0..29 from the same start reproduces the same masters (resume = same state)
    m2 = b["masters"].astype(np.float64)
    for step in range(30):
        _, _, m2 = zo.zo_step(wl, b["layout"], b["frozen"], m2, b["tokens"], b["labels"], SEED, step, prec)
    assert np.array_equal(m, m2)
