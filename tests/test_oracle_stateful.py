"""Pins for the oracle of the stateful variant (Algorithm 2).

* a hand-computed instance of the printed recurrence (one element, numbers chosen to be exact in binary);
* q = 1: the master form equals the printed pair-only recurrence in binary64 (both members of the new pair);
* exact arithmetic: the noise read back from a stored pair is the noise that made it, so the stateful update equals
  Algorithm 1's seed-replayed update;
* binary32: the read-back direction differs from the regenerated one by at most the rounding of theta +- eps z,
  and the two updates stay within a few ulps of each other;
* planted mistakes (a dropped 1/2, a wrong sign of the update, eps forgotten) are caught by the pins above.
"""
import numpy as np
import pytest

import workloads as W
from oracle import stateful, zo
from oracle.precision import Precision
from small_workloads import C1


def test_printed_recurrence_by_hand():
    # master 1.0, eps z_old = 0.5 (eps = 0.5, z_old = 1): pair (1.5, 0.5); g = 2, eta = 0.125: update = 0.25;
    # new z = eps * randn = 0.25  ->  B[0] = 1.5 - 0.5 - 0.25 + 0.25 = 1.0,  B[1] = 0.5 + 0.5 - 0.25 - 0.25 = 0.5
    b0, b1 = stateful.mobile_pair_step(np.array([1.5]), np.array([0.5]), g=2.0, eta=0.125, eps=0.5,
                                       z_scaled=np.array([0.25]))
    assert b0[0] == 1.0 and b1[0] == 0.5
    # the new pair is centred on master - update = 0.75 with half-width 0.25
    assert (b0[0] + b1[0]) / 2 == 0.75 and (b0[0] - b1[0]) / 2 == 0.25


def _setup(q=3, perturb_A=True, seed=7):
    w = C1.with_(q=q, perturb_A=perturb_A)
    lay = W.lora_layout(w)
    masters = W.make_lora_masters(w, seed, b_std=0.02)
    return w, lay, masters


def test_master_form_equals_printed_recurrence_for_q1():
    w, lay, masters = _setup(q=1)
    ex = Precision("exact")
    eps, lr, g = 1e-2, 1e-3, np.array([0.37])
    pairs = stateful.make_pairs(masters, lay, 11, 0, 1, eps, True, ex)
    new, new_pairs = stateful.stateful_update_and_reperturb(masters, pairs, g, lay, 11, 1, eps, lr, True, ex)
    z_next = float(np.float32(eps)) * zo.draw_z(lay, 11, 1, 0, masters.size, True).astype(np.float64)
    b0, b1 = stateful.mobile_pair_step(pairs[0][0], pairs[0][1], g[0], float(np.float32(lr)), float(np.float32(eps)), z_next)
    assert np.abs(b0 - new_pairs[0][0]).max() <= 1e-15
    assert np.abs(b1 - new_pairs[0][1]).max() <= 1e-15
    assert np.abs((b0 + b1) / 2 - new).max() <= 1e-15


@pytest.mark.parametrize("perturb_A", [True, False])
def test_exact_arithmetic_equals_seed_replay(perturb_A):
    w, lay, masters = _setup(q=3, perturb_A=perturb_A)
    ex = Precision("exact")
    eps, lr = 1e-3, 1e-2
    g = np.array([0.8, -1.7, 0.05])
    pairs = stateful.make_pairs(masters, lay, 5, 4, 3, eps, perturb_A, ex)
    a = stateful.stateful_update(masters, pairs, g, eps, lr, ex)
    b = zo.zo_update(masters, g, lay, 5, 4, lr, perturb_A, ex)
    assert np.abs(a - b).max() <= 1e-12 * max(1.0, np.abs(b).max())
    if not perturb_A:                       # LoRA-FA: A is neither perturbed nor moved
        for t in lay:
            if t.factor == 0:
                sl = slice(t.offset, t.offset + t.rows * t.cols)
                assert np.array_equal(a[sl], masters[sl].astype(np.float64))


def test_binary32_read_back_direction_and_update():
    w, lay, masters = _setup(q=2)
    p32 = Precision("f32")
    eps, lr = float(np.float32(1e-3)), 1e-2
    g = np.array([1.3, -0.4])
    pairs = stateful.make_pairs(masters, lay, 9, 2, 2, eps, True, p32)
    for k in range(2):
        z = zo.draw_z(lay, 9, 2, k, masters.size, True)
        zh = stateful.recovered_noise(pairs[k][0], pairs[k][1], eps, p32)
        assert zh.dtype == np.float32
        # theta +- eps z is rounded to an ulp of theta: the recovered direction is off by at most ~ulp(theta)/eps
        bound = 2.0 ** -23 * (np.abs(masters) + eps * np.abs(z)) / eps + 2.0 ** -22 * np.abs(z)
        assert (np.abs(zh.astype(np.float64) - z) <= bound).all()
    a = stateful.stateful_update(masters, pairs, g, eps, lr, p32)
    b = zo.zo_update(masters, g, lay, 9, 2, lr, True, p32)
    assert a.dtype == np.float32
    assert np.abs(a.astype(np.float64) - b).max() <= 4 * 2.0 ** -23 * np.abs(b).max()
    assert not np.array_equal(a, masters)


def test_planted_mistakes_are_caught():
    w, lay, masters = _setup(q=2)
    ex = Precision("exact")
    eps, lr = 1e-3, 1e-2
    g = np.array([1.3, -0.4])
    pairs = stateful.make_pairs(masters, lay, 9, 2, 2, eps, True, ex)
    good = zo.zo_update(masters, g, lay, 9, 2, lr, True, ex)
    m64 = masters.astype(np.float64)
    scale = np.abs(good - m64).max()

    def variant(half=0.5, sign=-1.0, use_eps=True):
        acc = np.zeros(masters.size)
        for k in range(2):
            d = (pairs[k][0] - pairs[k][1]) * half
            acc += g[k] * (d / float(np.float32(eps)) if use_eps else d)
        return m64 + sign * float(np.float32(lr)) * acc / 2

    assert np.abs(variant() - good).max() <= 1e-9 * scale
    for kw in (dict(half=1.0), dict(sign=+1.0), dict(use_eps=False)):
        assert np.abs(variant(**kw) - good).max() > 0.4 * scale
