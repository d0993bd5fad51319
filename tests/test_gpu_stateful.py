"""GPU parity for the stateful variant (Algorithm 2): update read back from the stored pairs and re-perturbation
in one kernel, bit-exact to the oracle; a training run of several steps with it against the oracle's run."""
import numpy as np
import pytest

import workloads as W
from oracle import stateful, zo
from oracle.precision import Precision
from gpu_helpers import make_bundle, gpu_model
from small_workloads import C1

pytestmark = pytest.mark.gpu
SEED = 0x0BAD_5EED_1234


def _bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("name,perturb_A", [("c1_tiny_fp32", 1), ("c1_tiny_fp32", 0), ("c2_opt125m", 1)])
def test_update_regen_bit_exact_from_given_losses(name, perturb_A):
    import torch
    w = W.get_workload(name).with_(n_layers=2, perturb_A=perturb_A)
    b = make_bundle(w, b_std=0.01)
    mdl = gpu_model(b)
    lay, prec = b["layout"], Precision("f32")           # masters and copies are binary32 in every model dtype
    masters = b["masters"].copy()
    mdl.regen_noise(SEED, 5)
    pairs = stateful.make_pairs(masters, lay, SEED, 5, w.q, w.eps, bool(perturb_A), prec)
    rng = np.random.default_rng(3)
    for step in (6, 7):                                  # two passes: the second reads pairs the kernel itself wrote
        losses = np.float32(rng.normal(0.7, 1e-3, size=2 * w.q))
        mdl.losses[:2 * w.q] = torch.from_numpy(losses).cuda()
        g_gpu = mdl.zo_update_regen(step).cpu().numpy()
        g = zo.projected_grads(losses, w.eps)
        assert np.array_equal(_bits(g_gpu), _bits(g.astype(np.float32)))
        masters, pairs = stateful.stateful_update_and_reperturb(masters, pairs, g, lay, SEED, step, w.eps, w.lr,
                                                                bool(perturb_A), prec)
        assert np.array_equal(_bits(mdl.masters.cpu().numpy()), _bits(masters))
        for k in range(w.q):
            for s in range(2):
                assert np.array_equal(_bits(mdl.perturbed_copy(2 * k + s).cpu().numpy()), _bits(pairs[k][s]))


def test_stateful_training_run_matches_oracle_fp32():
    """Five steps of forward + update_regen on the tiny fp32 workload: losses and masters as the oracle's run."""
    import torch
    from oracle.model import copy_loss
    w = C1
    b = make_bundle(w, b_std=0.01)
    mdl = gpu_model(b)
    lay, prec = b["layout"], Precision("f32")
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    masters = b["masters"].copy()
    mdl.regen_noise(SEED, 0)
    pairs = stateful.make_pairs(masters, lay, SEED, 0, w.q, w.eps, True, prec)
    for step in range(5):
        got = mdl.forward_perturbed(tok, lab).cpu().numpy()
        want = np.array([copy_loss(w, b["frozen"], zo.split_factors(lay, pairs[k][s]), b["tokens"], b["labels"], prec)
                         for k in range(w.q) for s in range(2)], dtype=np.float32)
        assert np.array_equal(_bits(got), _bits(want)), (step, got, want)
        mdl.zo_update_regen(step + 1)
        g = zo.projected_grads(want, w.eps)
        masters, pairs = stateful.stateful_update_and_reperturb(masters, pairs, g, lay, SEED, step + 1, w.eps, w.lr, True, prec)
        assert np.array_equal(_bits(mdl.masters.cpu().numpy()), _bits(masters))
    # and the run stays within a few ulps of Algorithm 1's (regenerate + replay) run from the same start
    m2 = gpu_model(b)
    for step in range(5):
        m2.zo_step(tok, lab, SEED, step)
    a, c = mdl.masters.cpu().numpy().astype(np.float64), m2.masters.cpu().numpy().astype(np.float64)
    moved = np.abs(c - b["masters"]).max()
    assert moved > 0 and np.abs(a - c).max() <= 1e-3 * moved + 8 * 2.0 ** -23 * np.abs(c).max()
