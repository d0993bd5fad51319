"""GPU parity: per-copy losses, projected gradients and updated LoRA factors of the HIP path against
the oracle on the same seeded inputs.

Tolerances (relative, norm-wise over the q projected gradients of a step, because a single g_k is a
zero-mean random projection and can be arbitrarily close to 0): fp32 models 1e-4, bf16 models 2e-2;
updated LoRA vector after the steps 1e-3 (fp32) / 2e-2 (bf16: B starts at 0, so the updated B is
a sum of g_k z_k and inherits the tolerance of g).
"""
import numpy as np
import pytest

import workloads as W
from gpu_helpers import make_bundle, gpu_model, gpu_steps, oracle_steps, rel_err
from small_workloads import MICRO, MINI_LLAMA, MINI_OPT

pytestmark = pytest.mark.gpu


def _check(w, b, steps, g_tol, loss_tol, theta_tol):
    Lg, Gg, Mg = gpu_steps(b, steps)
    Lo, Go, Mo = oracle_steps(b, steps)
    print(f"\n{w.name}: loss rel err {rel_err(Lg, Lo):.3e}; g rel err per step "
          f"{[f'{rel_err(Gg[s], Go[s]):.2e}' for s in range(steps)]}; theta rel err {rel_err(Mg, Mo):.3e}")
    assert np.abs(Lg - Lo).max() <= loss_tol * np.abs(Lo).max()
    for s in range(steps):
        assert rel_err(Gg[s], Go[s]) <= g_tol, (s, Gg[s], Go[s])
    assert rel_err(Mg, Mo) <= theta_tol
    return Lg, Gg, Mg


def test_c1_tiny_fp32_five_steps():
    w = W.get_workload("c1_tiny_fp32")
    _check(w, make_bundle(w), 5, g_tol=1e-4, loss_tol=1e-6, theta_tol=1e-3)


def test_c1_ten_steps_updated_factors():
    w = W.get_workload("c1_tiny_fp32")
    _check(w, make_bundle(w, b_std=0.01), 10, g_tol=1e-4, loss_tol=1e-6, theta_tol=1e-3)


@pytest.mark.parametrize("wl", [MINI_LLAMA, MINI_OPT, MINI_OPT.with_(loss_mode="next_token_all_pos", act="gelu", lora_scale=2.0),
                                MINI_LLAMA.with_(loss_mode="last_pos_label_subset", label_tokens=(3, 9), perturb_A=False)],
                         ids=["llama", "opt_fullvocab", "opt_nexttoken_gelu_scale2", "llama_lastpos_lorafa"])
def test_small_fp32_models_all_architectures(wl):
    _check(wl, make_bundle(wl, b_std=0.02), 3, g_tol=1e-4, loss_tol=1e-6, theta_tol=1e-3)


EDGE = {
    # the smallest legal batch: one query, one sequence of two tokens (a single next-token position)
    "q1_E1_S2": MICRO.with_(lora_rank=4, q=1, E=1, S=2, loss_mode="next_token_all_pos"),
    # odd sizes everywhere: 5 queries, 3 sequences of 7 tokens, sequence length below max_seq
    "q5_E3_S7": MINI_LLAMA.with_(q=5, E=3, S=7),
    # the largest rank on the output projection alone; the smallest on the key projection alone
    "rank64_o_only": MINI_LLAMA.with_(lora_rank=64, lora_targets=("o",)),
    "rank4_k_only": MINI_OPT.with_(lora_rank=4, lora_targets=("k",)),
    # untied head on the OPT-style model, sequences as long as the position table
    "opt_untied_full_positions": MINI_OPT.with_(tie_embeddings=False, S=10, max_seq=10),
    # many queries on a tiny batch (the q = 64 limit of the noise kernels' query loop is exercised by test_gpu_noise)
    "q16_E1": MICRO.with_(lora_rank=4, q=16, E=1),
}


@pytest.mark.parametrize("name", list(EDGE))
def test_edge_shapes_fp32(name):
    wl = EDGE[name]
    _check(wl, make_bundle(wl, b_std=0.02), 2, g_tol=1e-4, loss_tol=1e-6, theta_tol=1e-3)


def test_eps_zero_gives_bit_identical_losses_equal_to_the_unperturbed_oracle():
    import torch
    from oracle import zo
    from oracle.model import copy_loss
    from oracle.precision import Precision
    for name in ("c1_tiny_fp32",):
        w = W.get_workload(name)
        b = make_bundle(w, b_std=0.02)
        m = gpu_model(b)
        m.regen_noise(3456, 0, eps=0.0)
        l = m.forward_perturbed(torch.from_numpy(b["tokens"]).cuda(), torch.from_numpy(b["labels"]).cuda()).cpu().numpy()
        assert np.all(l == l[0])
        base = copy_loss(w, b["frozen"], zo.split_factors(b["layout"], b["masters"]), b["tokens"], b["labels"], Precision("f32"))
        assert abs(float(l[0]) - base) <= 1e-6 * abs(base)


def test_sign_flip_swaps_losses_on_gpu():
    """Running with -eps is not allowed by the ABI; instead check l(+)/l(-) against the oracle's swap partner:
    the oracle with negated noise must equal the GPU losses with each pair exchanged."""
    from oracle import zo
    from oracle.precision import Precision
    w = W.get_workload("c1_tiny_fp32")
    b = make_bundle(w, b_std=0.02)
    Lg, _, _ = gpu_steps(b, 1)
    neg = zo.perturbed_losses(w, b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"], 3456, 0,
                              Precision("f32"), eps=-w.eps)
    swapped = Lg[0].reshape(-1, 2)[:, ::-1].reshape(-1)
    assert np.abs(swapped - neg).max() <= 1e-6 * np.abs(neg).max()
    assert rel_err(swapped[0::2] - swapped[1::2], neg[0::2] - neg[1::2]) <= 1e-4


def test_resume_from_masters_seed_and_step_is_bit_identical():
    w = W.get_workload("c1_tiny_fp32")
    b = make_bundle(w)
    _, _, full = gpu_steps(b, 6)
    _, _, half = gpu_steps(b, 3)
    b2 = dict(b, masters=half)
    _, _, resumed = gpu_steps(b2, 3, first_step=3)
    assert np.array_equal(full.view(np.uint32), resumed.view(np.uint32))


def test_q1_is_the_sequential_two_pass_special_case():
    """q = 1 batched (2 copies) equals two single-copy evaluations of the oracle (MeZO with LoRA)."""
    w = W.get_workload("c1_tiny_fp32").with_(q=1)
    _check(w, make_bundle(w, b_std=0.02), 2, g_tol=1e-4, loss_tol=1e-6, theta_tol=1e-3)
