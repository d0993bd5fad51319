"""GPU parity for bf16 workloads.

With bf16 operands and eps = 1e-3 the perturbation is about one bf16 ulp of the adapted projections, and one
rounding flip upstream re-rolls the roundings downstream, so the end-to-end two-point difference of two
correct implementations (fp32 vs fp64 accumulation) drifts apart by more than the 2e-2 target; the tests
therefore check (1) every stage on the oracle's own inputs (no error build-up), element by element,
(2) end-to-end losses to the bf16 noise floor, and (3) g_k against the drift measured between the oracle and
a jittered copy of itself.
"""
import numpy as np
import pytest

import workloads as W
from gpu_helpers import (make_bundle, gpu_model, gpu_steps, oracle_steps, oracle_traces, rel_err, JitterPrecision)
from small_workloads import MINI_LLAMA, MINI_OPT

pytestmark = pytest.mark.gpu

CASES = {
    "mini_llama": MINI_LLAMA.with_(dtype="bf16"),
    "mini_opt": MINI_OPT.with_(dtype="bf16", loss_mode="next_token_all_pos"),
    "c2_2layers": W.get_workload("c2_opt125m").with_(n_layers=2),
    # 96 rows per copy: block tiles of 128 rows span two copies, every 32-row MFMA tile still belongs to one
    "c2_ragged_copies": W.get_workload("c2_opt125m").with_(n_layers=1, q=3, E=1, S=96),
    # Llama-style shapes that the MFMA kernels accept: adapters on q, k, v, o with r = 16, grouped-query
    # attention, rotary positions, SwiGLU (gate|up tiles fused), next-token loss over the whole vocabulary
    "llama_mfma": W.Workload(
        name="llama_mfma", n_layers=2, d_model=256, n_heads=4, n_kv_heads=2, d_ffn=384, vocab=1000, max_seq=64,
        act="swiglu", norm="rmsnorm", pos="rope", has_bias=False, tie_embeddings=False, dtype="bf16",
        lora_rank=16, lora_targets=("q", "k", "v", "o"), loss_mode="next_token_all_pos", q=2, E=2, S=64, steps=1),
}
# weight-only int8 block linears (codes widened in the GEMM's operand load, scale on the accumulator)
CASES["c2_int8"] = CASES["c2_2layers"].with_(weight_quant="int8")
CASES["llama_mfma_int8"] = CASES["llama_mfma"].with_(weight_quant="int8")
# weight-only 4-bit normal-float block linears (dequantised to bf16 once per pass, right before each GEMM); the
# miniature runs them through the shape-agnostic kernels
CASES["c2_nf4"] = CASES["c2_2layers"].with_(weight_quant="nf4")
CASES["llama_mfma_nf4"] = CASES["llama_mfma"].with_(weight_quant="nf4")
CASES["mini_llama_nf4"] = MINI_LLAMA.with_(dtype="bf16", d_ffn=128, weight_quant="nf4")


@pytest.mark.parametrize("name,eps,b_std", [("mini_llama", 1e-3, 0.01), ("mini_opt", 1e-3, 0.01),
                                            ("c2_2layers", 1e-3, 0.01), ("c2_2layers", 5e-2, 0.05),
                                            ("llama_mfma", 1e-3, 0.01), ("llama_mfma", 5e-2, 0.05),
                                            ("c2_ragged_copies", 5e-2, 0.05),
                                            ("c2_int8", 1e-3, 0.01), ("c2_int8", 5e-2, 0.05),
                                            ("llama_mfma_int8", 1e-3, 0.01), ("llama_mfma_int8", 5e-2, 0.05),
                                            ("c2_nf4", 1e-3, 0.01), ("c2_nf4", 5e-2, 0.05),
                                            ("llama_mfma_nf4", 1e-3, 0.01), ("llama_mfma_nf4", 5e-2, 0.05),
                                            ("mini_llama_nf4", 1e-3, 0.01)])
def test_each_stage_on_oracle_inputs(name, eps, b_std):
    """Second c2 case: perturbation and B large enough that the low-rank term moves the projections by
    O(10%), so a wrong or missing per-copy term cannot hide under the rounding tolerance."""
    import torch
    w = CASES[name].with_(eps=eps)
    b = make_bundle(w, b_std=b_std)
    H, losses = oracle_traces(b)
    m = gpu_model(b)
    m.regen_noise(3456, 0)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    h0 = m.embed(tok).cpu().numpy()
    assert np.array_equal(h0, H[0])                                    # exact: one fp32 add per element
    for l in range(w.n_layers):
        h = torch.from_numpy(H[l]).cuda()
        m.run_layers(h, l, l + 1, w.E, w.S)
        got = h.cpu().numpy().astype(np.float64)
        want = H[l + 1].astype(np.float64)
        rms = np.sqrt(np.mean(want ** 2))
        diff = np.abs(got - want)
        frac_exact = np.mean(got == want)
        print(f"\n{name} layer {l}: rms {rms:.3e}  max|d|/rms {diff.max() / rms:.3e}  rms|d|/rms "
              f"{np.sqrt(np.mean(diff ** 2)) / rms:.3e}  bit-equal {frac_exact:.4f}")
        # one block of the oracle itself moves by rms 1.1e-3 / max 1.4e-2 (of rms h) at workload-2 widths when its
        # operands are jittered by 1e-7 before rounding (the size of fp32 accumulation error)
        assert np.sqrt(np.mean(diff ** 2)) <= 3e-3 * rms
        assert diff.max() <= 5e-2 * rms
    hl = torch.from_numpy(H[-1]).cuda()
    got = m.head_loss(hl, tok, lab).cpu().numpy().astype(np.float64)
    print(f"{name} head: max rel err {np.abs(got - losses).max() / np.abs(losses).max():.3e}")
    assert np.abs(got - losses).max() <= 1e-4 * np.abs(losses).max()


def _g_bound(floor_g):
    """Bound on the norm-wise error of g that a wrong sign (error 2), a swapped pair (2) or a dropped perturbation (1)
    cannot pass; None when the oracle's own g moves by >= 0.1 under a 1e-6 operand jitter (nothing to assert)."""
    return min(max(2e-2, 6.0 * floor_g), 0.5) if floor_g < 0.1 else None


@pytest.mark.parametrize("name", list(CASES))
def test_end_to_end_losses_and_drift_of_g(name):
    """The workloads' own eps = 1e-3: per-copy losses to the bf16 bar; g against the oracle only where the oracle's
    own two-point differences stand above its rounding floor (else: reported, 'parity unpinned' at this eps; the eps
    sweep below pins the estimate where the difference is measurable)."""
    from oracle import zo
    w = CASES[name]
    b = make_bundle(w, b_std=0.01)
    Lg, Gg, _ = gpu_steps(b, 1)
    Lo, Go, _ = oracle_steps(b, 1)
    jl = zo.perturbed_losses(w, b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"], 3456, 0,
                             JitterPrecision(1e-6, 1))
    Gj = zo.projected_grads(jl.astype(np.float32), w.eps)
    floor_l = np.abs(jl - Lo[0]).max() / np.abs(Lo[0]).max()
    floor_g = rel_err(Gj, Go[0])
    err_l = np.abs(Lg[0] - Lo[0]).max() / np.abs(Lo[0]).max()
    err_g = rel_err(Gg[0], Go[0])
    print(f"\n{name}: loss err {err_l:.3e} (oracle-vs-jittered-oracle {floor_l:.3e}); g err {err_g:.3e} "
          f"(oracle-vs-jittered-oracle {floor_g:.3e}); g gpu {Gg[0]}, oracle {Go[0]}")
    assert err_l <= 2e-2            # the bf16 bar for per-copy losses
    assert err_l <= max(8.0 * floor_l, 1e-4)        # and no further from the oracle than a few of its own floors
    bound = _g_bound(floor_g)
    if bound is None:
        print(f"{name}: eps = {w.eps}: the oracle's own g moves by {floor_g:.2f} under a 1e-6 operand jitter - "
              f"g is not assertable at this eps (parity unpinned); see the eps sweep")
    else:
        assert err_g <= bound, (err_g, floor_g)


SWEEP = dict(CASES)


def _sweep_cases():
    from test_gpu_workloads import CASES as WIDE
    SWEEP.update({"c3_width": WIDE["c3_width"], "c4_width": WIDE["c4_width"]})
    return ["c2_2layers", "llama_mfma", "c3_width", "c4_width"]


@pytest.mark.parametrize("name", _sweep_cases())
def test_two_point_estimate_against_the_oracle_over_eps(name):
    """The end-to-end bf16 estimate g_k = (l_k+ - l_k-) / (2 eps) against the oracle for eps = 1e-3 (the workloads'),
    1e-2 (the paper's own MobiZO value, hyper-parameter table of Appendix D) and 5e-2, with B ~ 0.05 so that the
    low-rank path carries weight.  The rounding noise of a bf16 forward pass does not depend on eps, the two-point
    difference grows with it: the error of g must fall roughly as 1 / eps, meet the 2e-2 bar (or the oracle's own
    floor) at the largest eps, every g_k that stands above the floor must have the oracle's sign, and the differences
    between the per-copy losses - which the 2e-2 bar on the losses themselves cannot see - must match the oracle's."""
    from oracle import zo
    w0 = SWEEP[name]
    errs, floors = {}, {}
    for eps in (1e-3, 1e-2, 5e-2):
        w = w0.with_(eps=eps)
        b = make_bundle(w, b_std=0.05)
        Lg, Gg, _ = gpu_steps(b, 1)
        Lo, Go, _ = oracle_steps(b, 1)
        # the floor: how far the oracle's own estimate moves under two different 1e-6 operand jitters (the larger one:
        # with q values per step a single sample of the floor scatters by a factor of a few)
        floors[eps], floor_d, abs_floor = 0.0, 0.0, 0.0
        for jseed in (1, 2):
            jl = zo.perturbed_losses(w, b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"], 3456, 0,
                                     JitterPrecision(1e-6, jseed)).astype(np.float32).astype(np.float64)
            Gj = zo.projected_grads(jl, eps)
            floors[eps] = max(floors[eps], rel_err(Gj, Go[0]))
            floor_d = max(floor_d, rel_err(jl[1:] - jl[0], Lo[0][1:] - Lo[0][0]))
            abs_floor = max(abs_floor, np.abs(Gj - Go[0]).max())
        errs[eps] = rel_err(Gg[0], Go[0])
        # differences between the copies' losses (all against copy 0): what the perturbations do to the loss
        err_d = rel_err(Lg[0][1:] - Lg[0][0], Lo[0][1:] - Lo[0][0])
        print(f"\n{name} eps {eps:g}: g gpu {np.array2string(Gg[0], precision=4)} oracle {np.array2string(Go[0], precision=4)}\n"
              f"   g error {errs[eps]:.3e} (oracle vs jittered oracle {floors[eps]:.3e});  loss differences error {err_d:.3e} "
              f"(floor {floor_d:.3e});  losses error {np.abs(Lg[0] - Lo[0]).max() / np.abs(Lo[0]).max():.2e}", flush=True)
        for k in range(w.q):                       # sign of every estimate that stands above the floor
            if abs(Go[0][k]) > 4.0 * abs_floor:
                assert np.sign(Gg[0][k]) == np.sign(Go[0][k]), (eps, k, Gg[0], Go[0])
        bound = _g_bound(floors[eps])
        if bound is not None:
            assert errs[eps] <= bound, (eps, errs[eps], floors[eps])
            assert err_d <= min(max(2e-2, 6.0 * floor_d), 0.5), (eps, err_d, floor_d)
    # the largest eps must be assertable and meet the 2e-2 bar
    assert floors[5e-2] < 0.1
    assert errs[5e-2] <= 2e-2
    # 50 times the perturbation: the error of g falls by an order of magnitude or was already at the bar
    assert errs[5e-2] <= max(0.2 * errs[1e-3], 2e-2), errs


def test_ten_steps_at_a_measurable_eps_track_the_oracle():
    """Ten full ZO steps (noise, batched pass, estimate, seed-replayed update) at eps = 5e-2 on workload-2 widths:
    the updated LoRA factors against the oracle's.  B starts at N(0, 0.05^2); the update of a step is lr g z / q,
    so the error of theta relative to the MOVEMENT of theta is the accumulated error of g."""
    w = CASES["c2_2layers"].with_(eps=5e-2, q=2, E=4, lr=1e-3)
    b = make_bundle(w, b_std=0.05)
    Lg, Gg, Mg = gpu_steps(b, 10)
    Lo, Go, Mo = oracle_steps(b, 10)
    moved = np.linalg.norm(Mo.astype(np.float64) - b["masters"])
    err_theta = rel_err(Mg, Mo)
    err_move = float(np.linalg.norm(Mg.astype(np.float64) - Mo) / moved)
    err_g = [rel_err(Gg[s], Go[s]) for s in range(10)]
    print(f"\n10 steps at eps 5e-2: theta error {err_theta:.2e} (relative to theta), {err_move:.2e} (relative to its "
          f"movement {moved:.3e}); g errors per step {np.array2string(np.array(err_g), precision=3)}")
    assert err_theta <= 1e-3                       # the bar on the updated factors
    assert err_move <= 5e-2                        # and on what the ten updates did (inherits the error of g)
    assert max(err_g) <= 0.1 and np.median(err_g) <= 2e-2


def test_eps_zero_bit_identical_copies_bf16():
    import torch
    w = CASES["c2_2layers"]
    b = make_bundle(w, b_std=0.01)
    m = gpu_model(b)
    m.regen_noise(3456, 0, eps=0.0)
    l = m.forward_perturbed(torch.from_numpy(b["tokens"]).cuda(), torch.from_numpy(b["labels"]).cuda()).cpu().numpy()
    assert np.all(l == l[0])


def test_same_widths_in_fp32_meet_the_fp32_bar():
    """The same path at workload-2 widths with fp32 storage / fp64 accumulation: g within 1e-4."""
    w = W.get_workload("c2_opt125m").with_(n_layers=2, dtype="f32", vocab=2048, label_tokens=(1234, 77), E=2, q=2)
    b = make_bundle(w)
    Lg, Gg, Mg = gpu_steps(b, 2)
    Lo, Go, Mo = oracle_steps(b, 2)
    print(f"\nfp32 at c2 widths: loss err {rel_err(Lg, Lo):.2e}, g err {[rel_err(Gg[s], Go[s]) for s in range(2)]}, theta {rel_err(Mg, Mo):.2e}")
    assert np.abs(Lg - Lo).max() <= 1e-6 * np.abs(Lo).max()
    assert all(rel_err(Gg[s], Go[s]) <= 1e-4 for s in range(2))
    assert rel_err(Mg, Mo) <= 1e-3


@pytest.mark.parametrize("name", ["c2_2layers", "llama_mfma"])
def test_mfma_path_agrees_with_shape_agnostic_path(name):
    """Same rounding points, different kernels: one block on identical inputs, element by element."""
    import torch
    import paper_2409_15520_amd as M
    w = CASES[name].with_(eps=5e-2)
    b = make_bundle(w, b_std=0.05)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    outs = []
    for simple in (False, True):
        M.mpz_debug_set_kernel_path(m.handle, simple)
        m.regen_noise(3456, 0)
        h = m.embed(tok)
        m.run_layers(h, 0, 1, w.E, w.S)
        outs.append(h.cpu().numpy().astype(np.float64))
    rms = np.sqrt(np.mean(outs[1] ** 2))
    d = np.abs(outs[0] - outs[1])
    print(f"\n{name}: mfma vs simple: max|d|/rms {d.max() / rms:.3e} rms|d|/rms {np.sqrt(np.mean(d ** 2)) / rms:.3e}")
    assert np.sqrt(np.mean(d ** 2)) <= 3e-3 * rms and d.max() <= 5e-2 * rms
