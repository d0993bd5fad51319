"""GPU checks at the full sizes of the five workloads, in the launch configuration bench.py times.

Workload 2 is small enough for the oracle: all 2q per-copy losses of one full-depth step are compared.  At the full
sizes of workloads 3-5 the oracle would take hours, so properties that hold at any size stand in: eps = 0 makes all
copies bit-identical; a copy evaluated alone gets bit for bit the loss it gets inside the batched pass (the batched
MP-LoRA pass changes the schedule, not the numbers); the two copies of a query differ once eps > 0; at random
initialisation the next-token loss sits at the entropy of a uniform guess, ln V."""
import math

import numpy as np
import pytest

import workloads as W
from gpu_helpers import make_bundle, gpu_model, oracle_steps
from oracle import zo
from oracle.model import decoder_layer, head_loss
from oracle.precision import Precision

pytestmark = pytest.mark.gpu


def test_workload2_full_depth_losses_against_the_oracle():
    import torch
    w = W.get_workload("c2_opt125m")
    b = make_bundle(w, b_std=0.01)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    m.regen_noise(3456, 0)
    got = m.forward_perturbed(tok, lab).cpu().numpy().astype(np.float64)
    want, _, _ = oracle_steps(b, 1)
    print(f"\nworkload 2, 12 layers: max rel loss error {np.abs(got - want[0]).max() / np.abs(want[0]).max():.2e}")
    assert np.abs(got - want[0]).max() <= 2e-2 * np.abs(want[0]).max()


@pytest.mark.parametrize("name", ["c3_opt1p3b", "c4_llama1p1b", "c5_llama7b"])
def test_full_size_properties(name):
    import torch
    import paper_2409_15520_amd as M
    w = W.get_workload(name)
    frozen = M.device_random_weights(w, 1234)
    masters = W.make_lora_masters(w, 99, b_std=0.01)
    m = M.ZoModel(w, frozen, masters)
    tok = torch.from_numpy(W.make_tokens(w, 2345)).cuda()
    lab = torch.from_numpy(W.make_labels(w, 2345)).cuda()
    n = 2 * w.q
    m.regen_noise(3456, 0)
    batched = m.forward_perturbed(tok, lab).cpu().numpy().copy()
    assert np.isfinite(batched).all()
    if w.loss_mode == "next_token_all_pos":      # thousands of positions: the mean sits at the entropy of a uniform guess
        assert np.abs(batched - math.log(w.vocab)).max() < 0.15 * math.log(w.vocab), batched
    else:                                        # a handful of two-way decisions with O(1) random logit gaps
        assert (batched > 0).all() and (batched < 5.0).all(), batched
    # every copy is its own model (fp32 losses a few 1e-4 apart: one chance collision is allowed for)
    assert len(set(batched.tolist())) >= n - 1
    # one copy alone, and the last query's pair alone: bit for bit the batched numbers
    m.losses.zero_()
    m.forward_copies(tok, lab, 1, 1)
    m.forward_copies(tok, lab, n - 2, 2)
    part = m.losses[:n].cpu().numpy()
    for c in (1, n - 2, n - 1):
        assert part[c].view(np.uint32) == batched[c].view(np.uint32), (c, part[c], batched[c])
    # eps = 0: all copies are the unperturbed model
    m.regen_noise(3456, 0, eps=0.0)
    same = m.forward_perturbed(tok, lab).cpu().numpy()
    assert np.all(same.view(np.uint32) == same.view(np.uint32)[0])
    m.close()
    del m, frozen
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["c3_opt1p3b", "c4_llama1p1b", "c5_llama7b"])
def test_full_width_block_on_sampled_sequences(name):
    """One block of the workload at its full d, FFN, heads, q, E and S (host-drawn weights of one layer): the stacked
    batch of all 2q copies goes through the GPU block; the oracle evaluates two (copy, sequence) pairs of it, each
    with that copy's perturbed factors, on the same input rows.  Tolerances as in the small-shape stage tests."""
    import torch
    w = W.get_workload(name).with_(n_layers=1, eps=5e-2)
    b = make_bundle(w, b_std=0.05)
    m = gpu_model(b)
    m.regen_noise(3456, 0)
    n, rpc, d = 2 * w.q, w.E * w.S, w.d_model
    g = torch.Generator(device="cuda")
    g.manual_seed(7)
    h = torch.randn(n * rpc, d, generator=g, device="cuda", dtype=torch.float32)
    h_in = h.clone()
    m.run_layers(h, 0, 1, w.E, w.S)
    prec = Precision("bf16")
    lw = b["frozen"]["layers"][0]
    for c, e in ((1, 0), (n - 2, w.E - 1)):
        k, sign = c // 2, (+1 if c % 2 == 0 else -1)
        z = zo.draw_z(b["layout"], 3456, 0, k, b["masters"].size, w.perturb_A)
        lora = zo.split_factors(b["layout"], zo.perturb(b["masters"], z, sign, w.eps, prec))
        r0 = c * rpc + e * w.S
        x = h_in[r0:r0 + w.S].cpu().numpy().astype(np.float64)[None]
        want = decoder_layer(w, lw, 0, x, lora, prec)[0]
        got = h[r0:r0 + w.S].cpu().numpy().astype(np.float64)
        rms = np.sqrt(np.mean(want ** 2))
        diff = np.abs(got - want)
        moved = np.sqrt(np.mean((want - x[0]) ** 2)) / rms
        print(f"\n{name} copy {c} sequence {e}: rms {rms:.3e}, block moved the stream by {moved:.3f} rms, "
              f"max|d|/rms {diff.max() / rms:.3e}, rms|d|/rms {np.sqrt(np.mean(diff ** 2)) / rms:.3e}", flush=True)
        assert moved > 0.01                                   # the block does something at this scale
        assert np.sqrt(np.mean(diff ** 2)) <= 3e-3 * rms
        assert diff.max() <= 5e-2 * rms
    # final norm, head and loss at the full batch (whole-vocabulary cross-entropy fused into the head GEMM for
    # workloads 3 and 4): two copies against the oracle on the same residual rows
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    got = m.head_loss(h, tok, lab).cpu().numpy().astype(np.float64)
    for c in (1, n - 2):
        hc = h[c * rpc:(c + 1) * rpc].cpu().numpy().astype(np.float64).reshape(w.E, w.S, d)
        want = head_loss(w, b["frozen"], hc, b["tokens"], b["labels"], prec)
        print(f"{name} head + loss copy {c}: {got[c]:.6f} vs {want:.6f}", flush=True)
        assert abs(got[c] - want) <= 1e-4 * abs(want)
    m.close()
    del m, h, h_in
    torch.cuda.empty_cache()
