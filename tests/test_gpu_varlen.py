"""GPU parity on batches of unequal length: right-padded (losses over real tokens only) and packed (the same batch
without its padding: every kernel runs over real tokens only)."""
import numpy as np
import pytest

import workloads as W
from oracle import zo
from oracle.precision import Precision
from gpu_helpers import make_bundle, gpu_model
from small_workloads import C1, MINI_LLAMA, MINI_OPT
from test_gpu_bf16 import CASES as BF16_CASES

pytestmark = pytest.mark.gpu
SEED = 3456


def _bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("w", [C1, MINI_LLAMA, MINI_OPT, MINI_OPT.with_(loss_mode="next_token_all_pos")],
                         ids=lambda w: f"{w.name}-{w.loss_mode}")
def test_fp32_losses_bit_identical_on_padded_batches(w):
    import torch
    b = make_bundle(w, b_std=0.01)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    m.regen_noise(SEED, 0)
    full = m.forward_perturbed(tok, lab).cpu().numpy().copy()
    same = m.forward_perturbed(tok, lab, torch.full((w.E,), w.S, dtype=torch.int32, device="cuda")).cpu().numpy()
    assert np.array_equal(_bits(full), _bits(same))                       # full lengths: the fixed-length pass
    for pad in (0.2, 0.45):
        lengths = W.make_lengths(w, 11, pad_fraction=pad)
        got = m.forward_perturbed(tok, lab, torch.from_numpy(lengths).cuda()).cpu().numpy()
        want = zo.perturbed_losses(w, b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"], SEED, 0,
                                   Precision("f32"), lengths=lengths).astype(np.float32)
        assert np.array_equal(_bits(got), _bits(want)), (lengths, got, want)
        assert not np.array_equal(_bits(got), _bits(full))
    # lengths outside [2, S] are clamped, not dereferenced out of bounds
    wild = torch.tensor([0] + [10 ** 6] * (w.E - 1), dtype=torch.int32, device="cuda")
    clamped = np.array([2] + [w.S] * (w.E - 1))
    got = m.forward_perturbed(tok, lab, wild).cpu().numpy()
    want = zo.perturbed_losses(w, b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"], SEED, 0,
                               Precision("f32"), lengths=clamped).astype(np.float32)
    assert np.array_equal(_bits(got), _bits(want))


@pytest.mark.parametrize("name", ["c2_2layers", "llama_mfma", "mini_opt"])
def test_bf16_head_on_padded_batches(name):
    """The stages before the head do not depend on the lengths, so the head is checked on the oracle's own residual
    stream: fused whole-vocabulary head (llama_mfma, mini_opt) and the two-label head (c2)."""
    import torch
    from oracle.model import head_loss
    from gpu_helpers import oracle_traces
    w = BF16_CASES[name]
    b = make_bundle(w, b_std=0.01)
    H, _ = oracle_traces(b)
    m = gpu_model(b)
    m.regen_noise(SEED, 0)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    lengths = W.make_lengths(w, 4, pad_fraction=0.35)
    n = 2 * w.q
    hl = H[-1].reshape(n, w.E, w.S, w.d_model)
    prec = Precision("bf16")
    want = np.array([head_loss(w, b["frozen"], hl[c].astype(np.float64), b["tokens"], b["labels"], prec, lengths=lengths)
                     for c in range(n)])
    import paper_2409_15520_amd as M
    m_lengths = torch.from_numpy(lengths).cuda()
    got = m.head_loss(torch.from_numpy(H[-1]).cuda(), tok, lab, lengths=m_lengths).cpu().numpy().astype(np.float64)
    print(f"\n{name} padded head: {np.abs(got - want).max() / np.abs(want).max():.2e}")
    assert np.abs(got - want).max() <= 1e-4 * np.abs(want).max()
    full = m.head_loss(torch.from_numpy(H[-1]).cuda(), tok, lab).cpu().numpy().astype(np.float64)
    assert np.abs(full - want).max() > 1e-4 * np.abs(want).max()           # the lengths do change the loss


@pytest.mark.parametrize("w", [C1, MINI_LLAMA, MINI_OPT, MINI_OPT.with_(loss_mode="next_token_all_pos")],
                         ids=lambda w: f"{w.name}-{w.loss_mode}")
def test_fp32_packed_batches_match_the_oracle_bit_for_bit(w):
    """Packed rows change where a token sits, not what is computed for it: the losses are the oracle's losses of the
    padded batch (which never looks at the padding), bit for bit, also with sequences of a single token pair and at
    full length."""
    import torch
    b = make_bundle(w, b_std=0.01)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    m.regen_noise(SEED, 0)
    cases = [W.make_lengths(w, 11, pad_fraction=0.2), W.make_lengths(w, 12, pad_fraction=0.45),
             np.full(w.E, w.S, dtype=np.int32), np.array([2] + [w.S] * (w.E - 1), dtype=np.int32)]
    for lengths in cases:
        got = m.forward_perturbed_packed(tok, lab, torch.from_numpy(lengths).cuda()).cpu().numpy()
        want = zo.perturbed_losses(w, b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"], SEED, 0,
                                   Precision("f32"), lengths=lengths).astype(np.float32)
        assert np.array_equal(_bits(got), _bits(want)), (lengths, got, want)


@pytest.mark.parametrize("name", ["c2_2layers", "llama_mfma", "mini_opt", "c2_ragged_copies"])
def test_bf16_packed_batches_equal_the_padded_pass(name):
    """MFMA kernels: a row's GEMM, bottleneck and attention results do not depend on the rows around it, so the packed
    pass must reproduce the padded pass of the same batch; both are within the bf16 bar of the oracle."""
    import torch
    w = BF16_CASES[name]
    b = make_bundle(w, b_std=0.01)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    m.regen_noise(SEED, 0)
    for seed, pad in ((11, 0.2), (12, 0.45)):
        lengths = W.make_lengths(w, seed, pad_fraction=pad)
        ld = torch.from_numpy(lengths).cuda()
        padded = m.forward_perturbed(tok, lab, ld).cpu().numpy().copy()
        packed = m.forward_perturbed_packed(tok, lab, ld).cpu().numpy().copy()
        want = zo.perturbed_losses(w, b["layout"], b["frozen"], b["masters"], b["tokens"], b["labels"], SEED, 0,
                                   Precision("bf16"), lengths=lengths)
        print(f"\n{name} pad {pad}: lengths {lengths.tolist()}: packed vs padded max diff "
              f"{np.abs(packed - padded).max():.2e}, vs oracle {np.abs(packed - want).max() / np.abs(want).max():.2e}")
        assert np.abs(packed - padded).max() <= 1e-6 * np.abs(padded).max()
        assert np.abs(packed - want).max() <= 2e-2 * np.abs(want).max()


def test_packed_argument_errors():
    import torch
    import paper_2409_15520_amd as M
    w = MINI_OPT
    b = make_bundle(w)
    m = gpu_model(b)
    tok = torch.zeros(64, dtype=torch.int32, device="cuda")
    lab = torch.zeros(w.E, dtype=torch.int32, device="cuda")
    cu = torch.tensor([0, 5, 12, 20], dtype=torch.int32, device="cuda")
    out = m.losses.data_ptr()
    with pytest.raises(M.MpzError):                                   # before mpz_regen_noise
        M.mpz_forward_perturbed_packed(m.handle, tok.data_ptr(), lab.data_ptr(), cu.data_ptr(), 3, 20, 8, out)
    m.regen_noise(SEED, 0)
    M.mpz_forward_perturbed_packed(m.handle, tok.data_ptr(), lab.data_ptr(), cu.data_ptr(), 3, 20, 8, out)
    for E, total, max_len in ((0, 20, 8), (3, 20, 1), (3, 20, w.S + 1), (3, 5, 8), (3, 25, 8), (3, w.E * w.S + 1, w.S)):
        with pytest.raises(M.MpzError):
            M.mpz_forward_perturbed_packed(m.handle, tok.data_ptr(), lab.data_ptr(), cu.data_ptr(), E, total, max_len, out)
    with pytest.raises(M.MpzError):
        M.mpz_forward_perturbed_packed(m.handle, tok.data_ptr(), lab.data_ptr(), None, 3, 20, 8, out)
