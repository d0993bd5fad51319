"""GPU: evaluating the copies one at a time (or in groups) gives each copy exactly the loss of the batched pass,
for the fp32 path and for the bf16 MFMA path, so the batched MP-LoRA pass changes the schedule, not the numbers."""
import numpy as np
import pytest

import workloads as W
from gpu_helpers import make_bundle, gpu_model, oracle_steps
from small_workloads import MINI_LLAMA
from test_gpu_bf16 import CASES

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("w", [W.get_workload("c1_tiny_fp32"), MINI_LLAMA, CASES["c2_2layers"], CASES["llama_mfma"]],
                         ids=["c1", "mini_llama_f32", "c2_2layers", "llama_mfma"])
def test_sequential_and_grouped_passes_are_bit_identical_to_the_batched_pass(w):
    import torch
    b = make_bundle(w, b_std=0.01)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    m.regen_noise(3456, 0)
    batched = m.forward_perturbed(tok, lab).cpu().numpy().copy()
    m.losses.zero_()
    seq = m.forward_sequential(tok, lab, group=1).cpu().numpy().copy()
    m.losses.zero_()
    outer = m.forward_sequential(tok, lab, group=2).cpu().numpy().copy()
    assert np.array_equal(batched.view(np.uint32), seq.view(np.uint32))
    assert np.array_equal(batched.view(np.uint32), outer.view(np.uint32))
    assert len(set(batched.tolist())) == 2 * w.q              # copies really differ
    # the outer loop alone: all + copies in one pass, all - copies in another (every second copy each)
    m.losses.zero_()
    signs = m.forward_outer_only(tok, lab).cpu().numpy().copy()
    assert np.array_equal(batched.view(np.uint32), signs.view(np.uint32))
    # and against the oracle, which evaluates the 2q copies one by one (Algorithm 1 as printed): the sequential and the
    # outer-loop-only passes give its losses - to fp32 rounding on the fp32 path, to the bf16 bar on the MFMA path
    want = oracle_steps(b, 1)[0][0]
    tol = 1e-6 if w.dtype == "f32" else 2e-2
    for nm, got in (("sequential", seq), ("pairs", outer), ("outer loop only", signs)):
        err = np.abs(got.astype(np.float64) - want).max() / np.abs(want).max()
        print(f"\n{w.name} {nm} pass vs oracle: max rel loss error {err:.2e}")
        assert err <= tol, (nm, got, want)
    # and a strided pass touches nothing but its own copies' losses
    if w.q >= 2:
        import paper_2409_15520_amd as M
        m.losses.fill_(-1.0)
        M.mpz_forward_copies_strided(m.handle, tok.data_ptr(), lab.data_ptr(), w.E, w.S, 1, w.q, 2, m.losses.data_ptr())
        part = m.losses[:2 * w.q].cpu().numpy()
        assert np.array_equal(part[1::2].view(np.uint32), batched[1::2].view(np.uint32)) and np.all(part[0::2] == -1.0)


def test_copy_range_errors():
    import torch
    import paper_2409_15520_amd as M
    w = W.get_workload("c1_tiny_fp32")
    b = make_bundle(w)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    with pytest.raises(M.MpzError) as e:
        m.forward_copies(tok, lab, 0, 1)
    assert e.value.status == 5
    m.regen_noise(1, 0)
    for cb, nc in ((-1, 1), (0, 0), (3, 2), (4, 1)):
        with pytest.raises(M.MpzError) as e:
            m.forward_copies(tok, lab, cb, nc)
        assert e.value.status == 3
    for cb, nc, step in ((0, 2, 0), (0, 3, 2), (1, 2, 3), (2, 2, 2)):          # 2q = 4 copies
        with pytest.raises(M.MpzError) as e:
            M.mpz_forward_copies_strided(m.handle, tok.data_ptr(), lab.data_ptr(), w.E, w.S, cb, nc, step, m.losses.data_ptr())
        assert e.value.status == 3
    torch.cuda.synchronize()


@pytest.mark.parametrize("name", ["c2_2layers", "c2_int8"])
def test_two_halves_schedule_changes_no_bit(name):
    """Small models run the pass as two halves of q copies on two streams; with the hook off it is one pass on the
    caller's stream.  Losses of three consecutive steps (update in between) are bit-identical, also when the caller's
    stream is not the default one."""
    import torch
    import paper_2409_15520_amd as M
    w = CASES[name]
    b = make_bundle(w, b_std=0.01)
    side = torch.cuda.Stream()
    runs = []
    for enable, stream in ((True, None), (False, None), (True, side)):
        ctx = torch.cuda.stream(stream) if stream is not None else torch.cuda.stream(torch.cuda.current_stream())
        with ctx:
            m = gpu_model(b)
            M.mpz_debug_set_two_halves(m.handle, enable)
            tok = torch.from_numpy(b["tokens"]).cuda()
            lab = torch.from_numpy(b["labels"]).cuda()
            out = []
            for step in range(3):
                m.regen_noise(3456, step)
                out.append(m.forward_perturbed(tok, lab).clone())
                m.zo_update()
            torch.cuda.current_stream().synchronize()
            runs.append(torch.stack(out).cpu().numpy())
    assert np.array_equal(runs[0].view(np.uint32), runs[1].view(np.uint32))
    assert np.array_equal(runs[0].view(np.uint32), runs[2].view(np.uint32))


FEW_TOKENS = {   # passes over 128 stacked tokens: every projection splits K (three blocks deep: both fusions across blocks)
    "llama_few_tokens": W.get_workload("c4_llama1p1b").with_(n_layers=3, q=1, E=1, S=64),
    "opt_few_tokens": W.get_workload("c3_opt1p3b").with_(n_layers=3, q=1, E=2, S=32, vocab=4096, max_seq=64),
}


@pytest.mark.parametrize("name", ["c2_2layers", "llama_mfma", "c2_ragged_copies", "llama_few_tokens", "opt_few_tokens"])
def test_fused_norm_and_bottleneck_kernel_changes_no_bit(name):
    """The first pre-norm of a block and the LoRA bottleneck of its q/k/v projections run as one kernel where the
    shapes allow, and in passes over few tokens the reduction of a split-K projection into the residual stream runs
    as one kernel with the pre-norm that follows; with the hook off each is two kernels.  Same arithmetic, same
    order: identical losses."""
    import torch
    import paper_2409_15520_amd as M
    w = CASES[name] if name in CASES else FEW_TOKENS[name]
    b = make_bundle(w, b_std=0.05)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    out = []
    for enable in (True, False):
        M.mpz_debug_set_fused_norm_lora(m.handle, enable)
        m.regen_noise(3456, 0)
        out.append(m.forward_perturbed(tok, lab).cpu().numpy().copy())
    assert np.array_equal(out[0].view(np.uint32), out[1].view(np.uint32)), out


RANK4_MFMA = W.Workload(
    name="rank4_mfma", n_layers=2, d_model=256, n_heads=4, n_kv_heads=4, d_ffn=512, vocab=512, max_seq=64,
    act="relu", norm="layernorm", pos="learned", has_bias=True, tie_embeddings=True, dtype="bf16",
    lora_rank=4, lora_targets=("q", "o"), loss_mode="last_pos_full_vocab", q=3, E=2, S=64, steps=1, label_tokens=(5, 300))


@pytest.mark.parametrize("w,perturb_A", [(CASES["c2_2layers"], True), (CASES["llama_mfma"], True), (CASES["llama_mfma"], False),
                                         (RANK4_MFMA, True), (CASES["mini_llama"], True)],
                         ids=["c2_2layers_r8_qv", "llama_mfma_r16_qkvo", "llama_mfma_lora_fa", "rank4_qo", "mini_llama_fallback"])
def test_noise_written_straight_into_the_operand_layouts_changes_no_bit(w, perturb_A):
    """bf16 models: mpz_regen_noise writes the perturbed factors directly as bf16 hi / lo MFMA operands (one kernel, no
    fp32 copies); with the hook off it writes fp32 copies and packs them.  Same factors, so the same losses, and the
    fp32 copies - made on demand for the test hook, for the stateful update and for shapes the MFMA kernels refuse
    (the miniature model) - are the same bits too."""
    import torch
    import paper_2409_15520_amd as M
    w = w.with_(perturb_A=perturb_A)
    b = make_bundle(w, b_std=0.05)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    losses, copies, after = [], [], []
    for fused in (True, False):
        M.mpz_debug_set_fused_perturb_pack(m.handle, fused)
        m.masters.copy_(torch.from_numpy(b["masters"]).cuda())
        m.regen_noise(3456, 5, eps=5e-2)
        losses.append(m.forward_perturbed(tok, lab).cpu().numpy().copy())
        copies.append(m.perturbed_copy(2 * w.q - 1).cpu().numpy().copy())
        m.zo_update_regen(6)                       # the stateful update reads the stored fp32 pairs
        losses.append(m.forward_perturbed(tok, lab).cpu().numpy().copy())
        after.append(m.masters.cpu().numpy().copy())
    assert len(set(losses[0].tolist())) == 2 * w.q
    assert np.array_equal(losses[0].view(np.uint32), losses[2].view(np.uint32)), (losses[0], losses[2])
    assert np.array_equal(losses[1].view(np.uint32), losses[3].view(np.uint32)), (losses[1], losses[3])
    assert np.array_equal(copies[0].view(np.uint32), copies[1].view(np.uint32))
    assert np.array_equal(after[0].view(np.uint32), after[1].view(np.uint32))
