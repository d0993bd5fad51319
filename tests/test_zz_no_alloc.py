"""GPU: mpz_forward_perturbed_noalloc (per-pass activations in the library's static device array, no allocation)
against mpz_forward_perturbed (activations in the caller's workspace), through the C ABI: the same losses bit for bit,
on two calls in a row, the second on a smaller batch; and a pass that does not fit the array is refused before
anything is launched."""
import numpy as np
import pytest

import workloads as W
from gpu_helpers import make_bundle, gpu_model
from small_workloads import MINI_LLAMA

pytestmark = pytest.mark.gpu

LLAMA_MFMA = W.Workload(
    name="llama_mfma", n_layers=2, d_model=256, n_heads=4, n_kv_heads=2, d_ffn=384, vocab=1000, max_seq=64,
    act="swiglu", norm="rmsnorm", pos="rope", has_bias=False, tie_embeddings=False, dtype="bf16",
    lora_rank=16, lora_targets=("q", "k", "v", "o"), loss_mode="next_token_all_pos", q=2, E=2, S=64, steps=1)
C2_SMALL = W.get_workload("c2_opt125m").with_(n_layers=2, q=2, E=1, S=128)


@pytest.mark.parametrize("w", [W.get_workload("c1_tiny_fp32"), MINI_LLAMA, LLAMA_MFMA, C2_SMALL],
                         ids=["c1_fp32", "mini_llama_fp32", "llama_mfma_bf16", "c2_small_bf16"])
def test_noalloc_pass_equals_workspace_pass_on_two_calls_in_a_row(w):
    import torch
    import paper_2409_15520_amd as M
    b = make_bundle(w, b_std=0.05)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    n = 2 * w.q
    m.regen_noise(3456, 0, eps=5e-2)
    # the second call is smaller: fewer sequences if there are several, and a shorter sequence
    E2, S2 = max(1, w.E // 2), w.S // 2
    tok2 = tok[:E2, :S2].contiguous()
    lab2 = lab[:E2].contiguous()
    want1 = m.forward_perturbed(tok, lab).cpu().numpy().copy()
    want2 = m.forward_perturbed(tok2, lab2).cpu().numpy().copy()
    out = torch.full((n,), -1.0, dtype=torch.float32, device="cuda")
    M.mpz_forward_perturbed_noalloc(m.handle, tok.data_ptr(), lab.data_ptr(), w.E, w.S, out.data_ptr())
    got1 = out.cpu().numpy().copy()
    out.fill_(-1.0)
    M.mpz_forward_perturbed_noalloc(m.handle, tok2.data_ptr(), lab2.data_ptr(), E2, S2, out.data_ptr())
    got2 = out.cpu().numpy().copy()
    torch.cuda.synchronize()
    print(f"\n{w.name}: first call {got1}, second (E {E2}, S {S2}) {got2}")
    assert np.isfinite(want1).all() and len(set(want1.tolist())) == n      # the copies really differ
    assert np.array_equal(got1.view(np.uint32), want1.view(np.uint32)), (got1, want1)
    assert np.array_equal(got2.view(np.uint32), want2.view(np.uint32)), (got2, want2)
    assert not np.array_equal(want1, want2)
    # the workspace pass still gives the same numbers afterwards
    again = m.forward_perturbed(tok, lab).cpu().numpy()
    assert np.array_equal(again.view(np.uint32), want1.view(np.uint32))


def test_noalloc_pass_refuses_what_does_not_fit_and_launches_nothing():
    import torch
    import paper_2409_15520_amd as M
    w = W.get_workload("c2_opt125m").with_(n_layers=1)        # 8192 stacked tokens: the residual stream alone is 24 MiB
    b = make_bundle(w)
    m = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    out = torch.full((2 * w.q,), -1.0, dtype=torch.float32, device="cuda")
    with pytest.raises(M.MpzError) as e:                      # call order first
        M.mpz_forward_perturbed_noalloc(m.handle, tok.data_ptr(), lab.data_ptr(), w.E, w.S, out.data_ptr())
    assert e.value.status == 5
    m.regen_noise(3456, 0)
    assert M.mpz_noalloc_scratch_bytes() == 16 << 20
    with pytest.raises(M.MpzError) as e:
        M.mpz_forward_perturbed_noalloc(m.handle, tok.data_ptr(), lab.data_ptr(), w.E, w.S, out.data_ptr())
    assert e.value.status == 4 and "16777216" in str(e.value)
    torch.cuda.synchronize()
    assert (out.cpu().numpy() == -1.0).all()
    # a batch of the same model that fits goes through
    tok1, lab1 = tok[:1, :64].contiguous(), lab[:1].contiguous()
    M.mpz_forward_perturbed_noalloc(m.handle, tok1.data_ptr(), lab1.data_ptr(), 1, 64, out.data_ptr())
    torch.cuda.synchronize()
    assert np.isfinite(out.cpu().numpy()).all() and (out.cpu().numpy() > 0).all()
