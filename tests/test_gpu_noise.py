"""GPU parity: the regenerated noise, the perturbed copies and the update are bit-exact to the oracle."""
import numpy as np
import pytest

import workloads as W
from oracle import noise as N
from oracle import zo
from oracle.precision import Precision
from gpu_helpers import make_bundle, gpu_model

pytestmark = pytest.mark.gpu
SEED = 0x1234_5678_9ABC


def _bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def test_normal_transform_bit_exact_over_all_uniform_inputs():
    """Every one of the 2^23 distinct uniforms goes through ln/sqrt and through sin/cos once."""
    import torch
    import paper_2409_15520_amd as M
    m = np.arange(2**23, dtype=np.uint32)
    rng = np.random.default_rng(1)
    words = np.empty((2**23, 4), dtype=np.uint32)
    words[:, 0] = (m << 9) | rng.integers(0, 512, size=m.size, dtype=np.uint32)     # low 9 bits are ignored
    words[:, 1] = rng.permutation(m) << 9
    words[:, 2] = rng.permutation(m) << 9
    words[:, 3] = (m << 9) | 0x1FF
    dw = torch.from_numpy(words.view(np.int32)).cuda()
    out = torch.empty((2**23, 4), dtype=torch.float32, device="cuda")
    M.mpz_debug_normals_from_words(dw.data_ptr(), 2**23, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = np.stack(N.normals_from_words(words[:, 0], words[:, 1], words[:, 2], words[:, 3]), axis=1)
    assert np.array_equal(_bits(got), _bits(want))


@pytest.mark.parametrize("name", ["c1_tiny_fp32", "c2_opt125m", "c4_llama1p1b", "c5_llama7b"])
def test_noise_tensors_perturbed_copies_and_update_bit_exact(name):
    """Two blocks of each layout: ranks 4 / 8 on q, v (workloads 1, 2), rank 16 on q, k, v, o with the narrow k / v of
    grouped-query attention (workload 4, its 16 queries), rank 16 at d = 4096 (workload 5)."""
    import torch
    w = W.get_workload(name).with_(n_layers=2)
    if name in ("c4_llama1p1b", "c5_llama7b"):               # the frozen weights play no part here: a small vocabulary
        w = w.with_(vocab=512, E=1, S=64, max_seq=64, label_tokens=(3, 400))
    b = make_bundle(w, b_std=0.01)
    mdl = gpu_model(b)
    lay = b["layout"]
    for t in lay:                                            # every factor, two (step, k) coordinates
        for step, k in ((0, 0), (7, w.q - 1)):
            z = mdl.debug_noise(SEED, step, k, t.tensor_id, t.rows * t.cols).cpu().numpy()
            assert np.array_equal(_bits(z), _bits(N.noise_tensor(SEED, step, k, t.tensor_id, t.rows * t.cols)))
    # perturbed copies theta + (+/-) eps z_k
    mdl.regen_noise(SEED, 3)
    prec = Precision(w.dtype)
    for k in range(w.q):
        z = zo.draw_z(lay, SEED, 3, k, b["masters"].size, True)
        for s, sign in enumerate((+1, -1)):
            got = mdl.perturbed_copy(2 * k + s).cpu().numpy()
            assert np.array_equal(_bits(got), _bits(zo.perturb(b["masters"], z, sign, w.eps, prec)))
    # update from given losses
    losses = np.float32(np.random.default_rng(2).normal(0.7, 1e-4, size=2 * w.q))
    mdl.losses[:2 * w.q] = torch.from_numpy(losses).cuda()
    g = mdl.zo_update(lr=1e-2).cpu().numpy()
    g_ref = zo.projected_grads(losses, w.eps)
    assert np.array_equal(_bits(g), _bits(g_ref.astype(np.float32)))
    new_ref = zo.zo_update(b["masters"], g_ref, lay, SEED, 3, 1e-2, True, prec)
    assert np.array_equal(_bits(mdl.masters.cpu().numpy()), _bits(new_ref))


def test_lora_fa_mode_shares_A_and_leaves_it_unchanged():
    import torch
    w = W.get_workload("c1_tiny_fp32").with_(perturb_A=False)
    b = make_bundle(w, b_std=0.01)
    mdl = gpu_model(b)
    mdl.regen_noise(SEED, 0)
    c0, c1 = mdl.perturbed_copy(0).cpu().numpy(), mdl.perturbed_copy(3).cpu().numpy()
    mdl.losses[:4] = torch.tensor([0.7, 0.6, 0.5, 0.8], device="cuda")
    mdl.zo_update(lr=1e-2)
    new = mdl.masters.cpu().numpy()
    for t in b["layout"]:
        sl = slice(t.offset, t.offset + t.rows * t.cols)
        if t.factor == 0:
            assert np.array_equal(c0[sl], b["masters"][sl]) and np.array_equal(c1[sl], b["masters"][sl])
            assert np.array_equal(new[sl], b["masters"][sl])
        else:
            assert not np.array_equal(c0[sl], c1[sl]) and not np.array_equal(new[sl], b["masters"][sl])
    # B's stream is the same as when A is perturbed too
    z = N.noise_tensor(SEED, 0, 0, b["layout"][1].tensor_id, b["layout"][1].rows * b["layout"][1].cols)
    t = b["layout"][1]
    want = b["masters"][t.offset:t.offset + z.size] + np.float32(w.eps) * z
    assert np.array_equal(_bits(c0[t.offset:t.offset + z.size]), _bits(want))


def test_state_machine_and_argument_errors_on_device_handle():
    import torch
    import paper_2409_15520_amd as M
    w = W.get_workload("c1_tiny_fp32")
    b = make_bundle(w)
    mdl = gpu_model(b)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    with pytest.raises(M.MpzError) as e:
        mdl.forward_perturbed(tok, lab)
    assert e.value.status == 5
    mdl.regen_noise(SEED, 0, eps=0.0)
    mdl.forward_perturbed(tok, lab)
    with pytest.raises(M.MpzError) as e:                     # eps = 0: quotient undefined
        mdl.zo_update()
    assert e.value.status == 2
    mdl.regen_noise(SEED, 0)
    with pytest.raises(M.MpzError) as e:
        mdl.forward_perturbed(tok[:, :1].contiguous(), lab)    # S < 2
    assert e.value.status == 3
    with pytest.raises(M.MpzError) as e:
        mdl.forward_perturbed(tok, None)                     # this loss mode needs labels
    assert e.value.status == 1
    torch.cuda.synchronize()
