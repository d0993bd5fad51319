"""GPU parity at FULL DEPTH on workloads 3, 4 and 5, in the launch configuration bench.py times: the whole batched
pass (the workload's own q, E, S: all 2q copies) runs on the GPU; copies 0 and 1 (query 0, + and -) are compared
with the oracle's two single-copy evaluations of the same step (Algorithm 1, inner loop for k = 0; Section 3: the
copies are independent, so these two check the batched pass at every depth).

The oracle's numbers are stored in tests/golden/full_depth_query0_<workload>.json, written by
tests/golden/make_full_depth_golden.py, which calls only oracle/ and workloads/ (a full-depth oracle pass takes
minutes to an hour on the host).  Both sides draw the frozen weights from workloads/hashed.py (an integer hash:
the same bits on the host and on the device).  Two settings: the workload's own (eps = 1e-3, B = 0), and a strong
one (eps = 5e-2, B ~ 0.05) in which a wrong per-copy factor at any depth would move the loss far beyond the
tolerance.  Tolerances come from the stored jittered-oracle run (the distance two correct bf16 implementations can
have), not from the 2e-2 bar, which could not see a perturbation at all."""
import json
import os

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_hashed_weights_are_the_same_bits_on_host_and_device():
    import torch
    from workloads.hashed import hashed_normal
    for shape, no in (((257, 1031), 3), ((4096, 4096), 16 * 31 + 22)):
        host = hashed_normal(shape, no, 1234, device="cpu")
        dev = hashed_normal(shape, no, 1234, device="cuda").cpu()
        assert torch.equal(host.view(torch.int32), dev.view(torch.int32))
        assert abs(float(host.std()) - 0.02) < 2e-4 and abs(float(host.mean())) < 1e-4


@pytest.mark.parametrize("name", ["c3_opt1p3b", "c4_llama1p1b", "c5_llama7b"])
def test_full_depth_query0_against_the_oracle(name):
    import torch
    import paper_2409_15520_amd as M
    path = os.path.join(GOLDEN, f"full_depth_query0_{name}.json")
    if not os.path.exists(path):
        pytest.skip(f"{path} has not been written yet (tests/golden/make_full_depth_golden.py {name})")
    gold = json.load(open(path))
    w = W.get_workload(name)
    seeds = gold["seeds"]
    frozen = W.make_frozen_weights_hashed(w, seeds["weights"], device="cuda")
    tok = torch.from_numpy(W.make_tokens(w, seeds["tokens"])).cuda()
    lab = torch.from_numpy(W.make_labels(w, seeds["tokens"])).cuda()
    for sname, rec in gold["settings"].items():
        masters = W.make_lora_masters(w, seeds["lora"], b_std=rec["b_std"])
        m = M.ZoModel(w, frozen, masters)
        m.regen_noise(seeds["noise"], 0, eps=rec["eps"])
        got = m.forward_perturbed(tok, lab).cpu().numpy().astype(np.float64)
        assert np.isfinite(got).all()
        want, jit = np.array(rec["losses_bf16"]), np.array(rec["losses_bf16_jitter"])
        floor_l = np.abs(jit - want).max() / np.abs(want).max()
        err_l = np.abs(got[:2] - want).max() / np.abs(want).max()
        d_got, d_want, d_jit = got[0] - got[1], want[0] - want[1], jit[0] - jit[1]
        floor_d = abs(d_jit - d_want) / abs(d_want)
        err_d = abs(d_got - d_want) / abs(d_want)
        print(f"\n{name} [{sname}: eps {rec['eps']}, B std {rec['b_std']}] full depth, {2 * w.q} copies: "
              f"l0+ {got[0]:.7f} (oracle {want[0]:.7f})  l0- {got[1]:.7f} (oracle {want[1]:.7f})\n"
              f"   loss error {err_l:.2e} (oracle vs jittered oracle {floor_l:.2e});  l0+ - l0- = {d_got:.3e} "
              f"(oracle {d_want:.3e}): error {err_d:.2e} (oracle vs jittered oracle {floor_d:.2e});  "
              f"g_0 = {d_got / (2 * rec['eps']):.5f} (oracle {d_want / (2 * rec['eps']):.5f})", flush=True)
        # per-copy losses: within a few times the distance between two runs of the oracle itself
        assert err_l <= max(6.0 * floor_l, 1e-4), (err_l, floor_l)
        # the two-point difference (= 2 eps g_0): the 2e-2 bar where the oracle's own floor allows it, else a bound that
        # a wrong sign (error 2), a dropped perturbation (1) or a wrong per-copy factor at some depth (O(1)) cannot
        # pass; where the oracle's own difference moves by 20 % or more under the jitter nothing can be asserted
        if floor_d < 0.2:
            assert err_d <= min(max(2e-2, 6.0 * floor_d), 0.5), (err_d, floor_d)
            assert np.sign(d_got) == np.sign(d_want)
        else:
            print(f"   {name} [{sname}]: the oracle's own two-point difference moves by {floor_d:.2f} under a 1e-6 "
                  f"operand jitter: g_0 is not assertable here (parity of g unpinned at this setting)", flush=True)
        if sname == "strong":
            assert floor_d < 0.2, "the strong setting is meant to lift the two-point difference above the rounding floor"
        m.close()
        del m
    del frozen
    torch.cuda.empty_cache()
