#!/usr/bin/env python3
"""Writes tests/golden/full_depth_query0_<workload>.json: the oracle's losses of query 0 (the + and the - copy) of
ONE full-depth step of workloads 3, 4 and 5 at their own E and S - the loss evaluations of Algorithm 1's inner loop
for k = 0, each an independent single-copy forward pass (Section 3: the copies are independent, so two of the 2q
suffice to check a batched pass at full depth).

Calls only oracle/ and workloads/ (never the HIP library).  Weights come from the integer-hash generator
(workloads/hashed.py), which the GPU test reproduces bit for bit on the device.  Two settings per workload:
  "workload": the workload's own recipe, eps = 1e-3, B = 0;
  "strong":   eps = 5e-2 and B ~ N(0, 0.05^2), where the per-copy low-rank term moves the projections by O(10 %), so
              that a wrong per-copy factor at any depth shows in the loss.
Each is evaluated twice: with the bf16 rounding contract, and with the jittered contract (operands nudged by 1e-6
relative before rounding), whose distance from the first is the floor two correct bf16 implementations can differ by.

  python tests/golden/make_full_depth_golden.py [c3_opt1p3b c4_llama1p1b c5_llama7b]     (minutes to an hour each)
"""
import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

import workloads as W  # noqa: E402
from oracle import zo  # noqa: E402
from oracle.model import copy_loss  # noqa: E402
from oracle.precision import Precision, JitterPrecision  # noqa: E402

SEEDS = {"weights": 1234, "lora": 99, "tokens": 2345, "noise": 3456}
SETTINGS = {"workload": dict(eps=None, b_std=0.0), "strong": dict(eps=5e-2, b_std=0.05)}


def golden_for(name):
    w = W.get_workload(name)
    lay = W.lora_layout(w)
    t0 = time.time()
    frozen = W.make_frozen_weights_hashed(w, SEEDS["weights"])
    tokens, labels = W.make_tokens(w, SEEDS["tokens"]), W.make_labels(w, SEEDS["tokens"])
    print(f"{name}: weights drawn in {time.time() - t0:.0f} s", flush=True)
    out = {"workload": name, "seeds": SEEDS, "step": 0, "query": 0,
           "source": "oracle/ (copy_loss, bf16 rounding contract), Algorithm 1 inner loop for k = 0",
           "weights": "workloads.make_frozen_weights_hashed", "settings": {}}
    for sname, st in SETTINGS.items():
        eps = w.eps if st["eps"] is None else st["eps"]
        masters = W.make_lora_masters(w, SEEDS["lora"], b_std=st["b_std"])
        z = zo.draw_z(lay, SEEDS["noise"], 0, 0, masters.size, w.perturb_A)
        rec = {"eps": eps, "b_std": st["b_std"]}
        for pname, prec in (("bf16", Precision("bf16")), ("bf16_jitter", JitterPrecision(1e-6, 1))):
            losses = []
            for sign in (+1, -1):
                t0 = time.time()
                theta = zo.perturb(masters, z, sign, eps, Precision("bf16"))
                l = copy_loss(w, frozen, zo.split_factors(lay, theta), tokens, labels, prec)
                losses.append(float(np.float32(l)))
                print(f"{name} {sname} {pname} sign {sign:+d}: loss {l:.9f}  ({time.time() - t0:.0f} s)", flush=True)
            rec["losses_" + pname] = losses
        out["settings"][sname] = rec
    path = os.path.join(HERE, f"full_depth_query0_{name}.json")
    with open(path, "w") as f:
        json.dump(out, f, indent=1)
        f.write("\n")
    print("wrote", path, flush=True)


if __name__ == "__main__":
    for nm in (sys.argv[1:] or ["c3_opt1p3b", "c4_llama1p1b", "c5_llama7b"]):
        golden_for(nm)
