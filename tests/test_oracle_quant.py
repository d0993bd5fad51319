"""Pins for the oracle's weight-only int8 linears: the effective weight is code x per-channel scale, exactly.

* a hand-computed 2x2 instance;
* a model with int8 blocks equals the same model run on the float64 product matrices passed in as ordinary weights
  (the quantised path adds nothing but the dequantisation);
* scales are per OUTPUT channel: transposing the broadcast changes the loss.
"""
import numpy as np

import workloads as W
from oracle import zo
from oracle.model import _weight, copy_loss
from oracle.precision import Precision
from small_workloads import MINI_LLAMA, MINI_OPT


def test_weight_by_hand():
    lw = {"w_o": np.array([[2, -3], [5, 7]], dtype=np.int8), "s_o": np.array([0.5, 0.25], dtype=np.float32)}
    assert np.array_equal(_weight(lw, "o"), np.array([[1.0, -0.75], [2.5, 1.75]]))
    lw = {"w_o": np.array([[2.0, -3.0]], dtype=np.float32)}
    assert np.array_equal(_weight(lw, "o"), np.array([[2.0, -3.0]]))


def test_quantised_model_equals_model_on_product_matrices():
    for base in (MINI_LLAMA, MINI_OPT):
        w = base.with_(weight_quant="int8")
        frozen = W.make_frozen_weights(w, 1234)
        lay = W.lora_layout(w)
        masters = W.make_lora_masters(w, 99, b_std=0.02)
        lora = zo.split_factors(lay, masters.astype(np.float64))
        tokens, labels = W.make_tokens(w, 5), W.make_labels(w, 5)
        prec = Precision("exact")
        a = copy_loss(w, frozen, lora, tokens, labels, prec)
        dense = dict(frozen)
        dense["layers"] = []
        for lw in frozen["layers"]:
            d2 = dict(lw)
            for n in ("qkv", "o", "up", "down"):
                assert lw["w_" + n].dtype == np.int8 and lw["s_" + n].dtype == np.float32
                assert lw["s_" + n].shape == (lw["w_" + n].shape[1],)
                d2["w_" + n] = lw["w_" + n].astype(np.float64) * lw["s_" + n].astype(np.float64)[None, :]
                d2["s_" + n] = None
            dense["layers"].append(d2)
        b = copy_loss(base, dense, lora, tokens, labels, prec)
        assert a == b
        # per-output-channel: scaling along the input dimension instead gives another model
        wrong = dict(frozen)
        wrong["layers"] = []
        for lw in frozen["layers"]:
            d2 = dict(lw)
            q, s = lw["w_o"], lw["s_o"]                         # square: both broadcasts are legal shapes
            d2["w_o"] = q.astype(np.float64) * s.astype(np.float64)[:, None]
            d2["s_o"] = None
            wrong["layers"].append(d2)
        assert copy_loss(w, wrong, lora, tokens, labels, prec) != a
        # the synthetic weights have the recipe's scale
        std = np.std(_weight(frozen["layers"][0], "up"))
        assert 0.015 < std < 0.025
