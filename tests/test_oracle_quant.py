"""Pins for the oracle's weight-only quantised linears.

int8: the effective weight is code x per-channel scale, exactly.

* a hand-computed 2x2 instance;
* a model with int8 blocks equals the same model run on the float64 product matrices passed in as ordinary weights
  (the quantised path adds nothing but the dequantisation);
* scales are per OUTPUT channel: transposing the broadcast changes the loss.

4-bit normal float: level[code] x block maximum, rounded to the operand type.

* the level table against its definition (quantiles of the standard normal, computed here with scipy), its
  structure (seven negative levels, an exact zero, eight positive ones, ends at -1 and 1);
* a hand-computed block; nearest-level encoding of the dequantised values gives the codes back;
* a model with 4-bit blocks equals the same model on the dequantised matrices; blocks run along the INPUT dimension.
"""
import numpy as np

import workloads as W
from oracle import zo
from oracle.model import NF4_LEVELS, _weight, copy_loss, nf4_dequant
from oracle.precision import Precision
from small_workloads import MINI_LLAMA, MINI_OPT


def test_weight_by_hand():
    lw = {"w_o": np.array([[2, -3], [5, 7]], dtype=np.int8), "s_o": np.array([0.5, 0.25], dtype=np.float32)}
    assert np.array_equal(_weight(lw, "o", Precision("exact")), np.array([[1.0, -0.75], [2.5, 1.75]]))
    lw = {"w_o": np.array([[2.0, -3.0]], dtype=np.float32)}
    assert np.array_equal(_weight(lw, "o", Precision("bf16")), np.array([[2.0, -3.0]]))


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
        std = np.std(_weight(frozen["layers"][0], "up", prec))
        assert 0.015 < std < 0.025


def test_nf4_levels_are_the_normal_quantiles():
    """Q-LoRA's construction: 8 + 1 probabilities from delta to 1/2 on the positive side (the 1/2 itself dropped),
    7 + 1 on the negative side, delta = (1 - 1/(2*15) + 1 - 1/(2*16)) / 2 - one more positive level than negative ones,
    an exact zero, then division by the largest magnitude."""
    from scipy.stats import norm
    delta = 0.5 * ((1.0 - 1.0 / 30.0) + (1.0 - 1.0 / 32.0))
    pos = norm.ppf(np.linspace(delta, 0.5, 9)[:-1])
    neg = -norm.ppf(np.linspace(delta, 0.5, 8)[:-1])
    want = np.sort(np.concatenate([neg, [0.0], pos]))
    want /= np.abs(want).max()
    assert NF4_LEVELS.dtype == np.float32 and NF4_LEVELS.shape == (16,)
    assert np.abs(NF4_LEVELS.astype(np.float64) - want).max() < 5e-7
    assert NF4_LEVELS[0] == -1.0 and NF4_LEVELS[7] == 0.0 and NF4_LEVELS[15] == 1.0
    assert (np.diff(NF4_LEVELS) > 0).all() and (NF4_LEVELS[:7] < 0).all() and (NF4_LEVELS[8:] > 0).all()


def test_nf4_block_by_hand_and_round_trip():
    codes = np.zeros((128, 2), dtype=np.uint8)
    codes[:, 0] = np.arange(128) % 16
    codes[:, 1] = 15 - np.arange(128) % 16
    absmax = np.array([[0.5, 2.0], [0.25, 1.0]], dtype=np.float32)       # [k_in / 64, k_out]
    w = nf4_dequant(codes, absmax)
    assert w.dtype == np.float32 and w.shape == (128, 2)
    assert w[0, 0] == -0.5 and w[7, 0] == 0.0 and w[15, 0] == 0.5       # first block of channel 0: maximum 0.5
    assert w[64, 0] == -0.25 and w[64 + 15, 0] == 0.25                  # second block: 0.25
    assert w[0, 1] == 2.0 and w[15, 1] == -2.0 and w[64, 1] == 1.0      # channel 1: maxima 2 and 1
    assert w[8, 0] == np.float32(0.07958029955625534) * np.float32(0.5)
    # nearest level of w / absmax is the code again (powers of two: the division is exact)
    a = np.repeat(absmax, 64, axis=0)
    back = np.abs((w / a)[..., None] - NF4_LEVELS[None, None, :]).argmin(axis=-1)
    assert np.array_equal(back, codes)
    # operand rounding: bf16 mode rounds the product, exact mode keeps the binary32 product
    lw = {"w_o": codes, "s_o": absmax}
    assert np.array_equal(_weight(lw, "o", Precision("exact")), w.astype(np.float64))
    wb = _weight(lw, "o", Precision("bf16"))
    assert np.array_equal(wb, Precision("bf16").operand(w)) and not np.array_equal(wb, w.astype(np.float64))


def test_nf4_model_equals_model_on_dequantised_matrices():
    base = MINI_LLAMA.with_(d_ffn=128)
    w = base.with_(weight_quant="nf4")
    frozen = W.make_frozen_weights(w, 1234)
    lay = W.lora_layout(w)
    masters = W.make_lora_masters(w, 99, b_std=0.02)
    lora = zo.split_factors(lay, masters.astype(np.float64))
    tokens, labels = W.make_tokens(w, 5), W.make_labels(w, 5)
    for mode in ("exact", "bf16"):
        prec = Precision(mode)
        a = copy_loss(w, frozen, lora, tokens, labels, prec)
        dense, wrong = dict(frozen), dict(frozen)
        dense["layers"], wrong["layers"] = [], []
        for lw in frozen["layers"]:
            d2 = dict(lw)
            for n in ("qkv", "o", "up", "down"):
                c, s = lw["w_" + n], lw["s_" + n]
                assert c.dtype == np.uint8 and c.max() <= 15 and s.dtype == np.float32
                assert s.shape == (c.shape[0] // 64, c.shape[1])
                full = NF4_LEVELS[c] * np.repeat(s, 64, axis=0)          # binary32 product
                d2["w_" + n] = prec.operand(full)
                d2["s_" + n] = None
            dense["layers"].append(d2)
            d3 = dict(d2)
            c, s = lw["w_o"], lw["s_o"]                                 # [64, 64] codes, [1, 64] maxima
            d3["w_o"] = prec.operand(NF4_LEVELS[c] * np.repeat(s.T, 64, axis=1))   # blocks along the output dimension
            wrong["layers"].append(d3)
        assert copy_loss(base, dense, lora, tokens, labels, prec) == a
        assert copy_loss(base, wrong, lora, tokens, labels, prec) != a
    std = np.std(_weight(frozen["layers"][0], "up", Precision("exact")))
    assert 0.015 < std < 0.035
