"""Pins for the oracle's single-copy loss (CPU only).

* against an independent evaluation built from PyTorch library routines with merged LoRA weights
  (all three architectures / loss modes, non-zero B, scaled-up weights so every nonlinearity matters);
* closed forms: zero head gives ln 2 / ln V; B = 0 makes the loss independent of A;
* rotary embedding: relative-position property.
"""
import math

import numpy as np
import pytest
import torch

import workloads as W
from oracle import zo
from oracle.model import copy_loss, _rope, rope_tables, _attention
from oracle.precision import Precision

from small_workloads import C1, MINI_LLAMA, MINI_OPT, MICRO, bundle
from torch_reference import torch_loss

EXACT = Precision("exact")


def _oracle_loss(b, flat, w=None):
    w = w or b["w"]
    return copy_loss(w, b["frozen"], zo.split_factors(b["layout"], flat), b["tokens"], b["labels"], EXACT)


@pytest.mark.parametrize("wl", [C1, MINI_LLAMA, MINI_OPT, MICRO], ids=lambda w: w.name)
@pytest.mark.parametrize("scale", [1.0, 8.0])
def test_loss_matches_torch_library_evaluation(wl, scale):
    b = bundle(wl, b_std=0.05, scale_weights=scale)
    flat = b["masters"].astype(np.float64)
    got = _oracle_loss(b, flat)
    want = float(torch_loss(wl, b["frozen"], b["layout"], torch.from_numpy(flat), b["tokens"], b["labels"]))
    assert got == pytest.approx(want, rel=1e-12, abs=1e-13)


def test_lora_scale_and_loss_modes_match_torch():
    for mode in ("last_pos_label_subset", "last_pos_full_vocab", "next_token_all_pos"):
        wl = MINI_OPT.with_(loss_mode=mode, lora_scale=2.0, act="gelu")
        b = bundle(wl, b_std=0.1, scale_weights=6.0)
        flat = b["masters"].astype(np.float64)
        want = float(torch_loss(wl, b["frozen"], b["layout"], torch.from_numpy(flat), b["tokens"], b["labels"]))
        assert _oracle_loss(b, flat) == pytest.approx(want, rel=1e-12)


def test_zero_head_gives_log_of_class_count():
    for wl, want in ((C1, math.log(2.0)), (MINI_OPT.with_(tie_embeddings=False), math.log(64.0)),
                     (MINI_LLAMA, math.log(80.0))):
        b = bundle(wl, b_std=0.05)
        b["frozen"]["lm_head"] = np.zeros_like(b["frozen"]["lm_head"])
        assert _oracle_loss(b, b["masters"].astype(np.float64)) == pytest.approx(want, rel=1e-14)


def test_zero_B_makes_loss_independent_of_A():
    b = bundle(C1)                                    # B = 0 at initialisation (Section 2)
    flat = b["masters"].astype(np.float64)
    base = _oracle_loss(b, flat)
    rng = np.random.default_rng(0)
    other = flat.copy()
    for t in b["layout"]:
        if t.factor == 0:
            other[t.offset:t.offset + t.rows * t.cols] = rng.standard_normal(t.rows * t.cols)
    assert _oracle_loss(b, other) == base
    # and equals the un-adapted base model (no LoRA at all) evaluated by the torch routines
    none = float(torch_loss(C1, b["frozen"], [], torch.zeros(1, dtype=torch.float64), b["tokens"], b["labels"]))
    assert base == pytest.approx(none, rel=1e-13)


def test_rope_depends_only_on_relative_position():
    S, dh = 16, 8
    cos, sin = rope_tables(S, dh, 10000.0, EXACT)
    rng = np.random.default_rng(3)
    qv, kv = rng.standard_normal(dh), rng.standard_normal(dh)
    x = np.broadcast_to(qv, (1, S, 1, dh)).copy()
    y = np.broadcast_to(kv, (1, S, 1, dh)).copy()
    xr, yr = _rope(x, cos, sin)[0, :, 0], _rope(y, cos, sin)[0, :, 0]
    dots = xr @ yr.T                                  # [S, S]: position i of q with position j of k
    for off in range(-3, 4):
        diag = np.diagonal(dots, offset=off)
        assert np.allclose(diag, diag[0], rtol=1e-12, atol=1e-12)
    assert np.allclose(xr[0], qv)                     # position 0 is the identity
    assert np.allclose(np.linalg.norm(xr, axis=-1), np.linalg.norm(qv))
    assert not np.allclose(np.diagonal(dots, 1)[0], np.diagonal(dots, 2)[0])


def test_attention_is_causal_and_grouped():
    rng = np.random.default_rng(4)
    E, S, H, Hkv, dh = 1, 6, 4, 2, 8
    q = rng.standard_normal((E, S, H, dh))
    k = rng.standard_normal((E, S, Hkv, dh))
    v = rng.standard_normal((E, S, Hkv, dh))
    out = _attention(q, k, v, H, Hkv, EXACT).reshape(E, S, H, dh)
    assert np.allclose(out[0, 0, 0], v[0, 0, 0]) and np.allclose(out[0, 0, 3], v[0, 0, 1])
    k2, v2 = k.copy(), v.copy()
    k2[0, 4:], v2[0, 4:] = 9.0, -7.0                  # the future must not leak into positions < 4
    out2 = _attention(q, k2, v2, H, Hkv, EXACT).reshape(E, S, H, dh)
    assert np.array_equal(out[0, :4], out2[0, :4]) and not np.allclose(out[0, 4:], out2[0, 4:])


def test_rounded_modes_stay_close_to_exact():
    b = bundle(C1, b_std=0.02)
    lora = zo.split_factors(b["layout"], b["masters"])
    ex = copy_loss(C1, b["frozen"], lora, b["tokens"], b["labels"], EXACT)
    f32 = copy_loss(C1, b["frozen"], lora, b["tokens"], b["labels"], Precision("f32"))
    bf = copy_loss(C1, b["frozen"], lora, b["tokens"], b["labels"], Precision("bf16"))
    assert f32 == float(np.float32(f32)) and abs(f32 - ex) < 2e-7
    assert abs(bf - ex) < 5e-3 and bf != ex


def test_bf16_factor_split_is_hi_plus_lo():
    p = Precision("bf16")
    x = np.float32([0.0201171875, -1.2345678e-3, 3.0, 1e-8])
    eff = p.lora_factor(x)
    assert np.abs(eff - x.astype(np.float64)).max() <= np.abs(x).max() * 2.0**-16
    hi = p.operand(x)
    assert np.array_equal(p.operand(eff - hi), eff - hi)      # the remainder is itself a bf16 number
