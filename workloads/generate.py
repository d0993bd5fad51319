"""Seeded generators for synthetic weights, LoRA masters, tokens and labels.

Recipe (stands in for the pretrained checkpoints and task prompts the paper uses, which are
not available): every weight matrix, bias and embedding ~ N(0, 0.02^2); norm gains 1 and
norm biases 0; LoRA A ~ N(0, 0.02^2) and B = 0 (Section 2, "Low-Rank Adaptation"); token
ids i.i.d. uniform over the vocabulary, full-length sequences; labels uniform on {0, 1}.
For bf16 workloads the weights are rounded to bf16-representable values here, so that both
consumers start from identical bits.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .configs import Workload, lora_layout


def to_bf16_values(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable float32 (ties to even)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32)
    rounded = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def _normal(rng: np.random.Generator, shape, std: float, bf16: bool) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    x *= np.float32(std)
    return to_bf16_values(x) if bf16 else x


def _int8_weight(rng: np.random.Generator, shape):
    """Synthetic weight-only int8 linear [k_in, k_out]: codes ~ round(N(0, 32^2)) clipped to [-127, 127] and one
    float32 scale per output channel, 0.02/32 times a factor in [0.75, 1.25] (so the product is ~ N(0, 0.02^2) and
    a per-channel mix-up is visible)."""
    q = np.clip(np.rint(rng.standard_normal(shape, dtype=np.float32) * np.float32(32.0)), -127, 127).astype(np.int8)
    s = (np.float32(0.02 / 32.0) * (np.float32(0.75) + np.float32(0.5) * rng.random(shape[1], dtype=np.float32)))
    return q, s.astype(np.float32)


def _nf4_weight(rng: np.random.Generator, shape):
    """Synthetic weight-only 4-bit linear [k_in, k_out]: one code in 0..15 per element (uniform: the 4-bit normal-float
    levels are equal-probability bins of a normal weight) and one float32 absolute maximum per block of 64
    consecutive input channels of one output channel, [k_in / 64, k_out], 0.048 times a factor in [0.75, 1.25]
    (0.048 = 0.02 times the expected largest of 64 standard normals, about 2.4)."""
    if shape[0] % 64:
        raise ValueError("4-bit blocks hold 64 input channels: k_in must be a multiple of 64")
    codes = rng.integers(0, 16, size=shape, dtype=np.uint8)
    absmax = np.float32(0.048) * (np.float32(0.75) + np.float32(0.5) * rng.random((shape[0] // 64, shape[1]), dtype=np.float32))
    return codes, absmax.astype(np.float32)


def make_frozen_weights(w: Workload, seed: int, n_layers: Optional[int] = None) -> Dict[str, object]:
    """Frozen parameters as float32 arrays (bf16-representable when w.dtype == 'bf16').

    Layout: every linear is [k_in, k_out] row-major so that y = x W.  `w_qkv` is the column
    concatenation [W_q | W_k | W_v]; for SwiGLU `w_up` is [W_gate | W_up].  `emb` is
    [vocab, d]; `lm_head` is [vocab, d] (the same array as `emb` when embeddings are tied).
    Norm gains/biases are float32.  With w.weight_quant == "int8" the four linears of a block are int8 codes
    `w_*` [k_in, k_out] with float32 scales `s_*` [k_out] (embeddings and the head stay in the model dtype); with
    "nf4" they are uint8 codes 0..15 `w_*` [k_in, k_out] with float32 block maxima `s_*` [k_in / 64, k_out].
    """
    L = w.n_layers if n_layers is None else n_layers
    bf = w.dtype == "bf16"
    rng = np.random.default_rng(seed)
    d, f = w.d_model, w.d_ffn
    n_qkv = d + 2 * w.d_kv
    n_up = 2 * f if w.act == "swiglu" else f
    out: Dict[str, object] = {}
    out["emb"] = _normal(rng, (w.vocab, d), 0.02, bf)
    out["pos_emb"] = _normal(rng, (w.max_seq, d), 0.02, bf) if w.pos == "learned" else None
    layers = []
    for _ in range(L):
        lw = {
            "ln1_g": np.ones(d, np.float32),
            "ln1_b": np.zeros(d, np.float32) if w.norm == "layernorm" else None,
            "w_qkv": _normal(rng, (d, n_qkv), 0.02, bf),
            "b_qkv": _normal(rng, (n_qkv,), 0.02, False) if w.has_bias else None,
            "w_o": _normal(rng, (d, d), 0.02, bf),
            "b_o": _normal(rng, (d,), 0.02, False) if w.has_bias else None,
            "ln2_g": np.ones(d, np.float32),
            "ln2_b": np.zeros(d, np.float32) if w.norm == "layernorm" else None,
            "w_up": _normal(rng, (d, n_up), 0.02, bf),
            "b_up": _normal(rng, (n_up,), 0.02, False) if w.has_bias else None,
            "w_down": _normal(rng, (f, d), 0.02, bf),
            "b_down": _normal(rng, (d,), 0.02, False) if w.has_bias else None,
        }
        if w.weight_quant == "int8":
            for name in ("qkv", "o", "up", "down"):
                lw["w_" + name], lw["s_" + name] = _int8_weight(rng, lw["w_" + name].shape)
        elif w.weight_quant == "nf4":
            for name in ("qkv", "o", "up", "down"):
                lw["w_" + name], lw["s_" + name] = _nf4_weight(rng, lw["w_" + name].shape)
        elif w.weight_quant != "none":
            raise ValueError(f"unknown weight_quant {w.weight_quant!r}")
        layers.append(lw)
    out["layers"] = layers
    out["lnf_g"] = np.ones(d, np.float32)
    out["lnf_b"] = np.zeros(d, np.float32) if w.norm == "layernorm" else None
    out["lm_head"] = out["emb"] if w.tie_embeddings else _normal(rng, (w.vocab, d), 0.02, bf)
    return out


def make_lora_masters(w: Workload, seed: int, n_layers: Optional[int] = None,
                      b_std: float = 0.0) -> np.ndarray:
    """Flat float32 master vector in the canonical layout: A ~ N(0, 0.02^2), B = 0.

    `b_std` > 0 draws B ~ N(0, b_std^2) instead, for tests that need a non-trivial B.
    """
    ww = w if n_layers is None else w.with_(n_layers=n_layers)
    lay = lora_layout(ww)
    total = lay[-1].offset + lay[-1].rows * lay[-1].cols
    rng = np.random.default_rng(seed)
    flat = np.zeros(total, np.float32)
    for t in lay:
        n = t.rows * t.cols
        if t.factor == 0:
            flat[t.offset:t.offset + n] = rng.standard_normal(n, dtype=np.float32) * np.float32(0.02)
        elif b_std > 0.0:
            flat[t.offset:t.offset + n] = rng.standard_normal(n, dtype=np.float32) * np.float32(b_std)
    return flat


def make_tokens(w: Workload, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(0, w.vocab, size=(w.E, w.S), dtype=np.int32)


def make_labels(w: Workload, seed: int) -> np.ndarray:
    """Class ids in {0, 1}, one per sequence (used by the last-position loss modes)."""
    rng = np.random.default_rng(seed + 7919)
    return rng.integers(0, 2, size=(w.E,), dtype=np.int32)


def make_lengths(w: Workload, seed: int, pad_fraction: float = 0.3) -> np.ndarray:
    """Sequence lengths for a right-padded batch: the longest sequence fills S, the others are uniform on
    [2, S] scaled so that about `pad_fraction` of the E*S slots are padding (the paper reports 24-58 % padding at
    batch 16 and 1-38 % at batch 4 on its tasks; those datasets are not available here)."""
    rng = np.random.default_rng(seed + 104729)
    lo = max(2, int(round(w.S * (1.0 - 2.0 * pad_fraction))))
    lengths = rng.integers(lo, w.S + 1, size=(w.E,), dtype=np.int32)
    lengths[rng.integers(0, w.E)] = w.S
    return lengths
