"""Oracle: loss of ONE perturbed copy of the LoRA-adapted decoder on one token batch.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

This is the function l = L((theta_l, theta_f); B) that Algorithm 1 (the loss evaluation inside its inner loop) evaluates for each
perturbed parameter vector.  Every adapted linear is the LoRA layer of Section 2,
y = x W + x A B (here with an explicit scale s: y = x W + b + s (x A) B), which is what one path
of the MP-LoRA equation Y = X W + (X A) (.) B of Section 3 computes.  The decoder around it
(pre-norm blocks, causal attention, LayerNorm/RMSNorm, learned positions or rotary embedding,
ReLU/GELU/SwiGLU, cross-entropy) is the standard architecture of the evaluated model
families (Section 4), written out in its plain definition: one copy at a time, whole-tensor
NumPy operations, binary64 sums, no tiling, no fusion.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np
from scipy.special import erf

from .precision import Precision

TARGETS = ("q", "k", "v", "o")


def _norm(h, gain, bias, kind: str, eps: float):
    if kind == "layernorm":
        mu = h.mean(axis=-1, keepdims=True)
        var = ((h - mu) ** 2).mean(axis=-1, keepdims=True)
        y = (h - mu) / np.sqrt(var + eps) * gain
        return y + bias if bias is not None else y
    ms = (h ** 2).mean(axis=-1, keepdims=True)          # RMSNorm
    return h / np.sqrt(ms + eps) * gain


def rope_tables(S: int, d_head: int, theta: float, prec: Precision) -> Tuple[np.ndarray, np.ndarray]:
    """cos/sin of p * theta^(-2i/d_head), p < S, i < d_head/2 (stored in binary32 unless exact)."""
    i = np.arange(d_head // 2, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / d_head)
    ang = np.arange(S, dtype=np.float64)[:, None] * inv_freq[None, :]
    return prec.stream(np.cos(ang)), prec.stream(np.sin(ang))


def _rope(x, cos, sin):
    """Rotate pairs (i, i + d_head/2) of x [E, S, H, d_head] by the position angle."""
    half = x.shape[-1] // 2
    a, b = x[..., :half], x[..., half:]
    c, s = cos[None, :, None, :], sin[None, :, None, :]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def _lora_delta(x, lora, layer: int, target: str, scale: float, prec: Precision):
    """s (x A) B for one adapted linear, or None when the target carries no adapter."""
    key = (layer, TARGETS.index(target))
    if key not in lora:
        return None
    A, B = lora[key]
    t = prec.operand(scale * (x @ prec.lora_factor(A)))
    return t @ prec.lora_factor(B)


# The sixteen levels of the 4-bit normal-float type of Q-LoRA (Dettmers et al. 2023, appendix "NormalFloat 4-bit
# data type"), which Appendix D builds on: quantiles of N(0, 1) scaled to [-1, 1] with an exact zero - seven negative
# levels, zero, eight positive ones - as binary32 values.
NF4_LEVELS = np.array([
    -1.0, -0.6961928009986877, -0.5250730514526367, -0.39491748809814453, -0.28444138169288635,
    -0.18477343022823334, -0.09105003625154495, 0.0, 0.07958029955625534, 0.16093020141124725,
    0.24611230194568634, 0.33791524171829224, 0.44070982933044434, 0.5626170039176941, 0.7229568362236023, 1.0],
    dtype=np.float32)
NF4_BLOCK = 64


def nf4_dequant(codes: np.ndarray, absmax: np.ndarray) -> np.ndarray:
    """Weight [k_in, k_out] in binary32 from 4-bit codes [k_in, k_out] (0..15) and one absolute maximum per block of
    64 consecutive input channels of an output channel, [k_in / 64, k_out]: level[code] x absmax, one binary32
    multiplication per element (reading: blocks run along the input dimension, no second quantisation of the
    maxima)."""
    codes = np.asarray(codes)
    assert codes.dtype == np.uint8 and codes.max(initial=0) < 16 and codes.shape[0] % NF4_BLOCK == 0
    a = np.repeat(np.asarray(absmax, dtype=np.float32), NF4_BLOCK, axis=0)
    assert a.shape == codes.shape
    return NF4_LEVELS[codes] * a


def _weight(lw, name: str, prec: Precision) -> np.ndarray:
    """Frozen weight [k_in, k_out] of a block in binary64.  With weight-only quantisation (Appendix D, "MobiZO with
    weight-only quantization": weights are stored in a low-bit format and dequantised for the forward pass) the
    stored form is either an int8 code per element and a scale per output channel - the weight is their exact
    product (reading: no rounding to the 16-bit operand type on the way) - or a 4-bit normal-float code per element
    and a maximum per block of 64, dequantised to the operand type as the appendix describes (binary32 product,
    then the operand rounding)."""
    W = np.asarray(lw["w_" + name])
    s = lw.get("s_" + name)
    if s is None:
        return W.astype(np.float64)
    if W.dtype == np.uint8:
        return np.asarray(prec.operand(nf4_dequant(W, s)), dtype=np.float64)
    return W.astype(np.float64) * np.asarray(s, dtype=np.float64)[None, :]


def _linear(x, W, b, delta=None):
    y = x @ np.asarray(W, dtype=np.float64)
    if b is not None:
        y = y + b
    if delta is not None:
        y = y + delta
    return y


def _attention(q, k, v, n_heads: int, n_kv: int, prec: Precision):
    """Causal softmax attention; q [E,S,H,dh], k/v [E,S,Hkv,dh] -> [E,S,H*dh]."""
    E, S, H, dh = q.shape
    group = n_heads // n_kv
    out = np.empty((E, S, H, dh))
    mask = np.triu(np.ones((S, S), dtype=bool), k=1)
    scale = prec.stream(1.0 / np.sqrt(dh))
    for h in range(H):
        kh = h // group
        s = prec.stream(np.einsum("esd,etd->est", q[:, :, h], k[:, :, kh])) * scale
        s = np.where(mask[None], -np.inf, s)
        p = prec.operand(np.exp(s - s.max(axis=-1, keepdims=True)))
        out[:, :, h] = np.einsum("est,etd->esd", p, v[:, :, kh]) / p.sum(axis=-1, keepdims=True)
    return out.reshape(E, S, H * dh)


def _cross_entropy(logits, target):
    """-log softmax(logits)[target] row-wise; logits [N, C], target [N]."""
    m = logits.max(axis=-1, keepdims=True)
    lse = m[:, 0] + np.log(np.exp(logits - m).sum(axis=-1))
    return lse - logits[np.arange(logits.shape[0]), target]


def embed(w, frozen, tokens: np.ndarray, prec: Precision):
    """Token (+ learned position) embedding -> residual stream h [E, S, d]."""
    S = tokens.shape[1]
    h = np.asarray(frozen["emb"], dtype=np.float64)[tokens]
    if w.pos == "learned":
        h = h + np.asarray(frozen["pos_emb"], dtype=np.float64)[None, :S]
    return prec.stream(h)


def decoder_layer(w, lw, li: int, h, lora, prec: Precision):
    """One pre-norm decoder block on h [E, S, d] with this copy's LoRA factors."""
    E, S, d = h.shape
    H, Hkv, dh = w.n_heads, w.n_kv_heads, w.d_head
    norm_eps = float(np.float32(w.norm_eps))            # hyper-parameters are binary32 numbers
    scale = float(np.float32(w.lora_scale))
    x = prec.operand(_norm(h, lw["ln1_g"], lw["ln1_b"], w.norm, norm_eps))
    Wqkv, bqkv = _weight(lw, "qkv", prec), lw["b_qkv"]
    cols = {"q": (0, d), "k": (d, d + w.d_kv), "v": (d + w.d_kv, d + 2 * w.d_kv)}
    proj = {}
    for name, (c0, c1) in cols.items():
        b = bqkv[c0:c1] if bqkv is not None else None
        proj[name] = _linear(x, Wqkv[:, c0:c1], b, _lora_delta(x, lora, li, name, scale, prec))
    qh = proj["q"].reshape(E, S, H, dh)
    kh = proj["k"].reshape(E, S, Hkv, dh)
    vh = proj["v"].reshape(E, S, Hkv, dh)
    if w.pos == "rope":
        cos, sin = rope_tables(S, dh, w.rope_theta, prec)
        qh, kh = _rope(qh, cos, sin), _rope(kh, cos, sin)
    qh, kh, vh = prec.operand(qh), prec.operand(kh), prec.operand(vh)
    attn = prec.operand(_attention(qh, kh, vh, H, Hkv, prec))
    h = prec.stream(h + _linear(attn, _weight(lw, "o", prec), lw["b_o"], _lora_delta(attn, lora, li, "o", scale, prec)))

    x = prec.operand(_norm(h, lw["ln2_g"], lw["ln2_b"], w.norm, norm_eps))
    up = _linear(x, _weight(lw, "up", prec), lw["b_up"])
    if w.act == "relu":
        u = np.maximum(up, 0.0)
    elif w.act == "gelu":
        u = 0.5 * up * (1.0 + erf(up / np.sqrt(2.0)))
    else:                                                                    # SwiGLU
        gate, lin = up[..., :w.d_ffn], up[..., w.d_ffn:]
        u = gate / (1.0 + np.exp(-gate)) * lin
    u = prec.operand(u)
    return prec.stream(h + _linear(u, _weight(lw, "down", prec), lw["b_down"]))


def head_loss(w, frozen, h, tokens: np.ndarray, labels, prec: Precision, lengths=None) -> float:
    """Final norm, LM head and the mean cross-entropy of this copy in the configured loss mode.

    `lengths` (optional, one per sequence, 2 <= length <= S): sequences are right-padded to S as in the paper's batches
    (Section 3 discusses the padding that batching sequences of unequal length brings); only real tokens carry a loss.
    Next-token mode: positions p < length - 1; last-position modes: position length - 1.  The mean runs over the
    copy's loss positions."""
    E, S, d = h.shape
    norm_eps = float(np.float32(w.norm_eps))
    head = np.asarray(frozen["lm_head"], dtype=np.float64)                       # [V, d]
    lengths = np.full(E, S, dtype=np.int64) if lengths is None else np.asarray(lengths, dtype=np.int64)
    if w.loss_mode == "next_token_all_pos":
        xf = prec.operand(_norm(h[:, :S - 1], frozen["lnf_g"], frozen["lnf_b"], w.norm, norm_eps))
        logits = prec.stream(xf.reshape(-1, d) @ head.T)
        ce = _cross_entropy(logits, tokens[:, 1:].reshape(-1)).reshape(E, S - 1)
        valid = np.arange(S - 1)[None, :] < (lengths[:, None] - 1)
        ce = ce[valid]                                                           # row-major: sequence, then position
    else:
        last = h[np.arange(E), lengths - 1]
        xf = prec.operand(_norm(last, frozen["lnf_g"], frozen["lnf_b"], w.norm, norm_eps))
        labels = np.asarray(labels)
        if w.loss_mode == "last_pos_label_subset":
            logits = prec.stream(xf @ head[list(w.label_tokens)].T)              # [E, 2]
            ce = _cross_entropy(logits, labels)
        else:                                                                    # last_pos_full_vocab
            logits = prec.stream(xf @ head.T)
            ce = _cross_entropy(logits, np.asarray(w.label_tokens)[labels])
    return float(prec.stream(prec.stream(ce).mean()))


def copy_loss(w, frozen: Dict[str, object], lora: Dict[Tuple[int, int], Tuple[np.ndarray, np.ndarray]],
              tokens: np.ndarray, labels, prec: Precision, trace=None, lengths=None) -> float:
    """Loss of one copy.  `lora[(layer, target_index)] = (A_c, B_c)` are that copy's factors.
    If `trace` is a list, the residual stream after the embedding and after every block is appended."""
    h = embed(w, frozen, tokens, prec)
    if trace is not None:
        trace.append(h)
    for li, lw in enumerate(frozen["layers"]):
        h = decoder_layer(w, lw, li, h, lora, prec)
        if trace is not None:
            trace.append(h)
    return head_loss(w, frozen, h, tokens, labels, prec, lengths)
