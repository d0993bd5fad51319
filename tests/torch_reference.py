"""An independent binary64 evaluation of the same decoder loss, built from PyTorch CPU library
routines (layer_norm / rms_norm, scaled_dot_product_attention, gelu / silu, cross_entropy)
and with the LoRA factors MERGED into the weights (W + s A B) instead of applied as (x A) B.
Used only to pin the oracle; differentiable, so it also yields the exact LoRA gradient.
"""
import math

import torch
import torch.nn.functional as F

TARGETS = ("q", "k", "v", "o")


def _t(x):
    return None if x is None else torch.as_tensor(x, dtype=torch.float64)


def _norm(h, g, b, w):
    eps = float(torch.tensor(w.norm_eps, dtype=torch.float32))      # hyper-parameters are binary32 numbers
    if w.norm == "layernorm":
        return F.layer_norm(h, (w.d_model,), _t(g), _t(b), eps)
    return F.rms_norm(h, (w.d_model,), _t(g), eps)


def _rope_complex(x, S, dh, theta):
    """Rotary embedding as a complex multiplication: (x_i + j x_{i+dh/2}) * exp(j p theta^(-2i/dh))."""
    half = dh // 2
    inv = theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / dh)
    ang = torch.arange(S, dtype=torch.float64)[:, None] * inv[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)                     # [S, half]
    xc = torch.complex(x[..., :half], x[..., half:]) * rot[None, :, None, :]
    return torch.cat([xc.real, xc.imag], dim=-1)


def torch_loss(w, frozen, layout, lora_flat, tokens, labels):
    """lora_flat: 1-D float64 tensor (may require grad) in the canonical layout."""
    E, S = tokens.shape
    d, H, Hkv, dh = w.d_model, w.n_heads, w.n_kv_heads, w.d_head
    fac = {}
    for t in layout:
        fac[(t.layer, t.target, t.factor)] = lora_flat[t.offset:t.offset + t.rows * t.cols].reshape(t.rows, t.cols)
    tok = torch.as_tensor(tokens, dtype=torch.long)
    h = F.embedding(tok, _t(frozen["emb"]))
    if w.pos == "learned":
        h = h + _t(frozen["pos_emb"])[:S]
    for li, lw in enumerate(frozen["layers"]):
        def merged(W, c0, c1, tname):
            Wm = _t(W)[:, c0:c1]
            ti = TARGETS.index(tname)
            if (li, ti, 0) in fac:
                Wm = Wm + w.lora_scale * fac[(li, ti, 0)] @ fac[(li, ti, 1)]
            return Wm
        x = _norm(h, lw["ln1_g"], lw["ln1_b"], w)
        Wqkv = torch.cat([merged(lw["w_qkv"], 0, d, "q"), merged(lw["w_qkv"], d, d + w.d_kv, "k"),
                          merged(lw["w_qkv"], d + w.d_kv, d + 2 * w.d_kv, "v")], dim=1)
        qkv = F.linear(x, Wqkv.T, _t(lw["b_qkv"]))
        q, k, v = qkv.split([d, w.d_kv, w.d_kv], dim=-1)
        q = q.reshape(E, S, H, dh)
        k = k.reshape(E, S, Hkv, dh)
        v = v.reshape(E, S, Hkv, dh)
        if w.pos == "rope":
            q, k = _rope_complex(q, S, dh, w.rope_theta), _rope_complex(k, S, dh, w.rope_theta)
        a = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2),
                                           is_causal=True, enable_gqa=(H != Hkv))
        a = a.transpose(1, 2).reshape(E, S, d)
        h = h + F.linear(a, merged(lw["w_o"], 0, d, "o").T, _t(lw["b_o"]))
        x = _norm(h, lw["ln2_g"], lw["ln2_b"], w)
        up = F.linear(x, _t(lw["w_up"]).T, _t(lw["b_up"]))
        if w.act == "relu":
            u = F.relu(up)
        elif w.act == "gelu":
            u = F.gelu(up)
        else:
            u = F.silu(up[..., :w.d_ffn]) * up[..., w.d_ffn:]
        h = h + F.linear(u, _t(lw["w_down"]).T, _t(lw["b_down"]))
    hf = _norm(h, frozen["lnf_g"], frozen["lnf_b"], w)
    head = _t(frozen["lm_head"])
    if w.loss_mode == "next_token_all_pos":
        logits = F.linear(hf[:, :-1], head).reshape(-1, w.vocab)
        return F.cross_entropy(logits, tok[:, 1:].reshape(-1))
    last = hf[:, -1]
    lab = torch.as_tensor(labels, dtype=torch.long)
    if w.loss_mode == "last_pos_label_subset":
        return F.cross_entropy(F.linear(last, head[list(w.label_tokens)]), lab)
    return F.cross_entropy(F.linear(last, head), torch.as_tensor(w.label_tokens, dtype=torch.long)[lab])
