"""Frozen weights from an integer hash, identical bit for bit on the host and on the GPU.

The NumPy generator of `generate.py` draws a 7B-shaped model in minutes and its arrays must then be uploaded; this one
is for the full-size workloads, where the oracle (on the host) and the library (on the device) must start from the
same weights and neither side can wait that long.  Every weight is a function of (seed, tensor number, flat index) alone:

    h     = mix64(index + (tensor number << 40) + seed * 0x9E3779B97F4A7C15)     (the SplitMix64 finaliser)
    level = bits 24..39 of h                                                     (uniform on 0 .. 65535)
    value = bf16(std * QUANTILE[level])         QUANTILE[i] = inverse normal CDF at (i + 1/2) / 65536, binary32

so the values are N(0, std^2) quantised to 65536 equally likely levels, then rounded to bf16 like every stored weight.
Only 64-bit integer arithmetic (which wraps the same way everywhere), one table lookup, one binary32 multiplication
and the bf16 rounding are involved, so `device="cpu"` and `device="cuda"` give the same bits.  The table is computed
on the host in binary64 by whichever side calls.  Flat indices follow the OUTPUT-MAJOR layout the library reads
(`[k_out, k_in]`, element (n, k) at n * k_in + k); the host dictionary holds the same matrices as `[k_in, k_out]`
transposed views, the layout the oracle reads.  Nothing of the method's arithmetic is here.
"""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np

from .configs import Workload

_MASK64 = (1 << 64) - 1


def _i64(v: int) -> int:
    """The 64-bit pattern v as a signed Python int (torch int64 scalars are signed)."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_QUANTILES = None


def normal_quantile_table() -> np.ndarray:
    """QUANTILE[i] = inverse standard normal CDF at (i + 1/2) / 65536, as binary32."""
    global _QUANTILES
    if _QUANTILES is None:
        from scipy.special import ndtri
        _QUANTILES = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0).astype(np.float32)
    return _QUANTILES


def hashed_levels(i0: int, i1: int, tensor_no: int, seed: int, device: str = "cpu"):
    """int64 tensor of the levels 0 .. 65535 of flat indices i0 .. i1-1 of tensor `tensor_no`."""
    import torch
    z = torch.arange(i0, i1, dtype=torch.int64, device=device)
    z += _i64((tensor_no << 40) + seed * 0x9E3779B97F4A7C15)
    # SplitMix64 finaliser; >> on int64 is arithmetic, the masks make it logical
    z ^= (z >> 30) & ((1 << 34) - 1)
    z *= _i64(0xBF58476D1CE4E5B9)
    z ^= (z >> 27) & ((1 << 37) - 1)
    z *= _i64(0x94D049BB133111EB)
    z ^= (z >> 31) & ((1 << 33) - 1)
    return (z >> 24) & 0xFFFF


def hashed_normal(shape, tensor_no: int, seed: int, std: float = 0.02, bf16: bool = True, device: str = "cpu"):
    """float32 tensor of `shape` (bf16-representable values when bf16): std * QUANTILE[level], row-major flat index."""
    import torch
    n = int(np.prod(shape))
    table = torch.from_numpy(normal_quantile_table()).to(device)
    out = torch.empty(n, dtype=torch.float32, device=device)
    chunk = 1 << 26                                            # bounds the int64 temporaries
    for i0 in range(0, n, chunk):
        i1 = min(n, i0 + chunk)
        out[i0:i1] = table[hashed_levels(i0, i1, tensor_no, seed, device)] * np.float32(std)
    if bf16:
        out = out.to(torch.bfloat16).to(torch.float32)
    return out.reshape(shape)


def make_frozen_weights_hashed(w: Workload, seed: int, device: str = "cpu") -> Dict[str, object]:
    """Frozen parameters of workload w (plain bf16 / fp32 weights, no weight-only quantisation) from the hash.

    device = "cpu": NumPy float32 arrays in the oracle's layout (linears `[k_in, k_out]`, as transposed views), the
    dictionary `workloads.make_frozen_weights` returns.  Any other device: torch tensors on that device in the
    library's layout (`[k_out, k_in]`, model dtype), marked `_device_output_major` for the binding.
    Tensor numbers: 0 token embedding, 1 learned positions, 2 head (untied), 16 l + (0 q/k/v, 1 its bias, 2 o, 3 its bias,
    4 up (gate | up), 5 its bias, 6 down, 7 its bias) + 16 for block l.  Norm gains 1, norm biases 0."""
    import torch
    if w.weight_quant != "none":
        raise ValueError("hashed weights are plain bf16 / fp32 weights")
    host = device == "cpu"
    bf = w.dtype == "bf16"
    st = torch.bfloat16 if bf else torch.float32
    d, f = w.d_model, w.d_ffn
    n_qkv, n_up = d + 2 * w.d_kv, (2 * f if w.act == "swiglu" else f)

    def mat(n_out, n_in, no):
        t = hashed_normal((n_out, n_in), no, seed, 0.02, bf, device)
        return t.numpy().T if host else t.to(st)

    def vec(n, no):
        t = hashed_normal((n,), no, seed, 0.02, False, device)
        return t.numpy() if host else t

    def table(rows, cols, no):
        t = hashed_normal((rows, cols), no, seed, 0.02, bf, device)
        return t.numpy() if host else t.to(st)

    def const(n, v):
        return np.full(n, v, np.float32) if host else torch.full((n,), v, dtype=torch.float32, device=device)

    ln = w.norm == "layernorm"
    out: Dict[str, object] = {"emb": table(w.vocab, d, 0),
                              "pos_emb": table(w.max_seq, d, 1) if w.pos == "learned" else None, "layers": []}
    if not host:
        out["_device_output_major"] = True
    for l in range(w.n_layers):
        b0 = 16 * l + 16
        lw = {"ln1_g": const(d, 1.0), "ln1_b": const(d, 0.0) if ln else None,
              "w_qkv": mat(n_qkv, d, b0), "b_qkv": vec(n_qkv, b0 + 1) if w.has_bias else None,
              "w_o": mat(d, d, b0 + 2), "b_o": vec(d, b0 + 3) if w.has_bias else None,
              "ln2_g": const(d, 1.0), "ln2_b": const(d, 0.0) if ln else None,
              "w_up": mat(n_up, d, b0 + 4), "b_up": vec(n_up, b0 + 5) if w.has_bias else None,
              "w_down": mat(d, f, b0 + 6), "b_down": vec(d, b0 + 7) if w.has_bias else None}
        if not host:
            lw.update({"s_qkv": None, "s_o": None, "s_up": None, "s_down": None})
        out["layers"].append(lw)
    out["lnf_g"], out["lnf_b"] = const(d, 1.0), (const(d, 0.0) if ln else None)
    out["lm_head"] = out["emb"] if w.tie_embeddings else table(w.vocab, d, 2)
    return out
