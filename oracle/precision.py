"""Oracle: where the configured storage precision rounds a tensor.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

The method itself (Algorithm 1; the MP-LoRA layer equation of Section 3) is stated over the
reals; mode "exact" evaluates it in binary64 with no intermediate rounding.  The workloads fix
a storage precision ("fp32", or "bf16 weights with fp32 accumulation"), and the two-point
difference l(+) - l(-) is so small next to l that two implementations are only comparable when
they round the same tensors at the same places.  Modes "f32" and "bf16" therefore round

* operand(x): every tensor that is stored in the GEMM operand type (norm outputs, q/k/v,
  attention probabilities, attention output, FFN activation, the LoRA bottleneck x A) to
  that type (bf16: first to binary32, then to bf16, ties to even - the accumulator it is
  rounded from is binary32), and
* stream(x): the residual stream, logits, per-position losses and per-copy loss to binary32,

while every sum in between is accumulated in binary64.
"""
from __future__ import annotations

import numpy as np


def _bf16_rne(x32: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(x32, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


class Precision:
    def __init__(self, mode: str):
        assert mode in ("exact", "f32", "bf16")
        self.mode = mode

    @property
    def exact(self) -> bool:
        return self.mode == "exact"

    def operand(self, x):
        x = np.asarray(x, dtype=np.float64)
        if self.mode == "exact":
            return x
        x32 = x.astype(np.float32)
        if self.mode == "bf16":
            x32 = _bf16_rne(x32)
        return x32.astype(np.float64)

    def stream(self, x):
        x = np.asarray(x, dtype=np.float64)
        if self.mode == "exact":
            return x
        return x.astype(np.float32).astype(np.float64)

    def lora_factor(self, x):
        """A perturbed LoRA factor as the GEMM sees it.

        bf16 mode: the binary32 factor is split as hi + lo with hi = bf16(x), lo = bf16(x - hi), so a
        perturbation of a few bf16 ulps of A is not rounded away; f32 mode: the binary32 value.
        """
        x = np.asarray(x)
        if self.mode == "exact":
            return x.astype(np.float64)
        x32 = x.astype(np.float32)
        if self.mode == "f32":
            return x32.astype(np.float64)
        hi = _bf16_rne(x32)
        lo = _bf16_rne(x32 - hi)                  # x32 - hi is exact in binary32
        return hi.astype(np.float64) + lo.astype(np.float64)


class JitterPrecision(Precision):
    """Diagnostic, not part of the method: the bf16 contract with every operand nudged by a relative error of
    fp32-accumulation size before it is rounded - a stand-in for 'the same arithmetic with another summation
    order'.  The distance between a run with this class and a run with Precision("bf16") measures how far two
    correct implementations of a bf16 workload can drift apart (the floor the parity tests quote)."""

    def __init__(self, rel: float = 1e-6, seed: int = 0):
        super().__init__("bf16")
        self.rel, self.rng = rel, np.random.default_rng(seed)

    def operand(self, x):
        x = np.asarray(x, dtype=np.float64)
        return super().operand(x * (1.0 + self.rel * self.rng.standard_normal(x.shape)))
