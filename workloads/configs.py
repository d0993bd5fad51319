"""Workload descriptions: decoder shapes and zeroth-order hyper-parameters.

The five named workloads are the decoder shapes the paper evaluates (OPT-, TinyLlama- and
Llama-2-shaped models, Section 4 and Appendix D) plus a tiny fp32 model for exact checks.
Every field is a plain shape or hyper-parameter; nothing here computes anything.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, NamedTuple, Tuple

TARGETS = ("q", "k", "v", "o")          # canonical LoRA target order


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int
    max_seq: int
    act: str                 # "relu" | "gelu" | "swiglu"
    norm: str                # "layernorm" | "rmsnorm"
    pos: str                 # "learned" | "rope"
    has_bias: bool
    tie_embeddings: bool
    dtype: str               # "f32" | "bf16": storage / GEMM operand type
    lora_rank: int
    lora_targets: Tuple[str, ...]
    loss_mode: str           # "last_pos_label_subset" | "last_pos_full_vocab" | "next_token_all_pos"
    q: int                   # queries per step (outer loop, Algorithm 1)
    E: int                   # sequences per perturbed copy (effective batch size)
    S: int                   # sequence length
    steps: int
    eps: float = 1e-3        # perturbation scale
    lr: float = 1e-4         # learning rate
    lora_scale: float = 1.0
    perturb_A: bool = True   # False = LoRA-FA: A frozen and shared, only B perturbed (Section 3)
    norm_eps: float = 1e-5
    rope_theta: float = 10000.0
    label_tokens: Tuple[int, int] = (0, 1)
    weight_quant: str = "none"   # "none" | "int8" | "nf4": weight-only quantisation of the block linears (Appendix D)

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    @property
    def n_copies(self) -> int:
        return 2 * self.q

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.d_head

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    "c1_tiny_fp32": Workload(
        name="c1_tiny_fp32", n_layers=2, d_model=128, n_heads=4, n_kv_heads=4, d_ffn=512, vocab=512,
        max_seq=32, act="gelu", norm="layernorm", pos="learned", has_bias=True, tie_embeddings=True,
        dtype="f32", lora_rank=4, lora_targets=("q", "v"), loss_mode="last_pos_label_subset",
        q=2, E=2, S=32, steps=5, label_tokens=(17, 401)),
    "c2_opt125m": Workload(
        name="c2_opt125m", n_layers=12, d_model=768, n_heads=12, n_kv_heads=12, d_ffn=3072, vocab=50272,
        max_seq=128, act="relu", norm="layernorm", pos="learned", has_bias=True, tie_embeddings=True,
        dtype="bf16", lora_rank=8, lora_targets=("q", "v"), loss_mode="last_pos_label_subset",
        q=4, E=8, S=128, steps=20, label_tokens=(1234, 40321)),
    "c3_opt1p3b": Workload(
        name="c3_opt1p3b", n_layers=24, d_model=2048, n_heads=32, n_kv_heads=32, d_ffn=8192, vocab=50272,
        max_seq=256, act="relu", norm="layernorm", pos="learned", has_bias=True, tie_embeddings=True,
        dtype="bf16", lora_rank=8, lora_targets=("q", "v"), loss_mode="next_token_all_pos",
        q=8, E=8, S=256, steps=1),
    "c4_llama1p1b": Workload(
        name="c4_llama1p1b", n_layers=22, d_model=2048, n_heads=32, n_kv_heads=4, d_ffn=5632, vocab=32000,
        max_seq=512, act="swiglu", norm="rmsnorm", pos="rope", has_bias=False, tie_embeddings=False,
        dtype="bf16", lora_rank=16, lora_targets=("q", "k", "v", "o"), loss_mode="next_token_all_pos",
        q=16, E=4, S=512, steps=1),
    "c5_llama7b": Workload(
        name="c5_llama7b", n_layers=32, d_model=4096, n_heads=32, n_kv_heads=32, d_ffn=11008, vocab=32000,
        max_seq=512, act="swiglu", norm="rmsnorm", pos="rope", has_bias=False, tie_embeddings=False,
        dtype="bf16", lora_rank=16, lora_targets=("q", "v"), loss_mode="last_pos_label_subset",
        q=4, E=2, S=512, steps=1, label_tokens=(3869, 1939)),
}


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


class LoraTensor(NamedTuple):
    layer: int
    target: int        # index into TARGETS
    factor: int        # 0 = A [k_in, r], 1 = B [r, k_out]
    tensor_id: int     # (layer*4 + target)*2 + factor
    offset: int        # element offset in the flat fp32 master vector
    rows: int
    cols: int


def lora_layout(w: Workload) -> List[LoraTensor]:
    """Canonical order of the LoRA factors in the flat master vector.

    Layer-major; inside a layer the targets in the order q, k, v, o (those enabled); for each
    target A [k_in, r] then B [r, k_out], both row-major.
    """
    out: List[LoraTensor] = []
    off = 0
    r = w.lora_rank
    for layer in range(w.n_layers):
        for ti, t in enumerate(TARGETS):
            if t not in w.lora_targets:
                continue
            k_in = w.d_model
            k_out = w.d_model if t in ("q", "o") else w.d_kv
            for factor, (rows, cols) in enumerate(((k_in, r), (r, k_out))):
                out.append(LoraTensor(layer, ti, factor, (layer * 4 + ti) * 2 + factor, off, rows, cols))
                off += rows * cols
    return out
