"""Small variants of the workloads for CPU tests (same structure, reduced sizes)."""
import workloads as W

C1 = W.get_workload("c1_tiny_fp32")

# Llama-style miniature: RMSNorm, rotary positions, grouped-query attention, SwiGLU, untied head,
# adapters on all four projections, next-token loss - every code path of workloads 4 and 5.
MINI_LLAMA = W.Workload(
    name="mini_llama", n_layers=2, d_model=64, n_heads=4, n_kv_heads=2, d_ffn=96, vocab=80, max_seq=12,
    act="swiglu", norm="rmsnorm", pos="rope", has_bias=False, tie_embeddings=False, dtype="f32",
    lora_rank=4, lora_targets=("q", "k", "v", "o"), loss_mode="next_token_all_pos",
    q=3, E=2, S=12, steps=3)

# OPT-style miniature with ReLU and the full-vocabulary last-position loss.
MINI_OPT = W.Workload(
    name="mini_opt", n_layers=2, d_model=48, n_heads=3, n_kv_heads=3, d_ffn=96, vocab=64, max_seq=10,
    act="relu", norm="layernorm", pos="learned", has_bias=True, tie_embeddings=True, dtype="f32",
    lora_rank=4, lora_targets=("q", "v"), loss_mode="last_pos_full_vocab",
    q=2, E=3, S=10, steps=3, label_tokens=(5, 41))

# A one-layer model whose 256 LoRA parameters allow per-parameter finite differences.
MICRO = W.Workload(
    name="micro", n_layers=1, d_model=32, n_heads=2, n_kv_heads=2, d_ffn=64, vocab=64, max_seq=8,
    act="gelu", norm="layernorm", pos="learned", has_bias=True, tie_embeddings=True, dtype="f32",
    lora_rank=2, lora_targets=("q", "v"), loss_mode="last_pos_label_subset",
    q=2, E=2, S=8, steps=3, label_tokens=(3, 50))


def bundle(w, b_std=0.0, wseed=1234, lseed=99, tseed=2345, scale_weights=1.0):
    frozen = W.make_frozen_weights(w, wseed)
    if scale_weights != 1.0:                 # larger weights make attention / nonlinearities matter
        def sc(x):
            return None if x is None else x * scale_weights
        for lw in frozen["layers"]:
            for k in ("w_qkv", "w_o", "w_up", "w_down", "b_qkv", "b_o", "b_up", "b_down"):
                lw[k] = sc(lw[k])
        frozen["emb"] = sc(frozen["emb"])
        if w.tie_embeddings:
            frozen["lm_head"] = frozen["emb"]
        else:
            frozen["lm_head"] = sc(frozen["lm_head"])
        frozen["pos_emb"] = sc(frozen["pos_emb"])
    return dict(w=w, layout=W.lora_layout(w), frozen=frozen,
                masters=W.make_lora_masters(w, lseed, b_std=b_std),
                tokens=W.make_tokens(w, tseed), labels=W.make_labels(w, tseed))
