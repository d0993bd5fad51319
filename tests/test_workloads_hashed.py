"""CPU pins of the integer-hash weight generator (workloads/hashed.py): the hash against an independent big-integer
SplitMix64 finaliser, the level table against the normal quantiles, moments and independence of the values, and the
layouts the two consumers read (the oracle's [k_in, k_out] views of the library's [k_out, k_in] matrices)."""
import numpy as np
import pytest

import workloads as W
from workloads.hashed import hashed_levels, hashed_normal, normal_quantile_table


def _mix64(v):
    m = (1 << 64) - 1
    v &= m
    v ^= v >> 30
    v = (v * 0xBF58476D1CE4E5B9) & m
    v ^= v >> 27
    v = (v * 0x94D049BB133111EB) & m
    v ^= v >> 31
    return v


@pytest.mark.parametrize("i0,tensor_no,seed", [(0, 0, 1234), (10 ** 9, 16 * 31 + 22, 1234), (123456789, 2, 0xDEADBEEF)])
def test_levels_match_a_big_integer_implementation(i0, tensor_no, seed):
    got = hashed_levels(i0, i0 + 500, tensor_no, seed).numpy()
    for k in range(500):
        h = _mix64(i0 + k + (tensor_no << 40) + seed * 0x9E3779B97F4A7C15)
        assert int(got[k]) == (h >> 24) & 0xFFFF


def test_quantile_table_and_distribution():
    from scipy import stats
    q = normal_quantile_table()
    assert q.shape == (65536,) and np.all(np.diff(q) > 0) and abs(q[32768] + q[32767]) < 1e-7     # symmetric, increasing
    assert abs(stats.norm.cdf(q[40000]) - (40000.5 / 65536)) < 1e-7
    x = hashed_normal((1 << 20,), 7, 1234, std=0.02, bf16=False).numpy().astype(np.float64) / 0.02
    assert abs(x.mean()) < 4e-3 and abs(x.std() - 1.0) < 4e-3
    assert stats.kstest(x[:200000], "norm").pvalue > 1e-3
    assert abs(np.corrcoef(x[:-1], x[1:])[0, 1]) < 4e-3
    y = hashed_normal((1 << 20,), 8, 1234, std=0.02, bf16=False).numpy().astype(np.float64) / 0.02
    assert abs(np.corrcoef(x, y)[0, 1]) < 4e-3                                                     # tensors are independent


def test_host_dictionary_holds_the_library_layout_transposed():
    w = W.Workload(name="t", n_layers=2, d_model=64, n_heads=4, n_kv_heads=2, d_ffn=128, vocab=96, max_seq=16, act="swiglu",
                   norm="rmsnorm", pos="rope", has_bias=False, tie_embeddings=False, dtype="bf16", lora_rank=4,
                   lora_targets=("q", "v"), loss_mode="next_token_all_pos", q=1, E=1, S=16, steps=1)
    f = W.make_frozen_weights_hashed(w, 1234)
    lw = f["layers"][1]
    n_qkv = w.d_model + 2 * w.d_kv
    assert lw["w_qkv"].shape == (w.d_model, n_qkv) and lw["w_up"].shape == (w.d_model, 2 * w.d_ffn)
    assert lw["w_down"].shape == (w.d_ffn, w.d_model) and f["emb"].shape == (w.vocab, w.d_model)
    out_major = hashed_normal((n_qkv, w.d_model), 16 * 1 + 16, 1234).numpy()
    assert np.array_equal(lw["w_qkv"], out_major.T)
    assert np.array_equal(W.to_bf16_values(lw["w_o"]), lw["w_o"])                                  # bf16-representable
    assert f["lm_head"] is not f["emb"] and lw["b_qkv"] is None and f["pos_emb"] is None
