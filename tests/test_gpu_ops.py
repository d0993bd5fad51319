"""GPU parity of single operations of the bf16 path against the oracle's sub-routines on identical operands:
the MP-LoRA projection (shared W + per-copy rank-r term) before any rounding, and causal attention."""
import numpy as np
import pytest

import workloads as W
from oracle import zo
from oracle.model import _attention, _linear, _lora_delta
from oracle.precision import Precision
from gpu_helpers import make_bundle, gpu_model
from test_gpu_bf16 import CASES

pytestmark = pytest.mark.gpu
BF = Precision("bf16")


def _bf16_tensor(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda().to(torch.bfloat16).contiguous()


# 32768 stacked tokens: the bottleneck kernel switches to its 64-token blocks (one and two 32-column MFMA tiles)
BIG_T = {"c2_big_T": CASES["c2_2layers"].with_(q=4, E=32), "llama_mfma_big_T": CASES["llama_mfma"].with_(q=4, E=64),
         # a rank that the vectorised packing kernel does not take: the element-wise one writes the same operand layouts
         "c2_rank12": CASES["c2_2layers"].with_(lora_rank=12)}


@pytest.mark.parametrize("name,simple", [("c2_2layers", False), ("llama_mfma", False), ("c2_2layers", True),
                                         ("c2_ragged_copies", False), ("c2_big_T", False), ("llama_mfma_big_T", False),
                                         ("c2_rank12", False)])
def test_qkv_projection_matches_the_mp_lora_layer_equation(name, simple):
    import torch
    import paper_2409_15520_amd as M
    w = (BIG_T[name] if name in BIG_T else CASES[name]).with_(eps=5e-2, n_layers=1)
    b = make_bundle(w, b_std=0.05)
    m = gpu_model(b)
    M.mpz_debug_set_kernel_path(m.handle, simple)
    m.regen_noise(3456, 0)
    T, d, nqkv = 2 * w.q * w.E * w.S, w.d_model, w.d_model + 2 * w.d_kv
    x = BF.operand(np.random.default_rng(5).standard_normal((T, d)))
    xd = _bf16_tensor(x)
    out = torch.empty((T, nqkv), dtype=torch.float32, device="cuda")
    M.mpz_debug_qkv_projection(m.handle, xd.data_ptr(), 0, w.E, w.S, out.data_ptr())
    got = out.cpu().numpy().astype(np.float64)

    lw = b["frozen"]["layers"][0]
    cols = {"q": (0, d), "k": (d, d + w.d_kv), "v": (d + w.d_kv, nqkv)}
    rpc = w.E * w.S
    want = np.empty_like(got)
    lora_part = np.zeros_like(got)
    for k in range(w.q):
        z = zo.draw_z(b["layout"], 3456, 0, k, b["masters"].size, True)
        for s, sign in enumerate((+1, -1)):
            c = 2 * k + s
            lora = zo.split_factors(b["layout"], zo.perturb(b["masters"], z, sign, w.eps, BF))
            xc = x[c * rpc:(c + 1) * rpc]
            for tname, (c0, c1) in cols.items():
                delta = _lora_delta(xc, lora, 0, tname, w.lora_scale, BF)
                bias = lw["b_qkv"][c0:c1] if lw["b_qkv"] is not None else None
                want[c * rpc:(c + 1) * rpc, c0:c1] = _linear(xc, lw["w_qkv"][:, c0:c1], bias, delta)
                if delta is not None:
                    lora_part[c * rpc:(c + 1) * rpc, c0:c1] = delta
    rms = np.sqrt(np.mean(want ** 2))
    err = np.abs(got - want) / rms
    print(f"\n{name} simple={simple}: rms {rms:.3f}, low-rank term rms {np.sqrt(np.mean(lora_part ** 2)):.3f}, "
          f"max err/rms {err.max():.2e}, frac > 2e-5: {np.mean(err > 2e-5):.2e}")
    assert np.sqrt(np.mean(lora_part ** 2)) > 0.03 * rms           # the per-copy term is far above the tolerance
    # fp32 accumulation only; the rare larger deviations are bf16 flips of a bottleneck activation t
    assert np.mean(err > 2e-5) < 2e-3
    assert err.max() < 1e-2        # one flipped t (2^-8 relative) times a low-rank term of ~0.4 rms
    # different copies really get different factors
    assert np.abs(lora_part[:rpc] - lora_part[rpc:2 * rpc]).max() > 0.01 * rms


# S above 256 takes the instance of the head-width-64 kernel that is held to four waves per SIMD
@pytest.mark.parametrize("name,S,simple", [("c2_2layers", 128, False), ("c2_2layers", 100, False), ("llama_mfma", 64, False),
                                           ("llama_mfma", 37, False), ("c2_2layers", 100, True),
                                           ("c2_2layers", 512, False), ("llama_mfma", 300, False)])
def test_attention_matches_oracle_on_the_same_operands(name, S, simple):
    import torch
    import paper_2409_15520_amd as M
    w = CASES[name]
    b = make_bundle(w)
    m = gpu_model(b)
    M.mpz_debug_set_kernel_path(m.handle, simple)
    n_seq, H, Hkv, dh, d = 3, w.n_heads, w.n_kv_heads, w.d_head, w.d_model
    rng = np.random.default_rng(S)
    q = BF.operand(2.0 * rng.standard_normal((n_seq, S, H, dh)))
    k = BF.operand(2.0 * rng.standard_normal((n_seq, S, Hkv, dh)))
    v = BF.operand(rng.standard_normal((n_seq, S, Hkv, dh)))
    qkv = np.concatenate([q.reshape(n_seq * S, -1), k.reshape(n_seq * S, -1), v.reshape(n_seq * S, -1)], axis=1)
    qd = _bf16_tensor(qkv)
    out = torch.empty((n_seq * S, d), dtype=torch.bfloat16, device="cuda")
    M.mpz_debug_attention(m.handle, qd.data_ptr(), n_seq, S, out.data_ptr())
    got = out.float().cpu().numpy().astype(np.float64)
    want = BF.operand(_attention(q, k, v, H, Hkv, BF)).reshape(n_seq * S, d)
    ulp = np.maximum(np.abs(want), 1e-30) * 2.0 ** -7
    bad = np.abs(got - want) > 0
    print(f"\n{name} S={S} simple={simple}: bit-equal {1 - bad.mean():.5f}, max err in ulps {(np.abs(got - want) / ulp).max():.2f}")
    assert bad.mean() < 5e-3                      # rounding flips of P and of the output only
    # an output ulp, plus one flipped probability (2^-8 relative, p <= 1) times the largest |v|
    assert (np.abs(got - want) <= 1.01 * ulp + 2.0 ** -8 * np.abs(v).max()).all()


@pytest.mark.parametrize("cfg", [1, 6, 9, 10, 11, 12])
@pytest.mark.parametrize("M_,N_,K_", [(512, 512, 256), (300, 260, 192), (1024, 768, 64)])
def test_gemm_every_tile_configuration_and_ragged_edges(cfg, M_, N_, K_):
    """x W^T + bias with ReLU, fp32 output, against the fp64 product of the same bf16 operands."""
    import torch
    import paper_2409_15520_amd as M
    rng = np.random.default_rng(cfg * 1000 + M_)
    x = BF.operand(rng.standard_normal((M_, K_)))
    w = BF.operand(0.05 * rng.standard_normal((N_, K_)))
    bias = rng.standard_normal(N_).astype(np.float32)
    xd, wd = _bf16_tensor(x), _bf16_tensor(w)
    bd = torch.from_numpy(bias).cuda()
    out = torch.full((M_, N_), float("nan"), dtype=torch.float32, device="cuda")
    M.mpz_debug_gemm_bf16(M_, N_, K_, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), 0, out.data_ptr(), True,
                          torch.cuda.current_stream().cuda_stream, cfg)
    got = out.cpu().numpy().astype(np.float64)
    want = np.maximum(x @ w.T + bias, 0.0)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= 2e-6 * np.sqrt(K_) * np.abs(want).max()


# shapes whose tile configuration is chosen by the library (0): the 8-wave 128 x 128 tile, the 192 x 128 tile (N = 768
# with a long K), the 256 x 256 tile (512 or more of them), each with ragged edges, plus one row / one tile extremes
@pytest.mark.parametrize("M_,N_,K_,act,bf16_out", [
    (1, 4, 64, -1, False), (33, 68, 128, 1, True), (1000, 772, 320, 0, False), (8192, 768, 1536, -1, True),
    (8190, 764, 1600, 0, False), (8192, 4096, 128, 0, True), (8100, 4100, 192, 1, False), (4096, 8200, 64, -1, True)])
def test_gemm_with_the_tile_chosen_by_shape(M_, N_, K_, act, bf16_out):
    import torch
    import paper_2409_15520_amd as M
    from scipy.special import erf
    rng = np.random.default_rng(M_ * 7 + N_)
    x = BF.operand(rng.standard_normal((M_, K_)))
    w = BF.operand(0.05 * rng.standard_normal((N_, K_)))
    bias = rng.standard_normal(N_).astype(np.float32)
    xd, wd = _bf16_tensor(x), _bf16_tensor(w)
    bd = torch.from_numpy(bias).cuda()
    out = torch.full((M_, N_), float("nan"), dtype=torch.bfloat16 if bf16_out else torch.float32, device="cuda")
    M.mpz_debug_gemm_bf16(M_, N_, K_, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), act, out.data_ptr(), not bf16_out,
                          torch.cuda.current_stream().cuda_stream, 0)
    got = out.float().cpu().numpy().astype(np.float64)
    y = x @ w.T + bias
    want = y if act < 0 else (np.maximum(y, 0.0) if act == 0 else 0.5 * y * (1.0 + erf(y / np.sqrt(2.0))))
    assert np.isfinite(got).all()
    tol = 2e-6 * np.sqrt(K_) * np.abs(want).max()
    if bf16_out:
        assert np.abs(got - want).max() <= tol + 2.0 ** -8 * np.abs(want).max()      # one bf16 rounding of the result
    else:
        assert np.abs(got - want).max() <= tol


@pytest.mark.parametrize("cfg", [1, 6])
def test_swiglu_dual_gemm(cfg):
    import torch
    import paper_2409_15520_amd as M
    M_, F_, K_ = 520, 384, 128
    rng = np.random.default_rng(cfg)
    x = BF.operand(rng.standard_normal((M_, K_)))
    w = BF.operand(0.1 * rng.standard_normal((2 * F_, K_)))
    xd, wd = _bf16_tensor(x), _bf16_tensor(w)
    out = torch.zeros((M_, F_), dtype=torch.bfloat16, device="cuda")
    M.mpz_debug_gemm_bf16(M_, F_, K_, xd.data_ptr(), wd.data_ptr(), None, 2, out.data_ptr(), False,
                          torch.cuda.current_stream().cuda_stream, cfg)
    got = out.float().cpu().numpy().astype(np.float64)
    g, u = x @ w[:F_].T, x @ w[F_:].T
    want = BF.operand(g / (1.0 + np.exp(-g)) * u)
    ulp = np.maximum(np.abs(want), 1e-30) * 2.0 ** -7
    assert np.mean(got != want) < 2e-3 and (np.abs(got - want) <= 1.01 * ulp + 1e-7).all()


@pytest.mark.parametrize("tile_cfg", [0, 1, 6, 9, 11, 12])
@pytest.mark.parametrize("loss_mode", ["next_token_all_pos", "last_pos_full_vocab"])
def test_fused_head_cross_entropy(tile_cfg, loss_mode):
    """LM head with the cross-entropy folded into the GEMM (logits stay in the accumulators, per-tile maximum /
    sum of exponentials combined afterwards), for every wave-tile width, on a vocabulary that ends inside a tile:
    against the oracle's head on the same residual stream."""
    import torch
    import paper_2409_15520_amd as M
    from oracle.model import head_loss
    from oracle.precision import Precision
    w = W.Workload(name="head_ce", n_layers=1, d_model=256, n_heads=4, n_kv_heads=4, d_ffn=512, vocab=1000, max_seq=64,
                   act="relu", norm="layernorm", pos="learned", has_bias=True, tie_embeddings=False, dtype="bf16",
                   lora_rank=8, lora_targets=("q", "v"), loss_mode=loss_mode, label_tokens=(7, 993), q=2, E=3, S=64, steps=1)
    b = make_bundle(w, b_std=0.01)
    m = gpu_model(b)
    M.mpz_debug_set_tile_config(m.handle, tile_cfg)
    m.regen_noise(3456, 0)
    rng = np.random.default_rng(5)
    n = 2 * w.q
    h = (3.0 * rng.standard_normal((n, w.E, w.S, w.d_model))).astype(np.float32)
    tok = torch.from_numpy(b["tokens"]).cuda()
    lab = torch.from_numpy(b["labels"]).cuda()
    got = m.head_loss(torch.from_numpy(h.reshape(-1, w.d_model)).cuda(), tok, lab).cpu().numpy().astype(np.float64)
    prec = Precision("bf16")
    want = np.array([head_loss(w, b["frozen"], h[c].astype(np.float64), b["tokens"], b["labels"], prec) for c in range(n)])
    print(f"\nfused head {loss_mode} cfg {tile_cfg}: {got} vs {want}")
    assert np.abs(got - want).max() <= 2e-5 * np.abs(want).max()


@pytest.mark.parametrize("cfg", [1, 6, 11, 12])
@pytest.mark.parametrize("M_,N_,K_", [(512, 768, 256), (300, 260, 192), (1024, 384, 64)])
def test_gemm_int8_weights(cfg, M_, N_, K_):
    """x (codes * scale)^T + bias with ReLU, fp32 output, against the fp64 product: the codes are widened to bf16
    exactly and the per-output-channel scale multiplies the fp32 accumulator, so only accumulation order differs."""
    import torch
    import paper_2409_15520_amd as M
    rng = np.random.default_rng(cfg * 1000 + M_)
    x = BF.operand(rng.standard_normal((M_, K_)))
    codes = rng.integers(-127, 128, size=(N_, K_), dtype=np.int8)
    scale = (0.02 / 32 * (0.75 + 0.5 * rng.random(N_))).astype(np.float32)
    bias = rng.standard_normal(N_).astype(np.float32)
    xd = _bf16_tensor(x)
    cd, sd, bd = torch.from_numpy(codes).cuda(), torch.from_numpy(scale).cuda(), torch.from_numpy(bias).cuda()
    out = torch.full((M_, N_), float("nan"), dtype=torch.float32, device="cuda")
    M.mpz_debug_gemm_int8(M_, N_, K_, xd.data_ptr(), cd.data_ptr(), sd.data_ptr(), bd.data_ptr(), 0, out.data_ptr(), True,
                          torch.cuda.current_stream().cuda_stream, cfg)
    got = out.cpu().numpy().astype(np.float64)
    want = np.maximum(x @ (codes.astype(np.float64) * scale.astype(np.float64)[:, None]).T + bias, 0.0)
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= 2e-6 * np.sqrt(K_) * np.abs(want).max()


@pytest.mark.parametrize("cfg", [1, 6])
def test_swiglu_dual_gemm_int8_weights(cfg):
    import torch
    import paper_2409_15520_amd as M
    Mr, F, K = 512, 384, 256
    rng = np.random.default_rng(cfg + 40)
    x = BF.operand(rng.standard_normal((Mr, K)))
    codes = rng.integers(-127, 128, size=(2 * F, K), dtype=np.int8)
    scale = (0.05 / 32 * (0.75 + 0.5 * rng.random(2 * F))).astype(np.float32)
    xd = _bf16_tensor(x)
    cd, sd = torch.from_numpy(codes).cuda(), torch.from_numpy(scale).cuda()
    out = torch.full((Mr, F), float("nan"), dtype=torch.float32, device="cuda")
    M.mpz_debug_gemm_int8(Mr, F, K, xd.data_ptr(), cd.data_ptr(), sd.data_ptr(), None, 2, out.data_ptr(), True,
                          torch.cuda.current_stream().cuda_stream, cfg)
    got = out.cpu().numpy().astype(np.float64)
    wd = codes.astype(np.float64) * scale.astype(np.float64)[:, None]
    gate, up = x @ wd[:F].T, x @ wd[F:].T
    want = gate / (1.0 + np.exp(-gate)) * up
    assert np.abs(got - want).max() <= 1e-5 * np.abs(want).max()


@pytest.mark.parametrize("rows,K_", [(1, 64), (3, 192), (257, 4096), (1000, 768)])
def test_nf4_dequantisation_is_bit_exact(rows, K_):
    """level[code] * block maximum in binary32, rounded to bf16: the same bits as the oracle's dequantisation (sizes
    from one block to several thread blocks with a ragged tail; every code occurs)."""
    import torch
    import paper_2409_15520_amd as M
    from oracle.model import nf4_dequant
    rng = np.random.default_rng(rows * 7 + K_)
    codes = rng.integers(0, 16, size=(K_, rows), dtype=np.uint8)                   # oracle layout [k_in, k_out]
    codes[:16, 0] = np.arange(16)
    absmax = (0.048 * (0.5 + rng.random((K_ // 64, rows)))).astype(np.float32)
    want = BF.operand(nf4_dequant(codes, absmax)).T                                # [k_out, k_in]
    packed = M.pack_nf4_codes(np.ascontiguousarray(codes.T))
    assert packed.shape == (rows, K_ // 2) and packed.dtype == np.uint8
    cd = torch.from_numpy(np.ascontiguousarray(packed)).cuda()
    ad = torch.from_numpy(np.ascontiguousarray(absmax.T)).cuda()
    out = torch.full((rows, K_), float("nan"), dtype=torch.bfloat16, device="cuda")
    M.mpz_debug_dequant_nf4(cd.data_ptr(), ad.data_ptr(), out.data_ptr(), rows * K_, torch.cuda.current_stream().cuda_stream)
    got = out.float().cpu().numpy().astype(np.float64)
    assert np.array_equal(got, want)


# Split K (passes over at most 256 stacked tokens): k_splits blocks per output tile, fp32 partial sums, reduction kernel
# with the epilogue.  Shapes: the 7B-shaped projections at 64 / 128 tokens, ragged M and N, every tile the path picks
# (M <= 64: 128 x 64; M <= 128: 64 x 128; else 128 x 128), forced and chosen split counts.
@pytest.mark.parametrize("M_,N_,K_,act,resid,bf16_out,ks", [
    (128, 4096, 4096, -1, True, False, 0), (64, 12288, 4096, -1, False, True, 0), (128, 4096, 11008, -1, True, False, 0),
    (64, 768, 3072, 0, False, True, 4), (200, 1028, 2048, 1, True, False, 3), (33, 260, 1024, 0, True, True, 2),
    (256, 2048, 2048, -1, False, False, 0), (100, 516, 1536, -1, False, False, 24)])
def test_gemm_split_k(M_, N_, K_, act, resid, bf16_out, ks):
    import torch
    import paper_2409_15520_amd as M
    from scipy.special import erf
    rng = np.random.default_rng(M_ * 7 + N_ + ks)
    x = BF.operand(rng.standard_normal((M_, K_)))
    w = BF.operand(0.05 * rng.standard_normal((N_, K_)))
    bias = rng.standard_normal(N_).astype(np.float32)
    res = rng.standard_normal((M_, N_)).astype(np.float32) if resid else None
    xd, wd = _bf16_tensor(x), _bf16_tensor(w)
    bd = torch.from_numpy(bias).cuda()
    rd = torch.from_numpy(res).cuda() if resid else None
    cap = 64 * M_ * N_
    chosen = M.mpz_debug_gemm_splits(M_, N_, K_, False, cap)
    if ks == 0:
        assert chosen >= 2, "these shapes are meant to take the split-K path on their own"
    part = torch.full((cap,), float("nan"), dtype=torch.float32, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    outs = []
    for split in (True, False):
        out = torch.full((M_, N_), float("nan"), dtype=torch.bfloat16 if bf16_out else torch.float32, device="cuda")
        if split:
            M.mpz_debug_gemm_bf16_splitk(M_, N_, K_, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), act,
                                         rd.data_ptr() if resid else None, out.data_ptr(), not bf16_out, ks, part.data_ptr(), cap, st)
        else:                                      # the one-block kernel (no residual argument on this hook: added below)
            M.mpz_debug_gemm_bf16(M_, N_, K_, xd.data_ptr(), wd.data_ptr(), bd.data_ptr(), act, out.data_ptr(), not bf16_out, st, 0)
        outs.append(out.float().cpu().numpy().astype(np.float64))
    y = x @ w.T + bias
    y = np.maximum(y, 0.0) if act == 0 else (0.5 * y * (1.0 + erf(y / np.sqrt(2.0))) if act == 1 else y)
    want = y + (res if resid else 0.0)
    got = outs[0]
    assert np.isfinite(got).all()
    tol = 2e-6 * np.sqrt(K_) * np.abs(want).max()
    if bf16_out:
        assert np.abs(got - want).max() <= tol + 2.0 ** -8 * np.abs(want).max()
    else:
        assert np.abs(got - want).max() <= tol
        # against the one-block kernel: the same products summed in another order
        one = outs[1] + (res if resid else 0.0)
        assert np.abs(got - one).max() <= 4e-6 * np.abs(want).max()


@pytest.mark.parametrize("M_,ks", [(128, 0), (64, 4), (256, 2)])
def test_swiglu_dual_gemm_split_k(M_, ks):
    import torch
    import paper_2409_15520_amd as M
    F_, K_ = 1408, 2048
    rng = np.random.default_rng(M_ + ks)
    x = BF.operand(rng.standard_normal((M_, K_)))
    w = BF.operand(0.03 * rng.standard_normal((2 * F_, K_)))
    xd, wd = _bf16_tensor(x), _bf16_tensor(w)
    cap = 16 * M_ * 2 * F_
    if ks == 0:
        assert M.mpz_debug_gemm_splits(M_, F_, K_, True, cap) >= 2
    part = torch.full((cap,), float("nan"), dtype=torch.float32, device="cuda")
    out = torch.zeros((M_, F_), dtype=torch.bfloat16, device="cuda")
    M.mpz_debug_gemm_bf16_splitk(M_, F_, K_, xd.data_ptr(), wd.data_ptr(), None, 2, None, out.data_ptr(), False, ks,
                                 part.data_ptr(), cap, torch.cuda.current_stream().cuda_stream)
    got = out.float().cpu().numpy().astype(np.float64)
    g, u = x @ w[:F_].T, x @ w[F_:].T
    want = BF.operand(g / (1.0 + np.exp(-g)) * u)
    ulp = np.maximum(np.abs(want), 1e-30) * 2.0 ** -7
    # one bf16 rounding, plus the fp32 summation error of a K = 2048 gate (about 3e-6 absolute) carried through
    # SiLU'(g) u where the gate nearly cancels
    assert np.mean(got != want) < 2e-3 and (np.abs(got - want) <= 1.01 * ulp + 1e-5 * (1.0 + np.abs(u))).all()


@pytest.mark.parametrize("rb,seg,ks,mode", [(128, 128, 2, 0), (128, 128, 4, 3), (64, 256, 1, 1), (1, 4096, 2, 0), (32, 512, 2, 2)])
def test_read_probe_reads_its_own_tiles(rb, seg, ks, mode):
    """mpz_debug_hbm_read_probe (measurement hook): thread 0 of block (x, y) leaves the XOR of the 16-byte pieces it
    fetched: pieces 0, 256, 512, ... of every tile of rows [x rb, (x + 1) rb) and of share y of the row (plus, with mode
    bit 0, the same pieces of rows [0, rb)).  The host recomputes that from the buffer: the kernel reads what its
    description says, in bounds, every tile once."""
    import torch
    import paper_2409_15520_amd as M
    rows, row_bytes = 512 if rb > 1 else 8, 8192
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    buf = torch.randint(0, 2 ** 31 - 1, (rows * row_bytes // 4,), dtype=torch.int32, device="cuda", generator=g)
    nbx = rows // rb
    out = torch.zeros(nbx * ks, dtype=torch.int32, device="cuda")
    lds = (2 if mode & 1 else 1) * rb * seg if mode & 2 else 0
    M.mpz_debug_hbm_read_probe(buf.data_ptr(), rows, row_bytes, rb, seg, ks, lds, mode, out.data_ptr(),
                               torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    host = buf.cpu().numpy().view(np.uint32).reshape(rows, row_bytes // 16, 4)
    segc, L = seg // 16, rb * seg // 4096
    tiles = row_bytes // seg // ks
    want = np.zeros(nbx * ks, dtype=np.uint32)
    for y in range(ks):
        for x in range(nbx):
            acc = np.zeros(4, dtype=np.uint32)
            for t in range(tiles):
                for i in range(L):
                    c = 256 * i                                   # thread 0's pieces of a tile
                    r, col = c // segc, (y * tiles + t) * segc + c % segc
                    if mode & 2:                                  # through LDS: thread 0 reads back pieces (256 i) % (256 L) = 256 i
                        pass
                    acc ^= host[x * rb + r, col]
                    if mode & 1:
                        acc ^= host[r, col]
            want[y * nbx + x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3]
    got = out.cpu().numpy().view(np.uint32)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("M_,N_,K_,act,resid,ks", [(128, 512, 1024, -1, False, 2), (64, 388, 2048, -1, True, 4),
                                                   (128, 256, 1024, 2, False, 2), (100, 132, 4096, 0, False, 8),
                                                   (256, 4096, 4096, -1, True, 3)])
def test_gemm_nf4_codes_in_the_operand_load(M_, N_, K_, act, resid, ks):
    """Passes over few tokens read 4-bit weights as codes inside the split-K GEMM (looked up and scaled on the way into
    LDS) instead of from a dequantised bf16 buffer.  Same weights bf16(level[code] * max), same K order: the output has
    the bits of mpz_debug_dequant_nf4 followed by the bf16 split-K GEMM with the same split count and tile - for plain,
    residual, ReLU and stacked gate / up (SwiGLU) launches, whole and ragged tiles, token counts on both tile heights."""
    import torch
    import paper_2409_15520_amd as M
    st = torch.cuda.current_stream().cuda_stream
    g = torch.Generator(device="cuda")
    g.manual_seed(M_ * 31 + N_)
    rows = 2 * N_ if act == 2 else N_
    codes = torch.randint(0, 256, (rows, K_ // 2), dtype=torch.uint8, device="cuda", generator=g)
    absmax = (0.048 * (0.5 + torch.rand(rows, K_ // 64, device="cuda", generator=g))).float().contiguous()
    x = torch.randn(M_, K_, device="cuda", generator=g).to(torch.bfloat16)
    res = torch.randn(M_, N_, device="cuda", generator=g).float() if resid else None
    w = torch.empty(rows, K_, dtype=torch.bfloat16, device="cuda")
    M.mpz_debug_dequant_nf4(codes.data_ptr(), absmax.data_ptr(), w.data_ptr(), rows * K_, st)
    cap = ks * M_ * rows
    part = torch.empty(cap, dtype=torch.float32, device="cuda")
    outs = []
    for which in ("codes", "dense"):
        out = torch.full((M_, N_), float("nan"), dtype=torch.float32 if resid else torch.bfloat16, device="cuda")
        rp = res.data_ptr() if resid else None
        if which == "codes":
            M.mpz_debug_gemm_nf4_splitk(M_, N_, K_, x.data_ptr(), codes.data_ptr(), absmax.data_ptr(), None, act, rp,
                                        out.data_ptr(), resid, ks, part.data_ptr(), cap, st)
        else:
            tile = 9 if M_ <= 64 else 1                     # the tile the code path uses (128 features x 64 / 128 tokens)
            M.mpz_debug_gemm_bf16_splitk(M_, N_, K_, x.data_ptr(), w.data_ptr(), None, act, rp, out.data_ptr(), resid,
                                         ks + 1000 * tile, part.data_ptr(), cap, st)
        torch.cuda.synchronize()
        outs.append(out.float().cpu().numpy())
    assert np.isfinite(outs[0]).all()
    assert np.array_equal(outs[0].view(np.uint32), outs[1].view(np.uint32))
    # and it is the product: fp64 reference on the dequantised weights (tolerance: fp32 accumulation + one bf16 rounding)
    wd = w.float().cpu().numpy().astype(np.float64)
    xd = x.float().cpu().numpy().astype(np.float64)
    ref = xd @ wd[:N_].T
    if act == 2:
        up = xd @ wd[N_:].T
        ref = ref / (1.0 + np.exp(-ref)) * up
    elif act == 0:
        ref = np.maximum(ref, 0.0)
    if resid:
        ref = ref + res.cpu().numpy().astype(np.float64)
    tol = 1e-5 if resid else 1.0 / 128
    assert np.abs(outs[0] - ref).max() <= tol * (1.0 + np.abs(ref).max())
