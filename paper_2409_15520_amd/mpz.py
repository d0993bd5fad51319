"""ctypes binding of libmpz.so: argument marshalling only, every step runs in the HIP kernels.

PyTorch is used for device memory and the stream handle.  The library is loaded from this
package directory; if it has not been built (`python -m paper_2409_15520_amd.build`) loading
raises - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# MPZ_LIBRARY names another build of the same library (e.g. the host-sanitised one of build.py --sanitize-host)
_LIB_PATH = os.environ.get("MPZ_LIBRARY") or os.path.join(_PKG, "libmpz.so")
_lib = None

ACT = {"relu": 0, "gelu": 1, "swiglu": 2}
NORM = {"layernorm": 0, "rmsnorm": 1}
POS = {"learned": 0, "rope": 1}
DTYPE = {"f32": 0, "bf16": 1}
LOSS = {"last_pos_label_subset": 0, "last_pos_full_vocab": 1, "next_token_all_pos": 2}
TARGET_BIT = {"q": 1, "k": 2, "v": 4, "o": 8}


class MpzError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{mpz_status_string(status)}: {message}")
        self.status = status


class MpzConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("max_seq", C.c_int32),
                ("act", C.c_int32), ("norm", C.c_int32), ("norm_eps", C.c_float), ("pos", C.c_int32),
                ("rope_theta", C.c_float), ("has_bias", C.c_int32), ("dtype", C.c_int32),
                ("lora_rank", C.c_int32), ("lora_targets", C.c_uint32), ("lora_scale", C.c_float),
                ("perturb_A", C.c_int32), ("loss_mode", C.c_int32), ("label_token", C.c_int32 * 2),
                ("weight_quant", C.c_int32)]


class MpzLayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
                                          "w_up", "b_up", "w_down", "b_down", "s_qkv", "s_o", "s_up", "s_down")]


class MpzWeights(C.Structure):
    _fields_ = [("emb", C.c_void_p), ("pos_emb", C.c_void_p), ("lm_head", C.c_void_p), ("lnf_g", C.c_void_p),
                ("lnf_b", C.c_void_p), ("layers", C.POINTER(MpzLayerWeights))]


PROF_CATEGORIES = ("gemm", "attention", "norm", "lora_down", "noise", "update", "embed", "rope", "loss", "other", "pack")


class MpzProfileEntry(C.Structure):
    _fields_ = [("ms", C.c_double), ("launches", C.c_int64), ("flops", C.c_double), ("bytes", C.c_double)]


class MpzLoraTensor(C.Structure):
    _fields_ = [("layer", C.c_int32), ("target", C.c_int32), ("factor", C.c_int32), ("tensor_id", C.c_int32),
                ("offset", C.c_int64), ("rows", C.c_int32), ("cols", C.c_int32)]


def load_library() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2409_15520_amd.build` "
                          "(there is no fallback implementation)")
    lib = C.CDLL(_LIB_PATH)
    cfgp = C.POINTER(MpzConfig)
    lib.mpz_lora_numel.restype = C.c_size_t
    lib.mpz_lora_numel.argtypes = [cfgp]
    lib.mpz_lora_tensor_count.restype = C.c_int32
    lib.mpz_lora_tensor_count.argtypes = [cfgp]
    lib.mpz_lora_tensor_info.restype = C.c_int
    lib.mpz_lora_tensor_info.argtypes = [cfgp, C.c_int32, C.POINTER(MpzLoraTensor)]
    lib.mpz_workspace_bytes.restype = C.c_size_t
    lib.mpz_workspace_bytes.argtypes = [cfgp, C.c_int32, C.c_int32, C.c_int32]
    lib.mpz_init_model.restype = C.c_int
    lib.mpz_init_model.argtypes = [cfgp, C.POINTER(MpzWeights), C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32,
                                   C.c_int32, C.c_int32, C.c_void_p, C.POINTER(C.c_void_p)]
    lib.mpz_regen_noise.restype = C.c_int
    lib.mpz_regen_noise.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32, C.c_float]
    lib.mpz_forward_perturbed.restype = C.c_int
    lib.mpz_forward_perturbed.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.mpz_forward_perturbed_varlen.restype = C.c_int
    lib.mpz_forward_perturbed_varlen.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                                 C.c_void_p]
    lib.mpz_forward_copies.restype = C.c_int
    lib.mpz_forward_copies.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                       C.c_void_p]
    lib.mpz_zo_update.restype = C.c_int
    lib.mpz_zo_update.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_void_p]
    lib.mpz_zo_update_regen.restype = C.c_int
    lib.mpz_zo_update_regen.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_uint32, C.c_void_p]
    lib.mpz_debug_noise.restype = C.c_int
    lib.mpz_debug_noise.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32, C.c_int32, C.c_void_p]
    lib.mpz_debug_normals_from_words.restype = C.c_int
    lib.mpz_debug_normals_from_words.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.mpz_debug_perturbed_copy.restype = C.c_int
    lib.mpz_debug_perturbed_copy.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    lib.mpz_debug_embed.restype = C.c_int
    lib.mpz_debug_embed.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.mpz_debug_run_layers.restype = C.c_int
    lib.mpz_debug_run_layers.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32]
    lib.mpz_debug_head_loss.restype = C.c_int
    lib.mpz_debug_head_loss.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                        C.c_void_p]
    lib.mpz_debug_qkv_projection.restype = C.c_int
    lib.mpz_debug_qkv_projection.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
    lib.mpz_debug_attention.restype = C.c_int
    lib.mpz_debug_attention.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.mpz_debug_gemm_bf16.restype = C.c_int
    lib.mpz_debug_gemm_bf16.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.mpz_debug_set_tile_config.restype = C.c_int
    lib.mpz_debug_set_tile_config.argtypes = [C.c_void_p, C.c_int32]
    lib.mpz_debug_set_kernel_path.restype = C.c_int
    lib.mpz_debug_set_kernel_path.argtypes = [C.c_void_p, C.c_int32]
    lib.mpz_profile_begin.restype = C.c_int
    lib.mpz_profile_begin.argtypes = [C.c_void_p]
    lib.mpz_profile_end.restype = C.c_int
    lib.mpz_profile_end.argtypes = [C.c_void_p, C.POINTER(MpzProfileEntry)]
    lib.mpz_destroy.restype = None
    lib.mpz_destroy.argtypes = [C.c_void_p]
    lib.mpz_last_error.restype = C.c_char_p
    lib.mpz_last_error.argtypes = [C.c_void_p]
    lib.mpz_status_string.restype = C.c_char_p
    lib.mpz_status_string.argtypes = [C.c_int]
    _lib = lib
    return lib


def _check(status: int, handle=None):
    if status != 0:
        raise MpzError(status, mpz_last_error(handle))


# ---- the C entry points under their own names ----------------------------------------------------
def mpz_status_string(status: int) -> str:
    return load_library().mpz_status_string(int(status)).decode()


def mpz_last_error(handle=None) -> str:
    return load_library().mpz_last_error(handle).decode()


def mpz_lora_numel(cfg: MpzConfig) -> int:
    return int(load_library().mpz_lora_numel(C.byref(cfg)))


def mpz_lora_tensor_count(cfg: MpzConfig) -> int:
    return int(load_library().mpz_lora_tensor_count(C.byref(cfg)))


def mpz_lora_tensor_info(cfg: MpzConfig, i: int) -> MpzLoraTensor:
    out = MpzLoraTensor()
    _check(load_library().mpz_lora_tensor_info(C.byref(cfg), i, C.byref(out)))
    return out


def mpz_workspace_bytes(cfg: MpzConfig, q_max: int, E_max: int, S_max: int) -> int:
    return int(load_library().mpz_workspace_bytes(C.byref(cfg), q_max, E_max, S_max))


def mpz_init_model(cfg: MpzConfig, weights: MpzWeights, lora_masters_ptr: int, workspace_ptr: int,
                   workspace_bytes: int, q_max: int, E_max: int, S_max: int, stream_ptr: int):
    handle = C.c_void_p()
    _check(load_library().mpz_init_model(C.byref(cfg), C.byref(weights), lora_masters_ptr, workspace_ptr,
                                         workspace_bytes, q_max, E_max, S_max, stream_ptr, C.byref(handle)))
    return handle


def mpz_regen_noise(handle, seed: int, step: int, q: int, eps: float):
    _check(load_library().mpz_regen_noise(handle, seed, step, q, eps), handle)


def mpz_forward_perturbed(handle, tokens_ptr: int, labels_ptr: Optional[int], E: int, S: int, losses_ptr: int):
    _check(load_library().mpz_forward_perturbed(handle, tokens_ptr, labels_ptr, E, S, losses_ptr), handle)


def mpz_forward_perturbed_noalloc(handle, tokens_ptr: int, labels_ptr: Optional[int], E: int, S: int, losses_ptr: int):
    lib = load_library()
    lib.mpz_forward_perturbed_noalloc.restype = C.c_int
    lib.mpz_forward_perturbed_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    _check(lib.mpz_forward_perturbed_noalloc(handle, tokens_ptr, labels_ptr, E, S, losses_ptr), handle)


def mpz_noalloc_scratch_bytes() -> int:
    lib = load_library()
    lib.mpz_noalloc_scratch_bytes.restype = C.c_size_t
    lib.mpz_noalloc_scratch_bytes.argtypes = []
    return int(lib.mpz_noalloc_scratch_bytes())


def mpz_forward_perturbed_varlen(handle, tokens_ptr: int, labels_ptr: Optional[int], lengths_ptr: int, E: int, S: int,
                                 losses_ptr: int):
    _check(load_library().mpz_forward_perturbed_varlen(handle, tokens_ptr, labels_ptr, lengths_ptr, E, S, losses_ptr),
           handle)


def mpz_forward_copies_strided(handle, tokens_ptr: int, labels_ptr: Optional[int], E: int, S: int, copy_begin: int,
                               n_copies: int, copy_step: int, losses_ptr: int):
    lib = load_library()
    lib.mpz_forward_copies_strided.restype = C.c_int
    lib.mpz_forward_copies_strided.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                               C.c_int32, C.c_int32, C.c_void_p]
    _check(lib.mpz_forward_copies_strided(handle, tokens_ptr, labels_ptr, E, S, copy_begin, n_copies, copy_step, losses_ptr),
           handle)


def mpz_forward_perturbed_packed(handle, tokens_ptr: int, labels_ptr: Optional[int], cu_ptr: int, E: int,
                                 total_tokens: int, max_len: int, losses_ptr: int):
    lib = load_library()
    lib.mpz_forward_perturbed_packed.restype = C.c_int
    lib.mpz_forward_perturbed_packed.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                                                 C.c_int32, C.c_void_p]
    _check(lib.mpz_forward_perturbed_packed(handle, tokens_ptr, labels_ptr, cu_ptr, E, total_tokens, max_len, losses_ptr),
           handle)


def mpz_forward_copies(handle, tokens_ptr: int, labels_ptr: Optional[int], E: int, S: int, copy_begin: int,
                       n_copies: int, losses_ptr: int):
    _check(load_library().mpz_forward_copies(handle, tokens_ptr, labels_ptr, E, S, copy_begin, n_copies, losses_ptr),
           handle)


def mpz_zo_update(handle, losses_ptr: int, lr: float, proj_grads_ptr: Optional[int]):
    _check(load_library().mpz_zo_update(handle, losses_ptr, lr, proj_grads_ptr), handle)


def mpz_zo_update_regen(handle, losses_ptr: int, lr: float, next_step: int, proj_grads_ptr: Optional[int]):
    _check(load_library().mpz_zo_update_regen(handle, losses_ptr, lr, next_step, proj_grads_ptr), handle)


def mpz_debug_noise(handle, seed: int, step: int, k: int, tensor_id: int, z_ptr: int):
    _check(load_library().mpz_debug_noise(handle, seed, step, k, tensor_id, z_ptr), handle)


def mpz_debug_normals_from_words(words_ptr: int, n4: int, out_ptr: int, stream_ptr: int):
    _check(load_library().mpz_debug_normals_from_words(words_ptr, n4, out_ptr, stream_ptr))


def mpz_debug_perturbed_copy(handle, c: int, out_ptr: int):
    _check(load_library().mpz_debug_perturbed_copy(handle, c, out_ptr), handle)


def mpz_debug_embed(handle, tokens_ptr: int, E: int, S: int, h_ptr: int):
    _check(load_library().mpz_debug_embed(handle, tokens_ptr, E, S, h_ptr), handle)


def mpz_debug_run_layers(handle, h_ptr: int, layer_begin: int, layer_end: int, E: int, S: int):
    _check(load_library().mpz_debug_run_layers(handle, h_ptr, layer_begin, layer_end, E, S), handle)


def mpz_debug_head_loss(handle, h_ptr: int, tokens_ptr: int, labels_ptr: Optional[int], lengths_ptr: Optional[int], E: int,
                        S: int, losses_ptr: int):
    _check(load_library().mpz_debug_head_loss(handle, h_ptr, tokens_ptr, labels_ptr, lengths_ptr, E, S, losses_ptr), handle)


def mpz_debug_qkv_projection(handle, x_ptr: int, layer: int, E: int, S: int, out_ptr: int):
    _check(load_library().mpz_debug_qkv_projection(handle, x_ptr, layer, E, S, out_ptr), handle)


def mpz_debug_attention(handle, qkv_ptr: int, n_seq: int, S: int, out_ptr: int):
    _check(load_library().mpz_debug_attention(handle, qkv_ptr, n_seq, S, out_ptr), handle)


def mpz_debug_gemm_bf16(M: int, N: int, K: int, x_ptr: int, w_ptr: int, bias_ptr: Optional[int], act: int, out_ptr: int,
                        out_f32: bool, stream_ptr: int, tile_cfg: int = 0):
    _check(load_library().mpz_debug_gemm_bf16(M, N, K, x_ptr, w_ptr, bias_ptr, act, out_ptr, int(out_f32), tile_cfg,
                                              stream_ptr))


def mpz_debug_gemm_bf16_splitk(M: int, N: int, K: int, x_ptr: int, w_ptr: int, bias_ptr: Optional[int], act: int,
                               residual_ptr: Optional[int], out_ptr: int, out_f32: bool, k_splits: int, partial_ptr: int,
                               partial_elems: int, stream_ptr: int):
    lib = load_library()
    lib.mpz_debug_gemm_bf16_splitk.restype = C.c_int
    lib.mpz_debug_gemm_bf16_splitk.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                               C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
    _check(lib.mpz_debug_gemm_bf16_splitk(M, N, K, x_ptr, w_ptr, bias_ptr, act, residual_ptr, out_ptr, int(out_f32), k_splits,
                                          partial_ptr, partial_elems, stream_ptr))


def mpz_debug_gemm_nf4_splitk(M: int, N: int, K: int, x_ptr: int, codes_ptr: int, absmax_ptr: int, bias_ptr: Optional[int],
                              act: int, residual_ptr: Optional[int], out_ptr: int, out_f32: bool, k_splits: int,
                              partial_ptr: int, partial_elems: int, stream_ptr: int):
    lib = load_library()
    lib.mpz_debug_gemm_nf4_splitk.restype = C.c_int
    lib.mpz_debug_gemm_nf4_splitk.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_int32, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t,
                                              C.c_void_p]
    _check(lib.mpz_debug_gemm_nf4_splitk(M, N, K, x_ptr, codes_ptr, absmax_ptr, bias_ptr, act, residual_ptr, out_ptr,
                                         int(out_f32), k_splits, partial_ptr, partial_elems, stream_ptr))


def mpz_debug_gemm_splits(M: int, N: int, K: int, dual: bool, partial_elems: int) -> int:
    lib = load_library()
    lib.mpz_debug_gemm_splits.restype = C.c_int32
    lib.mpz_debug_gemm_splits.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_size_t]
    return int(lib.mpz_debug_gemm_splits(M, N, K, int(dual), partial_elems))


def mpz_debug_set_split_k(handle, enable: bool):
    lib = load_library()
    lib.mpz_debug_set_split_k.restype = C.c_int
    lib.mpz_debug_set_split_k.argtypes = [C.c_void_p, C.c_int32]
    _check(lib.mpz_debug_set_split_k(handle, int(enable)), handle)


def mpz_debug_gemm_int8(M: int, N: int, K: int, x_ptr: int, w_ptr: int, scale_ptr: int, bias_ptr: Optional[int], act: int,
                        out_ptr: int, out_f32: bool, stream_ptr: int, tile_cfg: int = 0):
    lib = load_library()
    lib.mpz_debug_gemm_int8.restype = C.c_int
    lib.mpz_debug_gemm_int8.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    _check(lib.mpz_debug_gemm_int8(M, N, K, x_ptr, w_ptr, scale_ptr, bias_ptr, act, out_ptr, int(out_f32), tile_cfg,
                                   stream_ptr))


def mpz_debug_mfma_probe(operands_ptr: int, blocks: int, iters: int, with_lds: int, out_ptr: int, stream_ptr: int):
    lib = load_library()
    lib.mpz_debug_mfma_probe.restype = C.c_int
    lib.mpz_debug_mfma_probe.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    _check(lib.mpz_debug_mfma_probe(operands_ptr, blocks, iters, int(with_lds), out_ptr, stream_ptr))


def mpz_debug_hbm_read_probe(buf_ptr: int, rows: int, row_bytes: int, rows_per_block: int, seg_bytes: int, k_splits: int,
                             lds_bytes: int, mode: int, out_ptr: int, stream_ptr: int):
    lib = load_library()
    lib.mpz_debug_hbm_read_probe.restype = C.c_int
    lib.mpz_debug_hbm_read_probe.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_int32, C.c_void_p, C.c_void_p]
    _check(lib.mpz_debug_hbm_read_probe(buf_ptr, rows, row_bytes, rows_per_block, seg_bytes, k_splits, lds_bytes, mode,
                                        out_ptr, stream_ptr))


def mpz_debug_dequant_nf4(codes_ptr: int, absmax_ptr: int, out_ptr: int, n_elems: int, stream_ptr: int):
    lib = load_library()
    lib.mpz_debug_dequant_nf4.restype = C.c_int
    lib.mpz_debug_dequant_nf4.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    _check(lib.mpz_debug_dequant_nf4(codes_ptr, absmax_ptr, out_ptr, n_elems, stream_ptr))


def pack_nf4_codes(codes):
    """Codes 0..15, one per byte, [rows, k_in] (a torch or numpy uint8 array) -> two per byte [rows, k_in / 2]: element
    2j of a row in the low nibble of byte j, element 2j + 1 in the high nibble (the library's layout)."""
    return codes[..., 0::2] | (codes[..., 1::2] << 4)


def mpz_debug_noise_alu_probe(n_groups: int, q: int, sink_ptr: int, stream_ptr: int):
    lib = load_library()
    lib.mpz_debug_noise_alu_probe.restype = C.c_int
    lib.mpz_debug_noise_alu_probe.argtypes = [C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    _check(lib.mpz_debug_noise_alu_probe(n_groups, q, sink_ptr, stream_ptr))


def mpz_debug_set_fused_norm_lora(handle, enable: bool):
    lib = load_library()
    lib.mpz_debug_set_fused_norm_lora.restype = C.c_int
    lib.mpz_debug_set_fused_norm_lora.argtypes = [C.c_void_p, C.c_int32]
    _check(lib.mpz_debug_set_fused_norm_lora(handle, int(enable)), handle)


def mpz_debug_set_fused_perturb_pack(handle, enable: bool):
    lib = load_library()
    lib.mpz_debug_set_fused_perturb_pack.restype = C.c_int
    lib.mpz_debug_set_fused_perturb_pack.argtypes = [C.c_void_p, C.c_int32]
    _check(lib.mpz_debug_set_fused_perturb_pack(handle, int(enable)), handle)


def mpz_debug_set_two_halves(handle, enable: bool):
    lib = load_library()
    lib.mpz_debug_set_two_halves.restype = C.c_int
    lib.mpz_debug_set_two_halves.argtypes = [C.c_void_p, C.c_int32]
    _check(lib.mpz_debug_set_two_halves(handle, int(enable)), handle)


def mpz_debug_last_pass_streams(handle) -> int:
    lib = load_library()
    lib.mpz_debug_last_pass_streams.restype = C.c_int32
    lib.mpz_debug_last_pass_streams.argtypes = [C.c_void_p]
    return int(lib.mpz_debug_last_pass_streams(handle))


def mpz_debug_set_tile_config(handle, tile_cfg: int):
    _check(load_library().mpz_debug_set_tile_config(handle, tile_cfg), handle)


def mpz_debug_set_kernel_path(handle, simple_only: bool):
    _check(load_library().mpz_debug_set_kernel_path(handle, int(simple_only)), handle)


def mpz_profile_begin(handle):
    _check(load_library().mpz_profile_begin(handle), handle)


def mpz_profile_end(handle):
    """Returns {category: dict(ms, launches, flops, bytes)} since mpz_profile_begin."""
    arr = (MpzProfileEntry * len(PROF_CATEGORIES))()
    _check(load_library().mpz_profile_end(handle, arr), handle)
    return {name: dict(ms=arr[i].ms, launches=arr[i].launches, flops=arr[i].flops, bytes=arr[i].bytes)
            for i, name in enumerate(PROF_CATEGORIES)}


def mpz_destroy(handle):
    load_library().mpz_destroy(handle)


# ---- marshalling helpers ---------------------------------------------------------------------------
def config_from_workload(w) -> MpzConfig:
    cfg = MpzConfig()
    cfg.struct_size = C.sizeof(MpzConfig)
    cfg.n_layers, cfg.d_model, cfg.n_heads, cfg.n_kv_heads = w.n_layers, w.d_model, w.n_heads, w.n_kv_heads
    cfg.d_ffn, cfg.vocab, cfg.max_seq = w.d_ffn, w.vocab, w.max_seq
    cfg.act, cfg.norm, cfg.norm_eps, cfg.pos = ACT[w.act], NORM[w.norm], w.norm_eps, POS[w.pos]
    cfg.rope_theta, cfg.has_bias, cfg.dtype = w.rope_theta, int(w.has_bias), DTYPE[w.dtype]
    cfg.lora_rank = w.lora_rank
    cfg.lora_targets = sum(TARGET_BIT[t] for t in w.lora_targets)
    cfg.lora_scale, cfg.perturb_A, cfg.loss_mode = w.lora_scale, int(w.perturb_A), LOSS[w.loss_mode]
    cfg.label_token[0], cfg.label_token[1] = w.label_tokens
    cfg.weight_quant = {"none": 0, "int8": 1, "nf4": 2}[getattr(w, "weight_quant", "none")]
    return cfg


def device_random_weights(w, seed: int, device: str = "cuda:0"):
    """Frozen weights drawn on the GPU (N(0, 0.02^2), norm gains 1 / biases 0), already output-major and in the
    model dtype: for benchmarks of the large workloads, where drawing and uploading host arrays would take minutes.
    Same structure as workloads.make_frozen_weights; not bit-compatible with it."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    st = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    d, f = w.d_model, w.d_ffn
    n_qkv, n_up = d + 2 * w.d_kv, (2 * f if w.act == "swiglu" else f)

    def rnd(*shape, dtype=st):
        return (torch.randn(*shape, generator=g, device=device, dtype=torch.float32) * 0.02).to(dtype)

    ones = lambda n: torch.ones(n, device=device, dtype=torch.float32)
    zeros = lambda n: torch.zeros(n, device=device, dtype=torch.float32)
    ln = w.norm == "layernorm"
    q8 = getattr(w, "weight_quant", "none") == "int8"
    q4 = getattr(w, "weight_quant", "none") == "nf4"

    def lin(n_out, n_in):
        """A block linear [k_out, k_in]: model dtype, (int8 codes, per-output-channel scales), or (4-bit codes packed
        two per byte, block maxima [k_out, k_in / 64])."""
        if q4:
            codes = torch.randint(0, 16, (n_out, n_in), generator=g, device=device, dtype=torch.uint8)
            absmax = 0.048 * (0.75 + 0.5 * torch.rand(n_out, n_in // 64, generator=g, device=device, dtype=torch.float32))
            return pack_nf4_codes(codes).contiguous(), absmax
        if not q8:
            return rnd(n_out, n_in), None
        codes = (torch.randn(n_out, n_in, generator=g, device=device, dtype=torch.float32) * 32.0).round_().clamp_(-127, 127)
        scale = (0.02 / 32.0) * (0.75 + 0.5 * torch.rand(n_out, generator=g, device=device, dtype=torch.float32))
        return codes.to(torch.int8), scale

    out = {"_device_output_major": True, "emb": rnd(w.vocab, d),
           "pos_emb": rnd(w.max_seq, d) if w.pos == "learned" else None, "layers": []}
    for _ in range(w.n_layers):
        (wq, sq), (wo, so), (wu, su), (wd, sd) = lin(n_qkv, d), lin(d, d), lin(n_up, d), lin(d, f)
        out["layers"].append({
            "ln1_g": ones(d), "ln1_b": zeros(d) if ln else None,
            "w_qkv": wq, "s_qkv": sq, "b_qkv": rnd(n_qkv, dtype=torch.float32) if w.has_bias else None,
            "w_o": wo, "s_o": so, "b_o": rnd(d, dtype=torch.float32) if w.has_bias else None,
            "ln2_g": ones(d), "ln2_b": zeros(d) if ln else None,
            "w_up": wu, "s_up": su, "b_up": rnd(n_up, dtype=torch.float32) if w.has_bias else None,
            "w_down": wd, "s_down": sd, "b_down": rnd(d, dtype=torch.float32) if w.has_bias else None})
    out["lnf_g"], out["lnf_b"] = ones(d), (zeros(d) if ln else None)
    out["lm_head"] = out["emb"] if w.tie_embeddings else rnd(w.vocab, d)
    return out


class ZoModel:
    """Device buffers + handle for one workload.  Holds the torch tensors the library borrows."""

    def __init__(self, w, frozen: Dict[str, object], masters: np.ndarray, q_max: Optional[int] = None,
                 E_max: Optional[int] = None, S_max: Optional[int] = None, device: str = "cuda:0"):
        import torch
        self.torch = torch
        self.w = w
        self.device = torch.device(device)
        self.cfg = config_from_workload(w)
        self.q_max, self.E_max, self.S_max = q_max or w.q, E_max or w.E, S_max or w.S
        st = torch.bfloat16 if w.dtype == "bf16" else torch.float32
        self._keep = []

        on_device = bool(frozen.get("_device_output_major", False))   # tensors already on the GPU, [k_out, k_in]

        def dev(a, dtype, transpose=False):
            if a is None:
                return None
            if on_device:
                t = a.to(dtype).contiguous()
            else:
                t = torch.from_numpy(np.ascontiguousarray(a.T if transpose else a))
                t = t.to(self.device).to(dtype).contiguous()
            self._keep.append(t)
            return t.data_ptr()

        L = len(frozen["layers"])
        assert L == w.n_layers
        layers = (MpzLayerWeights * L)()
        for i, lw in enumerate(frozen["layers"]):
            for name in ("ln1_g", "ln1_b", "b_qkv", "b_o", "ln2_g", "ln2_b", "b_up", "b_down"):
                setattr(layers[i], name, dev(lw[name], torch.float32))
            quant = getattr(w, "weight_quant", "none")
            for name in ("w_qkv", "w_o", "w_up", "w_down"):          # [k_in, k_out] -> output-major
                if quant == "nf4" and not on_device:                 # one code per byte -> two per byte along k_in
                    packed = pack_nf4_codes(np.ascontiguousarray(np.asarray(lw[name]).T))
                    setattr(layers[i], name, dev(packed, torch.uint8))
                else:
                    wt_dtype = {"none": st, "int8": torch.int8, "nf4": torch.uint8}[quant]
                    setattr(layers[i], name, dev(lw[name], wt_dtype, transpose=True))
            for name in ("s_qkv", "s_o", "s_up", "s_down"):          # nf4: [k_in / 64, k_out] -> [k_out, k_in / 64]
                setattr(layers[i], name, dev(lw.get(name), torch.float32, transpose=quant == "nf4")
                        if quant != "none" else None)
        self._layers = layers
        wt = MpzWeights()
        wt.emb = dev(frozen["emb"], st)
        wt.pos_emb = dev(frozen["pos_emb"], st)
        wt.lm_head = wt.emb if frozen["lm_head"] is frozen["emb"] else dev(frozen["lm_head"], st)
        wt.lnf_g = dev(frozen["lnf_g"], torch.float32)
        wt.lnf_b = dev(frozen["lnf_b"], torch.float32)
        wt.layers = layers
        self._weights = wt
        numel = mpz_lora_numel(self.cfg)
        assert numel == masters.size, (numel, masters.size)
        self.masters = torch.from_numpy(masters.astype(np.float32)).to(self.device)
        ws_bytes = mpz_workspace_bytes(self.cfg, self.q_max, self.E_max, self.S_max)
        if ws_bytes == 0:
            raise MpzError(2, "invalid configuration for mpz_workspace_bytes")
        self.workspace_bytes = ws_bytes
        self.frozen_bytes = sum(t.numel() * t.element_size() for t in self._keep)
        self.workspace = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=self.device)
        ws_ptr = (self.workspace.data_ptr() + 255) & ~255
        self.stream = torch.cuda.current_stream(self.device)
        self.handle = mpz_init_model(self.cfg, wt, self.masters.data_ptr(), ws_ptr, ws_bytes, self.q_max, self.E_max,
                                     self.S_max, self.stream.cuda_stream)
        self.losses = torch.zeros(2 * self.q_max, dtype=torch.float32, device=self.device)
        self.grads = torch.zeros(self.q_max, dtype=torch.float32, device=self.device)
        self.q = w.q

    def regen_noise(self, seed: int, step: int, q: Optional[int] = None, eps: Optional[float] = None):
        self.q = self.w.q if q is None else q
        mpz_regen_noise(self.handle, seed, step, self.q, self.w.eps if eps is None else eps)

    def forward_perturbed(self, tokens, labels=None, lengths=None):
        """tokens: int32 device tensor [E, S]; labels: int32 device tensor [E] or None; lengths: int32 device tensor [E]
        for a right-padded batch, or None.  Returns losses[2q] (device)."""
        E, S = tokens.shape
        if lengths is not None:
            mpz_forward_perturbed_varlen(self.handle, tokens.data_ptr(), None if labels is None else labels.data_ptr(),
                                         lengths.data_ptr(), E, S, self.losses.data_ptr())
            return self.losses[:2 * self.q]
        mpz_forward_perturbed(self.handle, tokens.data_ptr(), None if labels is None else labels.data_ptr(), E, S,
                              self.losses.data_ptr())
        return self.losses[:2 * self.q]

    def pack_batch(self, tokens, lengths):
        """The right-padded batch tokens [E, S] with lengths [E] (int32 device tensors) without its padding: the real
        tokens back to back, filler up to a multiple of 32 rows, and the sequence starts.  One host read of the lengths
        (the launches are sized by the total and the longest length).  Returns a tuple for forward_packed."""
        torch = self.torch
        E, S = tokens.shape
        len_host = lengths.cpu()
        total, max_len = int(len_host.sum()), int(len_host.max())
        rows = (total + 31) // 32 * 32
        cu = torch.zeros(E + 1, dtype=torch.int32, device=tokens.device)
        cu[1:] = torch.cumsum(lengths, 0)
        keep = torch.arange(S, device=tokens.device)[None, :] < lengths[:, None]
        packed = torch.zeros(rows, dtype=torch.int32, device=tokens.device)
        packed[:total] = tokens[keep]
        return packed, cu, E, total, max_len

    def forward_packed(self, batch, labels=None):
        """batch: what pack_batch returned (kept alive by the caller until the stream has consumed it)."""
        packed, cu, E, total, max_len = batch
        mpz_forward_perturbed_packed(self.handle, packed.data_ptr(), None if labels is None else labels.data_ptr(),
                                     cu.data_ptr(), E, total, max_len, self.losses.data_ptr())
        return self.losses[:2 * self.q]

    def forward_perturbed_packed(self, tokens, labels, lengths):
        """pack_batch + forward_packed.  Returns losses[2q] (device)."""
        self._packed_keep = self.pack_batch(tokens, lengths)
        return self.forward_packed(self._packed_keep, labels)

    def forward_outer_only(self, tokens, labels=None):
        """The outer loop alone: all q queries in one pass, first the + copies, then the - copies (two passes of q
        copies).  Returns losses[2q] (device), the same numbers as forward_perturbed."""
        E, S = tokens.shape
        lab = None if labels is None else labels.data_ptr()
        for sign in (0, 1):
            mpz_forward_copies_strided(self.handle, tokens.data_ptr(), lab, E, S, sign, self.q, 2, self.losses.data_ptr())
        return self.losses[:2 * self.q]

    def forward_copies(self, tokens, labels, copy_begin: int, n_copies: int):
        E, S = tokens.shape
        mpz_forward_copies(self.handle, tokens.data_ptr(), None if labels is None else labels.data_ptr(), E, S,
                           copy_begin, n_copies, self.losses.data_ptr())
        return self.losses[:2 * self.q]

    def forward_sequential(self, tokens, labels=None, group: int = 1):
        """All 2q copies in passes of `group` copies each (group = 1: one forward pass per perturbed copy)."""
        for c in range(0, 2 * self.q, group):
            self.forward_copies(tokens, labels, c, min(group, 2 * self.q - c))
        return self.losses[:2 * self.q]

    def zo_update(self, lr: Optional[float] = None):
        mpz_zo_update(self.handle, self.losses.data_ptr(), self.w.lr if lr is None else lr, self.grads.data_ptr())
        return self.grads[:self.q]

    def zo_update_regen(self, next_step: int, lr: Optional[float] = None):
        """Stateful variant: update from the stored pairs and re-perturb for `next_step` in one pass."""
        mpz_zo_update_regen(self.handle, self.losses.data_ptr(), self.w.lr if lr is None else lr, next_step,
                            self.grads.data_ptr())
        return self.grads[:self.q]

    def zo_step(self, tokens, labels, seed: int, step: int):
        self.regen_noise(seed, step)
        self.forward_perturbed(tokens, labels)
        self.zo_update()

    def debug_noise(self, seed: int, step: int, k: int, tensor_id: int, numel: int):
        z = self.torch.empty(numel, dtype=self.torch.float32, device=self.device)
        mpz_debug_noise(self.handle, seed, step, k, tensor_id, z.data_ptr())
        return z

    def perturbed_copy(self, c: int):
        out = self.torch.empty(self.masters.numel(), dtype=self.torch.float32, device=self.device)
        mpz_debug_perturbed_copy(self.handle, c, out.data_ptr())
        return out

    def embed(self, tokens):
        E, S = tokens.shape
        h = self.torch.empty((2 * self.q * E * S, self.w.d_model), dtype=self.torch.float32, device=self.device)
        mpz_debug_embed(self.handle, tokens.data_ptr(), E, S, h.data_ptr())
        return h

    def run_layers(self, h, layer_begin: int, layer_end: int, E: int, S: int):
        """In place on the fp32 device tensor h [2q*E*S, d]."""
        mpz_debug_run_layers(self.handle, h.data_ptr(), layer_begin, layer_end, E, S)
        return h

    def head_loss(self, h, tokens, labels=None, lengths=None):
        E, S = tokens.shape
        mpz_debug_head_loss(self.handle, h.data_ptr(), tokens.data_ptr(), None if labels is None else labels.data_ptr(),
                            None if lengths is None else lengths.data_ptr(), E, S, self.losses.data_ptr())
        return self.losses[:2 * self.q]

    def close(self):
        if getattr(self, "handle", None) is not None:
            mpz_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
