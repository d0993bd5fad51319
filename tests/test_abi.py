"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and its host-side logic (layout, workspace sizing, validation) behaves as documented."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads as W
import paper_2409_15520_amd as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mpz.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mpz_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = M.load_library()
    names = _declared_symbols()
    assert {"mpz_init_model", "mpz_regen_noise", "mpz_forward_perturbed", "mpz_zo_update"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_config_struct_size_matches():
    cfg = M.config_from_workload(W.get_workload("c1_tiny_fp32"))
    assert M.mpz_lora_numel(cfg) == 4096
    cfg.struct_size += 4
    assert M.mpz_lora_numel(cfg) == 0 and M.mpz_workspace_bytes(cfg, 2, 2, 32) == 0


@pytest.mark.parametrize("name", list(W.WORKLOADS))
def test_lora_layout_matches_canonical_order(name):
    w = W.get_workload(name)
    cfg = M.config_from_workload(w)
    lay = W.lora_layout(w)
    assert M.mpz_lora_tensor_count(cfg) == len(lay)
    assert M.mpz_lora_numel(cfg) == lay[-1].offset + lay[-1].rows * lay[-1].cols
    for i in (0, 1, len(lay) // 2, len(lay) - 1):
        t = M.mpz_lora_tensor_info(cfg, i)
        assert (t.layer, t.target, t.factor, t.tensor_id, t.offset, t.rows, t.cols) == tuple(lay[i])
    with pytest.raises(M.MpzError):
        M.mpz_lora_tensor_info(cfg, len(lay))


def test_workspace_grows_with_shape_and_rejects_bad_arguments():
    w = W.get_workload("c2_opt125m")
    cfg = M.config_from_workload(w)
    a = M.mpz_workspace_bytes(cfg, 4, 8, 128)
    assert a > 0 and a % 256 == 0
    assert M.mpz_workspace_bytes(cfg, 8, 8, 128) > a > M.mpz_workspace_bytes(cfg, 4, 4, 128)
    assert M.mpz_workspace_bytes(cfg, 0, 8, 128) == 0
    assert M.mpz_workspace_bytes(cfg, 4, 8, 129) == 0          # S_max > max_seq
    assert M.mpz_workspace_bytes(cfg, 65, 8, 128) == 0


@pytest.mark.parametrize("field,value", [("n_heads", 5), ("n_kv_heads", 5), ("lora_rank", 6), ("lora_targets", 0),
                                         ("lora_targets", 16), ("act", 3), ("dtype", 2), ("loss_mode", 7),
                                         ("vocab", 1), ("norm_eps", 0.0)])
def test_invalid_configs_are_rejected_on_the_host(field, value):
    cfg = M.config_from_workload(W.get_workload("c1_tiny_fp32"))
    setattr(cfg, field, value)
    assert M.mpz_lora_numel(cfg) == 0
    assert M.mpz_workspace_bytes(cfg, 2, 2, 32) == 0


def test_four_bit_weights_need_bf16_and_add_the_dequantisation_buffer():
    w = W.get_workload("c2_opt125m")
    cfg = M.config_from_workload(w)
    plain = M.mpz_workspace_bytes(cfg, 4, 8, 128)
    cfg4 = M.config_from_workload(w.with_(weight_quant="nf4"))
    assert cfg4.weight_quant == 2
    # one bf16 copy of the largest block linear (768 x 3072), rounded up to the 256-byte carving
    assert M.mpz_workspace_bytes(cfg4, 4, 8, 128) - plain == 768 * 3072 * 2
    cfg4.dtype = 0
    assert M.mpz_workspace_bytes(cfg4, 4, 8, 128) == 0
    cfg4.dtype, cfg4.weight_quant = 1, 3
    assert M.mpz_workspace_bytes(cfg4, 4, 8, 128) == 0
    with pytest.raises(M.MpzError):
        M.mpz_debug_dequant_nf4(None, None, None, 64, None)
    assert np.array_equal(M.pack_nf4_codes(np.array([[1, 2, 15, 0]], dtype=np.uint8)), np.array([[0x21, 0x0F]], dtype=np.uint8))


def test_label_tokens_must_be_distinct_and_in_vocab():
    cfg = M.config_from_workload(W.get_workload("c1_tiny_fp32"))
    cfg.label_token[1] = 512
    assert M.mpz_lora_numel(cfg) == 0
    cfg.label_token[1] = cfg.label_token[0]
    assert M.mpz_lora_numel(cfg) == 0
    cfg.loss_mode = 2                                            # next-token loss ignores the label words
    assert M.mpz_lora_numel(cfg) == 4096


def test_init_rejects_null_and_small_workspace_without_touching_the_device():
    lib = M.load_library()
    cfg = M.config_from_workload(W.get_workload("c1_tiny_fp32"))
    h = C.c_void_p()
    assert lib.mpz_init_model(C.byref(cfg), None, None, None, 0, 2, 2, 32, None, C.byref(h)) == 1   # MPZ_ERR_NULL
    assert "NULL" in M.mpz_last_error()
    assert lib.mpz_regen_noise(None, 1, 0, 1, 1e-3) == 1
    assert lib.mpz_forward_perturbed(None, None, None, 1, 2, None) == 1
    assert lib.mpz_zo_update(None, None, 1e-4, None) == 1
    assert M.mpz_status_string(0) == "MPZ_OK" and M.mpz_status_string(5) == "MPZ_ERR_STATE"
    # fake non-null addresses: validation fails before any of them is dereferenced
    L = (M.mpz.MpzLayerWeights * cfg.n_layers)()
    for lw in L:
        for n, _ in lw._fields_:
            setattr(lw, n, 0x1000)
    wt = M.mpz.MpzWeights(0x1000, 0x1000, 0x1000, 0x1000, 0x1000, L)
    need = M.mpz_workspace_bytes(cfg, 2, 2, 32)
    assert lib.mpz_init_model(C.byref(cfg), C.byref(wt), 0x1000, 0x1000, need - 1, 2, 2, 32, None, C.byref(h)) == 4
    assert "workspace too small" in M.mpz_last_error()
    assert lib.mpz_init_model(C.byref(cfg), C.byref(wt), 0x1000, 0x1001, need, 2, 2, 32, None, C.byref(h)) == 4
    assert lib.mpz_init_model(C.byref(cfg), C.byref(wt), 0x1000, 0x1000, need, 2, 2, 33, None, C.byref(h)) == 2
    # a valid init with no rotary tables enqueues nothing, so the state machine can be checked on the host
    assert lib.mpz_init_model(C.byref(cfg), C.byref(wt), 0x1000, 0x1000, need, 2, 2, 32, None, C.byref(h)) == 0
    assert lib.mpz_forward_perturbed(h, 0x1000, 0x1000, 2, 32, 0x1000) == 5          # before regen_noise
    assert lib.mpz_zo_update(h, 0x1000, 1e-4, None) == 5
    assert lib.mpz_zo_update_regen(h, 0x1000, 1e-4, 1, None) == 5                     # no stored pairs yet
    assert lib.mpz_zo_update_regen(None, None, 1e-4, 1, None) == 1
    assert lib.mpz_forward_perturbed_varlen(h, 0x1000, 0x1000, None, 2, 32, 0x1000) == 1     # NULL lengths
    assert lib.mpz_forward_perturbed_varlen(h, 0x1000, 0x1000, 0x1000, 2, 32, 0x1000) == 5   # before regen_noise
    assert lib.mpz_regen_noise(h, 1, 0, 3, 1e-3) == 3                                # q > q_max
    assert lib.mpz_regen_noise(h, 1, 0, 2, -1.0) == 2
    assert "eps" in M.mpz_last_error(h)
    lib.mpz_destroy(h)


def test_read_probe_rejects_what_its_kernel_could_not_read_in_bounds():
    """mpz_debug_hbm_read_probe launches only when every tile of every block lies inside [rows][row_bytes]: the checks
    run on the host, before any device call."""
    lib = M.load_library()
    lib.mpz_debug_hbm_read_probe.restype = C.c_int
    lib.mpz_debug_hbm_read_probe.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                             C.c_int32, C.c_void_p, C.c_void_p]
    ok = dict(rows=256, row_bytes=4096, rb=128, seg=128, ks=2, lds=0, mode=0)

    def call(buf=0x1000, out=0x1000, **kw):
        a = dict(ok, **kw)
        return lib.mpz_debug_hbm_read_probe(buf, a["rows"], a["row_bytes"], a["rb"], a["seg"], a["ks"], a["lds"], a["mode"], out, None)
    assert call(buf=None) == 1 and call(out=None) == 1                    # MPZ_ERR_NULL
    assert call(buf=0x1008) == 2                                          # MPZ_ERR_CONFIG: alignment
    assert call(rows=200) == 3                                            # MPZ_ERR_SHAPE from here: rows not a multiple of the rows per block
    assert call(ks=3) == 3                                                # a row does not split into 3 shares of whole tiles
    assert call(seg=24) == 3 and call(seg=0) == 3
    assert call(rb=96) == 3                                               # 96 x 128 B is not a whole number of 4 KiB
    assert call(rb=128, seg=1024, row_bytes=8192) == 3                    # 128 KiB tiles: more than a thread holds
    assert call(lds=200 * 1024) == 3
    assert call(mode=4) == 2 and call(mode=-1) == 2
    assert call(mode=2, lds=8192) == 3                                    # staging 16 KiB tiles needs 16 KiB of LDS
    assert call(mode=3, lds=16384) == 3                                   # ... and 32 KiB with the activation tile
