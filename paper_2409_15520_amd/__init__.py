"""MI355X-native MP-LoRA zeroth-order step: thin Python binding over the C-ABI library libmpz.so."""
from .mpz import (MpzError, MpzConfig, load_library, config_from_workload, ZoModel, device_random_weights,
                  mpz_lora_numel, mpz_lora_tensor_count, mpz_lora_tensor_info, mpz_workspace_bytes,
                  mpz_init_model, mpz_regen_noise, mpz_forward_perturbed, mpz_forward_perturbed_varlen, mpz_forward_perturbed_noalloc, mpz_noalloc_scratch_bytes, mpz_forward_perturbed_packed, mpz_forward_copies, mpz_forward_copies_strided, mpz_zo_update, mpz_zo_update_regen, mpz_debug_noise,
                  mpz_debug_normals_from_words, mpz_debug_perturbed_copy, mpz_debug_embed,
                  mpz_debug_run_layers, mpz_debug_head_loss, mpz_debug_set_kernel_path, mpz_debug_set_tile_config, mpz_debug_set_two_halves, mpz_debug_last_pass_streams, mpz_debug_set_fused_norm_lora, mpz_debug_set_fused_perturb_pack, mpz_debug_gemm_bf16, mpz_debug_gemm_int8, mpz_debug_gemm_bf16_splitk, mpz_debug_gemm_nf4_splitk, mpz_debug_gemm_splits, mpz_debug_set_split_k, mpz_debug_dequant_nf4, mpz_debug_mfma_probe, mpz_debug_hbm_read_probe, pack_nf4_codes, mpz_debug_noise_alu_probe, mpz_debug_qkv_projection, mpz_debug_attention, mpz_profile_begin, mpz_profile_end, PROF_CATEGORIES, mpz_destroy, mpz_last_error,
                  mpz_status_string)
