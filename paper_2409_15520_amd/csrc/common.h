// Internal declarations shared by the HIP translation units of libmpz (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace mpz {

// bf16 stored as its 16-bit pattern; conversions are explicit so rounding is visible in the code.
struct bf16_t { uint16_t bits; };

__host__ __device__ inline float bf16_to_f32(bf16_t v) {
  union { uint32_t u; float f; } c; c.u = ((uint32_t)v.bits) << 16; return c.f;
}
// round-to-nearest-even from binary32 (finite inputs)
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
  union { uint32_t u; float f; } c; c.f = f;
  uint32_t r = c.u + 0x7FFFu + ((c.u >> 16) & 1u);
  bf16_t o; o.bits = (uint16_t)(r >> 16); return o;
}

// two binary32 values -> two bf16 in one word (low half = a), round-to-nearest-even in hardware (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// SiLU(g) * u in binary32 for the bf16 models: g * u / (1 + 2^(-g log2 e)) with the hardware exp2 and reciprocal
// (1 ulp each; the result is rounded to bf16 right after).  One definition for the fused SwiGLU epilogue and the
// stand-alone kernel, so that both give the same bits.
__device__ __forceinline__ float silu_mul_f32(float g, float u) {
  const float e = __builtin_amdgcn_exp2f(g * -1.4426950408889634f);
  return g * __builtin_amdgcn_rcpf(1.0f + e) * u;
}

// Position of the LoRA factors inside one layer's slice of the flat master vector.
struct LoraLayerTable {
  int32_t n_tensors;          // 2 per adapted target
  int32_t per_layer;          // elements per layer
  int32_t off[9];             // start of tensor i inside the layer slice; off[n_tensors] = per_layer
  int32_t local_id[8];        // target*2 + factor
  int32_t rows[8], cols[8];
};

// ---- noise.hip -------------------------------------------------------------------------
void launch_perturb(hipStream_t st, const float* masters, float* pert /*[2q][P]*/, int64_t P,
                    const LoraLayerTable& tab, uint64_t seed, uint32_t step, int q, float eps, int perturb_A);
// the same perturbation written straight into the bf16 hi / lo MFMA operand layouts of all 2q copies (see
// launch_pack_factors for the layouts); supported for ranks 4 / 8 / 16 with K % 8 == 0 and k_out % 4 == 0
bool perturb_pack_supported(const LoraLayerTable& tab, int rank, int rp);
void launch_perturb_pack(hipStream_t st, const float* masters, void* packed, int64_t packed_per_copy,
                         const LoraLayerTable& tab, int n_layers, int rank, int rp, uint64_t seed, uint32_t step, int q,
                         float eps, int perturb_A);
void launch_update(hipStream_t st, float* masters, int64_t P, const LoraLayerTable& tab, uint64_t seed,
                   uint32_t step, int q, float eps, float lr, int perturb_A, const float* losses,
                   float* proj_grads_out);
// update from the stored perturbed pairs, then re-perturb with the noise of next_step (stateful variant, Algorithm 2)
void launch_noise_alu_probe(hipStream_t st, int64_t n_groups, int q, float* sink);
void launch_update_regen(hipStream_t st, float* masters, float* pert, int64_t P, const LoraLayerTable& tab, uint64_t seed,
                         uint32_t next_step, int q, float eps, float lr, int perturb_A, const float* losses,
                         float* proj_grads_out);
void launch_debug_noise(hipStream_t st, float* z_out, int64_t numel, uint64_t seed, uint32_t step, int k,
                        int tensor_id);
void launch_normals_from_words(hipStream_t st, const uint32_t* words, size_t n4, float* out);

// ---- simple_kernels.hip: straightforward kernels, any shape, fp32 (fp64 accumulate) or bf16 (fp32) --
struct LoraSeg {              // one adapted column range of a linear
  int32_t col_begin, col_end; // output columns [begin, end)
  const void* t;              // [T, t_stride] bottleneck activations OP(s x A_c), model dtype
  int32_t t_stride, t_off;    // row stride and first column of this target's r values
  const float* Bc;            // perturbed B copies: copy c at Bc + c*copy_stride, [r, k_out] row-major
  int64_t copy_stride;
};

struct MfmaLoraSeg {
  int32_t col_begin, col_end;   // adapted output columns, multiples of 128
  const void* tp;               // [T, rp] bf16: [t | t | 0], t = OP(s x A_c)
  const void* bp;               // packed B copies: copy c at bp + c*copy_stride, [k_out, rp] bf16 = [hi | lo | 0]
  int32_t rp;                   // padded 2r, multiple of 16
  int64_t copy_stride;          // elements
};

struct LinearArgs {
  int dtype;                  // MPZ_DTYPE_*
  int M, N, K;
  const void* x;              // [M, K] model dtype
  const void* w;              // [N, K] model dtype (output-major); int8 codes when w_scale is set
  const float* w_scale;       // [N] per-output-channel scales of int8 weights, or null
  const void* w_codes;        // 4-bit weights that have not been dequantised: codes [N, K / 2] and
  const float* w_absmax;      //   block maxima [N, K / 64]; w is then null until the launcher decides who dequantises
  const float* bias;          // [N] or null
  int n_seg; LoraSeg seg[3];
  int mfma_lora; MfmaLoraSeg mseg[3];   // the same segments in the MFMA kernels' operand layouts (when prepared)
  int rank; int rows_per_copy;
  int act;                    // -1 none, else MPZ_ACT_RELU / MPZ_ACT_GELU_ERF
  const float* residual;      // [M, N] fp32 added before the store, or null
  int out_kind;               // 0: model dtype, 1: fp32, 2: accumulate type staging (double for f32 models, float for bf16)
  void* out;                  // [M, N]
  // optional fused rotary embedding (MFMA path, model-dtype output): see MfmaGemmArgs
  const float* rope_cos; const float* rope_sin; int rope_cols, rope_dh, S;
  const int32_t* rope_pos;    // packed batches: position of row m % S inside its sequence (null: m % S itself)
};
void launch_linear_simple(hipStream_t st, const LinearArgs& a);

// row_pos (packed batches, else null): position of a copy's row inside its own sequence, [E * S]
void launch_embed(hipStream_t st, int dtype, const int32_t* tokens, const void* emb, const void* pos_emb,
                  const int32_t* row_pos, float* h, int n_copies, int E, int S, int d);
void launch_norm(hipStream_t st, int dtype, int kind, float eps, const float* h, int64_t h_row_stride,
                 const float* g, const float* b, void* out, int rows, int d);
// t[T, r_tot] = OP(scale * x A_c) for up to 4 targets sharing the input x
struct LoraDownArgs {
  int dtype; int T, K, rank, n_targets, rows_per_copy;
  const void* x; float scale;
  const float* Ac[4];         // perturbed A copies per target: copy c at Ac[i] + c*copy_stride, [K, r] row-major
  int64_t copy_stride;
  void* t;                    // [T, n_targets*rank] model dtype
};
void launch_lora_down_simple(hipStream_t st, const LoraDownArgs& a);
// q/k: rotate (optionally) and convert staging -> model dtype; v: convert. staging is [T, n_cols] accumulate type
// row_pos (packed batches, else null): position of row % S inside its own sequence
void launch_rope_convert(hipStream_t st, int dtype, const void* staging, void* out, int T, int S, int n_cols,
                         int d_head, int n_rot_heads, const float* cos_tab, const float* sin_tab, const int32_t* row_pos);
// cu == null: n_seq sequences of S rows back to back.  Packed batches: S is the longest sequence, sequence s of the
// n_seq = copies * E starts at row (s / E) * rows_per_copy + cu[s % E] and holds cu[s % E + 1] - cu[s % E] rows.
void launch_attention_simple(hipStream_t st, int dtype, const void* qkv, int qkv_stride, void* out, int n_seq, int S,
                             int H, int Hkv, int dh, const int32_t* cu, int E, int rows_per_copy);
void launch_swiglu(hipStream_t st, int dtype, const void* staging, void* out, int T, int f);
// per-row CE from fp32 logits; target[r] < 0 => row skipped (ce = 0)
void launch_ce_rows(hipStream_t st, int dtype, const float* logits, int64_t row_stride, int n_cols, const int32_t* target,
                    float* ce, int rows);
void launch_last_pos_subset_logits(hipStream_t st, int dtype, const void* xf, const void* head, int d, int rows,
                                   int tok0, int tok1, float* logits2);
void launch_make_targets(hipStream_t st, int mode, const int32_t* tokens, const int32_t* labels, const int32_t* lengths,
                         const int32_t* row_end, int tok0, int tok1, int32_t* target, int n_copies, int E, int S);
// packed batch: per row of a copy, its position in its sequence and the row after the sequence's last (-1: filler)
void launch_packed_index(hipStream_t st, const int32_t* cu, int E, int rows, int32_t* row_pos, int32_t* row_end);
void launch_gather_last_rows_packed(hipStream_t st, const float* h, const int32_t* cu, int n_copies, int E,
                                    int rows_per_copy, int d, float* out);
void launch_gather_last_rows(hipStream_t st, const float* h, const int32_t* lengths, int n_copies, int E, int S, int d,
                             float* out);
// losses[i * loss_stride] = mean of copy i's per-row losses
void launch_copy_mean(hipStream_t st, const float* ce, int rows_per_copy, int count_per_copy, const int32_t* lengths, int E,
                      int S, float* losses, int n_copies, int loss_stride);
void launch_fill_f32(hipStream_t st, float* p, float v, int64_t n);
// 4-bit normal-float codes (two per byte, low nibble first) + block maxima [n_elems / 64] -> bf16 [n_elems];
// n_elems % 64 == 0, rows of a multiple of 64 elements stored back to back
void launch_nf4_dequant(hipStream_t st, const void* codes, const float* absmax, void* out, int64_t n_elems);

// ---- gemm_mfma.hip: bf16 MFMA kernels (gfx950) ------------------------------------------------
struct MfmaGemmArgs {
  int M, N, K;                  // out[M, N] = x[M, K] w[N, K]^T ; dual: N = columns of ONE of the two tiles
  const void* x; const void* w;
  const float* w_scale;         // null: w is bf16.  Else w holds int8 codes [w_rows, K] and w_scale [w_rows] the
                                // per-output-channel scales: the product is x . (code * scale)
  const float* w_absmax;        // non-null (split-K launches only): w holds 4-bit normal-float codes [w_rows, K / 2]
                                // (element 2j of a row in the low nibble of byte j) and w_absmax [w_rows, K / 64] the
                                // block maxima; the operand load turns them into bf16(level[code] * max)
  int w_rows;                   // rows of w (N, or 2N for dual): bounds the weight buffer
  const float* bias;            // [N] (dual: [dual_offset + N]) or null
  int dual; int dual_offset;    // dual: second weight tile starts dual_offset rows below (SwiGLU gate | up)
  int n_seg; MfmaLoraSeg seg[3];
  int rows_per_copy;
  int act;                      // -1 none, MPZ_ACT_RELU, MPZ_ACT_GELU_ERF (ignored when dual: SiLU(gate) * up)
  const float* residual;        // [M, ldo] fp32 or null
  int out_f32; void* out; int ldo;
  int tile_cfg;                 // 0 = choose by shape; 1, 6, 9, 10, 11, 12 force that tile configuration (tests)
  // fused rotary embedding (bf16 output only): columns [0, rope_cols) are heads of width rope_dh rotated by the
  // position m % S with tables [max_seq, rope_dh / 2]; packed batches: position rope_pos[m % S] (S = rows per copy)
  const float* rope_cos; const float* rope_sin; int rope_cols, rope_dh, S;
  const int32_t* rope_pos;
  // fused cross-entropy (LM head): when ce_max is set nothing is stored to `out`; every wave tile writes, per token
  // row, the maximum and the sum of exp(logit - maximum) over its columns to slot [tile_n * waves_n + wave_n][M] of
  // ce_max / ce_sum, and the wave holding column ce_target[m] writes that logit to ce_tlogit[m]
  float* ce_max; float* ce_sum; float* ce_tlogit; const int32_t* ce_target;
  // split K (few stacked tokens: the weight stream is what takes the time, and one block per output tile would
  // leave most of the chip idle): k_splits > 1 blocks share an output tile, each takes a contiguous share of the
  // K-tiles and writes its raw fp32 sums to partial[split][M][ldp] (dual: the second weight tile N columns to the
  // right); bias, activation, rotary embedding, residual and the output type are then the reduction kernel's
  // (launch_gemm_mfma does both).  0 or 1: off.  defer_reduce: launch_gemm_mfma leaves the reduction to the caller
  // (launch_splitk_reduce_norm: the reduction in one kernel with the pre-norm that follows the projection).
  int k_splits; float* partial; int ldp; int defer_reduce;
};
// k_splits a launch of these arguments would use given room for `partial_capacity` floats (1 = no split)
int mfma_gemm_splits(const MfmaGemmArgs& a, size_t partial_capacity);
bool mfma_gemm_supported(const MfmaGemmArgs& a);
int mfma_gemm_ce_slots(const MfmaGemmArgs& a);      // partial slots per row the launch will write (depends on the tile)
// ce[m] = logsumexp over the slots - target logit (0 where ce_target[m] < 0)
void launch_ce_combine(hipStream_t st, int slots, int M, const float* ce_max, const float* ce_sum, const float* ce_tlogit,
                       const int32_t* ce_target, float* ce);
// hipSuccess, or the error of raising the kernel instance's dynamic LDS limit (then nothing was launched)
hipError_t launch_gemm_mfma(hipStream_t st, const MfmaGemmArgs& a);

struct MfmaLoraDownArgs {
  int T, K, rank, n_targets, rows_per_copy, rp;
  const void* x; float scale;
  const void* ap[3];            // packed A copies per target: copy c at ap[i] + c*copy_stride, [2][K / 8][r][8] bf16 (hi part, lo part; element (j, k) of a part at ((k / 8) r + j) 8 + k % 8)
  int64_t copy_stride;
  void* tp[3];                  // per target [T, rp] bf16
};
// measurement: `blocks` x 8 waves x iters x 8 MFMAs (32x32x16 bf16), fragments from operands [>= 12288 bf16], optionally
// re-read from LDS every step; out [blocks * 512] fp32
void launch_mfma_probe(hipStream_t st, const void* operands, int blocks, int iters, int with_lds, float* out);
// read-only traffic probe: tiles of rb rows x seg_bytes of a [rows][row_bytes] buffer, L = rb * seg_bytes / 4096 in {1,2,4,8,16}
hipError_t launch_hbm_read_probe(hipStream_t st, const void* buf, long rows, long row_bytes, int rb, int seg_bytes, int k_splits,
                                 int lds_bytes, int mode, uint32_t* out);
bool mfma_lora_down_supported(const MfmaLoraDownArgs& a);
void launch_lora_down_mfma(hipStream_t st, const MfmaLoraDownArgs& a);
void launch_pack_factors(hipStream_t st, const float* pert, int64_t P, int n_copies, const LoraLayerTable& tab,
                         int n_layers, int rank, int rp, void* packed, int64_t packed_per_copy);


// ---- attention_mfma.hip ---------------------------------------------------------------------------
bool attention_mfma_supported(int dh, int qkv_stride, int d);
// cu / E / rows_per_copy: as for launch_attention_simple
void launch_attention_mfma(hipStream_t st, const void* qkv, int qkv_stride, void* out, int n_seq, int S, int H, int Hkv,
                           int dh, const int32_t* cu, int E, int rows_per_copy);


// ---- rowwise.hip ----------------------------------------------------------------------------------
// norm_rows + lora_down_mfma in one kernel (h dense [T, d] fp32 -> out [T, d] bf16 and a.tp); a.x is ignored
bool norm_lora_supported(int d, const MfmaLoraDownArgs& a);
void launch_norm_lora(hipStream_t st, int kind, float eps, const float* h, const float* g, const float* b, void* out,
                      const MfmaLoraDownArgs& a);
bool norm_rows_supported(int d, int64_t h_row_stride);
// split-K projection into the residual stream + the pre-norm of the same rows in one kernel (same bits as the
// reduction kernel followed by launch_norm_rows); `a` is the GEMM launched with defer_reduce
bool splitk_reduce_norm_supported(const MfmaGemmArgs& a);
void launch_splitk_reduce_norm(hipStream_t st, const MfmaGemmArgs& a, int kind, float eps, const float* g, const float* b,
                               void* out);
void launch_norm_rows(hipStream_t st, int kind, float eps, const float* h, int64_t h_row_stride, const float* g,
                      const float* b, void* out, int rows, int d);

}  // namespace mpz
