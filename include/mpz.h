/*
 * mpz - MP-LoRA zeroth-order step on one AMD MI355X (gfx950).
 *
 * One "ZO step" is Algorithm 1 of the paper (MobiZO, arXiv 2409.15520): q queries (outer loop)
 * times the two signs (inner loop) give n = 2q perturbed copies of the LoRA factors; all copies
 * run through ONE batched forward pass that shares the frozen weights (the MP-LoRA layer of
 * Section 3, Y = X W + (X A) (.) B with per-copy factors); the per-copy losses give the
 * two-point estimates g_k (Algorithm 1, the projected gradient) and the update regenerates the noise from
 * its seed instead of storing it (Algorithm 1, the stored seeds and the update; Section 2, "ZO LLM Fine-Tuning").
 *
 * Conventions for every entry point
 *   - Pointers marked [dev] are device (HBM) addresses, [host] are host addresses.
 *   - The library allocates no device memory: the caller owns the frozen weights, the LoRA
 *     masters, token / label / loss buffers and one workspace, and keeps them alive for the
 *     lifetime of the model handle.  The handle itself is host memory owned by the library.
 *   - All device work is enqueued on the HIP stream given to mpz_init_model; no entry point
 *     synchronises with the device except mpz_init_model.  Outputs are valid once the caller
 *     has synchronised that stream.
 *   - Errors are returned as mpz_status; nothing throws or aborts across this boundary.
 *     Arguments are validated on the host before any launch.  mpz_last_error() returns a
 *     message for the last failing call on that handle (or on the calling thread when there
 *     is no handle).
 *   - Copy order: copy c = 2k + s uses +eps z_k for s = 0 and -eps z_k for s = 1, k < q.
 *     Stacked token row of (copy c, sequence e, position p) is (c*E + e)*S + p.
 *   - Storage layout of a linear y = x W (+ b), W in R^{k_in x k_out}: output-major, element
 *     (k, n) of W at w[n*k_in + k], in the model dtype (fp32 or bf16); biases and norm
 *     parameters are fp32.
 */
#ifndef MPZ_H
#define MPZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mpz_model mpz_model; /* opaque host-side handle */

typedef enum {
  MPZ_OK = 0,
  MPZ_ERR_NULL = 1,      /* a required pointer is NULL */
  MPZ_ERR_CONFIG = 2,    /* inconsistent or unsupported configuration / argument value */
  MPZ_ERR_SHAPE = 3,     /* q, E or S outside what the model was initialised for */
  MPZ_ERR_WORKSPACE = 4, /* workspace too small or misaligned */
  MPZ_ERR_STATE = 5,     /* call order violated (e.g. update without a preceding regen_noise) */
  MPZ_ERR_DEVICE = 6     /* a HIP runtime call failed */
} mpz_status;

enum { MPZ_ACT_RELU = 0, MPZ_ACT_GELU_ERF = 1, MPZ_ACT_SWIGLU = 2 };
enum { MPZ_NORM_LAYERNORM = 0, MPZ_NORM_RMSNORM = 1 };
enum { MPZ_POS_LEARNED = 0, MPZ_POS_ROPE = 1 };
enum { MPZ_DTYPE_F32 = 0, MPZ_DTYPE_BF16 = 1 };
enum { MPZ_WEIGHT_QUANT_NONE = 0, MPZ_WEIGHT_QUANT_INT8 = 1, MPZ_WEIGHT_QUANT_NF4 = 2 };
enum { MPZ_TARGET_Q = 1, MPZ_TARGET_K = 2, MPZ_TARGET_V = 4, MPZ_TARGET_O = 8 };
enum {
  MPZ_LOSS_LAST_POS_LABEL_SUBSET = 0, /* 2-way CE over two label-token logits at the last position */
  MPZ_LOSS_LAST_POS_FULL_VOCAB = 1,   /* CE over the whole vocabulary at the last position (Appendix D.2) */
  MPZ_LOSS_NEXT_TOKEN_ALL_POS = 2     /* position p predicts token p+1, p < S-1, whole vocabulary */
};

/* Model description.  Plain data; struct_size = sizeof(mpz_config) guards against layout drift. */
typedef struct {
  uint32_t struct_size;
  int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab, max_seq;
  int32_t act;            /* MPZ_ACT_* */
  int32_t norm;           /* MPZ_NORM_* */
  float norm_eps;
  int32_t pos;            /* MPZ_POS_* */
  float rope_theta;       /* rotary base; pairs (i, i + d_head/2), angle p * theta^(-2i/d_head) */
  int32_t has_bias;       /* linears carry biases (OPT-style) */
  int32_t dtype;          /* MPZ_DTYPE_*: storage type of weights and GEMM operands.
                             BF16 accumulates in fp32; F32 accumulates in fp64. */
  int32_t lora_rank;      /* r, a multiple of 4 */
  uint32_t lora_targets;  /* OR of MPZ_TARGET_* */
  float lora_scale;       /* s in y = x W + s (x A) B */
  int32_t perturb_A;      /* 1: A and B are perturbed and updated; 0: LoRA-FA of Section 3 -
                             A frozen and shared by all copies, only B perturbed and updated */
  int32_t loss_mode;      /* MPZ_LOSS_* */
  int32_t label_token[2]; /* vocabulary ids of the two label words (last-position modes) */
  int32_t weight_quant;   /* MPZ_WEIGHT_QUANT_*: weight-only quantisation of the four linears of every block
                             (Appendix D, "MobiZO with weight-only quantization").  INT8: w_* hold int8 codes and
                             s_* one fp32 scale per output channel, W = code * scale exactly; needs dtype BF16,
                             d_model and d_ffn multiples of 64 and E*S a multiple of 32 (MFMA path only).  The codes
                             are widened once per step for all 2q copies, inside the GEMM's operand load.
                             NF4: w_* hold 4-bit normal-float codes (the sixteen-level type of Q-LoRA, which the
                             appendix builds on), two per byte, rows of k_in / 2 bytes with element 2j in the low
                             nibble of byte j; s_* one fp32 absolute maximum per block of 64 consecutive input
                             channels, [k_out, k_in / 64]; W = bf16(level[code] * max).  Needs dtype BF16 and d_model,
                             d_ffn multiples of 64.  Each linear is dequantised into a workspace buffer right before
                             its GEMM, once per pass for all the copies of that pass; in a pass over at most 256
                             stacked tokens the GEMMs that split K look the codes up in their own operand load
                             instead (the same weights bit for bit, a quarter of the bytes read). */
} mpz_config;

/* Frozen parameters theta_f of one decoder block (Algorithm 1, input line).  All [dev], borrowed. */
typedef struct {
  const float* ln1_g; /* [d] */
  const float* ln1_b; /* [d] or NULL (RMSNorm) */
  const void* w_qkv;  /* [d + 2*d_kv, d] output-major: rows 0..d-1 = W_q, then W_k, then W_v */
  const float* b_qkv; /* [d + 2*d_kv] or NULL */
  const void* w_o;    /* [d, d] */
  const float* b_o;   /* [d] or NULL */
  const float* ln2_g;
  const float* ln2_b;
  const void* w_up;   /* [d_ffn, d]; SwiGLU: [2*d_ffn, d], rows 0..d_ffn-1 = gate, then up */
  const float* b_up;  /* [d_ffn] (SwiGLU: [2*d_ffn]) or NULL */
  const void* w_down; /* [d, d_ffn] */
  const float* b_down;/* [d] or NULL */
  /* weight_quant = INT8: per-output-channel scales, 16-byte aligned; the w_* above are then int8 with the same
   * [k_out, k_in] shapes.  NF4: block maxima [k_out, k_in / 64]; the w_* are packed codes [k_out, k_in / 2] bytes,
   * 4-byte aligned.  NONE: ignored. */
  const float* s_qkv; /* [d + 2*d_kv] (NF4: [d + 2*d_kv, d / 64]) */
  const float* s_o;   /* [d] (NF4: [d, d / 64]) */
  const float* s_up;  /* [d_ffn] (SwiGLU: [2*d_ffn]) (NF4: [rows, d / 64]) */
  const float* s_down;/* [d] (NF4: [d, d_ffn / 64]) */
} mpz_layer_weights;

typedef struct {
  const void* emb;      /* [dev] [vocab, d] token embedding, model dtype */
  const void* pos_emb;  /* [dev] [max_seq, d] learned positions, or NULL with MPZ_POS_ROPE */
  const void* lm_head;  /* [dev] [vocab, d] output-major head; may alias emb (tied) */
  const float* lnf_g;   /* [dev] [d] final norm */
  const float* lnf_b;   /* [dev] [d] or NULL */
  const mpz_layer_weights* layers; /* [host] n_layers entries, copied by mpz_init_model */
} mpz_weights;

/* One LoRA factor inside the flat fp32 master vector theta_l. */
typedef struct {
  int32_t layer;
  int32_t target;    /* 0 = Q, 1 = K, 2 = V, 3 = O */
  int32_t factor;    /* 0 = A [k_in, r], 1 = B [r, k_out], both row-major (Section 2, LoRA) */
  int32_t tensor_id; /* (layer*4 + target)*2 + factor: the noise stream coordinate */
  int64_t offset;    /* element offset in the master vector */
  int32_t rows, cols;
} mpz_lora_tensor;

/* Number of fp32 elements of the LoRA master vector theta_l: layer-major; within a layer the
 * enabled targets in the order Q, K, V, O; for each target A then B.  0 on an invalid config. */
size_t mpz_lora_numel(const mpz_config* cfg /*[host]*/);
/* Number of LoRA factors (2 per adapted linear), and the i-th one's description. */
int32_t mpz_lora_tensor_count(const mpz_config* cfg /*[host]*/);
mpz_status mpz_lora_tensor_info(const mpz_config* cfg /*[host]*/, int32_t i, mpz_lora_tensor* out /*[host]*/);

/* Bytes of workspace needed for up to q_max queries on E_max sequences of S_max tokens.
 * Holds the transient perturbed factor copies (Section 3, inner-loop parallelisation: only the
 * master factors persist, perturbed copies live for one pass), activations of ONE layer for all
 * n copies (nothing is retained across layers), and small tables.  0 on an invalid configuration. */
size_t mpz_workspace_bytes(const mpz_config* cfg /*[host]*/, int32_t q_max, int32_t E_max, int32_t S_max);

/* Build a model handle (Algorithm 1, input line: theta_l, theta_f, q, E).
 *   frozen        [host] struct of [dev] pointers, borrowed for the handle's lifetime
 *   lora_masters  [dev] fp32[mpz_lora_numel], theta_l, updated in place by mpz_zo_update
 *   workspace     [dev] 256-byte aligned, at least mpz_workspace_bytes(cfg, q_max, E_max, S_max)
 *   hip_stream    hipStream_t (NULL = default stream)
 * Uploads small tables (rotary cos/sin, layout) into the workspace and synchronises the stream once.
 * Errors: NULL, CONFIG (d_model % n_heads, n_heads % n_kv_heads, odd d_head with RoPE, rank not a
 * multiple of 4, label ids outside the vocabulary, S_max > max_seq, ...), WORKSPACE, DEVICE. */
mpz_status mpz_init_model(const mpz_config* cfg, const mpz_weights* frozen, float* lora_masters,
                          void* workspace, size_t workspace_bytes, int32_t q_max, int32_t E_max,
                          int32_t S_max, void* hip_stream, mpz_model** out);

/* Algorithm 1, seed / noise / perturbation steps for all q queries and both signs at once: regenerate z_k ~ N(0, I) from
 * the counter-based stream (seed, step, k) and write the n = 2q perturbed factor copies
 * theta_l + (+/-) eps z_k into the workspace.  z is never stored.  The stream: Philox4x32-10
 * keyed by seed, counter (element/4, tensor_id, step, k), Box-Muller in binary32 without libm.
 * eps = 0 is legal (all copies equal the masters).  Errors: NULL, SHAPE (q < 1 or q > q_max),
 * CONFIG (eps not finite or negative). */
mpz_status mpz_regen_noise(mpz_model* m, uint64_t seed, uint32_t step, int32_t q, float eps);

/* Algorithm 1, the loss evaluations of both loops for all copies in one batched pass (Section 3, MP-LoRA; outer- and
 * inner-loop parallelisation): every copy sees the same E x S token batch, the frozen weights
 * are shared, each copy's low-rank path uses its own perturbed factors.
 *   tokens      [dev] int32[E*S], ids in [0, vocab) (not checked on device)
 *   labels      [dev] int32[E] class ids in {0,1} for the last-position modes; ignored (may be
 *               NULL) for MPZ_LOSS_NEXT_TOKEN_ALL_POS
 *   losses_out  [dev] fp32[2q], mean loss of each copy over its loss positions
 * Requires a preceding mpz_regen_noise (its q is used).  Errors: NULL, STATE, SHAPE
 * (E < 1, E > E_max, S < 2, S > S_max). */
mpz_status mpz_forward_perturbed(mpz_model* m, const int32_t* tokens, const int32_t* labels,
                                 int32_t E, int32_t S, float* losses_out);

/* For callers that cannot allocate or size a workspace when they call (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): mpz_forward_perturbed with the per-pass activations (residual stream,
 * operand rows, bottleneck activations, loss scratch) in a file-scope device array of the library instead of the
 * caller's workspace.  Same arguments, same kernels, same losses bit for bit (the pass is issued on the model's stream
 * alone).  Calls no hipMalloc / hipFree and creates no stream or event.  The array holds
 * mpz_noalloc_scratch_bytes() = 16 MiB per GPU for the life of the process; a pass whose activations for
 * (2q, E, S) need more is refused with MPZ_ERR_WORKSPACE (the message states both sizes) and nothing is launched.
 * Inputs, outputs, the perturbed factor copies of mpz_regen_noise and the tables made by mpz_init_model stay where
 * they are (caller memory).  Every call on one GPU shares that GPU's array and nothing in it needs clearing (each
 * buffer is written before it is read), but calls that overlap in time on one GPU - two models, two streams - race:
 * serialise them.  Other errors as mpz_forward_perturbed, plus STATE while mpz_profile_begin is in effect or when the
 * current device is not the model's, and DEVICE when the array's address cannot be obtained. */
mpz_status mpz_forward_perturbed_noalloc(mpz_model* m, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                                         float* losses_out);
size_t mpz_noalloc_scratch_bytes(void);

/* The same pass restricted to the copies [copy_begin, copy_begin + n_copies) of the last mpz_regen_noise; writes
 * losses_out[copy_begin .. copy_begin + n_copies) and leaves the other entries untouched.  n_copies = 1 in a loop
 * over all 2q copies is the sequential evaluation that Section 3 starts from (one forward pass per perturbed
 * parameter vector, as in MeZO with q > 1, Appendix A); n_copies = q over the + copies and then the - copies is
 * outer-loop parallelisation alone.  Every copy's loss is bit-identical to what mpz_forward_perturbed gives it.
 * Errors as mpz_forward_perturbed, plus SHAPE for a range outside [0, 2q). */
mpz_status mpz_forward_copies(mpz_model* m, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                              int32_t copy_begin, int32_t n_copies, float* losses_out);

/* As mpz_forward_copies, for every copy_step-th copy: the pass evaluates copies copy_begin + copy_step * i, i <
 * n_copies, and writes losses_out[copy_begin + copy_step * i].  With copy_step = 2, copy_begin = 0 / 1 and n_copies = q
 * this is the outer loop alone (Section 3): all q queries in one pass, the + and the - perturbation in two passes.
 * Same losses, bit for bit, as the batched pass.  Errors as mpz_forward_copies (SHAPE also for copy_step < 1). */
mpz_status mpz_forward_copies_strided(mpz_model* m, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                                      int32_t copy_begin, int32_t n_copies, int32_t copy_step, float* losses_out);

/* mpz_forward_perturbed on a right-padded batch of sequences of unequal length (Section 3 argues that spending the
 * batch on q queries of E = B / q sequences shortens the padding that batching brings): sequence e has lengths[e] real
 * tokens, 2 <= lengths[e] <= S (values outside are clamped), followed by padding whose token ids are arbitrary but
 * inside the vocabulary.  Attention is causal, so no real token ever sees the padding; the loss is taken over real
 * tokens only: next-token mode averages over the positions p < lengths[e] - 1 of all sequences, the last-position
 * modes read position lengths[e] - 1.  With lengths[e] = S for all e the losses are bit-identical to
 * mpz_forward_perturbed.
 *   lengths   [dev] int32[E]
 * Errors as mpz_forward_perturbed, plus NULL for lengths and SHAPE for d_ffn < 2 d_model / element size. */
mpz_status mpz_forward_perturbed_varlen(mpz_model* m, const int32_t* tokens, const int32_t* labels, const int32_t* lengths,
                                        int32_t E, int32_t S, float* losses_out);

/* The same batch without the padding: the E sequences of unequal length lie back to back ("packed"), and every
 * copy of the stacked pass holds rows = total_tokens rounded up to a multiple of 32 (filler rows after the last
 * sequence; they belong to no sequence, see no attention and carry no loss).  Every row-wise kernel and every GEMM
 * then runs over real tokens only; attention runs per sequence on its own rows; positions (learned or rotary) count
 * from each sequence's first token.  The losses equal those of mpz_forward_perturbed_varlen on the padded form of
 * the same batch (bit for bit with the fp32 kernels).
 *   tokens       [dev] int32[rows]: the sequences' tokens back to back, then filler ids inside the vocabulary
 *   labels       [dev] int32[E] class ids (last-position modes) or NULL (next-token mode)
 *   cu_seqlens   [dev] int32[E + 1]: cu[0] = 0, sequence e holds rows cu[e] .. cu[e+1] - 1, cu[E] = total_tokens;
 *                every sequence holds at least one token and at most max_len (not checked on the device)
 *   max_len      the longest sequence, 2 <= max_len <= S_max (sizes the attention launch)
 * Errors: NULL; STATE (before mpz_regen_noise); SHAPE (E < 1, max_len or total_tokens out of range, rows >
 * E_max * S_max, in the last-position modes 2q E > 2 q_max E_max); DEVICE. */
mpz_status mpz_forward_perturbed_packed(mpz_model* m, const int32_t* tokens, const int32_t* labels,
                                        const int32_t* cu_seqlens, int32_t E, int32_t total_tokens, int32_t max_len,
                                        float* losses_out);

/* Algorithm 1, projected gradient and update: g_k = (l_{2k} - l_{2k+1}) / (2 eps) in fp64 from the fp32 losses, then
 * theta_l <- theta_l - lr (1/q) sum_k g_k z_k on the fp32 masters, z_k replayed from the (seed,
 * step, q, eps) of the last mpz_regen_noise.
 *   losses           [dev] fp32[2q]
 *   proj_grads_out   [dev] fp32[q] receives g_k, or NULL
 * Errors: NULL, STATE (no preceding regen_noise), CONFIG (that regen_noise used eps = 0: the
 * two-point quotient is undefined; lr not finite). */
mpz_status mpz_zo_update(mpz_model* m, const float* losses, float lr, float* proj_grads_out);

/* Stateful variant of the step (Algorithm 2, the "mobile" module, here for q queries and both factors): the
 * perturbed copies of the last mpz_regen_noise / mpz_zo_update_regen are still in the workspace, so the direction of
 * pair k is read back from them, diff_k = (theta_k(+) - theta_k(-)) / 2, instead of being regenerated:
 *   theta_l <- theta_l - sum_k (lr g_k / q) diff_k / eps,    g_k as in mpz_zo_update,
 * and, in the same pass over the factors, the pairs are re-centred on the new masters with fresh noise,
 * theta_l +- eps z'_k, z'_k drawn from (seed, next_step, k) with the seed, q and eps of the stored pairs.  One noise
 * generation per step instead of two; the model is left ready for the next mpz_forward_perturbed (no
 * mpz_regen_noise in between).  Up to the rounding of theta +- eps z, diff_k / eps is z_k and the result is that of
 * mpz_zo_update followed by mpz_regen_noise(seed, next_step, q, eps).
 *   losses           [dev] fp32[2q], proj_grads_out [dev] fp32[q] or NULL
 * Errors: NULL, STATE (no stored pairs: no mpz_regen_noise yet, or mpz_zo_update since), CONFIG (pairs made with
 * eps = 0; lr not finite). */
mpz_status mpz_zo_update_regen(mpz_model* m, const float* losses, float lr, uint32_t next_step, float* proj_grads_out);

/* Test hooks (not on the hot path). */
/* z for one LoRA factor of one query: z_out [dev] fp32[rows*cols], row-major. */
mpz_status mpz_debug_noise(mpz_model* m, uint64_t seed, uint32_t step, int32_t k, int32_t tensor_id,
                           float* z_out);
/* Measurement aid for the noise kernels: generates q normals-quadruples for each of n_groups counter values exactly
 * as mpz_regen_noise does (Philox call + Box-Muller transform), keeps them in registers and writes nothing (one
 * word per thread is stored only if a checksum hits an impossible value): the arithmetic ceiling of the generator,
 * against which the rate of the kernels that also move the factors is reported.  sink [dev] fp32[1]. */
mpz_status mpz_debug_noise_alu_probe(int64_t n_groups, int32_t q, float* sink, void* hip_stream);
/* The binary32 normal transform alone: words [dev] uint32[4*n4] -> normals [dev] fp32[4*n4]
 * (group j: words 4j..4j+3 -> Box-Muller pairs (0,1) and (2,3)).  hip_stream as in init. */
mpz_status mpz_debug_normals_from_words(const uint32_t* words, size_t n4, float* normals_out, void* hip_stream);
/* Copy c's perturbed factors as the forward pass sees them, in master layout: out [dev] fp32[numel]. */
mpz_status mpz_debug_perturbed_copy(mpz_model* m, int32_t c, float* out);

/* The three stages of mpz_forward_perturbed, run separately on a caller-held stacked residual
 * stream h [dev] fp32[2q*E*S, d_model] (rows in copy-major order), so that each stage can be checked
 * on given inputs: embedding -> h_out; decoder blocks [layer_begin, layer_end) in place on h; final
 * norm + head + per-copy mean loss from h (lengths: [dev] int32[E] as in mpz_forward_perturbed_varlen, or NULL).
 * Same preconditions and errors as mpz_forward_perturbed. */
mpz_status mpz_debug_embed(mpz_model* m, const int32_t* tokens, int32_t E, int32_t S, float* h_out);
mpz_status mpz_debug_run_layers(mpz_model* m, float* h, int32_t layer_begin, int32_t layer_end, int32_t E, int32_t S);
mpz_status mpz_debug_head_loss(mpz_model* m, const float* h, const int32_t* tokens, const int32_t* labels,
                               const int32_t* lengths, int32_t E, int32_t S, float* losses_out);

/* Test hooks for single operations of a bf16 / any model on caller-provided operands:
 * - the q/k/v projection of the MP-LoRA layer (Section 3: Y = X W + (X A)(.)B, plus bias) of block `layer` for all
 *   stacked copies: x [dev] model dtype [2q*E*S, d] -> out [dev] fp32 [2q*E*S, d + 2 d_kv], before the rotary
 *   embedding and before rounding to the operand type (bf16 models only);
 * - causal attention: qkv [dev] model dtype [n_seq*S, d + 2 d_kv] (q | k | v) -> out [dev] model dtype [n_seq*S, d]. */
mpz_status mpz_debug_qkv_projection(mpz_model* m, const void* x, int32_t layer, int32_t E, int32_t S, float* out);
mpz_status mpz_debug_attention(mpz_model* m, const void* qkv, int32_t n_seq, int32_t S, void* out);

/* Test / measurement hook: the bf16 MFMA GEMM alone, out[M, N] = act(x[M, K] w[N, K]^T + bias), all [dev], x and w bf16,
 * out bf16 or fp32 (out_f32), act = -1 (none), MPZ_ACT_RELU, MPZ_ACT_GELU_ERF, or MPZ_ACT_SWIGLU (then w has 2N rows,
 * gate then up, bias 2N, out = SiLU(gate) * up); tile_cfg 0 = chosen by shape; 1, 6, 9, 10, 11, 12 = that block-tile configuration (other numbers fall back to the choice by shape).  Errors: NULL, SHAPE (K % 64, N % 4). */
mpz_status mpz_debug_gemm_bf16(int32_t M, int32_t N, int32_t K, const void* x, const void* w, const float* bias,
                               int32_t act, void* out, int32_t out_f32, int32_t tile_cfg, void* hip_stream);
/* The same GEMM through the split-K path that passes over at most 256 stacked tokens take (k_splits blocks per output
 * tile stream disjoint shares of K and leave fp32 partial sums in `partial`; a second kernel adds them in a fixed order
 * and applies bias, activation, the fp32 residual [M, N] (may be NULL) and the output type).  k_splits = 0: the count
 * the library would choose for this shape (1 = no split: the one-block kernel runs); >= 2: forced.  partial [dev]
 * fp32[partial_elems], at least k_splits * M * N (SwiGLU: 2 N) elements.  mpz_debug_gemm_splits returns the chosen
 * count.  Errors: NULL, SHAPE. */
mpz_status mpz_debug_gemm_bf16_splitk(int32_t M, int32_t N, int32_t K, const void* x, const void* w, const float* bias,
                                      int32_t act, const float* residual, void* out, int32_t out_f32, int32_t k_splits,
                                      float* partial, size_t partial_elems, void* hip_stream);
int32_t mpz_debug_gemm_splits(int32_t M, int32_t N, int32_t K, int32_t dual, size_t partial_elems);
/* Test hook: allow (default) or forbid the split-K GEMMs inside a model's passes. */
mpz_status mpz_debug_set_split_k(mpz_model* m, int32_t enable);

/* Test hook: the split-K GEMM on 4-bit normal-float weights looked up in its own operand load (what a pass over at most
 * 256 stacked tokens does with weight_quant = NF4): w_codes [dev] [N, K / 2] bytes (SwiGLU: [2N, K / 2], gate rows then up
 * rows; two codes per byte, low nibble first), w_absmax [dev] [N or 2N, K / 64] fp32, 16- and 4-byte aligned; the other
 * arguments as mpz_debug_gemm_bf16_splitk with 2 <= k_splits <= 64.  The result has the bits of mpz_debug_dequant_nf4
 * followed by mpz_debug_gemm_bf16_splitk with the same k_splits.  Errors: NULL, SHAPE, DEVICE. */
mpz_status mpz_debug_gemm_nf4_splitk(int32_t M, int32_t N, int32_t K, const void* x, const void* w_codes, const float* w_absmax,
                                     const float* bias, int32_t act, const float* residual, void* out, int32_t out_f32,
                                     int32_t k_splits, float* partial, size_t partial_elems, void* hip_stream);

/* The same with weight-only int8 weights: w_codes [dev] int8 [N, K] (SwiGLU: [2N, K]), w_scale [dev] fp32 [N] ([2N]),
 * 16-byte aligned; out = act(x (codes * scale)^T + bias).  Tile configurations 1, 6, 11 and 12 only (others fall back to
 * the choice by shape). */
mpz_status mpz_debug_gemm_int8(int32_t M, int32_t N, int32_t K, const void* x, const void* w_codes, const float* w_scale,
                               const float* bias, int32_t act, void* out, int32_t out_f32, int32_t tile_cfg,
                               void* hip_stream);

/* Measurement hook: the matrix cores alone.  blocks x 8 waves each issue iters x 8 MFMAs (32x32x16 bf16, 32768 FLOP
 * each) on independent accumulators; the operand fragments are taken from operands [dev] bf16[12288] (16-byte aligned),
 * so the caller chooses the bit patterns; with_lds = 1 re-reads the 4 + 2 fragments of every step from LDS before its MFMAs,
 * 2 does the fragment reads alone (no MFMA: the LDS read rate).  out [dev] fp32[blocks * 512] receives checksums.  The caller times it (events around the call).
 * Errors: NULL, SHAPE, CONFIG. */
mpz_status mpz_debug_mfma_probe(const void* operands, int32_t blocks, int32_t iters, int32_t with_lds, float* out,
                                void* hip_stream);

/* Measurement hook: the read rate of the memory system for the access pattern of a GEMM's weight operand.  buf [dev] is
 * read as [rows][row_bytes] (16-byte aligned, never written); a block of 256 threads owns rows_per_block consecutive
 * rows and one of k_splits equal shares of each row, and walks its share in tiles of rows_per_block x seg_bytes, the next
 * tile in flight while the current one is consumed (rows_per_block = 128, seg_bytes = 128: the 128 x 64 bf16 tile of the
 * few-token GEMMs; rows_per_block = 1 with a long seg_bytes: one sequential stream per block).  lds_bytes of dynamic
 * LDS per block limit how many blocks a CU holds.  mode bit 0: every tile is accompanied by the tile of rows
 * 0 .. rows_per_block - 1 at the same row offset (what the activation operand of a GEMM adds: the same for all blocks);
 * bit 1: the tiles pass through LDS with two block barriers per tile (needs lds_bytes >= the staged bytes).  out [dev] uint32[rows / rows_per_block * k_splits] receives
 * checksums.  The caller times it.  Errors: NULL, CONFIG (alignment), SHAPE (rows % rows_per_block, row_bytes %
 * (seg_bytes * k_splits), rows_per_block * seg_bytes not 4, 8, 16, 32 or 64 KiB, lds_bytes outside [0, 160 KiB] or too small for mode bit 1). */
mpz_status mpz_debug_hbm_read_probe(const void* buf, int64_t rows, int64_t row_bytes, int32_t rows_per_block, int32_t seg_bytes,
                                    int32_t k_splits, int32_t lds_bytes, int32_t mode, uint32_t* out, void* hip_stream);

/* Test hook: the dequantisation of weight_quant = NF4 on its own: codes [dev] n_elems / 2 bytes (two codes per byte,
 * low nibble first), absmax [dev] [n_elems / 64] fp32, out [dev] [n_elems] bf16 = bf16(level[code] * max).
 * Errors: NULL, SHAPE (n_elems < 64 or not a multiple of 64). */
mpz_status mpz_debug_dequant_nf4(const void* codes, const float* absmax, void* out, int64_t n_elems, void* hip_stream);

/* Test hook: simple_only != 0 routes every stage through the shape-agnostic kernels (the only path of
 * fp32 models); 0 restores the default (bf16 models use the MFMA kernels wherever a shape allows).
 * Invalidates the perturbed copies: call mpz_regen_noise again. */
mpz_status mpz_debug_set_kernel_path(mpz_model* m, int32_t simple_only);

/* Test hook: allow (default) or forbid the two-halves schedule of mpz_forward_perturbed: for small models (every
 * GEMM on the 128-wide tiles, label-subset loss) the pass is issued as two halves of q copies each on the caller's
 * stream and on an internal second stream of the same priority, forked from and joined to the caller's stream by
 * events, so that the halves' kernels overlap.  Losses are bit-identical either way. */
mpz_status mpz_debug_set_two_halves(mpz_model* m, int32_t enable);
/* Number of streams the last mpz_forward_perturbed was issued on: 2 with the two-halves schedule, 1 without, 0
 * before the first pass (or for a NULL handle). */
int32_t mpz_debug_last_pass_streams(const mpz_model* m);

/* Test hook: allow (default) or forbid the kernels that fuse a pre-norm with its neighbour: a block's first pre-norm with
 * the LoRA bottleneck of the q/k/v projections in one pass over the residual rows (bf16 models with d_model 768, 1024
 * or 2048), and, in passes over few tokens, the reduction of a split-K projection into the residual stream with the
 * pre-norm that follows it.  Without them each runs as two kernels.  Same bits either way. */
mpz_status mpz_debug_set_fused_norm_lora(mpz_model* m, int32_t enable);

/* Test hook: allow (default) or forbid the kernel that writes the perturbed factors of a bf16 model straight into the
 * bf16 hi / lo MFMA operand layouts; without it mpz_regen_noise writes fp32 copies first and packs them in a second
 * kernel.  Same bits either way.  Invalidates the perturbed copies: call mpz_regen_noise again. */
mpz_status mpz_debug_set_fused_perturb_pack(mpz_model* m, int32_t enable);

/* Test hook: force one block-tile configuration (1, 6, 9, 10, 11 or 12; 0 = chosen by shape) for every MFMA GEMM of the model's
 * passes, so that small test shapes can exercise the configurations large workloads select.  Errors: NULL, CONFIG. */
mpz_status mpz_debug_set_tile_config(mpz_model* m, int32_t tile_cfg);

/* Measurement hook: between _begin and _end every kernel launch of the three hot-path calls is bracketed by HIP
 * events on the model's stream and booked under a category.  _end synchronises the stream and fills
 * out[MPZ_PROF_COUNT] [host] with, per category, the summed kernel time (ms), the number of launches, the
 * algorithmic FLOPs (GEMM: 2 M N K; attention: the causal-useful Q K^T and P V work) and the algorithmic bytes
 * (one read of each input, one write of each output).  Adds event overhead: do not enable it inside a region
 * whose wall-clock is reported.  Errors: NULL, STATE (end without begin), DEVICE. */
enum {
  MPZ_PROF_GEMM = 0,      /* base-weight GEMMs with the fused per-copy rank-r term, incl. the LM head */
  MPZ_PROF_ATTENTION = 1,
  MPZ_PROF_NORM = 2,
  MPZ_PROF_LORA_DOWN = 3, /* bottleneck t = s x A_c */
  MPZ_PROF_NOISE = 4,     /* regenerate noise, write the perturbed copies */
  MPZ_PROF_UPDATE = 5,    /* two-point estimate + seed-replayed update */
  MPZ_PROF_EMBED = 6,
  MPZ_PROF_ROPE = 7,
  MPZ_PROF_LOSS = 8,      /* targets, per-row cross-entropy, per-copy mean */
  MPZ_PROF_OTHER = 9,
  MPZ_PROF_PACK = 10,     /* perturbed copies -> bf16 hi/lo MFMA operand layouts */
  MPZ_PROF_COUNT = 11
};
typedef struct { double ms; int64_t launches; double flops; double bytes; } mpz_profile_entry;
mpz_status mpz_profile_begin(mpz_model* m);
mpz_status mpz_profile_end(mpz_model* m, mpz_profile_entry* out /*[host] MPZ_PROF_COUNT entries*/);

void mpz_destroy(mpz_model* m);
const char* mpz_last_error(const mpz_model* m /* may be NULL */);
const char* mpz_status_string(mpz_status s);

#ifdef __cplusplus
}
#endif
#endif /* MPZ_H */
