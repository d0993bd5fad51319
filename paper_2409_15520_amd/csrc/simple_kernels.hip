// Straightforward kernels for every step of the batched MP-LoRA forward pass (Section 3: one pass over
// n = 2q stacked copies, shared W, per-copy low-rank factors).  They take any shape and both storage
// types: fp32 storage accumulates in fp64 and rounds once per stored element, bf16 storage accumulates
// in fp32.  The bf16 hot path replaces the GEMM / attention kernels here with MFMA kernels; these stay
// as the fp32-model path and as the shape-agnostic fallback.
#include "common.h"
#include "../../include/mpz.h"

namespace mpz {
namespace {

template <typename ST> struct Traits;
template <> struct Traits<float> {
  using AT = double;
  static __device__ __forceinline__ AT load(const float* p, int64_t i) { return (double)p[i]; }
  static __device__ __forceinline__ void store(float* p, int64_t i, AT v) { p[i] = (float)v; }
  static __device__ __forceinline__ AT round_op(AT v) { return (double)(float)v; }
  // perturbed factor as the contraction sees it: the fp32 value itself
  static __device__ __forceinline__ AT factor(float v) { return (double)v; }
  static __device__ __forceinline__ AT exp_(AT v) { return exp(v); }
  static __device__ __forceinline__ AT erf_(AT v) { return erf(v); }
  static __device__ __forceinline__ AT log_(AT v) { return log(v); }
  static __device__ __forceinline__ AT rsqrt_(AT v) { return 1.0 / sqrt(v); }
};
template <> struct Traits<bf16_t> {
  using AT = float;
  static __device__ __forceinline__ AT load(const bf16_t* p, int64_t i) { return bf16_to_f32(p[i]); }
  static __device__ __forceinline__ void store(bf16_t* p, int64_t i, AT v) { p[i] = f32_to_bf16(v); }
  static __device__ __forceinline__ AT round_op(AT v) { return bf16_to_f32(f32_to_bf16(v)); }
  // bf16 hi + lo split of the fp32 factor (the sum is exact in fp32)
  static __device__ __forceinline__ AT factor(float v) {
    float hi = bf16_to_f32(f32_to_bf16(v));
    float lo = bf16_to_f32(f32_to_bf16(v - hi));
    return hi + lo;
  }
  static __device__ __forceinline__ AT exp_(AT v) { return expf(v); }
  static __device__ __forceinline__ AT erf_(AT v) { return erff(v); }
  static __device__ __forceinline__ AT log_(AT v) { return logf(v); }
  static __device__ __forceinline__ AT rsqrt_(AT v) { return 1.0f / sqrtf(v); }
};

template <typename T> __device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
template <typename T> __device__ __forceinline__ T wave_max(T v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { T other = __shfl_xor(v, o, 64); v = other > v ? other : v; }
  return v;
}
// block-wide reductions for 256-thread blocks, fixed order (deterministic)
template <typename T> __device__ __forceinline__ T block_sum(T v, T* red /*[4]*/) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  T r = red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r += red[i];
  return r;
}
template <typename T> __device__ __forceinline__ T block_max(T v, T* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  T r = red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = red[i] > r ? red[i] : r;
  return r;
}

// ---- embedding --------------------------------------------------------------------------------
template <typename ST>
__global__ void embed_kernel(const int32_t* __restrict__ tokens, const ST* __restrict__ emb, const ST* __restrict__ pos,
                             const int32_t* __restrict__ row_pos, float* __restrict__ h, int n_copies, int E, int S, int d) {
  using Tr = Traits<ST>;
  int64_t row = blockIdx.x;                       // (c*E + e)*S + p
  int rc = (int)(row % ((int64_t)E * S));         // row inside the copy = index into the token batch
  int p = row_pos != nullptr ? row_pos[rc] : rc % S;   // packed batch: position inside the row's own sequence
  int tok = tokens[rc];
  for (int i = threadIdx.x; i < d; i += blockDim.x) {
    typename Tr::AT v = Tr::load(emb, (int64_t)tok * d + i);
    if (pos != nullptr) v += Tr::load(pos, (int64_t)p * d + i);
    h[row * d + i] = (float)v;
  }
}

// ---- LayerNorm / RMSNorm: fp32 residual row -> operand type -------------------------------------
template <typename ST>
__global__ void __launch_bounds__(256) norm_kernel(int kind, float eps, const float* __restrict__ h, int64_t h_row_stride,
                                                   const float* __restrict__ g, const float* __restrict__ b,
                                                   ST* __restrict__ out, int d) {
  using Tr = Traits<ST>;
  using AT = typename Tr::AT;
  __shared__ AT red[4];
  const float* hr = h + (int64_t)blockIdx.x * h_row_stride;
  AT s = 0;
  for (int i = threadIdx.x; i < d; i += 256) s += (AT)hr[i];
  AT mean = 0;
  if (kind == MPZ_NORM_LAYERNORM) mean = block_sum(s, red) / (AT)d;
  AT v = 0;
  for (int i = threadIdx.x; i < d; i += 256) { AT c = (AT)hr[i] - mean; v += c * c; }
  AT var = block_sum(v, red) / (AT)d;
  AT rstd = Tr::rsqrt_(var + (AT)eps);
  for (int i = threadIdx.x; i < d; i += 256) {
    AT y = ((AT)hr[i] - mean) * rstd * (AT)g[i];
    if (b != nullptr) y += (AT)b[i];
    Tr::store(out, (int64_t)blockIdx.x * d + i, y);
  }
}

// ---- LoRA bottleneck t = OP(scale * x A_c), one thread per (row, bottleneck column) ------------------
template <typename ST>
__global__ void __launch_bounds__(256) lora_down_kernel(LoraDownArgs a) {
  using Tr = Traits<ST>;
  using AT = typename Tr::AT;
  int R = a.n_targets * a.rank;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)a.T * R) return;
  int m = (int)(idx / R), j = (int)(idx % R);
  int tgt = j / a.rank, jj = j % a.rank;
  int copy = m / a.rows_per_copy;
  const float* A = a.Ac[tgt] + (int64_t)copy * a.copy_stride;
  const ST* x = (const ST*)a.x + (int64_t)m * a.K;
  AT acc = 0;
  for (int k = 0; k < a.K; ++k) acc += Tr::load(x, k) * Tr::factor(A[(int64_t)k * a.rank + jj]);
  Tr::store((ST*)a.t, idx, acc * (AT)a.scale);
}

// ---- linear: out = epilogue(x W^T), 64x64 tile, 4x4 per thread -------------------------------------
template <typename ST>
__global__ void __launch_bounds__(256) linear_kernel(LinearArgs a) {
  using Tr = Traits<ST>;
  using AT = typename Tr::AT;
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ AT xs[BK][BM + 1];
  __shared__ AT ws[BK][BN + 1];
  const ST* x = (const ST*)a.x;
  const ST* w = (const ST*)a.w;
  int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  int lr = threadIdx.x / 4, lk = (threadIdx.x % 4) * 4;
  AT acc[4][4] = {};
  for (int k0 = 0; k0 < a.K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int k = k0 + lk + i;
      int m = m0 + lr, n = n0 + lr;
      xs[lk + i][lr] = (m < a.M && k < a.K) ? Tr::load(x, (int64_t)m * a.K + k) : (AT)0;
      ws[lk + i][lr] = (n < a.N && k < a.K) ? Tr::load(w, (int64_t)n * a.K + k) : (AT)0;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      AT xv[4], wv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { xv[i] = xs[k][ty * 4 + i]; wv[i] = ws[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += xv[i] * wv[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= a.M) continue;
    int copy = m / a.rows_per_copy;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= a.N) continue;
      AT v = acc[i][j];
      for (int s = 0; s < a.n_seg; ++s) {
        const LoraSeg& sg = a.seg[s];
        if (n >= sg.col_begin && n < sg.col_end) {
          int kout = sg.col_end - sg.col_begin;
          const ST* t = (const ST*)sg.t + (int64_t)m * sg.t_stride + sg.t_off;
          const float* B = sg.Bc + (int64_t)copy * sg.copy_stride + (n - sg.col_begin);
          AT dl = 0;
          for (int r = 0; r < a.rank; ++r) dl += Tr::load(t, r) * Tr::factor(B[(int64_t)r * kout]);
          v += dl;
        }
      }
      if (a.bias != nullptr) v += (AT)a.bias[n];
      if (a.act == MPZ_ACT_RELU) v = v > (AT)0 ? v : (AT)0;
      else if (a.act == MPZ_ACT_GELU_ERF) v = (AT)0.5 * v * ((AT)1 + Tr::erf_(v * (AT)0.70710678118654752440));
      int64_t o = (int64_t)m * a.N + n;
      if (a.residual != nullptr) v += (AT)a.residual[o];
      if (a.out_kind == 0) Tr::store((ST*)a.out, o, v);
      else if (a.out_kind == 1) ((float*)a.out)[o] = (float)v;
      else ((AT*)a.out)[o] = v;
    }
  }
}

// ---- rotary embedding + conversion of the q/k/v staging buffer -----------------------------------
template <typename ST>
__global__ void __launch_bounds__(256) rope_convert_kernel(const typename Traits<ST>::AT* __restrict__ stg, ST* __restrict__ out,
                                                           int64_t total, int S, int n_cols, int d_head, int n_rot_heads,
                                                           const float* __restrict__ cos_tab, const float* __restrict__ sin_tab,
                                                           const int32_t* __restrict__ row_pos) {
  using Tr = Traits<ST>;
  using AT = typename Tr::AT;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int col = (int)(idx % n_cols);
  int64_t row = idx / n_cols;
  int head = col / d_head, i = col % d_head, half = d_head / 2;
  AT v = stg[idx];
  if (head < n_rot_heads) {
    int p = (int)(row % S);
    if (row_pos != nullptr) p = row_pos[p];       // packed batch (S = rows per copy): position inside the sequence
    // binary32 staging (bf16 models): one rounded product and one fma, exactly as the GEMM's fused rotary epilogue
    if (i < half) {
      AT c = (AT)cos_tab[p * half + i], s = (AT)sin_tab[p * half + i];
      if constexpr (sizeof(AT) == 4) v = fmaf(v, c, -__fmul_rn(stg[idx + half], s));
      else v = v * c - stg[idx + half] * s;
    } else {
      AT c = (AT)cos_tab[p * half + i - half], s = (AT)sin_tab[p * half + i - half];
      if constexpr (sizeof(AT) == 4) v = fmaf(v, c, __fmul_rn(stg[idx - half], s));
      else v = v * c + stg[idx - half] * s;
    }
  }
  Tr::store(out, idx, v);
}

// ---- causal attention, one wave per (sequence, head, query position) --------------------------------
template <typename ST>
__global__ void __launch_bounds__(64) attention_kernel(const ST* __restrict__ qkv, int qkv_stride, ST* __restrict__ out,
                                                       int S, int H, int Hkv, int dh, float scale,
                                                       const int32_t* __restrict__ cu, int E, int rows_per_copy) {
  using Tr = Traits<ST>;
  using AT = typename Tr::AT;
  extern __shared__ unsigned char smem_raw[];
  AT* sc = (AT*)smem_raw;                 // [S] scores / probabilities
  AT* qv = sc + S;                        // [dh]
  int i = blockIdx.x % S;
  int head = (blockIdx.x / S) % H;
  int64_t seq = blockIdx.x / ((int64_t)S * H);
  int kvh = head / (H / Hkv);
  int d = H * dh, dkv = Hkv * dh;
  int64_t row0 = seq * S;
  if (cu != nullptr) {                    // packed batch: S is the longest sequence, this one may be shorter
    const int e = (int)(seq % E);
    row0 = (seq / E) * rows_per_copy + cu[e];
    if (i >= cu[e + 1] - cu[e]) return;   // block-uniform
  }
  int64_t row_i = row0 + i;
  const ST* qp = qkv + row_i * qkv_stride + head * dh;
  for (int c = threadIdx.x; c < dh; c += 64) qv[c] = Tr::load(qp, c);
  __syncthreads();
  AT mx = -1e30;
  for (int j = threadIdx.x; j <= i; j += 64) {
    const ST* kp = qkv + (row0 + j) * qkv_stride + d + kvh * dh;
    AT dot = 0;
    for (int c = 0; c < dh; ++c) dot += qv[c] * Tr::load(kp, c);
    AT s = (AT)(float)dot * (AT)scale;
    sc[j] = s;
    mx = s > mx ? s : mx;
  }
  mx = wave_max(mx);
  AT sum = 0;
  for (int j = threadIdx.x; j <= i; j += 64) {
    AT p = Tr::round_op(Tr::exp_(sc[j] - mx));
    sc[j] = p;
    sum += p;
  }
  sum = wave_sum(sum);
  __syncthreads();
  for (int c = threadIdx.x; c < dh; c += 64) {
    AT acc = 0;
    for (int j = 0; j <= i; ++j) acc += sc[j] * Tr::load(qkv, (row0 + j) * qkv_stride + d + dkv + kvh * dh + c);
    Tr::store(out, row_i * d + head * dh + c, acc / sum);
  }
}

template <typename ST>
__global__ void __launch_bounds__(256) swiglu_kernel(const typename Traits<ST>::AT* __restrict__ stg, ST* __restrict__ out,
                                                     int64_t total, int f) {
  using Tr = Traits<ST>;
  using AT = typename Tr::AT;
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  int64_t row = idx / f;
  int c = (int)(idx % f);
  AT g = stg[row * 2 * f + c], u = stg[row * 2 * f + f + c];
  if constexpr (sizeof(AT) == 4) Tr::store(out, idx, silu_mul_f32(g, u));      // bf16 models: as the fused epilogue
  else Tr::store(out, idx, g / ((AT)1 + Tr::exp_(-g)) * u);
}

// ---- loss ----------------------------------------------------------------------------------------
template <typename AT>
__global__ void __launch_bounds__(256) ce_rows_kernel(const float* __restrict__ logits, int64_t row_stride, int n_cols,
                                                      const int32_t* __restrict__ target, float* __restrict__ ce) {
  __shared__ AT red[4];
  int r = blockIdx.x;
  int tg = target[r];
  if (tg < 0) { if (threadIdx.x == 0) ce[r] = 0.f; return; }
  const float* lg = logits + (int64_t)r * row_stride;
  AT mx = -1e30;
  for (int c = threadIdx.x; c < n_cols; c += 256) { AT v = (AT)lg[c]; mx = v > mx ? v : mx; }
  mx = block_max(mx, red);
  AT s = 0;
  for (int c = threadIdx.x; c < n_cols; c += 256) {
    if constexpr (sizeof(AT) == 8) s += exp((AT)lg[c] - mx); else s += expf((AT)lg[c] - mx);
  }
  s = block_sum(s, red);
  if (threadIdx.x == 0) {
    AT lse;
    if constexpr (sizeof(AT) == 8) lse = mx + log(s); else lse = mx + logf(s);
    ce[r] = (float)(lse - (AT)lg[tg]);
  }
}

template <typename ST>
__global__ void __launch_bounds__(64) subset_logits_kernel(const ST* __restrict__ xf, const ST* __restrict__ head, int d,
                                                           int tok0, int tok1, float* __restrict__ logits2) {
  using Tr = Traits<ST>;
  using AT = typename Tr::AT;
  int r = blockIdx.x;
  AT a0 = 0, a1 = 0;
  for (int i = threadIdx.x; i < d; i += 64) {
    AT x = Tr::load(xf, (int64_t)r * d + i);
    a0 += x * Tr::load(head, (int64_t)tok0 * d + i);
    a1 += x * Tr::load(head, (int64_t)tok1 * d + i);
  }
  a0 = wave_sum(a0); a1 = wave_sum(a1);
  if (threadIdx.x == 0) { logits2[2 * r] = (float)a0; logits2[2 * r + 1] = (float)a1; }
}

// lengths (optional): sequences are right-padded to S; only real tokens carry a loss.  Values are clamped to [2, S].
__device__ __forceinline__ int seq_len(const int32_t* lengths, int e, int S) {
  if (lengths == nullptr) return S;
  int L = lengths[e];
  return L < 2 ? 2 : (L > S ? S : L);
}

__global__ void make_targets_kernel(int mode, const int32_t* __restrict__ tokens, const int32_t* __restrict__ labels,
                                    const int32_t* __restrict__ lengths, const int32_t* __restrict__ row_end, int tok0,
                                    int tok1, int32_t* __restrict__ target, int n_copies, int E, int S) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (mode == MPZ_LOSS_NEXT_TOKEN_ALL_POS) {
    if (idx >= (int64_t)n_copies * E * S) return;
    if (row_end != nullptr) {                     // packed batch (E = 1, S = rows per copy): the next row of the same sequence
      int rc = (int)(idx % S);
      target[idx] = (rc + 1 < row_end[rc]) ? tokens[rc + 1] : -1;
      return;
    }
    int p = (int)(idx % S), e = (int)((idx / S) % E);
    target[idx] = (p < seq_len(lengths, e, S) - 1) ? tokens[e * S + p + 1] : -1;
  } else {
    if (idx >= (int64_t)n_copies * E) return;
    int e = (int)(idx % E);
    int y = labels[e];
    target[idx] = (mode == MPZ_LOSS_LAST_POS_LABEL_SUBSET) ? y : (y == 0 ? tok0 : tok1);
  }
}

// residual rows of the last real token of every sequence, gathered into a dense [n_copies * E, d] block
__global__ void __launch_bounds__(256) gather_last_rows_kernel(const float* __restrict__ h,
                                                               const int32_t* __restrict__ lengths, int E, int S, int d,
                                                               float* __restrict__ out) {
  const int r = blockIdx.x, e = r % E;
  const float* src = h + ((int64_t)r * S + seq_len(lengths, e, S) - 1) * d;
  for (int i = threadIdx.x; i < d; i += 256) out[(int64_t)r * d + i] = src[i];
}

// Packed batch: the E sequences of a copy lie back to back, sequence e in rows cu[e] .. cu[e+1] - 1 (cu[0] = 0); rows
// from cu[E] up to the copy's padded row count are filler.  For every row of a copy: its position inside its
// sequence, and the row after its sequence's last one (-1 for filler rows).
__global__ void __launch_bounds__(256) packed_index_kernel(const int32_t* __restrict__ cu, int E, int rows,
                                                           int32_t* __restrict__ row_pos, int32_t* __restrict__ row_end) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  if (r >= cu[E]) { row_pos[r] = 0; row_end[r] = -1; return; }
  int lo = 0, hi = E;                             // the last e with cu[e] <= r (empty sequences are stepped over)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu[mid] <= r) lo = mid; else hi = mid;
  }
  row_pos[r] = r - cu[lo];
  row_end[r] = cu[lo + 1];
}

// last row of every sequence of a packed batch, gathered into a dense [n_copies * E, d] block
__global__ void __launch_bounds__(256) gather_last_rows_packed_kernel(const float* __restrict__ h,
                                                                      const int32_t* __restrict__ cu, int E,
                                                                      int rows_per_copy, int d, float* __restrict__ out) {
  const int r = blockIdx.x, e = r % E, c = r / E;
  int last = cu[e + 1] - 1;
  last = last < 0 ? 0 : last;
  const float* src = h + ((int64_t)c * rows_per_copy + last) * d;
  for (int i = threadIdx.x; i < d; i += 256) out[(int64_t)r * d + i] = src[i];
}

// mean of a copy's per-row losses: fp64, fixed summation order.  With lengths the divisor is the number of
// next-token positions of the padded batch, sum_e (length_e - 1).
__global__ void __launch_bounds__(256) copy_mean_kernel(const float* __restrict__ ce, int rows_per_copy, int count,
                                                        const int32_t* __restrict__ lengths, int E, int S,
                                                        float* __restrict__ losses, int loss_stride) {
  __shared__ double red[4];
  const float* p = ce + (int64_t)blockIdx.x * rows_per_copy;
  double s = 0;
  for (int i = threadIdx.x; i < rows_per_copy; i += 256) s += (double)p[i];
  s = block_sum(s, red);
  if (threadIdx.x == 0) {
    if (lengths != nullptr) {
      count = 0;
      for (int e = 0; e < E; ++e) count += seq_len(lengths, e, S) - 1;
    }
    losses[(int64_t)blockIdx.x * loss_stride] = (float)(s / (double)count);
  }
}

// 4-bit normal-float weights -> bf16 (Appendix D builds on Q-LoRA's data type: sixteen levels, the quantiles of
// N(0, 1) scaled to [-1, 1] with an exact zero; one binary32 maximum per block of 64 consecutive input channels).
// Layout: output-major rows of K / 2 bytes, element 2j of a row in the low nibble of byte j, element 2j + 1 in the
// high nibble; absmax [rows, K / 64].  A thread turns one 32-bit word (8 codes) into 16 bytes of bf16:
// level[code] * absmax in binary32, rounded to nearest even.  Rows are contiguous and K % 64 == 0, so word i
// belongs to block i / 8 whatever the row.
__global__ void __launch_bounds__(256) nf4_dequant_kernel(const uint32_t* __restrict__ codes,
                                                          const float* __restrict__ absmax, uint4* __restrict__ out,
                                                          int64_t words) {
  __shared__ float level[16];
  if (threadIdx.x < 16) {
    constexpr float kLevel[16] = {-1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
                                  -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
                                  0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f,
                                  0.33791524171829224f, 0.44070982933044434f, 0.5626170039176941f,
                                  0.7229568362236023f, 1.0f};
    level[threadIdx.x] = kLevel[threadIdx.x];
  }
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * 1024 + threadIdx.x;
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int64_t i = base + it * 256;
    if (i >= words) break;
    const uint32_t c = codes[i];
    const float a = absmax[i >> 3];
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = __fmul_rn(level[(c >> (4 * e)) & 15u], a);
    out[i] = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
  }
}

__global__ void fill_kernel(float* p, float v, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

inline unsigned nblk(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

}  // namespace

#define MPZ_DISPATCH(dtype, ...)                                  \
  do {                                                            \
    if ((dtype) == MPZ_DTYPE_F32) { using ST = float; __VA_ARGS__; } \
    else { using ST = bf16_t; __VA_ARGS__; }                      \
  } while (0)

void launch_embed(hipStream_t st, int dtype, const int32_t* tokens, const void* emb, const void* pos_emb,
                  const int32_t* row_pos, float* h,
                  int n_copies, int E, int S, int d) {
  unsigned rows = (unsigned)((int64_t)n_copies * E * S);
  MPZ_DISPATCH(dtype, (embed_kernel<ST><<<rows, 128, 0, st>>>(tokens, (const ST*)emb, (const ST*)pos_emb, row_pos, h, n_copies, E, S, d)));
}

void launch_norm(hipStream_t st, int dtype, int kind, float eps, const float* h, int64_t h_row_stride, const float* g,
                 const float* b, void* out, int rows, int d) {
  MPZ_DISPATCH(dtype, (norm_kernel<ST><<<rows, 256, 0, st>>>(kind, eps, h, h_row_stride, g, b, (ST*)out, d)));
}

void launch_lora_down_simple(hipStream_t st, const LoraDownArgs& a) {
  int64_t total = (int64_t)a.T * a.n_targets * a.rank;
  MPZ_DISPATCH(a.dtype, (lora_down_kernel<ST><<<nblk(total, 256), 256, 0, st>>>(a)));
}

void launch_linear_simple(hipStream_t st, const LinearArgs& a) {
  dim3 grid((a.N + 63) / 64, (a.M + 63) / 64);
  MPZ_DISPATCH(a.dtype, (linear_kernel<ST><<<grid, 256, 0, st>>>(a)));
}

void launch_rope_convert(hipStream_t st, int dtype, const void* staging, void* out, int T, int S, int n_cols, int d_head,
                         int n_rot_heads, const float* cos_tab, const float* sin_tab, const int32_t* row_pos) {
  int64_t total = (int64_t)T * n_cols;
  MPZ_DISPATCH(dtype, (rope_convert_kernel<ST><<<nblk(total, 256), 256, 0, st>>>(
                          (const typename Traits<ST>::AT*)staging, (ST*)out, total, S, n_cols, d_head, n_rot_heads, cos_tab, sin_tab, row_pos)));
}

void launch_attention_simple(hipStream_t st, int dtype, const void* qkv, int qkv_stride, void* out, int n_seq, int S, int H,
                             int Hkv, int dh, const int32_t* cu, int E, int rows_per_copy) {
  unsigned blocks = (unsigned)((int64_t)n_seq * H * S);
  MPZ_DISPATCH(dtype, (attention_kernel<ST><<<blocks, 64, (size_t)(S + dh) * sizeof(typename Traits<ST>::AT), st>>>(
                          (const ST*)qkv, qkv_stride, (ST*)out, S, H, Hkv, dh, (float)(1.0 / sqrt((double)dh)), cu, E,
                          rows_per_copy)));
}

void launch_swiglu(hipStream_t st, int dtype, const void* staging, void* out, int T, int f) {
  int64_t total = (int64_t)T * f;
  MPZ_DISPATCH(dtype, (swiglu_kernel<ST><<<nblk(total, 256), 256, 0, st>>>((const typename Traits<ST>::AT*)staging, (ST*)out, total, f)));
}

void launch_ce_rows(hipStream_t st, int dtype, const float* logits, int64_t row_stride, int n_cols, const int32_t* target,
                    float* ce, int rows) {
  if (dtype == MPZ_DTYPE_F32) ce_rows_kernel<double><<<rows, 256, 0, st>>>(logits, row_stride, n_cols, target, ce);
  else ce_rows_kernel<float><<<rows, 256, 0, st>>>(logits, row_stride, n_cols, target, ce);
}

void launch_last_pos_subset_logits(hipStream_t st, int dtype, const void* xf, const void* head, int d, int rows, int tok0,
                                   int tok1, float* logits2) {
  MPZ_DISPATCH(dtype, (subset_logits_kernel<ST><<<rows, 64, 0, st>>>((const ST*)xf, (const ST*)head, d, tok0, tok1, logits2)));
}

void launch_nf4_dequant(hipStream_t st, const void* codes, const float* absmax, void* out, int64_t n_elems) {
  const int64_t words = n_elems / 8;
  nf4_dequant_kernel<<<nblk((words + 3) / 4, 256), 256, 0, st>>>((const uint32_t*)codes, absmax, (uint4*)out, words);
}

void launch_make_targets(hipStream_t st, int mode, const int32_t* tokens, const int32_t* labels, const int32_t* lengths,
                         const int32_t* row_end, int tok0, int tok1, int32_t* target, int n_copies, int E, int S) {
  int64_t n = (mode == MPZ_LOSS_NEXT_TOKEN_ALL_POS) ? (int64_t)n_copies * E * S : (int64_t)n_copies * E;
  make_targets_kernel<<<nblk(n, 256), 256, 0, st>>>(mode, tokens, labels, lengths, row_end, tok0, tok1, target, n_copies, E, S);
}

void launch_packed_index(hipStream_t st, const int32_t* cu, int E, int rows, int32_t* row_pos, int32_t* row_end) {
  packed_index_kernel<<<nblk(rows, 256), 256, 0, st>>>(cu, E, rows, row_pos, row_end);
}

void launch_gather_last_rows_packed(hipStream_t st, const float* h, const int32_t* cu, int n_copies, int E,
                                    int rows_per_copy, int d, float* out) {
  gather_last_rows_packed_kernel<<<n_copies * E, 256, 0, st>>>(h, cu, E, rows_per_copy, d, out);
}

void launch_gather_last_rows(hipStream_t st, const float* h, const int32_t* lengths, int n_copies, int E, int S, int d,
                             float* out) {
  gather_last_rows_kernel<<<n_copies * E, 256, 0, st>>>(h, lengths, E, S, d, out);
}

void launch_copy_mean(hipStream_t st, const float* ce, int rows_per_copy, int count_per_copy, const int32_t* lengths, int E,
                      int S, float* losses, int n_copies, int loss_stride) {
  copy_mean_kernel<<<n_copies, 256, 0, st>>>(ce, rows_per_copy, count_per_copy, lengths, E, S, losses, loss_stride);
}

void launch_fill_f32(hipStream_t st, float* p, float v, int64_t n) {
  fill_kernel<<<nblk(n, 256), 256, 0, st>>>(p, v, n);
}

}  // namespace mpz
