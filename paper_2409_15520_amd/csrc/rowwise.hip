// Row-wise HBM-bound kernels of the bf16 hot path: LayerNorm / RMSNorm of the fp32 residual stream into the
// bf16 GEMM operand.  One 64-lane wave owns one token row, the row lives in registers (d / 64 floats per lane),
// statistics are two-pass in fp32 with wave-level reductions only; every access is 16 B (loads) or 8 B (stores)
// per lane and contiguous across the wave.
#include "common.h"
#include "../../include/mpz.h"

namespace mpz {
namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

__device__ __forceinline__ float wave_sum_f32(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <int NV>   // d = 256 * NV
__global__ void __launch_bounds__(256) norm_rows_kernel(int kind, float eps, const float* __restrict__ h, int64_t h_row_stride,
                                                        const float* __restrict__ g, const float* __restrict__ b,
                                                        uint16_t* __restrict__ out, int rows) {
  constexpr int D = 256 * NV;
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const f32x4* hr = (const f32x4*)(h + (int64_t)row * h_row_stride);
  f32x4 v[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) v[i] = hr[i * 64 + lane];
  float mean = 0.f;
  if (kind == MPZ_NORM_LAYERNORM) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    mean = wave_sum_f32(s) / (float)D;
  }
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i)
#pragma unroll
    for (int e = 0; e < 4; ++e) { float c = v[i][e] - mean; q += c * c; }
  const float rstd = 1.0f / sqrtf(wave_sum_f32(q) / (float)D + eps);
  u32x2* orow = (u32x2*)(out + (int64_t)row * D);
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    f32x4 gg = ((const f32x4*)g)[i * 64 + lane];
    float y[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = (v[i][e] - mean) * rstd * gg[e];
    if (b != nullptr) {
      f32x4 bb = ((const f32x4*)b)[i * 64 + lane];
#pragma unroll
      for (int e = 0; e < 4; ++e) y[e] += bb[e];
    }
    u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
    orow[i * 64 + lane] = pk;
  }
}

// ---- split-K reduction fused with the pre-norm that follows it -----------------------------------------------
// A projection whose output is the residual stream (h += x W) and whose K was split over blocks leaves raw fp32
// partial sums; the next kernel of the pass is the pre-norm of those rows.  One block per token row does both.  All
// four waves sum the row's partial sums (16-byte piece c = tid + 256 j: splits in order from split 0, bias, residual -
// the reduction kernel's operations per element, so h has the same bits), store h and leave the row in LDS; wave 0
// takes the statistics from there with norm_rows_kernel's lane mapping and order (the same bits again); all threads
// then scale their own pieces.  (A wave per row, as in norm_rows_kernel, leaves a pass of 128 rows with 128 waves that
// each walk k_splits x d floats one round trip after the other: measured at four times the two kernels it replaces.)
template <int NV>   // d = 256 * NV
__global__ void __launch_bounds__(256) splitk_reduce_norm_kernel(MfmaGemmArgs a, int kind, float eps,
                                                                 const float* __restrict__ g, const float* __restrict__ b,
                                                                 uint16_t* __restrict__ out) {
  constexpr int D = 256 * NV, NC = 64 * NV, J = (NC + 255) / 256;       // 16-byte pieces per row, per thread
  __shared__ __align__(16) float srow[D];
  __shared__ float stat[2];
  const int tid = threadIdx.x, lane = tid & 63, row = blockIdx.x;
  const size_t plane = (size_t)a.M * a.ldp;
  f32x4 v[J];
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = tid + 256 * j;
    if (c < NC) v[j] = ((const f32x4*)(a.partial + (size_t)row * a.ldp))[c];
  }
  // the other splits, four at a time: their pieces are all requested before the first is added (they come from other
  // XCDs' blocks, a fabric round trip each), and added in split order
  for (int s = 1; s < a.k_splits; s += 4) {
    const int ns = a.k_splits - s < 4 ? a.k_splits - s : 4;              // block-uniform
    f32x4 t4[4][J];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (u >= ns) break;
      const f32x4* ps = (const f32x4*)(a.partial + (s + u) * plane + (size_t)row * a.ldp);
#pragma unroll
      for (int j = 0; j < J; ++j) {
        const int c = tid + 256 * j;
        if (c < NC) t4[u][j] = ps[c];
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (u >= ns) break;
#pragma unroll
      for (int j = 0; j < J; ++j)
        if (tid + 256 * j < NC) v[j] += t4[u][j];
    }
  }
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = tid + 256 * j;
    if (c >= NC) continue;
    if (a.bias != nullptr) v[j] += ((const f32x4*)a.bias)[c];
    if (a.residual != nullptr) v[j] += ((const f32x4*)(a.residual + (size_t)row * a.ldo))[c];
    ((f32x4*)((float*)a.out + (size_t)row * a.ldo))[c] = v[j];
    ((f32x4*)srow)[c] = v[j];
  }
  __syncthreads();
  if (tid < 64) {
    f32x4 w[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) w[i] = ((const f32x4*)srow)[i * 64 + lane];
    float mean = 0.f;
    if (kind == MPZ_NORM_LAYERNORM) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) s += (w[i][0] + w[i][1]) + (w[i][2] + w[i][3]);
      mean = wave_sum_f32(s) / (float)D;
    }
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) { float c = w[i][e] - mean; q += c * c; }
    const float rstd = 1.0f / sqrtf(wave_sum_f32(q) / (float)D + eps);
    if (lane == 0) { stat[0] = mean; stat[1] = rstd; }
  }
  __syncthreads();
  const float mean = stat[0], rstd = stat[1];
  u32x2* orow = (u32x2*)(out + (int64_t)row * D);
#pragma unroll
  for (int j = 0; j < J; ++j) {
    const int c = tid + 256 * j;
    if (c >= NC) continue;
    const f32x4 gg = ((const f32x4*)g)[c];
    float y[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = (v[j][e] - mean) * rstd * gg[e];
    if (b != nullptr) {
      const f32x4 bb = ((const f32x4*)b)[c];
#pragma unroll
      for (int e = 0; e < 4; ++e) y[e] += bb[e];
    }
    orow[c] = u32x2{pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
  }
}

// ---- pre-norm fused with the LoRA bottleneck of the projections that read its output ------------------------
// One block = 32 token rows.  Phase A is norm_rows_kernel's arithmetic (each wave takes 8 of the rows, RB at a time
// so that their loads travel together); the bf16 row goes to global memory for the GEMM and to an LDS tile.  Phase B
// is lora_down_mfma_kernel's arithmetic on that tile - same K split over the 4 waves, same order of the partial sums,
// so t has the same bits - without reading x again, without chunk staging and without its launch.
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <int NV, int JT>   // d = 256 NV; JT 32-row MFMA tiles cover n_targets * rank bottleneck columns
__global__ void __launch_bounds__(256, NV <= 4 ? 2 : 1) norm_lora_kernel(int kind, float eps, const float* __restrict__ h,
                                                                       const float* __restrict__ g,
                                                                       const float* __restrict__ b,
                                                                       uint16_t* __restrict__ out, MfmaLoraDownArgs a) {
  constexpr int D = 256 * NV, XS = D + 8, RB = NV <= 4 ? 8 : 4;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xs = (uint16_t*)smem;                      // [32][XS]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lhalf = lane >> 5;
  const int m0 = blockIdx.x * 32;

  // ---- phase A: rows m0 + 8 wave + (0..7), RB at a time
#pragma unroll 1
  for (int r0 = 0; r0 < 8; r0 += RB) {
    f32x4 v[RB][NV];
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
      const f32x4* hr = (const f32x4*)(h + (int64_t)(m0 + wave * 8 + r0 + rr) * D);
#pragma unroll
      for (int i = 0; i < NV; ++i) v[rr][i] = hr[i * 64 + lane];
    }
#pragma unroll
    for (int rr = 0; rr < RB; ++rr) {
      float mean = 0.f;
      if (kind == MPZ_NORM_LAYERNORM) {
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) s += (v[rr][i][0] + v[rr][i][1]) + (v[rr][i][2] + v[rr][i][3]);
        mean = wave_sum_f32(s) / (float)D;
      }
      float q = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int e = 0; e < 4; ++e) { float c = v[rr][i][e] - mean; q += c * c; }
      const float rstd = 1.0f / sqrtf(wave_sum_f32(q) / (float)D + eps);
      const int row = wave * 8 + r0 + rr;
      u32x2* orow = (u32x2*)(out + (int64_t)(m0 + row) * D);
      u32x2* lrow_p = (u32x2*)(xs + row * XS);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        f32x4 gg = ((const f32x4*)g)[i * 64 + lane];
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (v[rr][i][e] - mean) * rstd * gg[e];
        if (b != nullptr) {
          f32x4 bb = ((const f32x4*)b)[i * 64 + lane];
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] += bb[e];
        }
        u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
        orow[i * 64 + lane] = pk;
        lrow_p[i * 64 + lane] = pk;
      }
    }
  }
  __syncthreads();

  // ---- phase B: t = scale * x (A_hi + A_lo) for the block's copy; wave w owns K-elements 256 ch + 64 w + (0..63)
  const int copy = m0 / a.rows_per_copy;
  const int R = a.n_targets * a.rank;
  const uint16_t* Ah[JT];
  const uint16_t* Al[JT];
  bool valid[JT];
#pragma unroll
  for (int t = 0; t < JT; ++t) {
    int j = t * 32 + lrow;
    valid[t] = j < R;
    int jj = valid[t] ? j : 0;
    int tgt = jj / a.rank, jr = jj % a.rank;
    const uint16_t* base = (const uint16_t*)a.ap[tgt] + (size_t)copy * a.copy_stride;
    Ah[t] = base + ((size_t)(wave * 8 + lhalf) * a.rank + jr) * 8;      // [2][K / 8][rank][8], as in lora_down_mfma_kernel
    Al[t] = Ah[t] + (size_t)D * a.rank;
  }
  f32x16 acc[JT];
#pragma unroll
  for (int t = 0; t < JT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  u32x4 fh[4][JT], fl[4][JT];
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
    for (int t = 0; t < JT; ++t) {
      fh[s4][t] = valid[t] ? *(const u32x4*)(Ah[t] + (size_t)(s4 * 16) * a.rank) : zero;
      fl[s4][t] = valid[t] ? *(const u32x4*)(Al[t] + (size_t)(s4 * 16) * a.rank) : zero;
    }
#pragma unroll
  for (int ch = 0; ch < NV; ++ch) {
    u32x4 ch_h[4][JT], ch_l[4][JT];
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
      for (int t = 0; t < JT; ++t) { ch_h[s4][t] = fh[s4][t]; ch_l[s4][t] = fl[s4][t]; }
    if (ch + 1 < NV) {                                   // the next chunk's factors travel during this chunk's MFMAs
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
        for (int t = 0; t < JT; ++t) {
          fh[s4][t] = valid[t] ? *(const u32x4*)(Ah[t] + (size_t)((ch + 1) * 256 + s4 * 16) * a.rank) : zero;
          fl[s4][t] = valid[t] ? *(const u32x4*)(Al[t] + (size_t)((ch + 1) * 256 + s4 * 16) * a.rank) : zero;
        }
    }
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const bf16x8 fx = __builtin_bit_cast(bf16x8, *(const u32x4*)(xs + lrow * XS + ch * 256 + wave * 64 + s4 * 16 + lhalf * 8));
#pragma unroll
      for (int t = 0; t < JT; ++t) {
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ch_h[s4][t]), fx, acc[t], 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ch_l[s4][t]), fx, acc[t], 0, 0, 0);
      }
    }
  }
  __syncthreads();                                       // every wave is done with the x tile: its memory takes the sums
  float* part = (float*)smem;                            // [3][JT][16][64]: partial sums of waves 1..3
  if (wave > 0) {
#pragma unroll
    for (int t = 0; t < JT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) part[(((wave - 1) * JT + t) * 16 + e) * 64 + lane] = acc[t][e];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int t = 0; t < JT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e)
      acc[t][e] = ((acc[t][e] + part[((0 * JT + t) * 16 + e) * 64 + lane]) + part[((1 * JT + t) * 16 + e) * 64 + lane]) +
                  part[((2 * JT + t) * 16 + e) * 64 + lane];
  const int m = m0 + lrow;
#pragma unroll
  for (int t = 0; t < JT; ++t)
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) {
      const int j = t * 32 + gq * 8 + lhalf * 4;
      if (j >= R) continue;
      const int tgt = j / a.rank, jr = j % a.rank;
      const u32x2 pk = {pack_bf16x2(acc[t][gq * 4] * a.scale, acc[t][gq * 4 + 1] * a.scale),
                        pack_bf16x2(acc[t][gq * 4 + 2] * a.scale, acc[t][gq * 4 + 3] * a.scale)};
      uint16_t* row = (uint16_t*)a.tp[tgt] + (size_t)m * a.rp;
      *(u32x2*)(row + jr) = pk;
      *(u32x2*)(row + a.rank + jr) = pk;
    }
  if (lhalf == 0)
    for (int tgt = 0; tgt < a.n_targets; ++tgt)
      for (int c = 2 * a.rank; c < a.rp; ++c) ((uint16_t*)a.tp[tgt])[(size_t)m * a.rp + c] = 0;
}

template <int NV, int JT>
void launch_norm_lora_t(hipStream_t st, int kind, float eps, const float* h, const float* g, const float* b, void* out,
                        const MfmaLoraDownArgs& a) {
  constexpr size_t lds = (size_t)32 * (256 * NV + 8) * 2;
  static bool attr_set = false;
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)norm_lora_kernel<NV, JT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_set = true;
  }
  norm_lora_kernel<NV, JT><<<a.T / 32, 256, lds, st>>>(kind, eps, h, g, b, (uint16_t*)out, a);
}

}  // namespace

// pre-norm + LoRA bottleneck in one kernel: d in {768, 1024, 2048} (the LDS tile of 32 rows must fit), dense rows.
// At d = 2048 the tile leaves room for one block per CU, whose two phases then do not overlap with another block's:
// measured, the fusion pays there only when the bottleneck is wide (more than 32 columns: three adapted projections
// of rank 16 take 11.2 instead of 12.0 ms per step on the 1.1B-shaped workload; two of rank 8 lose 0.4 ms on the
// 1.3B-shaped one).
bool norm_lora_supported(int d, const MfmaLoraDownArgs& a) {
  const bool wide = a.n_targets * a.rank > 32;
  return (d == 768 || d == 1024 || (d == 2048 && wide)) && a.K == d && mfma_lora_down_supported(a);
}

void launch_norm_lora(hipStream_t st, int kind, float eps, const float* h, const float* g, const float* b, void* out,
                      const MfmaLoraDownArgs& a) {
  const bool two = a.n_targets * a.rank > 32;
  switch (a.K / 256) {
    case 3: if (two) launch_norm_lora_t<3, 2>(st, kind, eps, h, g, b, out, a); else launch_norm_lora_t<3, 1>(st, kind, eps, h, g, b, out, a); break;
    case 4: if (two) launch_norm_lora_t<4, 2>(st, kind, eps, h, g, b, out, a); else launch_norm_lora_t<4, 1>(st, kind, eps, h, g, b, out, a); break;
    default: if (two) launch_norm_lora_t<8, 2>(st, kind, eps, h, g, b, out, a); else launch_norm_lora_t<8, 1>(st, kind, eps, h, g, b, out, a); break;
  }
}

bool splitk_reduce_norm_supported(const MfmaGemmArgs& a) {
  const int d = a.N;
  return a.k_splits > 1 && a.partial != nullptr && !a.dual && a.rope_cos == nullptr && a.act < 0 && a.out_f32 && a.ce_max == nullptr &&
         (d == 768 || d == 1024 || d == 2048 || d == 4096) && a.ldo == d && a.ldp % 4 == 0 && a.ldp >= d;
}

void launch_splitk_reduce_norm(hipStream_t st, const MfmaGemmArgs& a, int kind, float eps, const float* g, const float* b,
                               void* out) {
  const unsigned blocks = (unsigned)a.M;
  switch (a.N / 256) {
    case 3: splitk_reduce_norm_kernel<3><<<blocks, 256, 0, st>>>(a, kind, eps, g, b, (uint16_t*)out); break;
    case 4: splitk_reduce_norm_kernel<4><<<blocks, 256, 0, st>>>(a, kind, eps, g, b, (uint16_t*)out); break;
    case 8: splitk_reduce_norm_kernel<8><<<blocks, 256, 0, st>>>(a, kind, eps, g, b, (uint16_t*)out); break;
    default: splitk_reduce_norm_kernel<16><<<blocks, 256, 0, st>>>(a, kind, eps, g, b, (uint16_t*)out); break;
  }
}

bool norm_rows_supported(int d, int64_t h_row_stride) {
  return (d == 768 || d == 1024 || d == 2048 || d == 4096) && h_row_stride % 4 == 0;
}

void launch_norm_rows(hipStream_t st, int kind, float eps, const float* h, int64_t h_row_stride, const float* g,
                      const float* b, void* out, int rows, int d) {
  const unsigned blocks = (unsigned)((rows + 3) / 4);
  switch (d / 256) {
    case 3: norm_rows_kernel<3><<<blocks, 256, 0, st>>>(kind, eps, h, h_row_stride, g, b, (uint16_t*)out, rows); break;
    case 4: norm_rows_kernel<4><<<blocks, 256, 0, st>>>(kind, eps, h, h_row_stride, g, b, (uint16_t*)out, rows); break;
    case 8: norm_rows_kernel<8><<<blocks, 256, 0, st>>>(kind, eps, h, h_row_stride, g, b, (uint16_t*)out, rows); break;
    default: norm_rows_kernel<16><<<blocks, 256, 0, st>>>(kind, eps, h, h_row_stride, g, b, (uint16_t*)out, rows); break;
  }
}

}  // namespace mpz
