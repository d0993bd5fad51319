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

}  // namespace

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
