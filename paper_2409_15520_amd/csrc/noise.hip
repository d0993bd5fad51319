// Noise regeneration, perturbation and seed-replayed update (Algorithm 1: noise draw, perturbation
// and parameter update).  The stream is Philox4x32-10 words -> exact binary32 uniforms -> Box-Muller
// built only from binary32 multiplies and adds (never fused; this file is compiled with
// -ffp-contract=off) so that any IEEE-754 implementation yields the same bits.
#include "common.h"

namespace mpz {

namespace {

struct U4 { uint32_t x, y, z, w; };

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                            uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;   // round multipliers (Salmon et al., SC'11)
  constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;   // Weyl key increments
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += W0; k1 += W1;
  }
  return U4{c0, c1, c2, c3};
}

// -2 ln(u), u = ((x >> 9) + 1/2) 2^-23: exponent extraction + degree-10 polynomial of ln(1+t)/t.
__device__ __forceinline__ float neg2_ln_uniform(uint32_t x) {
  float u = ((float)(x >> 9) + 0.5f) * 0x1p-23f;
  uint32_t bits = __float_as_uint(u);
  int e = (int)(bits >> 23) - 127;
  uint32_t fb = (bits & 0x007FFFFFu) | 0x3F800000u;
  float f = __uint_as_float(fb);
  if (fb >= 0x3FB504F3u) { f = f * 0.5f; e += 1; }
  float ef = (float)e;
  float t = f - 1.0f;
  float p = 0x1.141476p-4f;
  p = p * t; p = p + -0x1.e058eap-4f;
  p = p * t; p = p + 0x1.e8676ep-4f;
  p = p * t; p = p + -0x1.fbdf42p-4f;
  p = p * t; p = p + 0x1.2312fep-3f;
  p = p * t; p = p + -0x1.555c8cp-3f;
  p = p * t; p = p + 0x1.99a71cp-3f;
  p = p * t; p = p + -0x1.000010p-2f;
  p = p * t; p = p + 0x1.555540p-2f;
  p = p * t; p = p + -0x1.000000p-1f;
  p = p * t; p = p + 0x1.000000p+0f;
  float lnf = p * t;
  float a = ef * 0x1.62e000p-1f;
  float b = ef * 0x1.0bfbe8p-15f;
  b = b + lnf;
  float ln_u = a + b;
  return ln_u * -2.0f;
}

// cos and sin of 2 pi u by octant folding on the 23-bit integer and degree-4 polynomials in y^2.
__device__ __forceinline__ void sincos_2pi_uniform(uint32_t x, float& cs, float& sn) {
  uint32_t m = x >> 9;
  uint32_t quad = m >> 21;
  uint32_t wq = m & 0x1FFFFFu;
  bool flip = wq >= 0x100000u;
  if (flip) wq = 0x1FFFFFu - wq;
  float y = ((float)wq + 0.5f) * 0x1p-21f;
  float w = y * y;
  float s = 0x1.4bc87ap-13f;
  s = s * w; s = s + -0x1.32ca9ep-8f;
  s = s * w; s = s + 0x1.466bbap-4f;
  s = s * w; s = s + -0x1.4abbcep-1f;
  s = s * w; s = s + 0x1.921fb6p+0f;
  s = s * y;
  float c = 0x1.d9c326p-11f;
  c = c * w; c = c + -0x1.55c57ap-6f;
  c = c * w; c = c + 0x1.03c1dcp-2f;
  c = c * w; c = c + -0x1.3bd3ccp+0f;
  c = c * w; c = c + 0x1.000000p+0f;
  if (flip) { float tmp = s; s = c; c = tmp; }
  switch (quad) {
    case 0: cs = c;  sn = s;  break;
    case 1: cs = -s; sn = c;  break;
    case 2: cs = -c; sn = -s; break;
    default: cs = s; sn = -c; break;
  }
}

// binary64 square root rounded to binary32 is the correctly rounded binary32 square root
// (53 >= 2*24 + 2), independent of how the compiler lowers sqrtf.
__device__ __forceinline__ float sqrt_rn(float v) { return (float)sqrt((double)v); }

__device__ __forceinline__ void normals4(const U4& w, float z[4]) {
  float r0 = sqrt_rn(neg2_ln_uniform(w.x));
  float c0, s0; sincos_2pi_uniform(w.y, c0, s0);
  z[0] = r0 * c0; z[1] = r0 * s0;
  float r1 = sqrt_rn(neg2_ln_uniform(w.z));
  float c1, s1; sincos_2pi_uniform(w.w, c1, s1);
  z[2] = r1 * c1; z[3] = r1 * s1;
}

// group g of four consecutive master elements -> (tensor id, group index inside the tensor, is-A)
__device__ __forceinline__ void locate(const LoraLayerTable& tab, int64_t g, uint32_t& tensor_id, uint32_t& j,
                                       bool& is_A) {
  int64_t elem = g * 4;
  int layer = (int)(elem / tab.per_layer);
  int rem = (int)(elem - (int64_t)layer * tab.per_layer);
  int i = 0;
  while (i + 1 < tab.n_tensors && rem >= tab.off[i + 1]) ++i;
  tensor_id = (uint32_t)(layer * 8 + tab.local_id[i]);
  j = (uint32_t)((rem - tab.off[i]) >> 2);
  is_A = (tab.local_id[i] & 1) == 0;
}

__global__ void __launch_bounds__(256) perturb_kernel(const float4* __restrict__ masters, float4* __restrict__ pert,
                                                      int64_t n_groups, LoraLayerTable tab, uint32_t k0, uint32_t k1,
                                                      uint32_t step, int q, float eps, int perturb_A) {
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  uint32_t tid, j; bool is_A;
  locate(tab, g, tid, j, is_A);
  float4 m = masters[g];
  bool frozen = is_A && !perturb_A;
  for (int k = 0; k < q; ++k) {
    float4 plus = m, minus = m;
    if (!frozen) {
      float z[4];
      normals4(philox4x32_10(j, tid, step, (uint32_t)k, k0, k1), z);
      float p0 = eps * z[0], p1 = eps * z[1], p2 = eps * z[2], p3 = eps * z[3];
      plus = make_float4(m.x + p0, m.y + p1, m.z + p2, m.w + p3);
      minus = make_float4(m.x - p0, m.y - p1, m.z - p2, m.w - p3);
    }
    pert[(int64_t)(2 * k) * n_groups + g] = plus;
    pert[(int64_t)(2 * k + 1) * n_groups + g] = minus;
  }
}

// Perturbation written straight into the bf16 MFMA operand layouts (the stacked pass of a bf16 model reads nothing
// else): value = master (+/-) eps z as in perturb_kernel, then hi = bf16(value), lo = bf16(value - hi).
//   A [K, r] of copy c  ->  [2][K / 8][r][8]: element (k, j) of the hi part at ((k / 8) r + j) 8 + k % 8, lo part K r further
//   B [r, k_out]        ->  [k_out][rp] = [hi(r) | lo(r) | 0]
// One thread = one query k (both signs) x one work item of a layer: for an A factor 8 consecutive rows k x 4 columns j
// (8 generator calls -> four 16-byte pieces of each part), for a B factor 4 rows j x 4 output features (4 calls ->
// an 8-byte piece of the hi and of the lo half of four packed rows).  Same generator coordinates as perturb_kernel:
// the two paths give the same factors.
// two values -> {hi pair, lo pair} (low half = first value); round-to-nearest-even conversions in hardware
__device__ __forceinline__ void split_bf16x2(float a, float b, uint32_t& hi, uint32_t& lo) {
  hi = pack_bf16x2(a, b);
  lo = pack_bf16x2(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xFFFF0000u));
}

template <int RANK>
__global__ void __launch_bounds__(256) perturb_pack_kernel(const float* __restrict__ masters, uint16_t* __restrict__ packed,
                                                           int64_t packed_per_copy, LoraLayerTable tab, int n_layers, int rp,
                                                           int items_per_layer, uint32_t k0, uint32_t k1, uint32_t step,
                                                           float eps, int perturb_A) {
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)items_per_layer * n_layers) return;
  const uint32_t kq = blockIdx.y;                       // query
  const int layer = (int)(idx / items_per_layer);
  int item = (int)(idx % items_per_layer);
  int i = 0;
  int64_t poff = 0;
  for (;; ++i) {                                        // which factor of the layer, and where its packed form starts
    const bool isB = tab.local_id[i] & 1;
    const int cnt = isB ? tab.cols[i] / 4 * (RANK / 4) : tab.rows[i] / 8 * (RANK / 4);
    if (item < cnt) break;
    item -= cnt;
    poff += isB ? (int64_t)tab.cols[i] * rp : (int64_t)2 * tab.rows[i] * tab.cols[i];
  }
  int64_t per_layer_packed = 0;
  for (int t = 0; t < tab.n_tensors; ++t)
    per_layer_packed += (tab.local_id[t] & 1) ? (int64_t)tab.cols[t] * rp : (int64_t)2 * tab.rows[t] * tab.cols[t];
  const uint32_t tensor_id = (uint32_t)(layer * 8 + tab.local_id[i]);
  const float* src = masters + (int64_t)layer * tab.per_layer + tab.off[i];
  uint16_t* dst_p = packed + (int64_t)(2 * kq) * packed_per_copy + (int64_t)layer * per_layer_packed + poff;
  uint16_t* dst_m = dst_p + packed_per_copy;
  if ((tab.local_id[i] & 1) == 0) {                     // A [K, r]
    const int K = tab.rows[i], chunk = item / (RANK / 4), j0 = (item % (RANK / 4)) * 4, kb = chunk * 8;
    const bool frozen = !perturb_A;
    uint32_t hp[4][4], lp[4][4], hm[4][4], lm[4][4];    // [column][pair of rows]
#pragma unroll
    for (int k2 = 0; k2 < 4; ++k2) {
      float vp[2][4], vm[2][4];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int64_t e = (int64_t)(kb + 2 * k2 + h) * RANK + j0;   // flat element index of (k, j0): a multiple of 4
        const float4 m = *(const float4*)(src + e);
        const float mv[4] = {m.x, m.y, m.z, m.w};
        float z[4] = {0.f, 0.f, 0.f, 0.f};
        if (!frozen) normals4(philox4x32_10((uint32_t)(e >> 2), tensor_id, step, kq, k0, k1), z);
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const float p = eps * z[jj];
          vp[h][jj] = frozen ? mv[jj] : mv[jj] + p;
          vm[h][jj] = frozen ? mv[jj] : mv[jj] - p;
        }
      }
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        split_bf16x2(vp[0][jj], vp[1][jj], hp[jj][k2], lp[jj][k2]);
        split_bf16x2(vm[0][jj], vm[1][jj], hm[jj][k2], lm[jj][k2]);
      }
    }
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int64_t o = ((int64_t)chunk * RANK + j0 + jj) * 8;
      *(u32x4*)(dst_p + o) = u32x4{hp[jj][0], hp[jj][1], hp[jj][2], hp[jj][3]};
      *(u32x4*)(dst_p + (int64_t)K * RANK + o) = u32x4{lp[jj][0], lp[jj][1], lp[jj][2], lp[jj][3]};
      *(u32x4*)(dst_m + o) = u32x4{hm[jj][0], hm[jj][1], hm[jj][2], hm[jj][3]};
      *(u32x4*)(dst_m + (int64_t)K * RANK + o) = u32x4{lm[jj][0], lm[jj][1], lm[jj][2], lm[jj][3]};
    }
  } else {                                              // B [r, k_out]: rows j0 .. j0+3, features n0 .. n0+3
    const int kout = tab.cols[i], j0 = (item % (RANK / 4)) * 4, n0 = (item / (RANK / 4)) * 4;
    float vp[4][4], vm[4][4];                           // [row j][feature]
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t e = (int64_t)(j0 + j) * kout + n0;
      const float4 m = *(const float4*)(src + e);
      const float mv[4] = {m.x, m.y, m.z, m.w};
      float z[4];
      normals4(philox4x32_10((uint32_t)(e >> 2), tensor_id, step, kq, k0, k1), z);
#pragma unroll
      for (int nn = 0; nn < 4; ++nn) {
        const float p = eps * z[nn];
        vp[j][nn] = mv[nn] + p;
        vm[j][nn] = mv[nn] - p;
      }
    }
#pragma unroll
    for (int nn = 0; nn < 4; ++nn) {
      uint16_t* rowp = dst_p + (int64_t)(n0 + nn) * rp;
      uint16_t* rowm = dst_m + (int64_t)(n0 + nn) * rp;
      uint32_t h0, h1, l0, l1;
      split_bf16x2(vp[0][nn], vp[1][nn], h0, l0);
      split_bf16x2(vp[2][nn], vp[3][nn], h1, l1);
      *(u32x2*)(rowp + j0) = u32x2{h0, h1};
      *(u32x2*)(rowp + RANK + j0) = u32x2{l0, l1};
      split_bf16x2(vm[0][nn], vm[1][nn], h0, l0);
      split_bf16x2(vm[2][nn], vm[3][nn], h1, l1);
      *(u32x2*)(rowm + j0) = u32x2{h0, h1};
      *(u32x2*)(rowm + RANK + j0) = u32x2{l0, l1};
      if (j0 == 0)
        for (int c = 2 * RANK; c < rp; c += 4) {
          *(u32x2*)(rowp + c) = u32x2{0u, 0u};
          *(u32x2*)(rowm + c) = u32x2{0u, 0u};
        }
    }
  }
}

constexpr int MAX_Q = 64;

__global__ void __launch_bounds__(256) update_kernel(float4* __restrict__ masters, int64_t n_groups, LoraLayerTable tab,
                                                     uint32_t k0, uint32_t k1, uint32_t step, int q, float eps, float lr,
                                                     int perturb_A, const float* __restrict__ losses,
                                                     float* __restrict__ proj_grads_out) {
  __shared__ float coef[MAX_Q];
  if ((int)threadIdx.x < q) {
    int k = threadIdx.x;
    double g = ((double)losses[2 * k] - (double)losses[2 * k + 1]) / (2.0 * (double)eps);
    float g32 = (float)g;
    coef[k] = (float)((double)lr * (double)g32 / (double)q);
    if (proj_grads_out != nullptr && blockIdx.x == 0) proj_grads_out[k] = g32;
  }
  __syncthreads();
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  uint32_t tid, j; bool is_A;
  locate(tab, g, tid, j, is_A);
  if (is_A && !perturb_A) return;
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  for (int k = 0; k < q; ++k) {
    float z[4];
    normals4(philox4x32_10(j, tid, step, (uint32_t)k, k0, k1), z);
    float c = coef[k];
    float t0 = c * z[0], t1 = c * z[1], t2 = c * z[2], t3 = c * z[3];
    a0 = a0 + t0; a1 = a1 + t1; a2 = a2 + t2; a3 = a3 + t3;
  }
  float4 m = masters[g];
  masters[g] = make_float4(m.x - a0, m.y - a1, m.z - a2, m.w - a3);
}

// Stateful variant (Algorithm 2, q queries, explicit master): the noise of the finished step is read back from
// the stored pair, diff_k = (theta_k(+) - theta_k(-)) / 2, update = sum_k (lr g_k / q) diff_k / eps, and the pair
// is re-centred on the new master with the noise of `next_step` - one noise generation per step instead of
// generate + replay.
__global__ void __launch_bounds__(256) update_regen_kernel(float4* __restrict__ masters, float4* __restrict__ pert,
                                                           int64_t n_groups, LoraLayerTable tab, uint32_t k0, uint32_t k1,
                                                           uint32_t next_step, int q, float eps, float lr, int perturb_A,
                                                           const float* __restrict__ losses,
                                                           float* __restrict__ proj_grads_out) {
  __shared__ float coef[MAX_Q];
  if ((int)threadIdx.x < q) {
    int k = threadIdx.x;
    double g = ((double)losses[2 * k] - (double)losses[2 * k + 1]) / (2.0 * (double)eps);
    float g32 = (float)g;
    coef[k] = (float)((double)lr * (double)g32 / (double)q);
    if (proj_grads_out != nullptr && blockIdx.x == 0) proj_grads_out[k] = g32;
  }
  __syncthreads();
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  uint32_t tid, j; bool is_A;
  locate(tab, g, tid, j, is_A);
  if (is_A && !perturb_A) return;               // the copies of a frozen factor already equal its master
  float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
  for (int k = 0; k < q; ++k) {
    const float4 pl = pert[(int64_t)(2 * k) * n_groups + g], mi = pert[(int64_t)(2 * k + 1) * n_groups + g];
    const float d0 = (pl.x - mi.x) * 0.5f, d1 = (pl.y - mi.y) * 0.5f, d2 = (pl.z - mi.z) * 0.5f, d3 = (pl.w - mi.w) * 0.5f;
    const float z0 = d0 / eps, z1 = d1 / eps, z2 = d2 / eps, z3 = d3 / eps;
    const float c = coef[k];
    const float t0 = c * z0, t1 = c * z1, t2 = c * z2, t3 = c * z3;
    a0 = a0 + t0; a1 = a1 + t1; a2 = a2 + t2; a3 = a3 + t3;
  }
  float4 m = masters[g];
  m = make_float4(m.x - a0, m.y - a1, m.z - a2, m.w - a3);
  masters[g] = m;
  for (int k = 0; k < q; ++k) {
    float z[4];
    normals4(philox4x32_10(j, tid, next_step, (uint32_t)k, k0, k1), z);
    const float p0 = eps * z[0], p1 = eps * z[1], p2 = eps * z[2], p3 = eps * z[3];
    pert[(int64_t)(2 * k) * n_groups + g] = make_float4(m.x + p0, m.y + p1, m.z + p2, m.w + p3);
    pert[(int64_t)(2 * k + 1) * n_groups + g] = make_float4(m.x - p0, m.y - p1, m.z - p2, m.w - p3);
  }
}

// the generator alone: same calls as perturb_kernel, no memory traffic
__global__ void __launch_bounds__(256) noise_alu_probe_kernel(int64_t n_groups, int q, float* __restrict__ sink) {
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  float acc = 0.f;
  for (int k = 0; k < q; ++k) {
    float z[4];
    normals4(philox4x32_10((uint32_t)g, 7u, 3u, (uint32_t)k, 0x12345678u, 0x9abcdef0u), z);
    acc += z[0] + z[1] + z[2] + z[3];
  }
  if (acc == 1.2345e30f) sink[0] = acc;
}

__global__ void __launch_bounds__(256) debug_noise_kernel(float4* __restrict__ z_out, int64_t n_groups, uint32_t k0,
                                                          uint32_t k1, uint32_t step, uint32_t k, uint32_t tensor_id) {
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n_groups) return;
  float z[4];
  normals4(philox4x32_10((uint32_t)g, tensor_id, step, k, k0, k1), z);
  z_out[g] = make_float4(z[0], z[1], z[2], z[3]);
}

__global__ void __launch_bounds__(256) normals_from_words_kernel(const uint4* __restrict__ words, size_t n4,
                                                                 float4* __restrict__ out) {
  size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= n4) return;
  uint4 w = words[g];
  float z[4];
  normals4(U4{w.x, w.y, w.z, w.w}, z);
  out[g] = make_float4(z[0], z[1], z[2], z[3]);
}

inline unsigned blocks_for(int64_t n, int per_block) { return (unsigned)((n + per_block - 1) / per_block); }

}  // namespace

void launch_perturb(hipStream_t st, const float* masters, float* pert, int64_t P, const LoraLayerTable& tab,
                    uint64_t seed, uint32_t step, int q, float eps, int perturb_A) {
  int64_t ng = P / 4;
  perturb_kernel<<<blocks_for(ng, 256), 256, 0, st>>>((const float4*)masters, (float4*)pert, ng, tab,
                                                      (uint32_t)seed, (uint32_t)(seed >> 32), step, q, eps, perturb_A);
}

bool perturb_pack_supported(const LoraLayerTable& tab, int rank, int rp) {
  if (!(rank == 4 || rank == 8 || rank == 16) || rp % 4) return false;
  for (int t = 0; t < tab.n_tensors; ++t) {
    const bool isB = tab.local_id[t] & 1;
    if (!isB && tab.rows[t] % 8) return false;
    if (isB && tab.cols[t] % 4) return false;
    if (tab.off[t] % 4) return false;
  }
  return tab.per_layer % 4 == 0;
}

void launch_perturb_pack(hipStream_t st, const float* masters, void* packed, int64_t packed_per_copy,
                         const LoraLayerTable& tab, int n_layers, int rank, int rp, uint64_t seed, uint32_t step, int q,
                         float eps, int perturb_A) {
  int items = 0;
  for (int t = 0; t < tab.n_tensors; ++t)
    items += (tab.local_id[t] & 1) ? tab.cols[t] / 4 * (rank / 4) : tab.rows[t] / 8 * (rank / 4);
  const dim3 grid(blocks_for((int64_t)items * n_layers, 256), (unsigned)q);
  const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
  uint16_t* pk = (uint16_t*)packed;
  if (rank == 4) perturb_pack_kernel<4><<<grid, 256, 0, st>>>(masters, pk, packed_per_copy, tab, n_layers, rp, items, k0, k1, step, eps, perturb_A);
  else if (rank == 8) perturb_pack_kernel<8><<<grid, 256, 0, st>>>(masters, pk, packed_per_copy, tab, n_layers, rp, items, k0, k1, step, eps, perturb_A);
  else perturb_pack_kernel<16><<<grid, 256, 0, st>>>(masters, pk, packed_per_copy, tab, n_layers, rp, items, k0, k1, step, eps, perturb_A);
}

void launch_update(hipStream_t st, float* masters, int64_t P, const LoraLayerTable& tab, uint64_t seed, uint32_t step,
                   int q, float eps, float lr, int perturb_A, const float* losses, float* proj_grads_out) {
  int64_t ng = P / 4;
  update_kernel<<<blocks_for(ng, 256), 256, 0, st>>>((float4*)masters, ng, tab, (uint32_t)seed, (uint32_t)(seed >> 32),
                                                     step, q, eps, lr, perturb_A, losses, proj_grads_out);
}

void launch_update_regen(hipStream_t st, float* masters, float* pert, int64_t P, const LoraLayerTable& tab, uint64_t seed,
                         uint32_t next_step, int q, float eps, float lr, int perturb_A, const float* losses,
                         float* proj_grads_out) {
  int64_t ng = P / 4;
  update_regen_kernel<<<blocks_for(ng, 256), 256, 0, st>>>((float4*)masters, (float4*)pert, ng, tab, (uint32_t)seed,
                                                           (uint32_t)(seed >> 32), next_step, q, eps, lr, perturb_A, losses,
                                                           proj_grads_out);
}

void launch_noise_alu_probe(hipStream_t st, int64_t n_groups, int q, float* sink) {
  noise_alu_probe_kernel<<<blocks_for(n_groups, 256), 256, 0, st>>>(n_groups, q, sink);
}

void launch_debug_noise(hipStream_t st, float* z_out, int64_t numel, uint64_t seed, uint32_t step, int k, int tensor_id) {
  int64_t ng = numel / 4;
  debug_noise_kernel<<<blocks_for(ng, 256), 256, 0, st>>>((float4*)z_out, ng, (uint32_t)seed, (uint32_t)(seed >> 32), step,
                                                          (uint32_t)k, (uint32_t)tensor_id);
}

void launch_normals_from_words(hipStream_t st, const uint32_t* words, size_t n4, float* out) {
  normals_from_words_kernel<<<blocks_for((int64_t)n4, 256), 256, 0, st>>>((const uint4*)words, n4, (float4*)out);
}

}  // namespace mpz
