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
