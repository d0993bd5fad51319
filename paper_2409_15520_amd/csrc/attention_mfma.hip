// Causal self-attention for the stacked copies (every copy is an ordinary batch row here: Section 3,
// the n copies of the input batch travel through the model side by side).  bf16 MFMA for Q K^T and P V,
// fp32 softmax.  Two passes over the keys: the first finds each query's exact row maximum, the second
// recomputes the scores (bit-identical), forms P = bf16(exp(s - max)) and accumulates P V and sum(P).
// Rounding P against the exact maximum makes the result independent of the key tiling, which a running
// ("online") maximum would not be.
//
// One block = one (sequence, head) and 128 queries, 4 waves x 32 queries.  MFMA orientation: rows = keys
// (A operand), columns = queries (B operand): a lane owns ONE query, so max / sum are in-lane plus one
// cross-half shuffle, and the score registers are directly the B operand of the P V product
// D[dv, q] = sum_key Vt[dv, key] P[key, q] (the key order inside an MFMA K-step is permuted identically
// on both operands).
#include "common.h"

namespace mpz {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int QB = 128;   // queries per block

// The softmax is VALU-bound at these head sizes (16 scores per lane and tile against 12 MFMAs), so the score
// path is kept to one fma and one hardware exp2 per element: exp(scale (s - max)) = exp2(s c - max c) with
// c = scale log2(e); masking only on tiles that touch the diagonal; bf16 rounding in hardware.

// KC = keys per LDS chunk.  When every key the block can see fits one chunk, K and V are loaded once and both
// passes run from LDS; otherwise each pass streams the chunks.
// MINB = blocks per CU the register allocation is held to: 2 leaves 134 registers (3 waves per SIMD), 4 squeezes the
// same code into 128 (4 waves per SIMD, no spills), which pays once a block streams several key chunks (S = 512:
// 11.9 -> 11.1 ms per step on the 1.1B-shaped workload) and costs 3 % at S = 256, where a block lives for two.
template <int DH, int KC, int MINB>
__global__ void __launch_bounds__(256, MINB) attention_mfma_kernel(const uint16_t* __restrict__ qkv, int qkv_stride,
                                                             uint16_t* __restrict__ out, int S_grid, int H, int Hkv,
                                                             float scale, const int32_t* __restrict__ cu, int E,
                                                             int rows_per_copy) {
  constexpr int KS = DH + 8;        // K chunk row stride (elements)
  constexpr int VS = KC + 8;        // V^T chunk row stride
  constexpr int NJ = DH / 16;       // MFMA K-steps over the head dimension
  constexpr int NT = DH / 32;       // 32-row output tiles over the head dimension
  __shared__ __align__(16) uint16_t sK[KC * KS];
  __shared__ __align__(16) uint16_t sVt[DH * VS];

  // Hardware deals consecutive workgroups round-robin to the 8 XCDs; give each XCD a contiguous range of the
  // (sequence, head, query block) order instead, so that the blocks that read one sequence's K and V (all query
  // blocks, and under grouped-query attention all heads of the group) share an L2.
  // (1.3B-shaped workload, S = 256: 5.4 -> 4.5 ms per step; with a single query block per head and no key sharing
  // there is nothing to share and the plain order is kept)
  int pid = blockIdx.x;
  const int qblocks = (S_grid + QB - 1) / QB;
  if (qblocks * (H / Hkv) > 1) {
    const int nblk = gridDim.x, per = nblk / 8, rem = nblk % 8;
    const int xcd = pid % 8, idx = pid / 8;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int qb = pid % qblocks;
  const int head = (pid / qblocks) % H;
  const int seq = pid / (qblocks * H);
  // padded batch: every sequence holds S_grid rows.  Packed batch: S_grid is the longest sequence; this one starts at
  // its copy's row cu[e] and may be shorter (query blocks past its end leave at once: block-uniform, before any barrier)
  int S = S_grid;
  size_t row0 = (size_t)seq * S_grid;
  if (cu != nullptr) {
    const int e = seq % E;
    const int start = cu[e];
    S = cu[e + 1] - start;
    row0 = (size_t)(seq / E) * rows_per_copy + start;
    if (qb * QB >= S) return;
  }
  const int kvh = head / (H / Hkv);
  const int d = H * DH, dkv = Hkv * DH;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // a scalar: the tile-visibility tests below are wave-uniform
  const int lrow = lane & 31, lhalf = lane >> 5;

  const int q0 = qb * QB + wave * 32;             // first query of this wave
  const int qi = q0 + lrow;                       // this lane's query
  const int qi_c = qi < S ? qi : S - 1;
  const uint16_t* kbase = qkv + row0 * qkv_stride + d + kvh * DH;
  const uint16_t* vbase = qkv + row0 * qkv_stride + d + dkv + kvh * DH;

  // Q fragments (B operand): query qi, head-dim elements j*16 + lhalf*8 .. +7
  bf16x8 fq[NJ];
  {
    const uint16_t* qp = qkv + (row0 + qi_c) * qkv_stride + head * DH + lhalf * 8;
#pragma unroll
    for (int j = 0; j < NJ; ++j) fq[j] = __builtin_bit_cast(bf16x8, *(const u32x4*)(qp + j * 16));
  }

  const int last_q_block = (qb * QB + QB - 1 < S ? qb * QB + QB - 1 : S - 1);
  const int n_chunks = last_q_block / KC + 1;     // key chunks any query of the block can see
  const int wave_last_q = q0 + 31;
  constexpr int CPR = DH / 8;                     // 16-byte chunks per key row

  // K / V chunks travel global -> registers -> LDS: the fetch of chunk c + 1 is issued right after chunk c has
  // been published, so its latency hides behind the MFMAs on chunk c.
  constexpr int KL = KC * CPR / 256;              // 16-byte pieces of a K chunk per thread
  constexpr int VL = (KC / 2) * CPR / 256;        // key pairs x 8 head-dim elements per thread
  static_assert(KC * CPR % 256 == 0 && (KC / 2) * CPR % 256 == 0, "chunks must deal out evenly");
  u32x4 rk[KL], rv0[VL], rv1[VL];
#define MPZ_FETCH_K(c)                                                             \
  _Pragma("unroll") for (int it = 0; it < KL; ++it) {                              \
    const int i = tid + 256 * it, key = i / CPR, ch = i % CPR;                     \
    int kg = (c) * KC + key; kg = kg < S ? kg : S - 1;                             \
    rk[it] = *(const u32x4*)(kbase + (size_t)kg * qkv_stride + ch * 8);            \
  }
#define MPZ_PUT_K()                                                                \
  _Pragma("unroll") for (int it = 0; it < KL; ++it) {                              \
    const int i = tid + 256 * it, key = i / CPR, ch = i % CPR;                     \
    *(u32x4*)(sK + key * KS + ch * 8) = rk[it];                                    \
  }
  // V^T into LDS: a thread takes two consecutive keys and 8 head-dim elements and writes 8 words
  // {V[key][dv], V[key+1][dv]}; consecutive lanes hold consecutive key pairs, so the 32-bit writes of a wave fall
  // into consecutive banks (a per-element 16-bit scatter would serialise on a handful of banks).  Inside every
  // group of 16 keys the pairs are stored in the order 0 1 4 5 2 3 6 7: the 8 keys of one MFMA K-step that a lane
  // half needs (k + 4 lhalf + (0..3) and k + 8 + 4 lhalf + (0..3)) are then 16 contiguous bytes.
#define MPZ_FETCH_V(c)                                                             \
  _Pragma("unroll") for (int it = 0; it < VL; ++it) {                              \
    const int i = tid + 256 * it, kp = i % (KC / 2), ch = i / (KC / 2);            \
    int k0 = (c) * KC + 2 * kp, k1 = k0 + 1;                                       \
    k0 = k0 < S ? k0 : S - 1; k1 = k1 < S ? k1 : S - 1;                            \
    rv0[it] = *(const u32x4*)(vbase + (size_t)k0 * qkv_stride + ch * 8);           \
    rv1[it] = *(const u32x4*)(vbase + (size_t)k1 * qkv_stride + ch * 8);           \
  }
#define MPZ_PUT_V()                                                                \
  _Pragma("unroll") for (int it = 0; it < VL; ++it) {                              \
    const int i = tid + 256 * it, kp = i % (KC / 2), ch = i / (KC / 2);            \
    const int pp = kp & 7;                                                         \
    uint32_t* dst = (uint32_t*)sVt + (kp & ~7) + ((pp & 1) | ((pp & 2) << 1) | ((pp & 4) >> 1)); \
    _Pragma("unroll") for (int e = 0; e < 4; ++e) {                                \
      dst[(ch * 8 + 2 * e) * (VS / 2)] = (rv0[it][e] & 0xFFFFu) | (rv1[it][e] << 16);        \
      dst[(ch * 8 + 2 * e + 1) * (VS / 2)] = (rv0[it][e] >> 16) | (rv1[it][e] & 0xFFFF0000u); \
    }                                                                              \
  }
  // raw scores (q . k, unscaled) of one 32-key tile against this wave's 32 queries; lane: query qi,
  // keys kt0 + (e/4)*8 + lhalf*4 + e%4.  Tiles that reach past the diagonal get -inf on the masked entries.
#define MPZ_SCORE_TILE(t_local, kt0, sacc)                                         \
  {                                                                                \
    _Pragma("unroll") for (int e = 0; e < 16; ++e) sacc[e] = 0.f;                  \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j) {                               \
      bf16x8 fk = __builtin_bit_cast(bf16x8, *(const u32x4*)(sK + ((t_local) * 32 + lrow) * KS + j * 16 + lhalf * 8)); \
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fk, fq[j], sacc, 0, 0, 0);    \
    }                                                                              \
    if ((kt0) + 31 > q0) {                                                         \
      _Pragma("unroll") for (int e = 0; e < 16; ++e) {                             \
        int key = (kt0) + (e >> 2) * 8 + lhalf * 4 + (e & 3);                      \
        sacc[e] = key <= qi ? sacc[e] : -INFINITY;                                 \
      }                                                                            \
    }                                                                              \
  }

  // ---- pass 1: exact row maximum ----
  float mx = -1e30f;
  MPZ_FETCH_K(0)
  if (n_chunks == 1) { MPZ_FETCH_V(0) }
  for (int c = 0; c < n_chunks; ++c) {
    __syncthreads();                              // every wave is done with the previous chunk
    MPZ_PUT_K()
    if (n_chunks == 1) { MPZ_PUT_V() }
    __syncthreads();
    if (n_chunks > 1) {                           // next chunk of this pass, or the first one of pass 2
      if (c + 1 < n_chunks) { MPZ_FETCH_K(c + 1) } else { MPZ_FETCH_K(0) MPZ_FETCH_V(0) }
    }
#pragma unroll
    for (int t = 0; t < KC / 32; ++t) {
      int kt0 = c * KC + t * 32;
      if (kt0 > wave_last_q) continue;            // tile entirely in this wave's future
      f32x16 sc;
      MPZ_SCORE_TILE(t, kt0, sc)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sc[e]);
    }
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float c1 = scale * 1.4426950408889634f;   // scale > 0: the maximum of the raw scores is the maximum
  const float mx2 = mx * c1;

  // ---- pass 2: P = bf16(exp(s - max)), O^T += V^T P, l += P ----
  f32x16 oacc[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[t][e] = 0.f;
  float lsum = 0.f;
  const bf16x2 ones = __builtin_bit_cast(bf16x2, 0x3f803f80u);
  for (int c = 0; c < n_chunks; ++c) {
    if (n_chunks > 1) {
      __syncthreads();
      MPZ_PUT_K()
      MPZ_PUT_V()
      __syncthreads();
      if (c + 1 < n_chunks) { MPZ_FETCH_K(c + 1) MPZ_FETCH_V(c + 1) }
    }
#pragma unroll
    for (int t = 0; t < KC / 32; ++t) {
      int kt0 = c * KC + t * 32;
      if (kt0 > wave_last_q) continue;
      f32x16 sc;
      MPZ_SCORE_TILE(t, kt0, sc)
      uint32_t pw[8];                             // 16 probabilities as bf16 pairs
#pragma unroll
      for (int e = 0; e < 16; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[e], c1, -mx2));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[e + 1], c1, -mx2));
        const uint32_t w = pack_bf16x2(p0, p1);
        pw[e >> 1] = w;
        lsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w), ones, lsum, false);   // the rounded values
      }
      // two MFMA K-steps of 16 keys: step h uses score registers 8h .. 8h+7, i.e. keys
      // kt0 + 16h + lhalf*4 + (0..3) and kt0 + 16h + 8 + lhalf*4 + (0..3)
#pragma unroll
      for (int hstep = 0; hstep < 2; ++hstep) {
        u32x4 pfrag = {pw[hstep * 4], pw[hstep * 4 + 1], pw[hstep * 4 + 2], pw[hstep * 4 + 3]};
        bf16x8 fp = __builtin_bit_cast(bf16x8, pfrag);
        const int kl = t * 32 + hstep * 16 + lhalf * 8;   // this half's 8 keys of the step, as stored
#pragma unroll
        for (int vt = 0; vt < NT; ++vt) {
          const u32x4 vfrag = *(const u32x4*)(sVt + (vt * 32 + lrow) * VS + kl);
          oacc[vt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vfrag), fp, oacc[vt], 0, 0, 0);
        }
      }
    }
  }
#undef MPZ_FETCH_K
#undef MPZ_PUT_K
#undef MPZ_FETCH_V
#undef MPZ_PUT_V
#undef MPZ_SCORE_TILE
  lsum += __shfl_xor(lsum, 32, 64);

  if (qi < S) {
    const float inv = 1.0f / lsum;
    uint16_t* op = out + (row0 + qi) * (size_t)d + head * DH;
#pragma unroll
    for (int vt = 0; vt < NT; ++vt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int dv = vt * 32 + g * 8 + lhalf * 4;
        u32x2 pk = {pack_bf16x2(oacc[vt][g * 4] * inv, oacc[vt][g * 4 + 1] * inv),
                    pack_bf16x2(oacc[vt][g * 4 + 2] * inv, oacc[vt][g * 4 + 3] * inv)};
        *(u32x2*)(op + dv) = pk;
      }
  }
}

}  // namespace

bool attention_mfma_supported(int dh, int qkv_stride, int d) {
  return (dh == 64 || dh == 128) && qkv_stride % 8 == 0 && d % 8 == 0;
}

void launch_attention_mfma(hipStream_t st, const void* qkv, int qkv_stride, void* out, int n_seq, int S, int H, int Hkv,
                           int dh, const int32_t* cu, int E, int rows_per_copy) {
  const int qblocks = (S + QB - 1) / QB;
  const unsigned blocks = (unsigned)((size_t)n_seq * H * qblocks);
  const float scale = (float)(1.0 / sqrt((double)dh));
  if (dh == 64 && S > 256)
    attention_mfma_kernel<64, 128, 4><<<blocks, 256, 0, st>>>((const uint16_t*)qkv, qkv_stride, (uint16_t*)out, S, H, Hkv, scale, cu, E, rows_per_copy);
  else if (dh == 64)
    attention_mfma_kernel<64, 128, 2><<<blocks, 256, 0, st>>>((const uint16_t*)qkv, qkv_stride, (uint16_t*)out, S, H, Hkv, scale, cu, E, rows_per_copy);
  else
    attention_mfma_kernel<128, 64, 2><<<blocks, 256, 0, st>>>((const uint16_t*)qkv, qkv_stride, (uint16_t*)out, S, H, Hkv, scale, cu, E, rows_per_copy);
}

}  // namespace mpz
