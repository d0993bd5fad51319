// bf16 MFMA GEMM for the shared-weight term of the MP-LoRA layer (Section 3: Y = X W + (X A) (.) B):
// the frozen weight tile is read once for all n = 2q stacked copies, and the per-copy rank-r term is
// folded into the same fp32 accumulators as extra K-steps whose "weight" operand is that copy's packed
// factor [B_hi | B_lo].  gfx950 only: v_mfma_f32_32x32x16_bf16, 64-lane waves, LDS-staged block tiles
// (128..256 square-ish, several configurations) with register-staged double buffering.
//
// Orientation: the MFMA "A" operand is a W tile (rows = output features n), the "B" operand an X tile
// (rows = tokens m), so every lane ends up with 4 consecutive n of one token: bias / residual / stores
// are 8- or 16-byte accesses along the contiguous output dimension.
#include <mutex>

#include "common.h"
#include "../../include/mpz.h"

namespace mpz {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;     // 16-byte chunk in registers (native vector type)
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ bf16x8 as_frag(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float gelu_erf(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752440f)); }
// the same arithmetic as a real call: where all of a block's accumulators are live around it, inlining erff 128 times
// would cost registers that the common path (no GELU) never needs
__device__ __noinline__ float gelu_erf_call(float v) { return gelu_erf(v); }

// Instruction interleave of one main-loop phase.  Issued as a burst, the tile's global loads occupy the address
// path for ~16 cycles each and its LDS stores for ~8, during which the issuing wave cannot feed the matrix core:
// spread them (and the fragment reads of the next K-step) between the MFMAs instead.
template <int MASK>
__device__ __forceinline__ void sched_one() { __builtin_amdgcn_sched_group_barrier(MASK, 1, 0); }

// entries I..HI-1 of a K-step's list of non-MFMA instructions: NDSR fragment reads first (the next step needs
// them soonest), then global loads and LDS stores alternating
template <int I, int HI, int NDSR, int NVM, int NDSW>
__device__ __forceinline__ void sched_others() {
  if constexpr (I < HI) {
    if constexpr (I < NDSR) sched_one<0x100>();
    else {
      constexpr int j = I - NDSR, pairs = NVM < NDSW ? NVM : NDSW;
      if constexpr (j < 2 * pairs) { if constexpr (j % 2 == 0) sched_one<0x020>(); else sched_one<0x200>(); }
      else if constexpr (NVM > NDSW) sched_one<0x020>();
      else sched_one<0x200>();
    }
    sched_others<I + 1, HI, NDSR, NVM, NDSW>();
  }
}

template <int NM, int NDSR, int NVM, int NDSW, int C = 0>
__device__ __forceinline__ void sched_step() {
  if constexpr (C < NM) {
    sched_one<0x008>();
    constexpr int NO = NDSR + NVM + NDSW;
    sched_others<C * NO / NM, (C + 1) * NO / NM, NDSR, NVM, NDSW>();
    sched_step<NM, NDSR, NVM, NDSW, C + 1>();
  }
}

// one phase: NF fragment reads of K-step 0, then KS steps of NM MFMAs, each carrying the next step's NF reads
// and its share of the tile's NUW + NUX fetch units (one global load each; WPU LDS stores per W unit, one per X unit)
template <int NM, int NF, int NUW, int NUX, int WPU, int KS, int S = 0>
__device__ __forceinline__ void sched_phase() {
  if constexpr (S == 0) __builtin_amdgcn_sched_group_barrier(0x100, NF, 0);
  if constexpr (S < KS) {
    constexpr int NU = NUW + NUX;
    constexpr int lo = (S * NU + KS - 1) / KS, hi = ((S + 1) * NU + KS - 1) / KS;   // this step's units
    constexpr int wlo = lo < NUW ? lo : NUW, whi = hi < NUW ? hi : NUW;
    constexpr int nvm = hi - lo, ndsw = (whi - wlo) * WPU + (hi - lo) - (whi - wlo);
    sched_step<NM, (S + 1 < KS ? NF : 0), nvm, ndsw>();
    sched_phase<NM, NF, NUW, NUX, WPU, KS, S + 1>();
  }
}

// 16 int8 codes (one 16-byte chunk along K) -> 16 bf16, exact: |code| <= 127 has 7 significant bits
__device__ __forceinline__ void i8x16_to_bf16(u32x4 in, u32x4& lo8, u32x4& hi8) {
  uint32_t o[8];
#pragma unroll
  for (int wd = 0; wd < 4; ++wd) {
    const uint32_t v = in[wd];
    const float f0 = (float)(int8_t)(v & 0xff), f1 = (float)(int8_t)((v >> 8) & 0xff);
    const float f2 = (float)(int8_t)((v >> 16) & 0xff), f3 = (float)(int8_t)(v >> 24);
    o[2 * wd] = pack_bf16x2(f0, f1);
    o[2 * wd + 1] = pack_bf16x2(f2, f3);
  }
  lo8 = u32x4{o[0], o[1], o[2], o[3]};
  hi8 = u32x4{o[4], o[5], o[6], o[7]};
}

// Block tile BN (output features) x BM (tokens), K-step BK, WGN x WGM waves, each wave (BN/WGN) x (BM/WGM) =
// NI x NJ MFMA tiles; two register sets of tiles in flight.  DUAL: two weight tiles (rows n and n + dual_offset:
// SwiGLU gate and up) against the same X tile.  LDS rows are padded by 16 B, which keeps ds_read_b128 of 32 rows
// conflict-free for BK = 32 and BK = 64.
// HP > 0: rotary embedding fused into the epilogue for head width 64 * HP (the partner column d_head/2 away sits in
// the same lane, HP MFMA tiles further), for output columns below rope_cols; the result is stored as bf16.
template <int BN, int BM, int BK, int WGN, int WGM, bool DUAL, int HP, int WQ>
__global__ void __launch_bounds__(64 * WGN * WGM, (BN * BM * (DUAL ? 2 : 1) <= 256 * 128 && WGN * WGM == 4 && !(BN == 192 && BK == 64)) ? 2 : 1)
gemm_bf16_kernel(MfmaGemmArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NW = DUAL ? 2 : 1;
  constexpr int LDS_STRIDE = BK + 8;
  constexpr int TILE_W = BN * LDS_STRIDE, TILE_X = BM * LDS_STRIDE;     // elements per operand tile per stage
  constexpr int NT = 64 * WGN * WGM;                                     // threads per block
  constexpr int TN = BN / WGN, TM = BM / WGM, NI = TN / 32, NJ = TM / 32;
  constexpr int CPR = BK / 8;                                            // 16-byte chunks per bf16 tile row
  constexpr int WCH = WQ == 2 ? BK / 32 : WQ == 1 ? BK / 16 : CPR;      // 16-byte chunks per W tile row (int8: 16 codes each, 4-bit: 32)
  constexpr int WSH = WQ == 2 ? 2 : WQ == 1 ? 1 : 0;                     // bytes of a bf16 weight >> WSH = bytes of a stored weight
  static_assert(WQ == 0 || WQ == 1 || (WQ == 2 && BK == 64 && !DUAL), "4-bit weights: one block of 64 input channels per K-tile");
  constexpr int LW = BN * WCH / NT, LX = BM * CPR / NT;                  // chunks per thread and tile
  static_assert(BN * WCH % NT == 0 && BM * CPR % NT == 0, "tile rows must deal out evenly to the threads");
  uint16_t* sW = (uint16_t*)smem;                        // [2 stages][NW][BN][LDS_STRIDE]
  constexpr int NSTG = 2;                                // LDS stages (and register sets) of operand tiles
  uint16_t* sX = sW + NSTG * NW * TILE_W;                // [stages][BM][LDS_STRIDE]

  // XCD-aware tile order: hardware deals consecutive workgroups round-robin to the 8 XCDs; give each XCD
  // a contiguous range of tiles so that neighbours in its L2 share X rows and the whole (small) W.
  const int tiles_n = (a.N + BN - 1) / BN, tiles_m = (a.M + BM - 1) / BM;
  const int nblk = tiles_n * tiles_m;
  int pid = blockIdx.x;
  {
    const int per = nblk / 8, rem = nblk % 8;              // XCD x owns per (+1 if x < rem) tiles
    const int xcd = pid % 8, idx = pid / 8;
    pid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  // Inside that range, walk groups of GM token-tiles with the token-tile index fastest: the blocks running
  // together on an XCD then form a compact patch of the output (few distinct X and W tiles per block), and a
  // W tile is finished after GM consecutive blocks instead of having to survive in L2 until the next row of tiles.
  constexpr int GM = 8;
  const int group = pid / (GM * tiles_n), first_m = group * GM;
  const int gsz = tiles_m - first_m < GM ? tiles_m - first_m : GM;
  const int rr = pid - group * GM * tiles_n;
  const int tile_m = first_m + rr % gsz, tile_n = rr / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = (wave / WGM) * TN, wm = (wave % WGM) * TM;   // wave tile origin inside the block tile
  const int lrow = lane & 31, lhalf = lane >> 5;

  // Operand fetch: raw buffer loads (per-thread byte offset in a VGPR, the K offset of the tile in an SGPR);
  // rows past the end of W or X fall outside the buffer and read as zero, so ragged M / N need no clamps.
  const __amdgpu_buffer_rsrc_t rsrcW =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.w), 0, (int)(((size_t)a.w_rows * a.K * 2) >> WSH), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcX =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.x), 0, (int)((size_t)a.M * a.K * 2), 0x00020000);
  uint32_t voffW[NW][LW], voffX[LX];
  int ldsW[LW], ldsX[LX];
#pragma unroll
  for (int i = 0; i < LW; ++i) {
    const int c = tid + NT * i, row = c / WCH, kc = (c % WCH) * (8 << WSH);
    voffW[0][i] = (((uint32_t)(n0 + row) * (uint32_t)a.K + kc) * 2u) >> WSH;
    if (DUAL) voffW[NW - 1][i] = (((uint32_t)(n0 + row + a.dual_offset) * (uint32_t)a.K + kc) * 2u) >> WSH;
    ldsW[i] = row * LDS_STRIDE + kc;
  }
  // 4-bit weights: the block maximum of the K-tile's 64 input channels travels with every chunk of codes, and the
  // sixteen levels sit in LDS (every lane of a wave may ask for another one; sixteen words lie in sixteen banks)
  __shared__ float nf4_level[WQ == 2 ? 16 : 1];
  __amdgpu_buffer_rsrc_t rsrcA = rsrcW;
  uint32_t voffA[LW];
  if constexpr (WQ == 2) {
    rsrcA = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.w_absmax), 0, (int)((size_t)a.w_rows * (a.K / 64) * 4), 0x00020000);
#pragma unroll
    for (int i = 0; i < LW; ++i) voffA[i] = (uint32_t)(n0 + (tid + NT * i) / WCH) * (uint32_t)(a.K / 64) * 4u;
    if (tid < 16) {
      constexpr float kLevel[16] = {-1.0f, -0.6961928009986877f, -0.5250730514526367f, -0.39491748809814453f,
                                    -0.28444138169288635f, -0.18477343022823334f, -0.09105003625154495f, 0.0f,
                                    0.07958029955625534f, 0.16093020141124725f, 0.24611230194568634f,
                                    0.33791524171829224f, 0.44070982933044434f, 0.5626170039176941f,
                                    0.7229568362236023f, 1.0f};
      nf4_level[tid] = kLevel[tid];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < LX; ++i) {
    const int c = tid + NT * i, row = c / CPR, kc = (c % CPR) * 8;
    voffX[i] = ((uint32_t)(m0 + row) * (uint32_t)a.K + kc) * 2u;
    ldsX[i] = row * LDS_STRIDE + kc;
  }
  u32x4 rw[NSTG][NW][LW], rx[NSTG][LX];
  float ra[NSTG][LW];                                    // 4-bit weights: block maxima of the chunks in rw
  // int8 weights: a fetched chunk is 16 codes; it becomes two 16-byte chunks of bf16 on its way into LDS
#define MPZ_PUT_W(ptr, v, am)                                                      \
  {                                                                                \
    if constexpr (WQ == 2) {                                                       \
      _Pragma("unroll") for (int wd_ = 0; wd_ < 4; ++wd_) {                        \
        const uint32_t c_ = (v)[wd_];                                              \
        float f_[8];                                                               \
        _Pragma("unroll") for (int e_ = 0; e_ < 8; ++e_) f_[e_] = __fmul_rn(nf4_level[(c_ >> (4 * e_)) & 15u], (am)); \
        *(u32x4*)((ptr) + 8 * wd_) = u32x4{pack_bf16x2(f_[0], f_[1]), pack_bf16x2(f_[2], f_[3]),  \
                                           pack_bf16x2(f_[4], f_[5]), pack_bf16x2(f_[6], f_[7])}; \
      }                                                                            \
    } else if constexpr (WQ == 1) {                                                \
      u32x4 lo8_, hi8_;                                                            \
      i8x16_to_bf16(v, lo8_, hi8_);                                                \
      *(u32x4*)(ptr) = lo8_;                                                       \
      *(u32x4*)((ptr) + 8) = hi8_;                                                 \
    } else {                                                                       \
      *(u32x4*)(ptr) = v;                                                          \
    }                                                                              \
  }
#define MPZ_LOAD_GLOBAL(set, kt)                                                   \
  {                                                                                \
    const int soff = ((kt) + kt0) * BK * 2;                                        \
    _Pragma("unroll") for (int d = 0; d < NW; ++d)                                 \
      _Pragma("unroll") for (int i = 0; i < LW; ++i)                               \
        rw[set][d][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, voffW[d][i], soff >> WSH, 0); \
    if constexpr (WQ == 2)                                                         \
      _Pragma("unroll") for (int i = 0; i < LW; ++i)                               \
        ra[set][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrcA, voffA[i], ((kt) + kt0) * 4, 0)); \
    _Pragma("unroll") for (int i = 0; i < LX; ++i)                                 \
      rx[set][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcX, voffX[i], soff, 0); \
    __builtin_amdgcn_sched_barrier(0);   /* keep the fetch here: the scheduler would sink it to its use */ \
  }
#define MPZ_STORE_LDS(set, stage)                                                  \
  {                                                                                \
    _Pragma("unroll") for (int d = 0; d < NW; ++d)                                 \
      _Pragma("unroll") for (int i = 0; i < LW; ++i)                               \
        MPZ_PUT_W(sW + ((stage) * NW + d) * TILE_W + ldsW[i], rw[set][d][i], ra[set][i]) \
    _Pragma("unroll") for (int i = 0; i < LX; ++i)                                 \
      *(u32x4*)(sX + (stage) * TILE_X + ldsX[i]) = rx[set][i];                     \
    __builtin_amdgcn_sched_barrier(0);                                             \
  }
#define MPZ_READ_FRAGS(buf, cw, cx, kk)                                           \
  {                                                                                \
    _Pragma("unroll") for (int d = 0; d < NW; ++d)                                 \
      _Pragma("unroll") for (int i = 0; i < NI; ++i)                               \
        fw[buf][d][i] = as_frag(*(const u32x4*)((cw) + d * TILE_W + (wn + i * 32 + lrow) * LDS_STRIDE + (kk) + lhalf * 8)); \
    _Pragma("unroll") for (int j = 0; j < NJ; ++j)                                 \
      fx[buf][j] = as_frag(*(const u32x4*)((cx) + (wm + j * 32 + lrow) * LDS_STRIDE + (kk) + lhalf * 8)); \
  }
#define MPZ_MFMAS(buf)                                                             \
  {                                                                                \
    _Pragma("unroll") for (int d = 0; d < NW; ++d)                                 \
      _Pragma("unroll") for (int i = 0; i < NI; ++i)                               \
        _Pragma("unroll") for (int j = 0; j < NJ; ++j)                             \
          acc[d][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][d][i], fx[buf][j], acc[d][i][j], 0, 0, 0); \
  }
// last tile(s): nothing left to fetch or store
#define MPZ_COMPUTE(stage)                                                         \
  {                                                                                \
    const uint16_t* cw = sW + (stage) * NW * TILE_W;                               \
    const uint16_t* cx = sX + (stage) * TILE_X;                                    \
    bf16x8 fw[1][NW][NI], fx[1][NJ];                                               \
    _Pragma("unroll") for (int kk = 0; kk < BK; kk += 16) {                        \
      MPZ_READ_FRAGS(0, cw, cx, kk)                                                \
      MPZ_MFMAS(0)                                                                 \
    }                                                                              \
  }
// One steady-state phase: MFMAs on LDS stage `cur` (tile kt) while tile kt+1 moves from register set `sset` into
// stage `nxt` and tile `ktl` = kt+2 is fetched into set `lset`.  LDS accesses keep their program order (the
// compiler cannot tell the stages apart), so that order is the intended one: the fragment reads of K-step s+1,
// then step s's share of the stores; sched_phase spreads them and the global loads between the MFMAs of step s.
#define MPZ_PHASE(cur, nxt, lset, sset, ktl)                                       \
  {                                                                                \
    const uint16_t* cw = sW + (cur) * NW * TILE_W;                                 \
    const uint16_t* cx = sX + (cur) * TILE_X;                                      \
    const int soff = ((ktl) + kt0) * BK * 2;                                       \
    bf16x8 fw[2][NW][NI], fx[2][NJ];                                               \
    MPZ_READ_FRAGS(0, cw, cx, 0)                                                   \
    _Pragma("unroll") for (int s = 0; s < KS; ++s) {                               \
      if (s + 1 < KS) MPZ_READ_FRAGS((s + 1) & 1, cw, cx, (s + 1) * 16)            \
      _Pragma("unroll") for (int c = 0; c < NV; ++c) {                             \
        if (c >= (s * NV + KS - 1) / KS && c < ((s + 1) * NV + KS - 1) / KS) {     \
          if (c < NW * LW) {                                                       \
            const int d = c / LW, i = c % LW;                                      \
            MPZ_PUT_W(sW + ((nxt) * NW + d) * TILE_W + ldsW[i], rw[sset][d][i], ra[sset][i]) \
            rw[lset][d][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcW, voffW[d][i], soff >> WSH, 0); \
            if constexpr (WQ == 2)                                                 \
              ra[lset][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrcA, voffA[i], ((ktl) + kt0) * 4, 0)); \
          } else {                                                                 \
            const int i = c - NW * LW;                                             \
            *(u32x4*)(sX + (nxt) * TILE_X + ldsX[i]) = rx[sset][i];                \
            rx[lset][i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcX, voffX[i], soff, 0); \
          }                                                                        \
        }                                                                          \
      }                                                                            \
      MPZ_MFMAS(s & 1)                                                             \
    }                                                                              \
    sched_phase<NM, NF, NW * LW, LX, WQ == 2 ? 4 : WQ == 1 ? 2 : 1, KS>();                            \
  }

  f32x16 acc[NW][NI][NJ];
#pragma unroll
  for (int d = 0; d < NW; ++d)
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[d][i][j][e] = 0.f;

  // K-tiles of this block: all of them, or with split K (grid.y = k_splits blocks per output tile, each leaving a raw
  // fp32 partial sum for the reduction kernel) the split's share.  A split's fetches past its last tile read the
  // next split's tiles (or zeros past the end): they land in the idle LDS stage and are never used.
  const int nk_all = a.K / BK;
  const int split = a.k_splits > 1 ? (int)blockIdx.y : 0;
  const int kt0 = a.k_splits > 1 ? (int)((long)nk_all * split / a.k_splits) : 0;
  const int nk = a.k_splits > 1 ? (int)((long)nk_all * (split + 1) / a.k_splits) - kt0 : nk_all;
  const bool raw = a.k_splits > 1;
  // Short-K GEMMs spend a visible share of a block's life after the main loop waiting for the low-rank operands:
  // small tiles fetch the fragments of a one-step segment (rank <= 8) now, behind the main loop (they are issued
  // first, so they have landed long before any tile load the loop waits for).
  constexpr bool PREF = !DUAL && NI * NJ <= 4;
  bf16x8 pre_fw[PREF ? NJ : 1][PREF ? NI : 1], pre_fx[PREF ? NJ : 1];
  int pre_seg = -1;
  if constexpr (PREF) {
    for (int s = 0; s < a.n_seg && split == 0; ++s)          // (with split K the low-rank term goes into split 0's sum)
      if (n0 >= a.seg[s].col_begin && n0 < a.seg[s].col_end && a.seg[s].rp == 16) pre_seg = s;
    if (pre_seg >= 0) {
      const MfmaLoraSeg& sg = a.seg[pre_seg];
      const uint16_t* tp = (const uint16_t*)sg.tp;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        int mt = m0 + wm + j * 32;
        mt = mt < a.M ? mt : a.M - 32;
        const uint16_t* bp = (const uint16_t*)sg.bp + (size_t)(mt / a.rows_per_copy) * sg.copy_stride;
        pre_fx[j] = as_frag(*(const u32x4*)(tp + (size_t)(mt + lrow) * sg.rp + lhalf * 8));
#pragma unroll
        for (int i = 0; i < NI; ++i)
          pre_fw[j][i] = as_frag(*(const u32x4*)(bp + (size_t)(n0 + wn + i * 32 + lrow - sg.col_begin) * sg.rp + lhalf * 8));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  }

  constexpr int NM = NW * NI * NJ, NF = NW * NI + NJ, NV = NW * LW + LX, KS = BK / 16;
  // Tile kt+1 sits in one register set (in flight or landed) while tile kt+2 is fetched into the other: a load
  // Tile kt+1 sits in one register set (in flight or landed) while tile kt+2 is fetched into the other: a load
  // has two MFMA phases to arrive before its LDS store needs it.  Loads past the last tile fall outside the
  // buffers (zeros); what they put into the idle LDS stage is never read.
  {
  MPZ_LOAD_GLOBAL(0, 0)
  MPZ_LOAD_GLOBAL(1, 1)                  // both in flight before the first wait
  MPZ_STORE_LDS(0, 0)
  __syncthreads();
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    MPZ_PHASE(0, 1, 0, 1, kt + 2)        // even phase: stage 0 is current, set 1 holds tile kt+1
    __syncthreads();
    MPZ_PHASE(1, 0, 1, 0, kt + 3)        // odd phase: stage 1 is current, set 0 holds tile kt+2
    __syncthreads();
  }
  if (kt < nk) MPZ_COMPUTE(0)            // odd number of tiles: the last one is already in stage 0
  }
#undef MPZ_LOAD_GLOBAL
#undef MPZ_PUT_W
#undef MPZ_READ_FRAGS
#undef MPZ_MFMAS
#undef MPZ_PHASE
#undef MPZ_STORE_LDS
#undef MPZ_COMPUTE

  // int8 weights: the accumulators hold x . codes; the per-output-channel scale turns them into x . W before
  // anything else (low-rank term, bias) is added
  if constexpr (WQ == 1) {
#pragma unroll
    for (int d = 0; d < NW; ++d)
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int n = n0 + wn + i * 32 + g * 8 + lhalf * 4;
          n = n < a.N ? n : 0;
          const f32x4 sc = *(const f32x4*)(a.w_scale + (d == 0 ? 0 : a.dual_offset) + n);
#pragma unroll
          for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[d][i][j][g * 4 + e] *= sc[e];
        }
  }

  // per-copy low-rank term: extra K-steps with the packed factor [B_hi | B_lo] of a copy against the duplicated
  // bottleneck activations [t | t].  Copies are whole multiples of 32 rows, so every 32-row MFMA tile belongs to
  // one copy (a block tile may span several); segments are aligned to the block tile.
  if (PREF && pre_seg >= 0) {
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int i = 0; i < NI; ++i)
        acc[0][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pre_fw[j][i], pre_fx[j], acc[0][i][j], 0, 0, 0);
  } else if constexpr (!DUAL) {
    for (int s = 0; s < a.n_seg && split == 0; ++s) {
      const MfmaLoraSeg& sg = a.seg[s];
      if (n0 < sg.col_begin || n0 >= sg.col_end) continue;
      const uint16_t* tp = (const uint16_t*)sg.tp;
      for (int ks = 0; ks < sg.rp; ks += 16) {
        // all fragments of the step first, then its MFMAs: the block waits for L2 once per step, not once per tile
        bf16x8 lx[NJ], lw[NJ][NI];
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          int mt = m0 + wm + j * 32;                       // first row of this MFMA tile
          mt = mt < a.M ? mt : a.M - 32;                   // tiles past the end compute discarded values in bounds
          const int copy = mt / a.rows_per_copy;
          const uint16_t* bp = (const uint16_t*)sg.bp + (size_t)copy * sg.copy_stride;
          lx[j] = as_frag(*(const u32x4*)(tp + (size_t)(mt + lrow) * sg.rp + ks + lhalf * 8));
#pragma unroll
          for (int i = 0; i < NI; ++i) {
            const int n = n0 + wn + i * 32 + lrow - sg.col_begin;
            lw[j][i] = as_frag(*(const u32x4*)(bp + (size_t)n * sg.rp + ks + lhalf * 8));
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
          for (int i = 0; i < NI; ++i)
            acc[0][i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lw[j][i], lx[j], acc[0][i][j], 0, 0, 0);
      }
    }
  }

  // Epilogue, part 1 (accumulator layout: a lane holds, for token m = lrow, features nb + g*8 + lhalf*4 + (0..3),
  // g = 0..3, of every MFMA tile): bias, activation or gating, rotary embedding -- everything that needs no
  // other token's data -- written back into acc[0].
  const bool relu = !DUAL && a.act == MPZ_ACT_RELU;
  if (!raw) {
#pragma unroll
  for (int i = 0; i < NI; ++i)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      int n = n0 + wn + i * 32 + g * 8 + lhalf * 4;
      n = n < a.N ? n : 0;                                 // columns past N are never stored
      f32x4 bg = {0.f, 0.f, 0.f, 0.f}, bu = bg;
      if (a.bias != nullptr) {
        bg = *(const f32x4*)(a.bias + n);
        if (DUAL) bu = *(const f32x4*)(a.bias + a.dual_offset + n);
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float v = acc[0][i][j][g * 4 + e] + bg[e];
          if (DUAL) {
            const float u = acc[NW - 1][i][j][g * 4 + e] + bu[e];
            v = silu_mul_f32(v, u);                        // SiLU(gate) * up
          } else {
            v = (relu && !(v > 0.f)) ? 0.f : v;            // a select, not a branch per element
          }
          acc[0][i][j][g * 4 + e] = v;
        }
    }
  }
  if (!raw && !DUAL && a.act == MPZ_ACT_GELU_ERF) {                // rare (no workload of the paper uses it): one cold loop
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[0][i][j][e] = gelu_erf_call(acc[0][i][j][e]);
  }
  if constexpr (HP > 0) {
    static_assert(!DUAL && NI >= 2 * HP && NI % (2 * HP) == 0, "a wave tile must hold whole heads");
    if (!raw && n0 < a.rope_cols) {
      // q / k columns: y_lo = x_lo cos - x_hi sin, y_hi = x_hi cos + x_lo sin with (lo, hi) = columns (c, c + d_head/2)
      const int half = 32 * HP;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        int m = m0 + wm + j * 32 + lrow;
        m = m < a.M ? m : a.M - 1;
        const int pos = a.rope_pos != nullptr ? a.rope_pos[m % a.S] : m % a.S;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          if ((i / HP) % 2 != 0) continue;                  // upper halves are rotated together with their lower half
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int c = (i % HP) * 32 + g * 8 + lhalf * 4;  // column inside the lower half of the head
            const f32x4 cs = *(const f32x4*)(a.rope_cos + (size_t)pos * half + c);
            const f32x4 sn = *(const f32x4*)(a.rope_sin + (size_t)pos * half + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float lo = acc[0][i][j][g * 4 + e], hi = acc[0][i + HP][j][g * 4 + e];
              // one rounded product, one fma: the same two operations as the stand-alone rotary kernel, so a pass
              // that takes that kernel (tile too narrow for a whole head) gives the same bits
              acc[0][i][j][g * 4 + e] = fmaf(lo, cs[e], -__fmul_rn(hi, sn[e]));
              acc[0][i + HP][j][g * 4 + e] = fmaf(hi, cs[e], __fmul_rn(lo, sn[e]));
            }
          }
        }
      }
    }
  }

  // Fused cross-entropy: the logits never leave the registers.  A lane holds NI * 16 columns of token row lrow
  // (the other half of the row's columns sits in lane ^ 32): row maximum, sum of exponentials against it, and
  // the target's logit if it falls into this wave tile.
  if (a.ce_max != nullptr) {
    constexpr float LOG2E = 1.4426950408889634f;
    const int slot = (n0 / BN) * WGN + wave / WGM;
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int m = m0 + wm + j * 32 + lrow;
      const int tg = m < a.M ? a.ce_target[m] : -1;
      float mx = -1e30f, tl = 0.f;
      bool has = false;
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int n = n0 + wn + i * 32 + g * 8 + lhalf * 4 + e;
            const float v = acc[0][i][j][g * 4 + e];
            if (n < a.N) mx = v > mx ? v : mx;
            if (n == tg) { tl = v; has = true; }
          }
      const float other = __shfl_xor(mx, 32);
      mx = other > mx ? other : mx;
      float sum = 0.f;
#pragma unroll
      for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int n = n0 + wn + i * 32 + g * 8 + lhalf * 4 + e;
            if (n < a.N) sum += __builtin_amdgcn_exp2f((acc[0][i][j][g * 4 + e] - mx) * LOG2E);
          }
      sum += __shfl_xor(sum, 32);
      if (m < a.M) {
        if (lhalf == 0) {
          a.ce_max[(size_t)slot * a.M + m] = mx;
          a.ce_sum[(size_t)slot * a.M + m] = sum;
        }
        if (has) a.ce_tlogit[m] = tl;
      }
    }
    return;
  }

  // Epilogue, part 2: each wave turns its tile around in a private LDS strip, 32 tokens at a time, so that a lane
  // ends up with 4 consecutive features of a token and consecutive lanes with consecutive features: residual reads
  // and output stores then cover whole 128-byte lines (straight from the accumulator layout a store instruction
  // would touch 32 token rows with 16 bytes each).
  constexpr int EPS = TN + 4;                              // strip row stride in floats: conflict-free 16-byte columns
  constexpr int LPR = TN / 4;                              // lanes per token row on the way out
  float* ep = (float*)smem + wave * 32 * EPS;
  __syncthreads();                                         // every wave is done with the operand stages
  // With split K the raw sums of this split go out instead (fp32, no bias / activation / residual; both weight tiles
  // of a dual launch, the second N columns to the right): partial[split][m][d N + n], row stride ldp.
  const int nd = raw ? NW : 1;
  const int ld = raw ? a.ldp : a.ldo;
  float* const praw = raw ? a.partial + (size_t)split * a.M * a.ldp : nullptr;
#pragma unroll
  for (int d = 0; d < NW; ++d) {
  if (d >= nd) break;
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 v = {acc[d][i][j][g * 4], acc[d][i][j][g * 4 + 1], acc[d][i][j][g * 4 + 2], acc[d][i][j][g * 4 + 3]};
        *(f32x4*)(ep + lrow * EPS + i * 32 + g * 8 + lhalf * 4) = v;
      }
    // RB pieces at a time: all their residual loads are issued before the first is used (a piece past M or N reads
    // a clamped, in-bounds address and is not stored), and the kind of output is decided outside the loops
    constexpr int R = 32 * LPR / 64, RB = R % 8 == 0 ? 8 : 4;
    static_assert(R % RB == 0, "pieces must deal out evenly to the batches");
#pragma unroll
    for (int r0 = 0; r0 < R; r0 += RB) {
      f32x4 v[RB];
      size_t o[RB];
      bool ok[RB];
#pragma unroll
      for (int r = 0; r < RB; ++r) {
        const int idx = (r0 + r) * 64 + lane, row = idx / LPR, c4 = idx % LPR;
        const int m = m0 + wm + j * 32 + row, n = n0 + wn + c4 * 4;
        ok[r] = m < a.M && n < a.N;
        o[r] = (size_t)(m < a.M ? m : a.M - 1) * ld + (n < a.N ? n : 0) + (raw ? d * a.N : 0);
        v[r] = *(const f32x4*)(ep + row * EPS + c4 * 4);
      }
      if (raw) {
#pragma unroll
        for (int r = 0; r < RB; ++r)
          if (ok[r]) *(f32x4*)(praw + o[r]) = v[r];
        continue;
      }
      if (a.residual != nullptr) {
        f32x4 rs[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) rs[r] = *(const f32x4*)(a.residual + o[r]);
#pragma unroll
        for (int r = 0; r < RB; ++r) v[r] += rs[r];
      }
      if (a.out_f32) {
#pragma unroll
        for (int r = 0; r < RB; ++r)
          if (ok[r]) *(f32x4*)((float*)a.out + o[r]) = v[r];
      } else {
#pragma unroll
        for (int r = 0; r < RB; ++r)
          if (ok[r]) {
            u32x2 pk = {pack_bf16x2(v[r][0], v[r][1]), pack_bf16x2(v[r][2], v[r][3])};
            *(u32x2*)((uint16_t*)a.out + o[r]) = pk;
          }
      }
    }
  }
  }
}

// Measurement: what the memory system delivers to a read-only kernel whose access pattern is that of a GEMM's weight
// operand.  The buffer is [rows][row_bytes]; a block owns `rb` consecutive rows and a 1/k_splits share of each row and
// walks it in tiles of rb rows x seg bytes (thread t takes the 16-byte chunks t, t + 256, ... of a tile, chunk c =
// 16 bytes number c % (seg / 16) of row c / (seg / 16): a wave's load covers 1024 / seg rows); the next tile is
// fetched before the current one is consumed.  rb = 128, seg = 128 is the 128 x 64 bf16 tile of the few-token GEMMs;
// rb = 1 and a long seg is a sequential stream per block.  `lds_bytes` of dynamic LDS limit the blocks per CU.  mode
// bit 0: every tile is accompanied by the tile of rows 0 .. rb - 1 at the same row offset (the activation operand:
// the same for all blocks, so it comes from L2); bit 1: the tiles go through LDS with two barriers per tile.
template <int L>
__global__ void __launch_bounds__(256) hbm_read_probe_kernel(const u32x4* __restrict__ buf, long row_chunks, int rb, int seg_chunks,
                                                             int tiles_per_split, int mode, uint32_t* __restrict__ out) {
  extern __shared__ __align__(16) unsigned char probe_smem[];
  u32x4* lds = (u32x4*)probe_smem;
  const int tid = threadIdx.x;
  const long koff = (long)blockIdx.y * tiles_per_split * seg_chunks;
  const u32x4* base = buf + (long)blockIdx.x * rb * row_chunks + koff;
  const u32x4* xbase = buf + koff;                       // mode bit 0: the tile of rows 0 .. rb - 1, shared by all blocks
  const bool with_x = mode & 1, via_lds = mode & 2;
  long off[L];
#pragma unroll
  for (int i = 0; i < L; ++i) {
    const int c = tid + 256 * i;
    off[i] = (long)(c / seg_chunks) * row_chunks + c % seg_chunks;
  }
  u32x4 cur[L], nxt[L], xcur[L], xnxt[L], acc = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < L; ++i) {
    cur[i] = base[off[i]];
    xcur[i] = with_x ? xbase[off[i]] : acc;
  }
  for (int t = 0; t < tiles_per_split; ++t) {
    const long adv = (long)(t + 1 < tiles_per_split ? t + 1 : t) * seg_chunks;
#pragma unroll
    for (int i = 0; i < L; ++i) {
      nxt[i] = base[adv + off[i]];
      xnxt[i] = with_x ? xbase[adv + off[i]] : acc;
    }
    if (via_lds) {                                       // mode bit 1: both tiles through LDS, two barriers per tile
      __syncthreads();
#pragma unroll
      for (int i = 0; i < L; ++i) {
        lds[tid + 256 * i] = cur[i];
        if (with_x) lds[256 * L + tid + 256 * i] = xcur[i];
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < L; ++i) {
        acc ^= lds[(tid * 7 + 256 * i) % (256 * L)];
        if (with_x) acc ^= lds[256 * L + (tid * 5 + 256 * i) % (256 * L)];
      }
    } else {
#pragma unroll
      for (int i = 0; i < L; ++i) acc ^= cur[i] ^ xcur[i];
    }
#pragma unroll
    for (int i = 0; i < L; ++i) { cur[i] = nxt[i]; xcur[i] = xnxt[i]; }
  }
  if (tid == 0) out[blockIdx.y * gridDim.x + blockIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}


// ---- measurement: the matrix cores alone, and with the main loop's fragment reads ---------------------------
// 8 waves per block (two per SIMD, the large tile's occupancy); a wave holds the 128 x 64 wave tile's 8 accumulator
// tiles and issues 8 MFMAs per step.  Operand fragments come from `operands` (the caller chooses the bit patterns:
// the rate the chip sustains depends on how many operand bits toggle).  with_lds = 0: fragments stay in registers;
// 1: the 4 + 2 fragments of every step are read from LDS again, as in gemm_bf16_kernel's main loop.
__global__ void __launch_bounds__(512, 1) mfma_probe_kernel(const uint16_t* __restrict__ operands, int iters, int with_lds,
                                                            float* __restrict__ out) {
  __shared__ __align__(16) uint16_t lds[(256 + 256) * 72];         // a 256 x 64 W tile and a 256 x 64 x tile, rows of 64 (+8)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lhalf = lane >> 5;
  for (int i = tid; i < (256 + 256) * 72 / 8; i += 512)
    *(u32x4*)(lds + i * 8) = *(const u32x4*)(operands + (size_t)(i % 1536) * 8);
  __syncthreads();
  const uint16_t* mw = lds + (wave / 4) * 128 * 72;                // this wave's 128 W rows and 64 x rows
  const uint16_t* mx = lds + (256 + (wave % 4) * 64) * 72;
  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  bf16x8 fw[4], fx[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) fw[i] = as_frag(*(const u32x4*)(mw + (i * 32 + lrow) * 72 + lhalf * 8));
#pragma unroll
  for (int j = 0; j < 2; ++j) fx[j] = as_frag(*(const u32x4*)(mx + (j * 32 + lrow) * 72 + lhalf * 8));
  if (with_lds == 2) {
    // LDS fragment reads alone (no MFMA), 24 in flight per wave (the 6 fragments of four K-steps) before any is
    // consumed: the rate at which the LDS delivers ds_read_b128 to the 8 waves of a CU
    u32x4 chk = {0u, 0u, 0u, 0u};
    for (int it = 0; it < iters; it += 4) {
      u32x4 r[4][6];
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
#pragma unroll
        for (int i = 0; i < 4; ++i) r[s4][i] = *(const u32x4*)(mw + (i * 32 + lrow) * 72 + s4 * 16 + lhalf * 8);
#pragma unroll
        for (int j = 0; j < 2; ++j) r[s4][4 + j] = *(const u32x4*)(mx + (j * 32 + lrow) * 72 + s4 * 16 + lhalf * 8);
      }
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
        for (int i = 0; i < 6; ++i) chk ^= r[s4][i];
      asm volatile("" ::: "memory");                       // the next round reads LDS again
    }
    out[(size_t)blockIdx.x * 512 + tid] = __uint_as_float(chk[0] ^ chk[1] ^ chk[2] ^ chk[3]);
    return;
  }
  for (int it = 0; it < iters; ++it) {
    if (with_lds) {
      const int kk = (it & 3) * 16;
#pragma unroll
      for (int i = 0; i < 4; ++i) fw[i] = as_frag(*(const u32x4*)(mw + (i * 32 + lrow) * 72 + kk + lhalf * 8));
#pragma unroll
      for (int j = 0; j < 2; ++j) fx[j] = as_frag(*(const u32x4*)(mx + (j * 32 + lrow) * 72 + kk + lhalf * 8));
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fx[j], acc[i][j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) sum += acc[i][j][e];
  out[(size_t)blockIdx.x * 512 + tid] = sum;
}

// ---- LoRA bottleneck: tp[m] = [t | t | 0], t = bf16(scale * x (A_hi + A_lo)) for the block's copy ----------
// HBM-bound (it reads x once).  One block = 32 tokens.  x streams through LDS in chunks of 256 K-elements with
// fully coalesced 16-byte loads (a wave reads two whole 512-byte row pieces per instruction; reading MFMA
// fragments straight from the row-major x would touch 32 rows per instruction), one chunk in flight in registers
// while the previous one is consumed.  Inside a chunk the 4 waves split K; their partial sums meet in LDS in a
// fixed order.  MFMA rows = bottleneck columns j of all targets that share the input x.
template <int JT>   // number of 32-row MFMA tiles covering n_targets * r bottleneck columns
__global__ void __launch_bounds__(256, 2) lora_down_mfma_kernel(MfmaLoraDownArgs a) {
  constexpr int KCH = 256, XS = KCH + 8;
  __shared__ __align__(16) uint16_t sx[3][32 * XS];
  __shared__ float part[3][JT][16][64];          // partial sums of waves 1..3
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, lrow = lane & 31, lhalf = lane >> 5;
  const int m0 = blockIdx.x * 32;
  const int copy = m0 / a.rows_per_copy;
  const int R = a.n_targets * a.rank;
  const uint16_t* X = (const uint16_t*)a.x + (size_t)m0 * a.K;
  // packed A: per copy and target [2][K / 8][rank][8] (hi part then lo part): the 16-byte pieces that the lanes of
  // a wave fetch for one MFMA operand (rank rows x 2 neighbouring chunks of 8 k) are contiguous
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
    Ah[t] = base + ((size_t)(wave * 8 + lhalf) * a.rank + jr) * 8;
    Al[t] = Ah[t] + (size_t)a.K * a.rank;
  }
  f32x16 acc[JT];
#pragma unroll
  for (int t = 0; t < JT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  const u32x4 zero = {0u, 0u, 0u, 0u};

  // chunk staging: piece p = tid + 256 i of the 32 x 256 chunk: row p / 32, 16-byte column p % 32
  int grow[4], gcol[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { int p = tid + 256 * i; grow[i] = p >> 5; gcol[i] = (p & 31) * 8; }
  // three chunks of x in flight (registers), three LDS buffers: a K = 768 row is fetched in one go
  constexpr int PD = 3;
  u32x4 st[PD][4];
  const int nch = a.K / KCH;
#pragma unroll
  for (int p = 0; p < PD; ++p)
    if (p < nch) {
#pragma unroll
      for (int i = 0; i < 4; ++i) st[p][i] = *(const u32x4*)(X + (size_t)grow[i] * a.K + p * KCH + gcol[i]);
    }
  for (int ch0 = 0; ch0 < nch; ch0 += PD) {
#pragma unroll
    for (int p = 0; p < PD; ++p) {
      const int ch = ch0 + p;
      if (ch >= nch) break;                        // block-uniform
      uint16_t* buf = sx[p];
      const int kg = ch * KCH;
      // this chunk's factor fragments (L2-resident) are fetched first, so that they travel while the x chunk is
      // stored and the block meets at the barrier
      u32x4 fh[4][JT], fl[4][JT];
      const int r16 = 16 * a.rank;                 // elements between the pieces of consecutive K-steps
#pragma unroll
      for (int t = 0; t < JT; ++t) {
        const uint16_t* ph = Ah[t] + kg * a.rank;
        const uint16_t* pl = Al[t] + kg * a.rank;
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          fh[s4][t] = valid[t] ? *(const u32x4*)(ph + s4 * r16) : zero;
          fl[s4][t] = valid[t] ? *(const u32x4*)(pl + s4 * r16) : zero;
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) *(u32x4*)(buf + grow[i] * XS + gcol[i]) = st[p][i];
      if (ch + PD < nch) {
#pragma unroll
        for (int i = 0; i < 4; ++i) st[p][i] = *(const u32x4*)(X + (size_t)grow[i] * a.K + (ch + PD) * KCH + gcol[i]);
      }
      __syncthreads();                             // chunk ch visible; its buffer was last read three chunks ago
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4) {
        bf16x8 fx = as_frag(*(const u32x4*)(buf + lrow * XS + wave * 64 + s4 * 16 + lhalf * 8));
#pragma unroll
        for (int t = 0; t < JT; ++t) {
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fh[s4][t]), fx, acc[t], 0, 0, 0);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(fl[s4][t]), fx, acc[t], 0, 0, 0);
        }
      }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int t = 0; t < JT; ++t)
#pragma unroll
      for (int e = 0; e < 16; ++e) part[wave - 1][t][e][lane] = acc[t][e];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int t = 0; t < JT; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = ((acc[t][e] + part[0][t][e][lane]) + part[1][t][e][lane]) + part[2][t][e][lane];
  // lane holds token m0 + lrow, bottleneck columns j = t*32 + g*8 + lhalf*4 + e
  const int m = m0 + lrow;
  // (ranks are multiples of 4: the 4 consecutive columns of a lane belong to one target and go out as one 8-byte store)
#pragma unroll
  for (int t = 0; t < JT; ++t)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int j = t * 32 + g * 8 + lhalf * 4;
      if (j >= R) continue;
      const int tgt = j / a.rank, jr = j % a.rank;
      const u32x2 pk = {pack_bf16x2(acc[t][g * 4] * a.scale, acc[t][g * 4 + 1] * a.scale),
                        pack_bf16x2(acc[t][g * 4 + 2] * a.scale, acc[t][g * 4 + 3] * a.scale)};
      uint16_t* row = (uint16_t*)a.tp[tgt] + (size_t)m * a.rp;
      *(u32x2*)(row + jr) = pk;
      *(u32x2*)(row + a.rank + jr) = pk;
    }
  // zero padding up to rp (done by lhalf 0 lanes; rp - 2 rank is 0 or 8)
  if (lhalf == 0)
    for (int tgt = 0; tgt < a.n_targets; ++tgt)
      for (int c = 2 * a.rank; c < a.rp; ++c) ((uint16_t*)a.tp[tgt])[(size_t)m * a.rp + c] = 0;
}

// ---- pack the perturbed fp32 factors into the bf16 hi/lo operand layouts ---------------------------------
// A [K, r] (master layout) -> ap [2][K / 8][r][8] (hi part, lo part);  B [r, k_out] -> bp [k_out][rp] = [hi(r) | lo(r) | 0]
__global__ void __launch_bounds__(256) pack_factors_kernel(const float* __restrict__ pert, int64_t P, int n_copies,
                                                           LoraLayerTable tab, int n_layers, int rank, int rp,
                                                           uint16_t* __restrict__ packed, int64_t packed_per_copy) {
  // one thread per master element
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)n_copies * P) return;
  int copy = (int)(idx / P);
  int64_t e = idx % P;
  int layer = (int)(e / tab.per_layer);
  int rem = (int)(e % tab.per_layer);
  int i = 0;
  while (i + 1 < tab.n_tensors && rem >= tab.off[i + 1]) ++i;
  int local = rem - tab.off[i];
  float v = pert[idx];
  uint16_t hi = f32_to_bf16(v).bits;
  bf16_t hb; hb.bits = hi;
  uint16_t lo = f32_to_bf16(v - bf16_to_f32(hb)).bits;
  // packed offset of tensor i inside a layer: A tensors take 2*rows*cols, B tensors take cols*rp
  int64_t poff = 0;
  for (int t = 0; t < i; ++t) poff += (tab.local_id[t] & 1) ? (int64_t)tab.cols[t] * rp : (int64_t)2 * tab.rows[t] * tab.cols[t];
  int64_t per_layer_packed = poff;
  for (int t = i; t < tab.n_tensors; ++t)
    per_layer_packed += (tab.local_id[t] & 1) ? (int64_t)tab.cols[t] * rp : (int64_t)2 * tab.rows[t] * tab.cols[t];
  uint16_t* dst = packed + (int64_t)copy * packed_per_copy + (int64_t)layer * per_layer_packed + poff;
  if ((tab.local_id[i] & 1) == 0) {              // A [K, r]: element (k, j) -> [k / 8][j][k % 8] of the hi and of the lo part
    int K = tab.rows[i];
    int k = local / rank, j = local % rank;
    if (K % 8 == 0) {
      const int64_t o = ((int64_t)(k / 8) * rank + j) * 8 + k % 8;
      dst[o] = hi;
      dst[(int64_t)K * rank + o] = lo;
    } else {                                      // no whole chunks: plain rows, which stay inside the factor's 2 r K elements
      dst[(int64_t)j * K + k] = hi;               // (the bottleneck kernels that read this buffer need K % 256 == 0)
      dst[(int64_t)(rank + j) * K + k] = lo;
    }
  } else {                                        // B [r, k_out]: element (j, n) -> [n][j] hi, [n][r + j] lo
    int kout = tab.cols[i];
    int j = local / kout, n = local % kout;
    dst[(int64_t)n * rp + j] = hi;
    dst[(int64_t)n * rp + rank + j] = lo;
    if (j == 0)
      for (int c = 2 * rank; c < rp; ++c) dst[(int64_t)n * rp + c] = 0;
  }
}


// The same packing with 16-byte accesses on the side that matters.  Work items per (copy, layer): for an A factor
// one thread per (chunk of 8 consecutive k, column j): consecutive lanes read consecutive floats of a row of A and
// write consecutive 16-byte pieces of the hi part and of the lo part; for a B factor one thread per output feature n (reads
// column n of B, contiguous across lanes; writes its whole packed row [hi | lo | 0]).
template <int RANK>
__global__ void __launch_bounds__(256) pack_factors_vec_kernel(const float* __restrict__ pert, int64_t P, int n_copies,
                                                               LoraLayerTable tab, int n_layers, int rp,
                                                               uint16_t* __restrict__ packed, int64_t packed_per_copy,
                                                               int items_per_layer) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_copy = (int64_t)items_per_layer * n_layers;
  if (idx >= per_copy * n_copies) return;
  const int copy = (int)(idx / per_copy);
  const int64_t r0 = idx % per_copy;
  const int layer = (int)(r0 / items_per_layer);
  int item = (int)(r0 % items_per_layer);
  int i = 0;
  int64_t poff = 0;
  for (;; ++i) {                                   // which factor of the layer, and where its packed form starts
    const bool isB = tab.local_id[i] & 1;
    const int cnt = isB ? tab.cols[i] : tab.rows[i] / 8 * RANK;
    if (item < cnt) break;
    item -= cnt;
    poff += isB ? (int64_t)tab.cols[i] * rp : (int64_t)2 * tab.rows[i] * tab.cols[i];
  }
  int64_t per_layer_packed = 0;
  for (int t = 0; t < tab.n_tensors; ++t)
    per_layer_packed += (tab.local_id[t] & 1) ? (int64_t)tab.cols[t] * rp : (int64_t)2 * tab.rows[t] * tab.cols[t];
  const float* src = pert + (int64_t)copy * P + (int64_t)layer * tab.per_layer + tab.off[i];
  uint16_t* dst = packed + (int64_t)copy * packed_per_copy + (int64_t)layer * per_layer_packed + poff;
  if ((tab.local_id[i] & 1) == 0) {                // A [K, r]: rows k0..k0+7 of column j -> piece [k0 / 8][j] of the hi and of the lo part
    const int K = tab.rows[i], chunk = item / RANK, j = item % RANK, k0 = chunk * 8;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = src[(int64_t)(k0 + e) * RANK + j];
    uint32_t hi[4], lo[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
      const bf16_t h0 = f32_to_bf16(v[e]), h1 = f32_to_bf16(v[e + 1]);
      const bf16_t l0 = f32_to_bf16(v[e] - bf16_to_f32(h0)), l1 = f32_to_bf16(v[e + 1] - bf16_to_f32(h1));
      hi[e / 2] = (uint32_t)h0.bits | ((uint32_t)h1.bits << 16);
      lo[e / 2] = (uint32_t)l0.bits | ((uint32_t)l1.bits << 16);
    }
    const u32x4 hv = {hi[0], hi[1], hi[2], hi[3]}, lv = {lo[0], lo[1], lo[2], lo[3]};
    *(u32x4*)(dst + (int64_t)item * 8) = hv;
    *(u32x4*)(dst + (int64_t)K * RANK + (int64_t)item * 8) = lv;
  } else {                                         // B [r, k_out]: column n -> packed row n = [hi(r) | lo(r) | 0]
    const int kout = tab.cols[i], n = item;
    uint16_t* row = dst + (int64_t)n * rp;
    uint16_t hb[RANK], lb[RANK];
#pragma unroll
    for (int j = 0; j < RANK; ++j) {
      const float x = src[(int64_t)j * kout + n];
      const bf16_t h = f32_to_bf16(x);
      hb[j] = h.bits;
      lb[j] = f32_to_bf16(x - bf16_to_f32(h)).bits;
    }
    if constexpr (RANK % 4 == 0) {
#pragma unroll
      for (int j = 0; j < RANK; j += 4) {
        const u32x2 hv = {(uint32_t)hb[j] | ((uint32_t)hb[j + 1] << 16), (uint32_t)hb[j + 2] | ((uint32_t)hb[j + 3] << 16)};
        const u32x2 lv = {(uint32_t)lb[j] | ((uint32_t)lb[j + 1] << 16), (uint32_t)lb[j + 2] | ((uint32_t)lb[j + 3] << 16)};
        *(u32x2*)(row + j) = hv;
        *(u32x2*)(row + RANK + j) = lv;
      }
    }
    for (int c = 2 * RANK; c < rp; ++c) row[c] = 0;
  }
}

// ---- tile configurations ----------------------------------------------------------------------------
// The numbered configurations (BN x BM x BK, waves) are listed where they are instantiated, in launch_gemm_mfma;
// choose_cfg picks among 6 (256 x 256 x 64, 8 waves: large problems), 12 and 1 (128 x 128 x 64 with 8 or 4 waves),
// 11 (192 x 128 x 64), 9 and 10 (128 x 64 and 64 x 64: problems with fewer tiles than CUs).  LDS = stages x (BN + BM) x (BK + 8) x 2 bytes, or the epilogue strips if those are larger.
template <int BN, int BM, int BK, int WGN, int WGM, bool DUAL, int HP = 0, int WQ = 0>
hipError_t launch_cfg(hipStream_t st, const MfmaGemmArgs& a) {
  constexpr size_t lds_stages = (size_t)2 * ((DUAL ? 2 : 1) * BN + BM) * (BK + 8) * 2;
  constexpr size_t lds_strips = (size_t)WGN * WGM * 32 * (BN / WGN + 4) * 4;          // epilogue: one strip per wave
  constexpr size_t lds = lds_stages > lds_strips ? lds_stages : lds_strips;
  // the kernel's dynamic LDS limit is raised once per instance (two host threads may arrive here together); a
  // refusal is remembered and makes every launch of this instance fail with that error instead of an opaque one
  static std::once_flag once;
  static hipError_t attr_status = hipSuccess;
  std::call_once(once, [] {
    attr_status = hipFuncSetAttribute((const void*)gemm_bf16_kernel<BN, BM, BK, WGN, WGM, DUAL, HP, WQ>,
                                      hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  });
  if (attr_status != hipSuccess) return attr_status;
  const int tiles = ((a.N + BN - 1) / BN) * ((a.M + BM - 1) / BM);
  const dim3 grid((unsigned)tiles, (unsigned)(a.k_splits > 1 ? a.k_splits : 1));
  gemm_bf16_kernel<BN, BM, BK, WGN, WGM, DUAL, HP, WQ><<<grid, 64 * WGN * WGM, lds, st>>>(a);
  return hipSuccess;
}

// block tile of configuration cfg (1, 6, 9, 10, 11, 12, 13; see launch_gemm_mfma)
int tile_bn(int cfg) { return (cfg == 10 || cfg == 13) ? 64 : cfg == 11 ? 192 : cfg == 6 ? 256 : 128; }
int tile_bm(int cfg) { return (cfg == 9 || cfg == 10) ? 64 : cfg == 6 ? 256 : 128; }
bool known_cfg(int cfg) { return cfg == 1 || cfg == 6 || (cfg >= 9 && cfg <= 13); }

bool cfg_ok(const MfmaGemmArgs& a, int cfg) {
  const int bn = tile_bn(cfg), bm = tile_bm(cfg);
  (void)bm;
  if (a.n_seg > 0 && (a.rows_per_copy % 32 || a.M % 32)) return false;
  for (int s = 0; s < a.n_seg; ++s)
    if (a.seg[s].col_begin % bn || a.seg[s].col_end % bn) return false;
  return true;
}

// split K: output features per block.  Wide or long-K projections stream through 128-feature tiles, the others through
// 64-feature tiles (twice the blocks); a dual launch has one tile shape.
int split_tile_bn(const MfmaGemmArgs& a) { return (a.dual || a.N >= 8192 || a.K >= 8192 || a.w_scale != nullptr || a.w_absmax != nullptr) ? 128 : 64; }

int choose_cfg(const MfmaGemmArgs& a) {
  // split K (at most 256 stacked tokens): a block takes all the tokens it can (the weights are then fetched from HBM
  // once) and as few output features as the low-rank segments allow, so that there are many blocks to stream them
  if (a.k_splits > 1) {
    const int forced = a.tile_cfg % 100;                 // measurement: tile_cfg = 100 k_splits + tile
    if (a.w_scale == nullptr && a.w_absmax == nullptr && (forced == 1 || forced == 9 || forced == 10 || forced == 12 || forced == 13) && cfg_ok(a, forced)) return forced;
    if (split_tile_bn(a) == 128 || !cfg_ok(a, 13)) return a.M <= 64 ? 9 : 1;     // 128 features x 64 or 128 tokens
    return a.M <= 64 ? 10 : 13;                                                   // 64 features x 64 or 128 tokens
  }
  const bool forced_ok = a.w_scale == nullptr || a.tile_cfg == 1 || a.tile_cfg == 6 || a.tile_cfg == 11 || a.tile_cfg == 12;   // int8: fewer instances
  if (forced_ok && known_cfg(a.tile_cfg) && cfg_ok(a, a.tile_cfg)) return a.tile_cfg;
  // enough 256 x 256 tiles to keep 256 CUs busy for several rounds -> biggest tile; else the largest tile that
  // still gives at least ~2 blocks per CU
  // The L2 -> CU path feeds about 64 B/clk per CU, which a 128 x 128 tile needs in full at MFMA peak; 256 x 256
  // halves that.  Use the big tile (8 waves of 128 x 64) once it yields two or more rounds of blocks on 256 CUs.
  const long t5 = (long)((a.N + 255) / 256) * ((a.M + 255) / 256);
  if (t5 >= 512 && cfg_ok(a, 6)) return 6;   // BK 64 with two tiles in flight: 128 KB of loads outstanding per CU
  // 128 x 128 tiles that fill between one and two blocks per CU leave half the chip with twice the work of the
  // other half; 192 x 128 tiles, one per CU, balance it (N = 768 projections of the 125M-class models)
  const long t1 = (long)((a.N + 127) / 128) * ((a.M + 127) / 128), t11 = (long)((a.N + 191) / 192) * ((a.M + 127) / 128);
  if (t1 > 256 && t1 < 512 && t11 <= 256 && a.N % 192 == 0 && a.K >= 1536 && a.rope_cos == nullptr && cfg_ok(a, 11)) return 11;
  // fewer 128 x 128 tiles than CUs (single-copy and single-query passes): 128 x 64 tiles, twice the blocks, and
  // 64 x 64 tiles if that is still less than one block per CU (one pass per copy on the 125M-shaped workload:
  // 8.2 -> 7.4 ms per step; 2 x 64 tokens through the 7B-shaped model: 75 -> 67 ms)
  if (t1 < 256 && a.rope_cos == nullptr && a.w_scale == nullptr && a.ce_max == nullptr && cfg_ok(a, 9))
    return (2 * t1 < 256 && cfg_ok(a, 10)) ? 10 : 9;
  // otherwise the 128 x 128 tile with 8 waves of 64 x 32 (16 waves per CU): a block of a short-K problem lives for
  // a dozen K-tiles, and what hides its first loads and last stores is other waves (10 % over 4 waves of 64 x 64
  // at K = 768, equal at long K)
  return 12;
}

int wave_cols(int cfg) { return (cfg == 10 || cfg == 13) ? 32 : cfg == 11 ? 96 : cfg == 6 ? 128 : 64; }   // BN / WGN of launch_gemm_mfma's table

// 64 token rows per block, the slots dealt to 4 waves: logsumexp over the per-wave-tile partials (online
// maximum / rescaled sum per thread, merged through LDS), minus the target's logit
__global__ void __launch_bounds__(256) ce_combine_kernel(int slots, int M, const float* __restrict__ ce_max,
                                                         const float* __restrict__ ce_sum,
                                                         const float* __restrict__ ce_tlogit,
                                                         const int32_t* __restrict__ ce_target, float* __restrict__ ce) {
  __shared__ float pm[4][64], psum[4][64];
  const int r = threadIdx.x & 63, part = threadIdx.x >> 6;
  const int m = blockIdx.x * 64 + r;
  float mx = -1e30f, s = 0.f;
  if (m < M) {
    for (int t = part; t < slots; t += 4) {
      const float v = ce_max[(size_t)t * M + m], sv = ce_sum[(size_t)t * M + m];
      if (v > mx) { s = s * expf(mx - v) + sv; mx = v; }
      else s += sv * expf(v - mx);
    }
  }
  pm[part][r] = mx; psum[part][r] = s;
  __syncthreads();
  if (part != 0 || m >= M) return;
  if (ce_target[m] < 0) { ce[m] = 0.f; return; }
  float gm = pm[0][r];
  for (int p = 1; p < 4; ++p) gm = pm[p][r] > gm ? pm[p][r] : gm;
  float gs = 0.f;
  for (int p = 0; p < 4; ++p) gs += psum[p][r] * expf(pm[p][r] - gm);
  ce[m] = gm + logf(gs) - ce_tlogit[m];
}

}  // namespace

int mfma_gemm_ce_slots(const MfmaGemmArgs& a0) {
  MfmaGemmArgs a = a0;
  if (a.ce_max == nullptr) a.ce_max = (float*)a.out;     // the caller asks before it has carved the buffers: the tile is chosen as for the launch
  const int cfg = choose_cfg(a);
  return ((a.N + tile_bn(cfg) - 1) / tile_bn(cfg)) * (tile_bn(cfg) / wave_cols(cfg));
}

void launch_ce_combine(hipStream_t st, int slots, int M, const float* ce_max, const float* ce_sum, const float* ce_tlogit,
                       const int32_t* ce_target, float* ce) {
  ce_combine_kernel<<<(M + 63) / 64, 256, 0, st>>>(slots, M, ce_max, ce_sum, ce_tlogit, ce_target, ce);
}

bool mfma_gemm_supported(const MfmaGemmArgs& a) {
  if (a.K % 64 || a.N % 4 || a.M < 1 || a.N < 1) return false;
  if ((size_t)a.M * a.K * 2 >= ((size_t)1 << 31) || (size_t)(a.dual ? 2 : 1) * a.N * a.K * 2 >= ((size_t)1 << 31)) return false;
  if (a.w_scale != nullptr && (a.K % 16 || ((uintptr_t)a.w_scale & 15))) return false;
  if (a.w_absmax != nullptr && (a.k_splits <= 1 || a.w_scale != nullptr || ((uintptr_t)a.w_absmax & 3) || ((uintptr_t)a.w & 15) ||
                                (a.dual && a.dual_offset != a.N) || (size_t)a.w_rows * (a.K / 64) * 4 >= ((size_t)1 << 31)))
    return false;
  for (int s = 0; s < a.n_seg; ++s)
    if (a.seg[s].rp % 16) return false;
  if (!cfg_ok(a, 1)) return false;
  if (a.dual && a.n_seg) return false;
  if (a.ce_max != nullptr && (a.dual || a.rope_cos != nullptr || !a.ce_sum || !a.ce_tlogit || !a.ce_target)) return false;
  if (a.k_splits > 1) {
    if (a.ce_max != nullptr || a.partial == nullptr || a.ldp < (a.dual ? 2 : 1) * a.N || a.ldp % 4 || a.ldo % 4) return false;
    if (a.rope_cos != nullptr && (a.dual || a.out_f32 || a.act >= 0 || a.residual != nullptr || !a.rope_sin || a.S < 1 ||
                                  a.rope_dh % 8 || a.rope_cols % a.rope_dh || a.rope_cols > a.N)) return false;
    return true;                                         // the rotation is the reduction kernel's: no tile constraints
  }
  if (a.rope_cos != nullptr) {
    // the rotated column range must end on a block-tile boundary, and a wave tile must hold whole heads
    const int cfg = choose_cfg(a), bn = tile_bn(cfg), tn = wave_cols(cfg);
    if (a.dual || a.out_f32 || a.act >= 0 || a.residual != nullptr || !a.rope_sin || a.S < 1) return false;
    if ((cfg != 6 && cfg != 1 && cfg != 12) || (a.rope_dh != 64 && a.rope_dh != 128) || a.rope_dh > tn) return false;
    if (a.rope_cols % bn || a.rope_cols > a.N || a.N % a.rope_dh) return false;
  }
  return true;
}

int mfma_gemm_splits(const MfmaGemmArgs& a, size_t partial_capacity) {
  if (a.tile_cfg >= 100) {                               // test / measurement: tile_cfg = 100 k_splits (+ tile) forces the count
    const int ks = a.tile_cfg / 100, nk = a.K / 64;
    return (ks >= 2 && ks <= nk && ks <= 64 && (size_t)ks * a.M * (a.dual ? 2 : 1) * a.N <= partial_capacity) ? ks : 1;
  }
  if (a.M > 256 || a.tile_cfg != 0 || a.ce_max != nullptr || partial_capacity == 0) return 1;
  // about one block per CU (measured on the 7B-shaped projections at 64 and 128 tokens: 2 - 8 splits are within 10 % of
  // each other, more only adds partial-sum traffic), every split at least 8 K-tiles long, and the partial sums
  // (written and read once) no more than the weight bytes
  const int bn = split_tile_bn(a);
  const int n_rows = (a.dual && a.dual_offset == a.N) ? 2 * a.N : a.N;     // stacked gate || up runs as one plain GEMM
  const long tiles = (long)((n_rows + bn - 1) / bn) * (a.M > 128 ? 2 : 1);
  if (tiles >= 256) return 1;                            // enough blocks without it
  // 4-bit codes looked up in the operand load: those blocks are bound by their own look-ups, not by memory, and a CU holds
  // two of them - as many splits as still fit that (measured best on all four 7B-shaped projections at 128 tokens)
  long ks = a.w_absmax != nullptr ? 512 / tiles : (255 + tiles) / tiles;
  const long by_k = a.K / 512, by_traffic = a.K / (4L * a.M);
  ks = ks < by_k ? ks : by_k;
  ks = ks < by_traffic ? ks : by_traffic;
  ks = ks < 16 ? ks : 16;
  while (ks > 1 && (size_t)ks * a.M * (a.dual ? 2 : 1) * a.N > partial_capacity) --ks;
  return ks >= 2 ? (int)ks : 1;
}

namespace {

// Sum of the k_splits partial sums in a fixed order (split 0 first), then what the one-block kernel does in its
// epilogue: bias, activation or SiLU(gate) * up, rotary embedding (same two operations per element), residual, output
// type.  One thread = 4 consecutive output features of one token (for rotated heads: of the lower half, and the 4
// partner features of the upper half).
__global__ void __launch_bounds__(256) splitk_reduce_kernel(MfmaGemmArgs a) {
  const int n4 = a.N / 4;
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)a.M * n4) return;
  const int m = (int)(idx / n4), n = (int)(idx % n4) * 4;
  const size_t plane = (size_t)a.M * a.ldp;
  auto sum4 = [&](int col) {
    const float* p = a.partial + (size_t)m * a.ldp + col;
    f32x4 v = *(const f32x4*)p;
    for (int s = 1; s < a.k_splits; ++s) v += *(const f32x4*)(p + s * plane);
    return v;
  };
  auto store4 = [&](int col, f32x4 v) {
    const size_t o = (size_t)m * a.ldo + col;
    if (a.residual != nullptr) v += *(const f32x4*)(a.residual + o);
    if (a.out_f32) *(f32x4*)((float*)a.out + o) = v;
    else *(u32x2*)((uint16_t*)a.out + o) = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
  };
  if (a.rope_cos != nullptr && n < a.rope_cols) {
    const int half = a.rope_dh / 2, c = n % a.rope_dh;
    if (c >= half) return;                               // done by the thread of the lower half
    f32x4 lo = sum4(n), hi = sum4(n + half);
    if (a.bias != nullptr) { lo += *(const f32x4*)(a.bias + n); hi += *(const f32x4*)(a.bias + n + half); }
    const int pos = a.rope_pos != nullptr ? a.rope_pos[m % a.S] : m % a.S;
    const f32x4 cs = *(const f32x4*)(a.rope_cos + (size_t)pos * half + c);
    const f32x4 sn = *(const f32x4*)(a.rope_sin + (size_t)pos * half + c);
    f32x4 ylo, yhi;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      ylo[e] = fmaf(lo[e], cs[e], -__fmul_rn(hi[e], sn[e]));
      yhi[e] = fmaf(hi[e], cs[e], __fmul_rn(lo[e], sn[e]));
    }
    store4(n, ylo);
    store4(n + half, yhi);
    return;
  }
  f32x4 v = sum4(n);
  if (a.bias != nullptr) v += *(const f32x4*)(a.bias + n);
  if (a.dual) {
    f32x4 u = sum4(a.N + n);
    if (a.bias != nullptr) u += *(const f32x4*)(a.bias + a.dual_offset + n);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = silu_mul_f32(v[e], u[e]);
  } else if (a.act == MPZ_ACT_RELU) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = v[e] > 0.f ? v[e] : 0.f;
  } else if (a.act == MPZ_ACT_GELU_ERF) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = gelu_erf(v[e]);
  }
  store4(n, v);
}

}  // namespace

hipError_t launch_gemm_mfma(hipStream_t st, const MfmaGemmArgs& a) {
  const bool q8 = a.w_scale != nullptr;      // int8 weights: the configurations the model path uses
  if (a.k_splits > 1) {                      // raw partial sums per split, then the reduction with the epilogue
    hipError_t e;
    // gate || up whose two weight blocks lie back to back: with raw partial sums the dual kernel has nothing to fuse, so
    // the launch is a plain GEMM over the 2 N stacked rows (column N + n of a partial row is up[n], which is the dual
    // kernel's raw layout), on the BK = 64 tile that fetches whole 128-byte lines
    MfmaGemmArgs b = a;
    if (a.dual && a.dual_offset == a.N) { b.dual = 0; b.N = 2 * a.N; }
    if (b.dual) e = q8 ? launch_cfg<128, 128, 32, 2, 2, true, 0, true>(st, a) : launch_cfg<128, 128, 32, 2, 2, true>(st, a);
    else if (a.w_absmax != nullptr)          // 4-bit codes looked up in the operand load: the two 128-feature tiles
      e = choose_cfg(b) == 9 ? launch_cfg<128, 64, 64, 2, 2, false, 0, 2>(st, b) : launch_cfg<128, 128, 64, 2, 2, false, 0, 2>(st, b);
    else
      switch (choose_cfg(b)) {
        case 9: e = q8 ? launch_cfg<128, 64, 64, 2, 2, false, 0, true>(st, b) : launch_cfg<128, 64, 64, 2, 2, false>(st, b); break;
        case 10: e = launch_cfg<64, 64, 64, 2, 2, false>(st, b); break;
        case 12: e = launch_cfg<128, 128, 64, 2, 4, false>(st, b); break;
        case 13: e = launch_cfg<64, 128, 64, 2, 2, false>(st, b); break;
        default: e = q8 ? launch_cfg<128, 128, 64, 2, 2, false, 0, true>(st, b) : launch_cfg<128, 128, 64, 2, 2, false>(st, b); break;
      }
    if (e != hipSuccess) return e;
    if (a.defer_reduce) return hipSuccess;
    const long items = (long)a.M * (a.N / 4);
    splitk_reduce_kernel<<<(unsigned)((items + 255) / 256), 256, 0, st>>>(a);
    return hipSuccess;
  }
  if (a.dual) {
    const long tb = (long)((a.N + 127) / 128) * ((a.M + 255) / 256);
    if ((a.tile_cfg == 0 && tb >= 512) || a.tile_cfg == 6)                 // 2 x 128 x 256, 8 waves
      return q8 ? launch_cfg<128, 256, 64, 2, 4, true, 0, true>(st, a) : launch_cfg<128, 256, 64, 2, 4, true>(st, a);
    return q8 ? launch_cfg<128, 128, 32, 2, 2, true, 0, true>(st, a) : launch_cfg<128, 128, 32, 2, 2, true>(st, a);
  }
  if (a.rope_cos != nullptr) {             // fused rotary epilogue: only the configurations the model path uses
    const int cfg = choose_cfg(a);
    if (cfg == 6) {
      if (a.rope_dh == 64) return q8 ? launch_cfg<256, 256, 64, 2, 4, false, 1, true>(st, a) : launch_cfg<256, 256, 64, 2, 4, false, 1>(st, a);
      return q8 ? launch_cfg<256, 256, 64, 2, 4, false, 2, true>(st, a) : launch_cfg<256, 256, 64, 2, 4, false, 2>(st, a);
    }
    if (cfg == 12) return q8 ? launch_cfg<128, 128, 64, 2, 4, false, 1, true>(st, a) : launch_cfg<128, 128, 64, 2, 4, false, 1>(st, a);
    return q8 ? launch_cfg<128, 128, 64, 2, 2, false, 1, true>(st, a) : launch_cfg<128, 128, 64, 2, 2, false, 1>(st, a);
  }
  if (q8) {
    switch (choose_cfg(a)) {
      case 6: return launch_cfg<256, 256, 64, 2, 4, false, 0, true>(st, a);
      case 11: return launch_cfg<192, 128, 64, 2, 2, false, 0, true>(st, a);
      case 12: return launch_cfg<128, 128, 64, 2, 4, false, 0, true>(st, a);
      default: return launch_cfg<128, 128, 64, 2, 2, false, 0, true>(st, a);
    }
  }
  switch (choose_cfg(a)) {
    case 6: return launch_cfg<256, 256, 64, 2, 4, false>(st, a);     // 8 waves of 128 x 64, BK 64 (147 KB LDS), 128 KB in flight
    case 9: return launch_cfg<128, 64, 64, 2, 2, false>(st, a);      // 4 waves of 64 x 32: more, smaller blocks
    case 10: return launch_cfg<64, 64, 64, 2, 2, false>(st, a);      // 4 waves of 32 x 32: the smallest blocks
    case 11: return launch_cfg<192, 128, 64, 2, 2, false>(st, a);    // 4 waves of 96 x 64, 92 KB LDS: 1 block per CU
    case 12: return launch_cfg<128, 128, 64, 2, 4, false>(st, a);    // 8 waves of 64 x 32: 16 waves per CU
    case 13: return launch_cfg<64, 128, 64, 2, 2, false>(st, a);     // 4 waves of 32 x 64: all of <= 128 tokens, few features
    default: return launch_cfg<128, 128, 64, 2, 2, false>(st, a);    // 1: 4 waves of 64 x 64
  }
}

hipError_t launch_hbm_read_probe(hipStream_t st, const void* buf, long rows, long row_bytes, int rb, int seg_bytes, int k_splits,
                                 int lds_bytes, int mode, uint32_t* out) {
  const long row_chunks = row_bytes / 16;
  const int seg_chunks = seg_bytes / 16, L = rb * seg_chunks / 256;
  const int tiles_per_split = (int)(row_bytes / seg_bytes / k_splits);
  const dim3 grid((unsigned)(rows / rb), (unsigned)k_splits);
#define MPZ_PROBE_CASE(LL)                                                                                              \
  case LL: {                                                                                                            \
    hipError_t e = hipFuncSetAttribute((const void*)hbm_read_probe_kernel<LL>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                       160 * 1024);                                                                     \
    if (e != hipSuccess) return e;                                                                                      \
    hbm_read_probe_kernel<LL><<<grid, 256, (size_t)lds_bytes, st>>>((const u32x4*)buf, row_chunks, rb, seg_chunks,     \
                                                                     tiles_per_split, mode, out);                       \
    return hipSuccess;                                                                                                  \
  }
  switch (L) {
    MPZ_PROBE_CASE(1) MPZ_PROBE_CASE(2) MPZ_PROBE_CASE(4) MPZ_PROBE_CASE(8) MPZ_PROBE_CASE(16)
    default: return hipErrorInvalidValue;
  }
#undef MPZ_PROBE_CASE
}

void launch_mfma_probe(hipStream_t st, const void* operands, int blocks, int iters, int with_lds, float* out) {
  mfma_probe_kernel<<<blocks, 512, 0, st>>>((const uint16_t*)operands, iters, with_lds, out);
}

bool mfma_lora_down_supported(const MfmaLoraDownArgs& a) {
  int R = a.n_targets * a.rank;
  return a.K % 256 == 0 && a.T % 32 == 0 && a.rows_per_copy % 32 == 0 && R <= 64 && a.rp % 8 == 0 && a.rank % 4 == 0;
}

void launch_lora_down_mfma(hipStream_t st, const MfmaLoraDownArgs& a) {
  int R = a.n_targets * a.rank;
  if (R <= 32) lora_down_mfma_kernel<1><<<a.T / 32, 256, 0, st>>>(a);
  else lora_down_mfma_kernel<2><<<a.T / 32, 256, 0, st>>>(a);
}

void launch_pack_factors(hipStream_t st, const float* pert, int64_t P, int n_copies, const LoraLayerTable& tab,
                         int n_layers, int rank, int rp, void* packed, int64_t packed_per_copy) {
  // vectorised variant: ranks 4 / 8 / 16 with every A factor's K a multiple of 8 and 8-byte-aligned packed rows
  bool vec = (rank == 4 || rank == 8 || rank == 16) && rp % 4 == 0;
  int items = 0;
  for (int t = 0; t < tab.n_tensors; ++t) {
    const bool isB = tab.local_id[t] & 1;
    if (!isB && tab.rows[t] % 8) vec = false;
    items += isB ? tab.cols[t] : tab.rows[t] / 8 * rank;
  }
  if (vec) {
    const int64_t total = (int64_t)items * n_layers * n_copies;
    const unsigned nb = (unsigned)((total + 255) / 256);
    if (rank == 4) pack_factors_vec_kernel<4><<<nb, 256, 0, st>>>(pert, P, n_copies, tab, n_layers, rp, (uint16_t*)packed, packed_per_copy, items);
    else if (rank == 8) pack_factors_vec_kernel<8><<<nb, 256, 0, st>>>(pert, P, n_copies, tab, n_layers, rp, (uint16_t*)packed, packed_per_copy, items);
    else pack_factors_vec_kernel<16><<<nb, 256, 0, st>>>(pert, P, n_copies, tab, n_layers, rp, (uint16_t*)packed, packed_per_copy, items);
    return;
  }
  int64_t total = (int64_t)n_copies * P;
  pack_factors_kernel<<<(unsigned)((total + 255) / 256), 256, 0, st>>>(pert, P, n_copies, tab, n_layers, rank, rp,
                                                                       (uint16_t*)packed, packed_per_copy);
}

}  // namespace mpz
