// C ABI of libmpz: argument validation, workspace carving and the launch sequence of one ZO step
// (Algorithm 1) over n = 2q stacked copies (Section 3, MP-LoRA with outer- and inner-loop
// parallelisation).  Host code only; every arithmetic step runs in the kernels it launches.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "common.h"
#include "../../include/mpz.h"

using namespace mpz;

// Scratch of mpz_forward_perturbed_noalloc: the activations of one pass, for callers that cannot hand over (or
// allocate) a workspace large enough at call time.  One copy per GPU, held until the process ends; its device address
// is looked up once per device (scratch_address) and only that pointer is ever given to kernels.
#define MPZ_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
static __device__ __align__(256) unsigned char scratch[MPZ_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up on first use per device), or null with *err set.
void* scratch_address(int* device_out, hipError_t* err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (device_out) *device_out = dev;
  if (dev < 0 || dev >= kMaxDevices) { *err = hipErrorInvalidDevice; return nullptr; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    *err = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || ptr == nullptr) { if (*err == hipSuccess) *err = hipErrorInvalidSymbol; return nullptr; }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

thread_local std::string g_last_error;

struct Carver {                                  // bump allocator over the caller's workspace
  unsigned char* base; size_t off = 0;
  explicit Carver(void* b) : base((unsigned char*)b) {}
  template <typename T> T* take(size_t count) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

struct Buffers {
  float* rope_cos = nullptr; float* rope_sin = nullptr;
  float* pert = nullptr;      // [2 q_max][P] perturbed factors, master layout, fp32
  float* h = nullptr;         // [T, d] residual stream, fp32
  void* x = nullptr;          // [T, d] norm output (GEMM operand)
  void* qkv = nullptr;        // [T, d + 2 d_kv]
  void* attn = nullptr;       // [T, d]
  void* t = nullptr;          // [T, 4 r] LoRA bottleneck activations
  void* u = nullptr;          // [T, d_ffn]
  void* stage = nullptr;      // accumulate-type staging for rotary q/k and SwiGLU gate|up
  float* logits = nullptr;    // [chunk_rows, vocab] or [n E, 2]
  float* ce = nullptr;        // [T] per-row losses
  int32_t* target = nullptr;  // [T]
  int chunk_rows = 0;
  void* packed = nullptr;     // [2 q_max][packed_per_copy] bf16 hi/lo operand layouts of the perturbed factors
  void* tp[3] = {nullptr, nullptr, nullptr};  // per target [T, rp] duplicated bottleneck activations
  void* wq = nullptr;         // 4-bit weights: the largest block linear, dequantised to bf16
  float* splitk = nullptr;    // partial sums of the split-K GEMMs of a pass over at most 256 stacked tokens
  size_t splitk_elems = 0;
  int32_t* row_pos = nullptr; // packed batches: per row of a copy, its position inside its sequence
  int32_t* row_end = nullptr; //   and the row after its sequence's last one (-1: filler row)
};

size_t elem_size(int dtype) { return dtype == MPZ_DTYPE_F32 ? 4 : 2; }
size_t acc_size(int dtype) { return dtype == MPZ_DTYPE_F32 ? 8 : 4; }

int count_targets(uint32_t m) { return __builtin_popcount(m & 15u); }

const char* validate_config(const mpz_config* c) {
  if (c->struct_size != sizeof(mpz_config)) return "struct_size does not match sizeof(mpz_config)";
  if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 || c->vocab < 2 ||
      c->max_seq < 2) return "non-positive model dimension";
  if (c->d_model % c->n_heads) return "d_model is not a multiple of n_heads";
  if (c->n_heads % c->n_kv_heads) return "n_heads is not a multiple of n_kv_heads";
  if (c->act < 0 || c->act > 2 || c->norm < 0 || c->norm > 1 || c->pos < 0 || c->pos > 1) return "unknown act/norm/pos";
  if (c->dtype != MPZ_DTYPE_F32 && c->dtype != MPZ_DTYPE_BF16) return "unknown dtype";
  if (c->pos == MPZ_POS_ROPE && ((c->d_model / c->n_heads) & 1)) return "rotary embedding needs an even d_head";
  if (c->pos == MPZ_POS_ROPE && !(c->rope_theta > 0.f)) return "rope_theta must be positive";
  if (c->lora_rank < 4 || c->lora_rank % 4 || c->lora_rank > 64) return "lora_rank must be a multiple of 4 in [4, 64]";
  if ((c->lora_targets & 15u) == 0 || (c->lora_targets & ~15u)) return "lora_targets must be a non-empty subset of Q|K|V|O";
  if (c->d_model % 4) return "d_model must be a multiple of 4";
  if (!(c->norm_eps > 0.f) || !std::isfinite(c->lora_scale)) return "norm_eps must be positive and lora_scale finite";
  if (c->loss_mode < 0 || c->loss_mode > 2) return "unknown loss_mode";
  if (c->weight_quant < MPZ_WEIGHT_QUANT_NONE || c->weight_quant > MPZ_WEIGHT_QUANT_NF4) return "unknown weight_quant";
  if (c->weight_quant == MPZ_WEIGHT_QUANT_NF4 && (c->dtype != MPZ_DTYPE_BF16 || c->d_model % 64 || c->d_ffn % 64))
    return "4-bit weights need dtype BF16 and d_model, d_ffn multiples of 64";
  if (c->weight_quant == MPZ_WEIGHT_QUANT_INT8 && (c->dtype != MPZ_DTYPE_BF16 || c->d_model % 64 || c->d_ffn % 64 ||
                                                   (c->n_kv_heads * (c->d_model / c->n_heads)) % 2))
    return "int8 weights need dtype BF16 and d_model, d_ffn multiples of 64";
  if (c->loss_mode != MPZ_LOSS_NEXT_TOKEN_ALL_POS) {
    for (int i = 0; i < 2; ++i)
      if (c->label_token[i] < 0 || c->label_token[i] >= c->vocab) return "label token id outside the vocabulary";
    if (c->label_token[0] == c->label_token[1]) return "the two label tokens must differ";
  }
  return nullptr;
}

void build_layout(const mpz_config* c, std::vector<mpz_lora_tensor>& out, LoraLayerTable& tab) {
  out.clear();
  int d = c->d_model, dkv = c->n_kv_heads * (c->d_model / c->n_heads), r = c->lora_rank;
  int64_t off = 0;
  memset(&tab, 0, sizeof(tab));
  for (int l = 0; l < c->n_layers; ++l) {
    int i = 0;
    for (int t = 0; t < 4; ++t) {
      if (!(c->lora_targets & (1u << t))) continue;
      int k_out = (t == 0 || t == 3) ? d : dkv;
      for (int f = 0; f < 2; ++f) {
        mpz_lora_tensor e;
        e.layer = l; e.target = t; e.factor = f; e.tensor_id = (l * 4 + t) * 2 + f; e.offset = off;
        e.rows = f == 0 ? d : r; e.cols = f == 0 ? r : k_out;
        if (l == 0) { tab.off[i] = (int32_t)off; tab.local_id[i] = t * 2 + f; tab.rows[i] = e.rows; tab.cols[i] = e.cols; }
        out.push_back(e);
        off += (int64_t)e.rows * e.cols;
        ++i;
      }
    }
    if (l == 0) { tab.n_tensors = i; tab.per_layer = (int32_t)off; tab.off[i] = (int32_t)off; }
  }
}

// What lives as long as the model handle: rotary tables, the perturbed factor copies that mpz_regen_noise leaves for
// the passes (master layout and MFMA operand layouts), the row tables of packed batches, the dequantisation buffer.
void carve_persistent(const mpz_config* c, int q_max, int E_max, int S_max, Carver& cv, Buffers& bb) {
  std::vector<mpz_lora_tensor> lay; LoraLayerTable tab;
  build_layout(c, lay, tab);
  const int64_t P = (int64_t)tab.per_layer * c->n_layers, n = 2 * (int64_t)q_max;
  const int64_t rpc_max = ((int64_t)E_max * S_max + 31) / 32 * 32;
  const int d = c->d_model, dh = d / c->n_heads, dkv = c->n_kv_heads * dh, f = c->d_ffn;
  if (c->pos == MPZ_POS_ROPE) {
    bb.rope_cos = cv.take<float>((size_t)c->max_seq * (dh / 2));
    bb.rope_sin = cv.take<float>((size_t)c->max_seq * (dh / 2));
  }
  bb.pert = cv.take<float>((size_t)(n * P));
  if (c->dtype == MPZ_DTYPE_BF16) {
    const int rp = (2 * c->lora_rank + 15) / 16 * 16;
    int64_t per_layer = 0;
    for (int i = 0; i < tab.n_tensors; ++i)
      per_layer += (tab.local_id[i] & 1) ? (int64_t)tab.cols[i] * rp : (int64_t)2 * tab.rows[i] * tab.cols[i];
    bb.packed = cv.take<uint16_t>((size_t)(n * per_layer * c->n_layers));
  }
  bb.row_pos = cv.take<int32_t>((size_t)rpc_max);
  bb.row_end = cv.take<int32_t>((size_t)rpc_max);
  if (c->weight_quant == MPZ_WEIGHT_QUANT_NF4) {
    const size_t n_qkv = (size_t)(d + 2 * dkv), n_up = (size_t)(c->act == MPZ_ACT_SWIGLU ? 2 * f : f);
    size_t big = n_qkv * d;
    if (n_up * d > big) big = n_up * d;
    if ((size_t)d * f > big) big = (size_t)d * f;
    bb.wq = cv.take<uint16_t>(big);
  }
}

// Room for the partial sums of a split-K GEMM (passes over at most 256 stacked tokens: mfma_gemm_splits keeps
// k_splits * M <= K / 4 and k_splits <= 16, and splits only K >= 1024): the largest of the block's four linears.
size_t splitk_capacity(const mpz_config* c, int64_t T) {
  if (c->dtype != MPZ_DTYPE_BF16) return 0;
  const int64_t Mx = T < 256 ? T : 256;
  const int d = c->d_model, dkv = c->n_kv_heads * (d / c->n_heads), f = c->d_ffn;
  const int64_t shapes[4][2] = {{d, d + 2 * dkv}, {d, d}, {d, c->act == MPZ_ACT_SWIGLU ? 2 * f : f}, {f, d}};   // K, columns
  int64_t cap = 0;
  for (const auto& s : shapes) {
    if (s[0] < 1024) continue;
    const int64_t rows = 16 * Mx < s[0] / 4 ? 16 * Mx : s[0] / 4;
    if (rows * s[1] > cap) cap = rows * s[1];
  }
  return (size_t)cap;
}

// What one pass needs and nothing outlives: the activations of ONE block for n stacked copies of rpc rows each
// (E sequences per copy), staging, and the loss scratch.  Every buffer is written by the pass before it is read.
void carve_activations(const mpz_config* c, int64_t n, int64_t rpc, int64_t E, Carver& cv, Buffers& bb) {
  const int64_t T = n * rpc;
  const int d = c->d_model, dh = d / c->n_heads, dkv = c->n_kv_heads * dh, f = c->d_ffn;
  const size_t es = elem_size(c->dtype), as = acc_size(c->dtype);
  bb.h = cv.take<float>((size_t)T * d);
  bb.x = cv.take<unsigned char>((size_t)T * d * es);
  bb.qkv = cv.take<unsigned char>((size_t)T * (d + 2 * dkv) * es);
  bb.attn = cv.take<unsigned char>((size_t)T * d * es);
  bb.t = cv.take<unsigned char>((size_t)T * 4 * c->lora_rank * es);
  bb.u = cv.take<unsigned char>((size_t)T * f * es);
  size_t stage_elems = 0;
  if (c->pos == MPZ_POS_ROPE) stage_elems = (size_t)T * (d + 2 * dkv);
  if (c->act == MPZ_ACT_SWIGLU && (size_t)T * 2 * f > stage_elems) stage_elems = (size_t)T * 2 * f;
  bb.stage = stage_elems ? cv.take<unsigned char>(stage_elems * as) : nullptr;
  const int64_t loss_rows = c->loss_mode == MPZ_LOSS_NEXT_TOKEN_ALL_POS ? T : n * E;
  if (c->loss_mode == MPZ_LOSS_LAST_POS_LABEL_SUBSET) {
    bb.chunk_rows = (int)loss_rows;
    bb.logits = cv.take<float>((size_t)loss_rows * 2);
  } else {
    bb.chunk_rows = (int)(loss_rows < 4096 ? loss_rows : 4096);
    bb.logits = cv.take<float>((size_t)bb.chunk_rows * c->vocab);
  }
  bb.ce = cv.take<float>((size_t)loss_rows);
  bb.target = cv.take<int32_t>((size_t)loss_rows);
  for (int i = 0; i < 3; ++i) bb.tp[i] = nullptr;
  if (c->dtype == MPZ_DTYPE_BF16) {
    const int rp = (2 * c->lora_rank + 15) / 16 * 16;
    for (int i = 0; i < 3; ++i) bb.tp[i] = cv.take<uint16_t>((size_t)T * rp);
  }
  bb.splitk_elems = splitk_capacity(c, T);
  bb.splitk = bb.splitk_elems ? cv.take<float>(bb.splitk_elems) : nullptr;
}

size_t carve(const mpz_config* c, int q_max, int E_max, int S_max, void* base, Buffers* b) {
  Carver cv(base);
  Buffers bb;
  carve_persistent(c, q_max, E_max, S_max, cv, bb);
  // rows per copy rounded up to whole 32-row tiles: a packed batch (mpz_forward_perturbed_packed) of anything that
  // fits as a padded batch then fits as well
  carve_activations(c, 2 * (int64_t)q_max, ((int64_t)E_max * S_max + 31) / 32 * 32, E_max, cv, bb);
  if (b) *b = bb;
  return (cv.off + 255) & ~(size_t)255;
}

}  // namespace

struct mpz_model {
  mpz_config cfg;
  std::vector<mpz_layer_weights> layers;
  mpz_weights w;
  float* masters = nullptr;
  hipStream_t stream = nullptr;
  int q_max = 0, E_max = 0, S_max = 0;
  Buffers buf;
  std::vector<mpz_lora_tensor> tensors;
  LoraLayerTable tab;
  int64_t P = 0;
  bool have_noise = false;
  uint64_t seed = 0; uint32_t step = 0; int q = 0; float eps = 0.f;
  int cb = 0, nc = 0;                           // copies cb + cstep i, i < nc, are processed by the current pass
  int cstep = 1;                                //   (their activations occupy rows [cb, cb + nc) * E * S of the workspace)
  bool fuse_norm_lora = true;                   // test hook: pre-norm and LoRA bottleneck in one kernel where shapes allow
  bool split_k = true;                          // test hook: split-K GEMMs for passes over few stacked tokens
  bool fuse_perturb_pack = true;                // test hook: noise -> bf16 operand layouts in one kernel (no fp32 copies)
  bool pert_valid = false;                      // buf.pert holds the fp32 copies of the last mpz_regen_noise (else only
                                                //   the bf16 operand layouts exist; ensure_pert regenerates them)
  int force_tile_cfg = 0;                       // test hook: GEMM block-tile configuration (0 = by shape)
  const int32_t* lengths = nullptr;             // [dev] per-sequence lengths of the pass in flight (right-padded batch), or null
  // packed (padding-free) batch of the pass in flight: cu [dev, E + 1] sequence starts inside a copy, `total` real
  // rows per copy, the longest sequence.  The pass then runs with one "sequence" of rows-per-copy rows per copy.
  struct Packed { const int32_t* cu = nullptr; int E = 0, total = 0, max_len = 0; } pk;
  const char* deferred = nullptr;               // set by a launch helper that had to refuse; reported by check_device
  hipError_t deferred_device = hipSuccess;      // a HIP error met while setting up a launch; reported by check_device
  // second stream for the two-halves schedule of small models (see forward_two_halves); default priority
  hipStream_t stream2 = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool two_halves = true;                       // test hook: allow that schedule
  int last_pass_streams = 0;                    // streams the last batched pass was issued on (0: none yet)
  int device = -1;                              // HIP device that was current at mpz_init_model
  size_t stage_row_bytes = 0;                   // staging bytes per stacked token (a copy range owns its rows of the buffer)
  std::string err;
  // optional per-launch timing by kernel category (mpz_profile_begin / _end)
  // bf16 MFMA path
  bool use_mfma = false;
  int rp = 0;                                   // padded 2r
  int64_t packed_per_layer = 0, packed_per_copy = 0;
  int64_t packed_off[8] = {0};                  // offset of tensor i inside a layer's packed block
  bool prof_on = false;
  std::vector<hipEvent_t> prof_ev;   // start/stop pairs
  std::vector<int> prof_cat;         // category of pair i
  size_t prof_used = 0;
  double prof_flops[MPZ_PROF_COUNT] = {0}, prof_bytes[MPZ_PROF_COUNT] = {0};
  ~mpz_model() {
    for (hipEvent_t e : prof_ev) (void)hipEventDestroy(e);
    if (ev_fork) (void)hipEventDestroy(ev_fork);
    if (ev_join) (void)hipEventDestroy(ev_join);
    if (stream2) (void)hipStreamDestroy(stream2);
  }
};

namespace {

mpz_status fail(mpz_model* m, mpz_status s, const std::string& msg) {
  g_last_error = msg;
  if (m) m->err = msg;
  return s;
}

mpz_status check_device(mpz_model* m, const char* where) {
  if (m && m->deferred) {                       // a launch helper refused (nothing was enqueued for that operation)
    const char* msg = m->deferred;
    m->deferred = nullptr;
    return fail(m, MPZ_ERR_SHAPE, std::string(where) + ": " + msg);
  }
  hipError_t e = hipGetLastError();
  if (m && m->deferred_device != hipSuccess) { e = m->deferred_device; m->deferred_device = hipSuccess; }
  if (e != hipSuccess) return fail(m, MPZ_ERR_DEVICE, std::string(where) + ": " + hipGetErrorString(e));
  return MPZ_OK;
}

const mpz_lora_tensor* find_tensor(const mpz_model* m, int layer, int target, int factor) {
  for (const auto& t : m->tensors)
    if (t.layer == layer && t.target == target && t.factor == factor) return &t;
  return nullptr;
}

// Brackets one launch with HIP events when profiling is on, and books its algorithmic work.
struct ProfScope {
  mpz_model* m; hipEvent_t e1 = nullptr;
  ProfScope(mpz_model* m_, int cat, double flops, double bytes) : m(m_) {
    if (!m->prof_on) return;
    if (m->prof_used + 2 > m->prof_ev.size()) {
      hipEvent_t x = nullptr, y = nullptr;
      if (hipEventCreate(&x) != hipSuccess || hipEventCreate(&y) != hipSuccess) return;
      m->prof_ev.push_back(x); m->prof_ev.push_back(y);
    }
    hipEvent_t e0 = m->prof_ev[m->prof_used]; e1 = m->prof_ev[m->prof_used + 1];
    if (m->prof_cat.size() < m->prof_ev.size() / 2) m->prof_cat.resize(m->prof_ev.size() / 2);
    m->prof_cat[m->prof_used / 2] = cat;
    m->prof_used += 2;
    m->prof_flops[cat] += flops; m->prof_bytes[cat] += bytes;
    (void)hipEventRecord(e0, m->stream);
  }
  void end() { if (e1) (void)hipEventRecord(e1, m->stream); e1 = nullptr; }   // close the bracket before the scope ends
  ~ProfScope() { end(); }
};

double esz(const mpz_model* m) { return m->cfg.dtype == MPZ_DTYPE_F32 ? 4.0 : 2.0; }

// Workspace pointers of the copies [m->cb, m->cb + m->nc): every activation buffer is row-major over the stacked
// tokens, so a range of copies is a range of rows; the whole-vocabulary loss scratch is shared (one pass at a time).
Buffers view(const mpz_model* m, int E, int S) {
  Buffers b = m->buf;
  const mpz_config& c = m->cfg;
  const size_t row0 = (size_t)m->cb * E * S, es = elem_size(c.dtype);
  const int d = c.d_model, dkv = c.n_kv_heads * (d / c.n_heads);
  b.pert += (size_t)m->cb * m->P;
  if (b.packed) b.packed = (uint16_t*)b.packed + (size_t)m->cb * m->packed_per_copy;
  b.h += row0 * d;
  b.x = (char*)b.x + row0 * d * es;
  b.qkv = (char*)b.qkv + row0 * (d + 2 * dkv) * es;
  b.attn = (char*)b.attn + row0 * d * es;
  b.t = (char*)b.t + row0 * 4 * c.lora_rank * es;
  b.u = (char*)b.u + row0 * c.d_ffn * es;
  for (int i = 0; i < 3; ++i)
    if (b.tp[i]) b.tp[i] = (uint16_t*)b.tp[i] + row0 * m->rp;
  const size_t loss0 = c.loss_mode == MPZ_LOSS_NEXT_TOKEN_ALL_POS ? row0 : (size_t)m->cb * E;
  b.ce += loss0; b.target += loss0;
  if (b.stage) b.stage = (char*)b.stage + row0 * m->stage_row_bytes;
  if (c.loss_mode == MPZ_LOSS_LAST_POS_LABEL_SUBSET) b.logits += loss0 * 2;   // [n E, 2]: a range owns its rows
  return b;
}

// The frozen weight of one block linear as the GEMM reads it.  4-bit weights are dequantised to bf16 here, into the
// one workspace buffer every linear shares (stream order keeps a GEMM ahead of the next dequantisation): once per
// pass, whatever the number of copies in it (Appendix D: the inner loop dequantises once per step).
// A pass over few stacked tokens is bound by the weight stream, and there the split-K GEMM looks the 4-bit codes up in
// its own operand load (a quarter of the bytes, no bf16 round trip through HBM): such a pass hands the codes on
// (w_codes / w_absmax) and gemm() dequantises only if the launch turns out not to split K.
struct WeightRef { const void* w; const float* scale; const void* codes; const float* absmax; };
const void* dequantised(mpz_model* m, const void* codes, const float* absmax, int N, int K) {
  ProfScope ps(m, MPZ_PROF_PACK, 0.0, (double)N * K * (0.5 + 4.0 / 64.0 + 2.0));
  launch_nf4_dequant(m->stream, codes, absmax, m->buf.wq, (int64_t)N * K);
  return m->buf.wq;
}
WeightRef weight_operand(mpz_model* m, const void* w, const float* s, int N, int K, int M) {
  if (m->cfg.weight_quant != MPZ_WEIGHT_QUANT_NF4) return {w, s, nullptr, nullptr};
  if (m->use_mfma && m->split_k && m->buf.splitk != nullptr && M <= 256) return {nullptr, nullptr, w, s};
  return {dequantised(m, w, s, N, K), nullptr, nullptr, nullptr};
}
void set_weight(LinearArgs& a, const WeightRef& r) { a.w = r.w; a.w_scale = r.scale; a.w_codes = r.codes; a.w_absmax = r.absmax; }
// Few stacked tokens: let k_splits blocks share an output tile (see MfmaGemmArgs).  Called once the shape and the
// epilogue of g are filled in, before mfma_gemm_supported.
void plan_split(const mpz_model* m, MfmaGemmArgs& g) {      // (g.w_absmax, if any, is already set: the tile depends on it)
  g.k_splits = 1; g.partial = nullptr; g.ldp = 0;
  if (m->buf.splitk == nullptr || !m->split_k) return;
  const int ks = mfma_gemm_splits(g, m->buf.splitk_elems);
  if (ks > 1) { g.k_splits = ks; g.partial = m->buf.splitk; g.ldp = (g.dual ? 2 : 1) * g.N; }
}

// A GEMM launch whose set-up error (the kernel's LDS limit could not be raised) is kept for check_device
void launch_checked(mpz_model* m, const MfmaGemmArgs& g) {
  const hipError_t e = launch_gemm_mfma(m->stream, g);
  if (e != hipSuccess && m->deferred_device == hipSuccess) m->deferred_device = e;
}

// Every base-weight GEMM of the pass goes through here (kernel selection and optional timing).  Returns false
// (nothing launched) only when a fused rotary epilogue was requested and the shape does not allow it.
// `then`: the pre-norm that reads this GEMM's output rows next (gains, optional biases, operand rows to write).  When
// the GEMM splits K, its reduction and that norm run as one kernel and then->done is set; otherwise the caller
// launches the norm itself.
struct NormAfter { const float* g; const float* b; void* x; bool done; };
bool gemm(mpz_model* m, const LinearArgs& a, NormAfter* then = nullptr) {
  const bool rope = a.rope_cos != nullptr;
  MfmaGemmArgs g{};
  bool use_mfma_gemm = false;
  if (m->use_mfma && a.dtype == MPZ_DTYPE_BF16 && (a.n_seg == 0 || a.mfma_lora)) {
    g.M = a.M; g.N = a.N; g.K = a.K; g.x = a.x; g.w = a.w; g.w_scale = a.w_scale; g.w_rows = a.N; g.bias = a.bias; g.dual = 0; g.dual_offset = 0;
    g.n_seg = a.n_seg; g.rows_per_copy = a.rows_per_copy;
    for (int i = 0; i < a.n_seg; ++i) g.seg[i] = a.mseg[i];
    g.tile_cfg = m->force_tile_cfg; g.out = a.out; g.ldo = a.N;
    if (rope) {
      g.act = -1; g.out_f32 = 0;
      g.rope_cos = a.rope_cos; g.rope_sin = a.rope_sin; g.rope_cols = a.rope_cols; g.rope_dh = a.rope_dh; g.S = a.S;
      g.rope_pos = a.rope_pos;
    } else {
      g.act = a.act; g.residual = a.residual;
      g.out_f32 = a.out_kind != 0;                 // bf16 models stage in fp32
    }
    // 4-bit weights nobody has dequantised yet: the split-K kernel reads the codes itself; a launch that does not
    // split K gets them dequantised below (the workspace buffer is where they will be)
    if (a.w_codes != nullptr) { g.w = a.w_codes; g.w_absmax = a.w_absmax; }
    plan_split(m, g);
    if (a.w_codes != nullptr && g.k_splits <= 1) { g.w = m->buf.wq; g.w_absmax = nullptr; }
    use_mfma_gemm = mfma_gemm_supported(g);
  }
  if (rope && !use_mfma_gemm) return false;         // nothing launched: the caller goes on without the fused rotation
  LinearArgs dense = a;                             // the same linear with weights every kernel can read
  if (a.w_codes != nullptr && !(use_mfma_gemm && g.k_splits > 1)) {
    dense.w = dequantised(m, a.w_codes, a.w_absmax, a.N, a.K);
    dense.w_codes = nullptr; dense.w_absmax = nullptr;
  }
  ProfScope ps(m, MPZ_PROF_GEMM, 2.0 * a.M * (double)a.N * a.K,
               rope ? 2.0 * ((double)a.M * a.K + (double)a.N * a.K + (double)a.M * a.N)
                    : esz(m) * ((double)a.M * a.K + (double)a.N * a.K) + (a.out_kind == 0 ? esz(m) : 4.0) * a.M * (double)a.N +
                          (a.residual ? 4.0 * a.M * (double)a.N : 0.0));
  if (use_mfma_gemm) {
    if (!rope && then != nullptr && m->fuse_norm_lora && splitk_reduce_norm_supported(g) && a.N == m->cfg.d_model) {
      g.defer_reduce = 1;
      launch_checked(m, g);
      ps.end();                                  // (the fused kernel is booked under the norm)
      ProfScope pn(m, MPZ_PROF_NORM, 0.0, (double)a.M * a.N * (4.0 * g.k_splits + 8.0 + esz(m)));
      launch_splitk_reduce_norm(m->stream, g, m->cfg.norm, m->cfg.norm_eps, then->g, then->b, then->x);
      then->done = true;
      return true;
    }
    launch_checked(m, g);
    return true;
  }
  if (a.w_scale != nullptr) {                  // no shape-agnostic kernel reads int8 weights: refuse, loudly
    m->deferred = "int8 weights: a GEMM of this pass has a shape the MFMA kernel does not take";
    return true;
  }
  launch_linear_simple(m->stream, dense);
  return true;
}

// SwiGLU up-projection: gate and up tiles in one kernel, u = SiLU(gate) * up rounded once
bool gemm_swiglu_mfma(mpz_model* m, const LinearArgs& a, int f, void* u_out) {
  if (!m->use_mfma) return false;
  MfmaGemmArgs g{};
  g.M = a.M; g.N = f; g.K = a.K; g.x = a.x; g.w = a.w; g.w_scale = a.w_scale; g.w_rows = 2 * f; g.bias = a.bias; g.dual = 1; g.dual_offset = f;
  g.rows_per_copy = a.rows_per_copy; g.act = -1; g.out_f32 = 0; g.out = u_out; g.ldo = f;
  g.tile_cfg = m->force_tile_cfg;
  if (a.w_codes != nullptr) { g.w = a.w_codes; g.w_absmax = a.w_absmax; }
  plan_split(m, g);
  const bool dequantise = a.w_codes != nullptr && g.k_splits <= 1;
  if (dequantise) { g.w = m->buf.wq; g.w_absmax = nullptr; }
  if (!mfma_gemm_supported(g)) return false;     // (nothing launched: the caller's plain GEMM dequantises for itself)
  if (dequantise) dequantised(m, a.w_codes, a.w_absmax, 2 * f, a.K);
  ProfScope ps(m, MPZ_PROF_GEMM, 2.0 * a.M * (double)(2 * f) * a.K,
               2.0 * ((double)a.M * a.K + 2.0 * f * a.K + (double)a.M * f));
  launch_checked(m, g);
  return true;
}

// index of (target, factor) among one layer's LoRA tensors
int tensor_slot(const mpz_model* m, int target, int factor) {
  for (int i = 0; i < m->tab.n_tensors; ++i)
    if (m->tab.local_id[i] == target * 2 + factor) return i;
  return 0;
}

// The fp32 perturbed copies (master layout) of the last mpz_regen_noise.  bf16 models whose pass runs on the MFMA
// kernels read only the bf16 operand layouts, so mpz_regen_noise writes those alone; whoever needs the fp32 form
// (a shape the MFMA kernels refuse, the stateful update, the test hook) regenerates it here from the same seed -
// the masters have not changed since, so these are the same factors.  Enqueued on the model's stream.
void ensure_pert(mpz_model* m) {
  if (m->pert_valid) return;
  ProfScope ps(m, MPZ_PROF_NOISE, 0.0, 4.0 * m->P * (1.0 + 2.0 * m->q));
  launch_perturb(m->stream, m->masters, m->buf.pert, m->P, m->tab, m->seed, m->step, m->q, m->eps, m->cfg.perturb_A);
  m->pert_valid = true;
}

// Will every adapted projection of a pass over copies of E x S rows take the MFMA low-rank path (the same checks as
// run_qkv / run_layers make when they choose)?  If not, the pass reads the fp32 copies.
bool lora_path_is_mfma(const mpz_model* m, int E, int S) {
  if (!m->use_mfma) return false;
  const mpz_config& c = m->cfg;
  // (judged for the largest pass, all 2q copies: what it allows, every smaller range of copies allows too)
  const int rpc = E * S, T = 2 * m->q * rpc, d = c.d_model, dkv = c.n_kv_heads * (d / c.n_heads), nqkv = d + 2 * dkv;
  const int col0[3] = {0, d, d + dkv}, col1[3] = {d, d + dkv, nqkv};
  MfmaLoraDownArgs md{};
  md.T = T; md.K = d; md.rank = c.lora_rank; md.rows_per_copy = rpc; md.rp = m->rp;
  MfmaGemmArgs probe{};
  probe.M = T; probe.N = nqkv; probe.K = d; probe.rows_per_copy = rpc;
  int nt = 0;
  for (int t = 0; t < 3; ++t)
    if (c.lora_targets & (1u << t)) {
      probe.seg[nt].col_begin = col0[t]; probe.seg[nt].col_end = col1[t]; probe.seg[nt].rp = m->rp;
      ++nt;
    }
  md.n_targets = nt; probe.n_seg = nt;
  if (nt && !(mfma_lora_down_supported(md) && mfma_gemm_supported(probe))) return false;
  if (c.lora_targets & MPZ_TARGET_O) {
    md.n_targets = 1;
    MfmaGemmArgs po{};
    po.M = T; po.N = d; po.K = d; po.rows_per_copy = rpc; po.n_seg = 1;
    po.seg[0].col_begin = 0; po.seg[0].col_end = d; po.seg[0].rp = m->rp;
    if (!(mfma_lora_down_supported(md) && mfma_gemm_supported(po))) return false;
  }
  return true;
}

// Called by every pass before its first launch, on the caller's stream: make the fp32 copies if this pass reads them.
void prepare_factors(mpz_model* m, int E, int S) {
  if (!m->pert_valid && !lora_path_is_mfma(m, E, S)) ensure_pert(m);
}

// fp32 residual rows -> operand type
void norm(mpz_model* m, const float* h, int64_t h_row_stride, const float* g, const float* b, void* out, int rows) {
  const mpz_config& c = m->cfg;
  ProfScope ps(m, MPZ_PROF_NORM, 0.0, (double)rows * c.d_model * (4.0 + esz(m)));
  if (m->use_mfma && norm_rows_supported(c.d_model, h_row_stride))
    launch_norm_rows(m->stream, c.norm, c.norm_eps, h, h_row_stride, g, b, out, rows, c.d_model);
  else
    launch_norm(m->stream, c.dtype, c.norm, c.norm_eps, h, h_row_stride, g, b, out, rows, c.d_model);
}

void run_embed(mpz_model* m, const int32_t* tokens, int E, int S, float* h) {
  const mpz_config& c = m->cfg;
  ProfScope ps(m, MPZ_PROF_EMBED, 0.0, (double)m->nc * E * S * (double)c.d_model * (4.0 + esz(m)));
  launch_embed(m->stream, c.dtype, tokens, m->w.emb, c.pos == MPZ_POS_ROPE ? nullptr : m->w.pos_emb,
               m->pk.cu ? m->buf.row_pos : nullptr, h, m->nc, E, S, c.d_model);
}

// q/k/v projections of the MP-LoRA layer for all stacked copies: x = b.x [T, d] -> out [T, d + 2 d_kv]
// rope: apply the rotary embedding to q and k and write the operand type to b.qkv (fused into the GEMM epilogue
// where the shape allows, else through the accumulate-type staging buffer); otherwise write `out` as `out_kind` says.
// norm_h != null: b.x has not been computed yet; it is the pre-norm of the residual rows norm_h [T, d], done here -
// in one kernel with the LoRA bottleneck where the shapes allow, else as the plain norm ahead of everything else.
void run_qkv(mpz_model* m, const Buffers& b, int l, int E, int S, bool rope, int out_kind, void* out,
             const float* norm_h = nullptr) {
  const mpz_config& c = m->cfg;
  hipStream_t st = m->stream;
  const mpz_layer_weights& lw = m->layers[l];
  const int n = m->nc, rpc = E * S, T = n * rpc;
  const int d = c.d_model, dh = d / c.n_heads, dkv = c.n_kv_heads * dh, r = c.lora_rank;
  const int nqkv = d + 2 * dkv;
  {
    // q/k/v projections of the MP-LoRA layer: shared W, per-copy (A_c, B_c)
    LoraDownArgs da{};
    da.dtype = c.dtype; da.T = T; da.K = d; da.rank = r; da.rows_per_copy = rpc; da.x = b.x; da.scale = c.lora_scale;
    da.copy_stride = m->P * m->cstep; da.t = b.t;
    LinearArgs qa{};
    qa.dtype = c.dtype; qa.M = T; qa.N = nqkv; qa.K = d; qa.x = b.x; qa.w = lw.w_qkv; qa.w_scale = lw.s_qkv; qa.bias = lw.b_qkv;
    qa.rank = r; qa.rows_per_copy = rpc; qa.act = -1; qa.residual = nullptr;
    const int col0[3] = {0, d, d + dkv}, col1[3] = {d, d + dkv, nqkv};
    int nt = 0;
    for (int t = 0; t < 3; ++t) {
      if (!(c.lora_targets & (1u << t))) continue;
      da.Ac[nt] = b.pert + find_tensor(m, l, t, 0)->offset;
      LoraSeg& sg = qa.seg[nt];
      sg.col_begin = col0[t]; sg.col_end = col1[t]; sg.t = b.t; sg.t_off = nt * r;
      sg.Bc = b.pert + find_tensor(m, l, t, 1)->offset; sg.copy_stride = m->P * m->cstep;
      ++nt;
    }
    for (int i = 0; i < nt; ++i) qa.seg[i].t_stride = nt * r;
    da.n_targets = nt; qa.n_seg = nt;
    const char* packed_l = (const char*)b.packed + (size_t)l * m->packed_per_layer * 2;
    bool lora_done = false;
    if (nt && m->use_mfma) {
      MfmaLoraDownArgs md{};
      md.T = T; md.K = d; md.rank = r; md.n_targets = nt; md.rows_per_copy = rpc; md.rp = m->rp; md.x = b.x;
      md.scale = c.lora_scale; md.copy_stride = m->packed_per_copy * m->cstep;
      int i = 0;
      for (int t = 0; t < 3; ++t) {
        if (!(c.lora_targets & (1u << t))) continue;
        int ia = tensor_slot(m, t, 0), ib = tensor_slot(m, t, 1);
        md.ap[i] = packed_l + m->packed_off[ia] * 2; md.tp[i] = b.tp[i];
        MfmaLoraSeg& ms = qa.mseg[i];
        ms.col_begin = col0[t]; ms.col_end = col1[t]; ms.tp = b.tp[i]; ms.bp = packed_l + m->packed_off[ib] * 2;
        ms.rp = m->rp; ms.copy_stride = m->packed_per_copy * m->cstep;
        ++i;
      }
      MfmaGemmArgs probe{};
      probe.M = T; probe.N = nqkv; probe.K = d; probe.n_seg = nt; probe.rows_per_copy = rpc;
      for (int k = 0; k < nt; ++k) probe.seg[k] = qa.mseg[k];
      if (mfma_lora_down_supported(md) && mfma_gemm_supported(probe)) {
        if (norm_h != nullptr && m->fuse_norm_lora && norm_lora_supported(d, md)) {
          // booked under the norm: one read of the fp32 rows, one write of the operand rows and of t
          ProfScope ps(m, MPZ_PROF_NORM, 4.0 * T * (double)d * nt * r, (double)T * d * (4.0 + esz(m)) + 2.0 * T * (double)nt * m->rp);
          launch_norm_lora(st, c.norm, c.norm_eps, norm_h, lw.ln1_g, lw.ln1_b, b.x, md);
          norm_h = nullptr;
        } else {
          if (norm_h != nullptr) { norm(m, norm_h, d, lw.ln1_g, lw.ln1_b, b.x, T); norm_h = nullptr; }
          ProfScope ps(m, MPZ_PROF_LORA_DOWN, 4.0 * T * (double)d * nt * r, 2.0 * T * ((double)d + (double)nt * m->rp));
          launch_lora_down_mfma(st, md);
        }
        qa.mfma_lora = 1; lora_done = true;
      }
    }
    if (norm_h != nullptr) { norm(m, norm_h, d, lw.ln1_g, lw.ln1_b, b.x, T); norm_h = nullptr; }
    if (nt && !lora_done) {
      if (!m->pert_valid) m->deferred = "internal: a pass needs the fp32 factor copies and they were not prepared";
      ProfScope ps(m, MPZ_PROF_LORA_DOWN, 2.0 * T * (double)d * nt * r, esz(m) * T * ((double)d + (double)nt * r));
      launch_lora_down_simple(st, da);
    }
    set_weight(qa, weight_operand(m, lw.w_qkv, lw.s_qkv, nqkv, d, T));
    if (rope) {
      qa.out_kind = 0; qa.out = b.qkv;
      qa.rope_cos = b.rope_cos; qa.rope_sin = b.rope_sin; qa.rope_cols = d + dkv; qa.rope_dh = dh; qa.S = S;
      qa.rope_pos = m->pk.cu ? b.row_pos : nullptr;
      if (gemm(m, qa)) return;
      qa.rope_cos = qa.rope_sin = nullptr;
      qa.out_kind = 2; qa.out = b.stage;
      gemm(m, qa);
      ProfScope ps(m, MPZ_PROF_ROPE, 0.0, (double)T * nqkv * (acc_size(c.dtype) + esz(m)));
      launch_rope_convert(st, c.dtype, b.stage, b.qkv, T, S, nqkv, dh, c.n_heads + c.n_kv_heads, b.rope_cos, b.rope_sin,
                          m->pk.cu ? b.row_pos : nullptr);
      return;
    }
    qa.out_kind = out_kind; qa.out = out;
    gemm(m, qa);
  }
}

// Decoder blocks [l0, l1) on the stacked residual stream h [T, d]: per adapted linear an optional
// bottleneck kernel, then the GEMM with the per-copy rank-r term.
void run_layers(mpz_model* m, float* h, int l0, int l1, int E, int S) {
  const mpz_config& c = m->cfg;
  hipStream_t st = m->stream;
  Buffers b = view(m, E, S);
  b.h = h;
  const int n = m->nc, rpc = E * S, T = n * rpc;
  const int d = c.d_model, dh = d / c.n_heads, dkv = c.n_kv_heads * dh, f = c.d_ffn, r = c.lora_rank;
  const int nqkv = d + 2 * dkv;
  const bool rope = c.pos == MPZ_POS_ROPE, swiglu = c.act == MPZ_ACT_SWIGLU;

  bool x_ready = false;                               // b.x already holds this block's first pre-norm (see the end of the loop)
  for (int l = l0; l < l1; ++l) {
    const mpz_layer_weights& lw = m->layers[l];
    run_qkv(m, b, l, E, S, rope, 0, b.qkv, x_ready ? nullptr : b.h);      // pre-norm, LoRA bottleneck, projection
    x_ready = false;

    {
      // causal-useful work: Q K^T and P V over the S (S + 1) / 2 visible (query, key) pairs of every head
      // (packed batches: booked as if every sequence had the longest one's length - an upper bound)
      const int aE = m->pk.cu ? m->pk.E : E, aS = m->pk.cu ? m->pk.max_len : S;
      ProfScope ps(m, MPZ_PROF_ATTENTION, 2.0 * n * aE * c.n_heads * (double)aS * (aS + 1) * dh, esz(m) * T * ((double)nqkv + d));
      if (m->use_mfma && attention_mfma_supported(dh, nqkv, d))
        launch_attention_mfma(st, b.qkv, nqkv, b.attn, n * aE, aS, c.n_heads, c.n_kv_heads, dh, m->pk.cu, aE, rpc);
      else
        launch_attention_simple(st, c.dtype, b.qkv, nqkv, b.attn, n * aE, aS, c.n_heads, c.n_kv_heads, dh, m->pk.cu, aE, rpc);
    }

    // output projection (+ adapter) added to the residual stream
    const char* packed_l = (const char*)b.packed + (size_t)l * m->packed_per_layer * 2;
    LoraDownArgs da{};
    da.dtype = c.dtype; da.T = T; da.K = d; da.rank = r; da.rows_per_copy = rpc; da.scale = c.lora_scale;
    da.copy_stride = m->P * m->cstep; da.t = b.t;
    LinearArgs oa{};
    oa.dtype = c.dtype; oa.M = T; oa.N = d; oa.K = d; oa.x = b.attn; oa.w = lw.w_o; oa.w_scale = lw.s_o; oa.bias = lw.b_o;
    oa.rank = r; oa.rows_per_copy = rpc; oa.act = -1; oa.residual = b.h; oa.out_kind = 1; oa.out = b.h;
    if (c.lora_targets & MPZ_TARGET_O) {
      LoraDownArgs oda = da;
      oda.x = b.attn; oda.n_targets = 1; oda.Ac[0] = b.pert + find_tensor(m, l, 3, 0)->offset;
      bool o_done = false;
      if (m->use_mfma) {
        MfmaLoraDownArgs md{};
        md.T = T; md.K = d; md.rank = r; md.n_targets = 1; md.rows_per_copy = rpc; md.rp = m->rp; md.x = b.attn;
        md.scale = c.lora_scale; md.copy_stride = m->packed_per_copy * m->cstep;
        md.ap[0] = packed_l + m->packed_off[tensor_slot(m, 3, 0)] * 2; md.tp[0] = b.tp[0];
        MfmaLoraSeg& ms = oa.mseg[0];
        ms.col_begin = 0; ms.col_end = d; ms.tp = b.tp[0]; ms.bp = packed_l + m->packed_off[tensor_slot(m, 3, 1)] * 2;
        ms.rp = m->rp; ms.copy_stride = m->packed_per_copy * m->cstep;
        MfmaGemmArgs probe{};
        probe.M = T; probe.N = d; probe.K = d; probe.n_seg = 1; probe.rows_per_copy = rpc; probe.seg[0] = ms;
        if (mfma_lora_down_supported(md) && mfma_gemm_supported(probe)) {
          { ProfScope ps(m, MPZ_PROF_LORA_DOWN, 4.0 * T * (double)d * r, 2.0 * T * ((double)d + (double)m->rp));
            launch_lora_down_mfma(st, md); }
          oa.mfma_lora = 1; o_done = true;
        }
      }
      if (!o_done) {
        if (!m->pert_valid) m->deferred = "internal: a pass needs the fp32 factor copies and they were not prepared";
        ProfScope ps(m, MPZ_PROF_LORA_DOWN, 2.0 * T * (double)d * r, esz(m) * T * ((double)d + (double)r));
        launch_lora_down_simple(st, oda);
      }
      oa.n_seg = 1;
      oa.seg[0].col_begin = 0; oa.seg[0].col_end = d; oa.seg[0].t = b.t; oa.seg[0].t_stride = r; oa.seg[0].t_off = 0;
      oa.seg[0].Bc = b.pert + find_tensor(m, l, 3, 1)->offset; oa.seg[0].copy_stride = m->P * m->cstep;
    }
    set_weight(oa, weight_operand(m, lw.w_o, lw.s_o, d, d, T));
    // feed-forward block: its pre-norm rides on the reduction of the output projection where that splits K
    NormAfter ffn_norm{lw.ln2_g, lw.ln2_b, b.x, false};
    gemm(m, oa, &ffn_norm);
    if (!ffn_norm.done) norm(m, b.h, d, lw.ln2_g, lw.ln2_b, b.x, T);
    LinearArgs ua{};
    ua.dtype = c.dtype; ua.M = T; ua.N = swiglu ? 2 * f : f; ua.K = d; ua.x = b.x; ua.w = lw.w_up; ua.w_scale = lw.s_up; ua.bias = lw.b_up;
    ua.rank = r; ua.rows_per_copy = rpc; ua.act = swiglu ? -1 : c.act;
    ua.out_kind = swiglu ? 2 : 0; ua.out = swiglu ? b.stage : b.u;
    set_weight(ua, weight_operand(m, lw.w_up, lw.s_up, swiglu ? 2 * f : f, d, T));
    if (!(swiglu && gemm_swiglu_mfma(m, ua, f, b.u))) {
      gemm(m, ua);
      if (swiglu) {
        ProfScope ps(m, MPZ_PROF_OTHER, 0.0, (double)T * f * (2.0 * acc_size(c.dtype) + esz(m)));
        launch_swiglu(st, c.dtype, b.stage, b.u, T, f);
      }
    }
    LinearArgs wa{};
    wa.dtype = c.dtype; wa.M = T; wa.N = d; wa.K = f; wa.x = b.u; wa.w = lw.w_down; wa.w_scale = lw.s_down; wa.bias = lw.b_down;
    wa.rank = r; wa.rows_per_copy = rpc; wa.act = -1; wa.residual = b.h; wa.out_kind = 1; wa.out = b.h;
    set_weight(wa, weight_operand(m, lw.w_down, lw.s_down, d, f, T));
    if (l + 1 < l1) {                                 // likewise the next block's first pre-norm
      NormAfter next_norm{m->layers[l + 1].ln1_g, m->layers[l + 1].ln1_b, b.x, false};
      gemm(m, wa, &next_norm);
      x_ready = next_norm.done;
    } else {
      gemm(m, wa);
    }
  }
}

// final norm, head and per-copy loss from the stacked residual stream h [T, d]
// LM head and cross-entropy in one pass (bf16 MFMA path): the GEMM keeps the logits in its accumulators and
// leaves, per token row and wave tile, a running maximum and sum of exponentials in the buffer that the unfused
// path uses for a chunk of logits; a second small kernel folds them into the row's loss.  Returns false (nothing
// launched) when the shape or the workspace does not allow it.
bool head_ce_fused(mpz_model* m, const Buffers& b, const void* x, int rows, int vocab, int d, int rpc,
                   const int32_t* target, float* ce) {
  const mpz_config& c = m->cfg;
  if (!(m->use_mfma && c.dtype == MPZ_DTYPE_BF16)) return false;
  MfmaGemmArgs g{};
  g.M = rows; g.N = vocab; g.K = d; g.x = x; g.w = m->w.lm_head; g.w_rows = vocab; g.rows_per_copy = rpc; g.act = -1;
  g.out_f32 = 1; g.out = b.logits; g.ldo = vocab; g.tile_cfg = m->force_tile_cfg;
  const int slots = mfma_gemm_ce_slots(g);
  const size_t need = ((size_t)2 * slots + 1) * rows, have = (size_t)b.chunk_rows * vocab;
  if (need > have) return false;
  g.ce_max = b.logits; g.ce_sum = b.logits + (size_t)slots * rows; g.ce_tlogit = b.logits + (size_t)2 * slots * rows;
  g.ce_target = target;
  if (!mfma_gemm_supported(g)) return false;
  { ProfScope ps(m, MPZ_PROF_GEMM, 2.0 * rows * (double)vocab * d,
                 2.0 * ((double)rows * d + (double)vocab * d) + 8.0 * slots * (double)rows);
    launch_checked(m, g); }
  { ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 8.0 * slots * (double)rows);
    launch_ce_combine(m->stream, slots, rows, g.ce_max, g.ce_sum, g.ce_tlogit, target, ce); }
  return true;
}

void run_head(mpz_model* m, const float* h, const int32_t* tokens, const int32_t* labels, int E, int S, float* losses_out) {
  const mpz_config& c = m->cfg;
  hipStream_t st = m->stream;
  Buffers b = view(m, E, S);
  b.h = const_cast<float*>(h);
  const int n = m->nc, rpc = E * S, T = n * rpc;
  const int d = c.d_model;
  const bool packed = m->pk.cu != nullptr;        // then E = 1 and S = rows per copy; the sequences are m->pk's
  const int Es = packed ? m->pk.E : E;            // sequences per copy
  const int nt_count = packed ? m->pk.total - m->pk.E : E * (S - 1);   // next-token positions per copy (full lengths)
  { ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 0.0);
    if (c.loss_mode == MPZ_LOSS_NEXT_TOKEN_ALL_POS)
      launch_make_targets(st, c.loss_mode, tokens, labels, m->lengths, packed ? b.row_end : nullptr, c.label_token[0],
                          c.label_token[1], b.target, n, E, S);
    else
      launch_make_targets(st, c.loss_mode, tokens, labels, nullptr, nullptr, c.label_token[0], c.label_token[1], b.target,
                          n, Es, S); }
  if (c.loss_mode == MPZ_LOSS_NEXT_TOKEN_ALL_POS) {
    norm(m, b.h, d, m->w.lnf_g, m->w.lnf_b, b.x, T);
    if (head_ce_fused(m, b, b.x, T, c.vocab, d, rpc, b.target, b.ce)) {
      ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 4.0 * T);
      launch_copy_mean(st, b.ce, rpc, nt_count, m->lengths, E, S, losses_out, n, m->cstep);
      return;
    }
    for (int r0 = 0; r0 < T; r0 += b.chunk_rows) {
      int rows = T - r0 < b.chunk_rows ? T - r0 : b.chunk_rows;
      LinearArgs la{};
      la.dtype = c.dtype; la.M = rows; la.N = c.vocab; la.K = d;
      la.x = (const unsigned char*)b.x + (size_t)r0 * d * elem_size(c.dtype);
      la.w = m->w.lm_head; la.act = -1; la.rows_per_copy = rpc; la.out_kind = 1; la.out = b.logits;
      gemm(m, la);
      { ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 4.0 * rows * (double)c.vocab);
        launch_ce_rows(st, c.dtype, b.logits, c.vocab, c.vocab, b.target + r0, b.ce + r0, rows); }
    }
    { ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 4.0 * T);
      launch_copy_mean(st, b.ce, rpc, nt_count, m->lengths, E, S, losses_out, n, m->cstep); }
  } else {
    const int rows_all = n * Es;
    if (m->lengths != nullptr || packed) {       // last real token of every sequence, gathered into the (idle) FFN buffer
      float* last = (float*)b.u;
      { ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 8.0 * rows_all * d);
        if (packed) launch_gather_last_rows_packed(st, b.h, m->pk.cu, n, Es, rpc, d, last);
        else launch_gather_last_rows(st, b.h, m->lengths, n, E, S, d, last); }
      norm(m, last, d, m->w.lnf_g, m->w.lnf_b, b.x, rows_all);
    } else {
      norm(m, b.h + (size_t)(S - 1) * d, (int64_t)S * d, m->w.lnf_g, m->w.lnf_b, b.x, rows_all);
    }
    if (c.loss_mode == MPZ_LOSS_LAST_POS_LABEL_SUBSET) {
      ProfScope ps(m, MPZ_PROF_LOSS, 0.0, esz(m) * (double)d * (rows_all + 2));
      launch_last_pos_subset_logits(st, c.dtype, b.x, m->w.lm_head, d, rows_all, c.label_token[0], c.label_token[1], b.logits);
      launch_ce_rows(st, c.dtype, b.logits, 2, 2, b.target, b.ce, rows_all);
    } else {
      const bool fused = head_ce_fused(m, b, b.x, rows_all, c.vocab, d, rpc, b.target, b.ce);
      for (int r0 = 0; r0 < rows_all && !fused; r0 += b.chunk_rows) {
        int rows = rows_all - r0 < b.chunk_rows ? rows_all - r0 : b.chunk_rows;
        LinearArgs la{};
        la.dtype = c.dtype; la.M = rows; la.N = c.vocab; la.K = d;
        la.x = (const unsigned char*)b.x + (size_t)r0 * d * elem_size(c.dtype);
        la.w = m->w.lm_head; la.act = -1; la.rows_per_copy = rpc; la.out_kind = 1; la.out = b.logits;
        gemm(m, la);
        { ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 4.0 * rows * (double)c.vocab);
        launch_ce_rows(st, c.dtype, b.logits, c.vocab, c.vocab, b.target + r0, b.ce + r0, rows); }
      }
    }
    { ProfScope ps(m, MPZ_PROF_LOSS, 0.0, 4.0 * rows_all);
      launch_copy_mean(st, b.ce, Es, Es, nullptr, Es, S, losses_out, n, m->cstep); }
  }
}

}  // namespace

extern "C" {

size_t mpz_lora_numel(const mpz_config* cfg) {
  if (!cfg || validate_config(cfg)) return 0;
  std::vector<mpz_lora_tensor> lay; LoraLayerTable tab;
  build_layout(cfg, lay, tab);
  return (size_t)tab.per_layer * cfg->n_layers;
}

int32_t mpz_lora_tensor_count(const mpz_config* cfg) {
  if (!cfg || validate_config(cfg)) return 0;
  return 2 * count_targets(cfg->lora_targets) * cfg->n_layers;
}

mpz_status mpz_lora_tensor_info(const mpz_config* cfg, int32_t i, mpz_lora_tensor* out) {
  if (!cfg || !out) return fail(nullptr, MPZ_ERR_NULL, "mpz_lora_tensor_info: NULL argument");
  if (const char* e = validate_config(cfg)) return fail(nullptr, MPZ_ERR_CONFIG, e);
  std::vector<mpz_lora_tensor> lay; LoraLayerTable tab;
  build_layout(cfg, lay, tab);
  if (i < 0 || i >= (int32_t)lay.size()) return fail(nullptr, MPZ_ERR_SHAPE, "tensor index out of range");
  *out = lay[i];
  return MPZ_OK;
}

size_t mpz_workspace_bytes(const mpz_config* cfg, int32_t q_max, int32_t E_max, int32_t S_max) {
  if (!cfg || validate_config(cfg)) return 0;
  if (q_max < 1 || q_max > 64 || E_max < 1 || S_max < 2 || S_max > cfg->max_seq) return 0;
  return carve(cfg, q_max, E_max, S_max, nullptr, nullptr);
}

mpz_status mpz_init_model(const mpz_config* cfg, const mpz_weights* frozen, float* lora_masters, void* workspace,
                          size_t workspace_bytes, int32_t q_max, int32_t E_max, int32_t S_max, void* hip_stream,
                          mpz_model** out) {
  if (!cfg || !frozen || !lora_masters || !workspace || !out) return fail(nullptr, MPZ_ERR_NULL, "mpz_init_model: NULL argument");
  *out = nullptr;
  if (const char* e = validate_config(cfg)) return fail(nullptr, MPZ_ERR_CONFIG, e);
  if (q_max < 1 || q_max > 64) return fail(nullptr, MPZ_ERR_CONFIG, "q_max must be in [1, 64]");
  if (E_max < 1 || S_max < 2 || S_max > cfg->max_seq) return fail(nullptr, MPZ_ERR_CONFIG, "E_max < 1 or S_max outside [2, max_seq]");
  if ((int64_t)2 * q_max * E_max * S_max > (int64_t)1 << 24) return fail(nullptr, MPZ_ERR_CONFIG, "more than 2^24 stacked tokens");
  if (!frozen->emb || !frozen->lm_head || !frozen->lnf_g || !frozen->layers)
    return fail(nullptr, MPZ_ERR_NULL, "mpz_init_model: NULL frozen weight");
  if (cfg->pos == MPZ_POS_LEARNED && !frozen->pos_emb) return fail(nullptr, MPZ_ERR_NULL, "learned positions need pos_emb");
  if (cfg->norm == MPZ_NORM_LAYERNORM && !frozen->lnf_b) return fail(nullptr, MPZ_ERR_NULL, "LayerNorm needs lnf_b");
  for (int l = 0; l < cfg->n_layers; ++l) {
    const mpz_layer_weights& lw = frozen->layers[l];
    if (!lw.ln1_g || !lw.ln2_g || !lw.w_qkv || !lw.w_o || !lw.w_up || !lw.w_down)
      return fail(nullptr, MPZ_ERR_NULL, "mpz_init_model: NULL layer weight");
    if (cfg->norm == MPZ_NORM_LAYERNORM && (!lw.ln1_b || !lw.ln2_b)) return fail(nullptr, MPZ_ERR_NULL, "LayerNorm needs biases");
    if (cfg->has_bias && (!lw.b_qkv || !lw.b_o || !lw.b_up || !lw.b_down))
      return fail(nullptr, MPZ_ERR_NULL, "has_bias set but a linear bias is NULL");
    if (cfg->weight_quant == MPZ_WEIGHT_QUANT_INT8) {
      if (!lw.s_qkv || !lw.s_o || !lw.s_up || !lw.s_down) return fail(nullptr, MPZ_ERR_NULL, "int8 weights need their scales");
      if ((((uintptr_t)lw.s_qkv | (uintptr_t)lw.s_o | (uintptr_t)lw.s_up | (uintptr_t)lw.s_down) & 15u) != 0)
        return fail(nullptr, MPZ_ERR_CONFIG, "int8 weight scales must be 16-byte aligned");
    }
    if (cfg->weight_quant == MPZ_WEIGHT_QUANT_NF4) {
      if (!lw.s_qkv || !lw.s_o || !lw.s_up || !lw.s_down) return fail(nullptr, MPZ_ERR_NULL, "4-bit weights need their block maxima");
      if ((((uintptr_t)lw.s_qkv | (uintptr_t)lw.s_o | (uintptr_t)lw.s_up | (uintptr_t)lw.s_down | (uintptr_t)lw.w_qkv |
            (uintptr_t)lw.w_o | (uintptr_t)lw.w_up | (uintptr_t)lw.w_down) & 3u) != 0)
        return fail(nullptr, MPZ_ERR_CONFIG, "4-bit codes and block maxima must be 4-byte aligned");
    }
  }
  if (((uintptr_t)workspace & 255u) != 0) return fail(nullptr, MPZ_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  size_t need = carve(cfg, q_max, E_max, S_max, nullptr, nullptr);
  if (workspace_bytes < need) {
    char msg[128];
    snprintf(msg, sizeof msg, "workspace too small: %zu bytes given, %zu needed", workspace_bytes, need);
    return fail(nullptr, MPZ_ERR_WORKSPACE, msg);
  }
  mpz_model* m = new (std::nothrow) mpz_model();
  if (!m) return fail(nullptr, MPZ_ERR_DEVICE, "out of host memory");
  m->cfg = *cfg;
  m->layers.assign(frozen->layers, frozen->layers + cfg->n_layers);
  if (!cfg->has_bias)
    for (auto& lw : m->layers) lw.b_qkv = lw.b_o = lw.b_up = lw.b_down = nullptr;
  if (cfg->norm == MPZ_NORM_RMSNORM)
    for (auto& lw : m->layers) lw.ln1_b = lw.ln2_b = nullptr;
  if (cfg->weight_quant == MPZ_WEIGHT_QUANT_NONE)
    for (auto& lw : m->layers) lw.s_qkv = lw.s_o = lw.s_up = lw.s_down = nullptr;
  m->w = *frozen;
  m->w.layers = m->layers.data();
  if (cfg->norm == MPZ_NORM_RMSNORM) m->w.lnf_b = nullptr;
  m->masters = lora_masters;
  m->stream = (hipStream_t)hip_stream;
  {
    hipError_t e = hipSuccess;                   // set-up of the allocation-free entry point: this device's scratch
    (void)scratch_address(&m->device, &e);       // address; a failure is reported by that entry point, not here
    (void)hipGetLastError();
  }
  m->q_max = q_max; m->E_max = E_max; m->S_max = S_max;
  build_layout(cfg, m->tensors, m->tab);
  m->P = (int64_t)m->tab.per_layer * cfg->n_layers;
  carve(cfg, q_max, E_max, S_max, workspace, &m->buf);
  {
    const int dh = cfg->d_model / cfg->n_heads, dkv = cfg->n_kv_heads * dh;
    size_t cols = cfg->pos == MPZ_POS_ROPE ? (size_t)cfg->d_model + 2 * dkv : 0;
    if (cfg->act == MPZ_ACT_SWIGLU && (size_t)2 * cfg->d_ffn > cols) cols = (size_t)2 * cfg->d_ffn;
    m->stage_row_bytes = cols * acc_size(cfg->dtype);
  }
  m->use_mfma = cfg->dtype == MPZ_DTYPE_BF16;
  m->rp = (2 * cfg->lora_rank + 15) / 16 * 16;
  for (int i = 0; i < m->tab.n_tensors; ++i) {
    m->packed_off[i] = m->packed_per_layer;
    m->packed_per_layer += (m->tab.local_id[i] & 1) ? (int64_t)m->tab.cols[i] * m->rp : (int64_t)2 * m->tab.rows[i] * m->tab.cols[i];
  }
  m->packed_per_copy = m->packed_per_layer * cfg->n_layers;
  if (cfg->pos == MPZ_POS_ROPE) {
    int dh = cfg->d_model / cfg->n_heads, half = dh / 2;
    std::vector<float> cs((size_t)cfg->max_seq * half), sn((size_t)cfg->max_seq * half);
    for (int i = 0; i < half; ++i) {
      double inv = std::pow((double)cfg->rope_theta, -2.0 * i / dh);
      for (int p = 0; p < cfg->max_seq; ++p) {
        double ang = p * inv;
        cs[(size_t)p * half + i] = (float)std::cos(ang);
        sn[(size_t)p * half + i] = (float)std::sin(ang);
      }
    }
    hipError_t e1 = hipMemcpyAsync(m->buf.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice, m->stream);
    hipError_t e2 = hipMemcpyAsync(m->buf.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice, m->stream);
    hipError_t e3 = hipStreamSynchronize(m->stream);
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess) {
      delete m;
      return fail(nullptr, MPZ_ERR_DEVICE, "uploading the rotary tables failed");
    }
  }
  *out = m;
  return MPZ_OK;
}

mpz_status mpz_regen_noise(mpz_model* m, uint64_t seed, uint32_t step, int32_t q, float eps) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_regen_noise: NULL model");
  if (q < 1 || q > m->q_max) return fail(m, MPZ_ERR_SHAPE, "q outside [1, q_max]");
  if (!std::isfinite(eps) || eps < 0.f) return fail(m, MPZ_ERR_CONFIG, "eps must be finite and non-negative");
  if (m->use_mfma && m->fuse_perturb_pack && perturb_pack_supported(m->tab, m->cfg.lora_rank, m->rp)) {
    // bf16 models: the noise goes straight into the bf16 hi / lo operand layouts; no fp32 copy is written
    ProfScope ps(m, MPZ_PROF_NOISE, 0.0, 4.0 * m->P + 2.0 * q * 2.0 * m->packed_per_copy);
    launch_perturb_pack(m->stream, m->masters, m->buf.packed, m->packed_per_copy, m->tab, m->cfg.n_layers, m->cfg.lora_rank,
                        m->rp, seed, step, q, eps, m->cfg.perturb_A);
    m->pert_valid = false;
  } else {
    {
      ProfScope ps(m, MPZ_PROF_NOISE, 0.0, 4.0 * m->P * (1.0 + 2.0 * q));
      launch_perturb(m->stream, m->masters, m->buf.pert, m->P, m->tab, seed, step, q, eps, m->cfg.perturb_A);
    }
    m->pert_valid = true;
    ProfScope ps_pack(m, MPZ_PROF_PACK, 0.0, m->use_mfma ? 2.0 * q * (4.0 * m->P + 2.0 * m->packed_per_copy) : 0.0);
    if (m->use_mfma)
      launch_pack_factors(m->stream, m->buf.pert, m->P, 2 * q, m->tab, m->cfg.n_layers, m->cfg.lora_rank, m->rp, m->buf.packed,
                          m->packed_per_copy);
  }
  m->have_noise = true; m->seed = seed; m->step = step; m->q = q; m->eps = eps;
  m->cb = 0; m->nc = 2 * q;
  return check_device(m, "mpz_regen_noise");
}

namespace {

// Small models (every GEMM of the pass stays on the 128-wide tiles) leave the chip part-empty around each kernel's
// first loads and last stores.  The copies are independent (Section 3), so the pass is issued as two halves of
// n/2 copies on two streams, layer by layer: the halves' kernels overlap and fill each other's edges (workload 2:
// 2.98 -> 2.68 ms per step).  Every copy's numbers are what the one-stream pass gives (a copy's rows never mix
// with another's).  The second stream forks from and joins the caller's stream through events, so the call keeps
// its ordering guarantees; it is not used while kernels are being timed one by one.
bool use_two_halves(mpz_model* m, int E, int S) {
  const mpz_config& c = m->cfg;
  const int n = 2 * m->q;
  if (!m->two_halves || m->prof_on || !m->use_mfma || n < 4 || n % 2 || m->lengths != nullptr || m->pk.cu != nullptr) return false;
  if (c.loss_mode != MPZ_LOSS_LAST_POS_LABEL_SUBSET) return false;           // the whole-vocabulary scratch is shared
  if (c.weight_quant == MPZ_WEIGHT_QUANT_NF4) return false;                  // so is the dequantised-weight buffer
  if (((n / 2) * E * S) % 32) return false;
  const long T = (long)n * E * S;
  if (m->split_k && m->buf.splitk != nullptr && T / 2 <= 256) return false;  // so is the split-K partial-sum buffer
  const int nqkv = c.d_model + 2 * c.n_kv_heads * (c.d_model / c.n_heads);
  if ((long)((nqkv + 255) / 256) * ((T + 255) / 256) >= 512) return false;   // large problems fill the chip alone
  if (!m->stream2) {
    if (hipStreamCreateWithFlags(&m->stream2, hipStreamNonBlocking) != hipSuccess) { m->stream2 = nullptr; (void)hipGetLastError(); return false; }
    if (hipEventCreateWithFlags(&m->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m->ev_join, hipEventDisableTiming) != hipSuccess) {
      (void)hipGetLastError();
      m->two_halves = false;
      return false;
    }
  }
  return true;
}

void forward_two_halves(mpz_model* m, const int32_t* tokens, const int32_t* labels, int E, int S, float* losses_out) {
  const int n = 2 * m->q, half = n / 2;
  hipStream_t main = m->stream, streams[2] = {m->stream, m->stream2};
  (void)hipEventRecord(m->ev_fork, main);                   // the perturbed factors are ready on the caller's stream
  (void)hipStreamWaitEvent(m->stream2, m->ev_fork, 0);
  const size_t rows = (size_t)half * E * S;
  // With the other half's kernels filling a block's first-load and last-store edges, the 128 x 128 tile does better
  // with 4 waves of 64 x 64 (a third fewer LDS fragment reads) than with the 8 waves of 64 x 32 that hide those edges
  // when a GEMM runs alone: 2.44 -> 2.37 ms per step on the 125M-shaped workload, 2.62 -> 2.77 without the halves.
  const int saved_cfg = m->force_tile_cfg;
  if (saved_cfg == 0) m->force_tile_cfg = 1;
  for (int step = -1; step <= m->cfg.n_layers; ++step)       // embedding, the blocks one by one, the head
    for (int hf = 0; hf < 2; ++hf) {
      m->stream = streams[hf]; m->cb = hf * half; m->nc = half;
      float* h = m->buf.h + (size_t)hf * rows * m->cfg.d_model;
      if (step < 0) run_embed(m, tokens, E, S, h);
      else if (step < m->cfg.n_layers) run_layers(m, h, step, step + 1, E, S);
      else run_head(m, h, tokens, labels, E, S, losses_out + hf * half);
    }
  m->stream = main; m->cb = 0; m->nc = n;
  m->force_tile_cfg = saved_cfg;
  (void)hipEventRecord(m->ev_join, m->stream2);
  (void)hipStreamWaitEvent(main, m->ev_join, 0);
}

}  // namespace

namespace {
// Argument checks shared by every pass over E x S token batches: nothing is enqueued on a refused call.
mpz_status validate_pass(mpz_model* m, const char* who, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                         const float* losses_out) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, std::string(who) + ": NULL model");
  if (!tokens || !losses_out) return fail(m, MPZ_ERR_NULL, std::string(who) + ": NULL tokens or losses_out");
  if (m->cfg.loss_mode != MPZ_LOSS_NEXT_TOKEN_ALL_POS && !labels) return fail(m, MPZ_ERR_NULL, std::string(who) + ": this loss mode needs labels");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, std::string(who) + " before mpz_regen_noise");
  if (E < 1 || E > m->E_max || S < 2 || S > m->S_max) return fail(m, MPZ_ERR_SHAPE, std::string(who) + ": E or S outside what the model was initialised for");
  if (m->cfg.weight_quant == MPZ_WEIGHT_QUANT_INT8 && ((E * S) % 32 || !m->use_mfma))
    return fail(m, MPZ_ERR_SHAPE, std::string(who) + ": int8 weights: E*S must be a multiple of 32 (MFMA kernels only)");
  return MPZ_OK;
}
}  // namespace

mpz_status mpz_forward_perturbed(mpz_model* m, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                                 float* losses_out) {
  if (const mpz_status st = validate_pass(m, "mpz_forward_perturbed", tokens, labels, E, S, losses_out)) return st;
  m->cb = 0; m->nc = 2 * m->q;
  prepare_factors(m, E, S);
  if (use_two_halves(m, E, S)) {
    m->last_pass_streams = 2;
    forward_two_halves(m, tokens, labels, E, S, losses_out);
    return check_device(m, "mpz_forward_perturbed");
  }
  m->last_pass_streams = 1;
  run_embed(m, tokens, E, S, m->buf.h);
  run_layers(m, m->buf.h, 0, m->cfg.n_layers, E, S);
  run_head(m, m->buf.h, tokens, labels, E, S, losses_out);
  return check_device(m, "mpz_forward_perturbed");
}

mpz_status mpz_forward_perturbed_noalloc(mpz_model* m, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                                         float* losses_out) {
  if (const mpz_status st = validate_pass(m, "mpz_forward_perturbed_noalloc", tokens, labels, E, S, losses_out)) return st;
  if (m->prof_on) return fail(m, MPZ_ERR_STATE, "mpz_forward_perturbed_noalloc: not while per-launch timing is on (it creates events)");
  const int64_t n = 2 * (int64_t)m->q, rpc = ((int64_t)E * S + 31) / 32 * 32;
  size_t need;
  {
    Carver sizing(nullptr);
    Buffers none;
    carve_activations(&m->cfg, n, rpc, E, sizing, none);
    need = sizing.off;
  }
  if (need > MPZ_NOALLOC_SCRATCH_BYTES) {
    char msg[192];
    snprintf(msg, sizeof msg, "mpz_forward_perturbed_noalloc: this pass needs %zu bytes of activations, the static scratch "
             "holds %zu: use mpz_forward_perturbed with a workspace", need, (size_t)MPZ_NOALLOC_SCRATCH_BYTES);
    return fail(m, MPZ_ERR_WORKSPACE, msg);
  }
  int dev = -1;
  hipError_t e = hipSuccess;
  void* ptr = scratch_address(&dev, &e);
  if (ptr == nullptr) return fail(m, MPZ_ERR_DEVICE, std::string("mpz_forward_perturbed_noalloc: hipGetSymbolAddress: ") + hipGetErrorString(e));
  if (dev != m->device) return fail(m, MPZ_ERR_STATE, "mpz_forward_perturbed_noalloc: the current device is not the one the model was initialised on");
  const Buffers saved = m->buf;
  Carver cv(ptr);
  carve_activations(&m->cfg, n, rpc, E, cv, m->buf);       // the persistent pointers (factor copies, tables) stay
  prepare_factors(m, E, S);
  m->cb = 0; m->nc = 2 * m->q;
  m->last_pass_streams = 1;                                // one stream: the second stream of small models is created on demand
  run_embed(m, tokens, E, S, m->buf.h);
  run_layers(m, m->buf.h, 0, m->cfg.n_layers, E, S);
  run_head(m, m->buf.h, tokens, labels, E, S, losses_out);
  m->buf = saved;
  return check_device(m, "mpz_forward_perturbed_noalloc");
}

size_t mpz_noalloc_scratch_bytes(void) { return MPZ_NOALLOC_SCRATCH_BYTES; }

mpz_status mpz_forward_perturbed_varlen(mpz_model* m, const int32_t* tokens, const int32_t* labels, const int32_t* lengths,
                                        int32_t E, int32_t S, float* losses_out) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_forward_perturbed_varlen: NULL model");
  if (!lengths) return fail(m, MPZ_ERR_NULL, "mpz_forward_perturbed_varlen: NULL lengths");
  if ((size_t)2 * m->cfg.d_ffn * elem_size(m->cfg.dtype) < (size_t)4 * m->cfg.d_model)
    return fail(m, MPZ_ERR_SHAPE, "mpz_forward_perturbed_varlen: d_ffn too small to stage the last-token rows");
  m->lengths = lengths;
  const mpz_status st = mpz_forward_perturbed(m, tokens, labels, E, S, losses_out);
  m->lengths = nullptr;
  return st;
}

mpz_status mpz_forward_perturbed_packed(mpz_model* m, const int32_t* tokens, const int32_t* labels,
                                        const int32_t* cu_seqlens, int32_t E, int32_t total_tokens, int32_t max_len,
                                        float* losses_out) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_forward_perturbed_packed: NULL model");
  if (!tokens || !cu_seqlens || !losses_out) return fail(m, MPZ_ERR_NULL, "mpz_forward_perturbed_packed: NULL tokens, cu_seqlens or losses_out");
  if (m->cfg.loss_mode != MPZ_LOSS_NEXT_TOKEN_ALL_POS && !labels) return fail(m, MPZ_ERR_NULL, "this loss mode needs labels");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "mpz_forward_perturbed_packed before mpz_regen_noise");
  const int64_t rows = ((int64_t)total_tokens + 31) / 32 * 32;      // rows per copy: the MFMA kernels want whole 32-row tiles per copy
  if (E < 1 || max_len < 2 || max_len > m->S_max || total_tokens < (int64_t)2 * E || total_tokens > (int64_t)E * max_len)
    return fail(m, MPZ_ERR_SHAPE, "mpz_forward_perturbed_packed: need E >= 1, 2 <= max_len <= S_max, 2 E <= total_tokens <= E max_len");
  if (rows > ((int64_t)m->E_max * m->S_max + 31) / 32 * 32)
    return fail(m, MPZ_ERR_SHAPE, "mpz_forward_perturbed_packed: more rows per copy than E_max * S_max (rounded up to 32)");
  if ((size_t)2 * m->cfg.d_ffn * elem_size(m->cfg.dtype) < (size_t)4 * m->cfg.d_model && m->cfg.loss_mode != MPZ_LOSS_NEXT_TOKEN_ALL_POS)
    return fail(m, MPZ_ERR_SHAPE, "mpz_forward_perturbed_packed: d_ffn too small to stage the last-token rows");
  if ((int64_t)2 * m->q * E > (int64_t)2 * m->q_max * m->E_max && m->cfg.loss_mode != MPZ_LOSS_NEXT_TOKEN_ALL_POS)
    return fail(m, MPZ_ERR_SHAPE, "mpz_forward_perturbed_packed: more sequences than E_max");
  if (m->cfg.weight_quant == MPZ_WEIGHT_QUANT_INT8 && !m->use_mfma)
    return fail(m, MPZ_ERR_SHAPE, "int8 weights: MFMA kernels only");
  m->pk.cu = cu_seqlens; m->pk.E = E; m->pk.total = total_tokens; m->pk.max_len = max_len;
  launch_packed_index(m->stream, cu_seqlens, E, (int)rows, m->buf.row_pos, m->buf.row_end);
  prepare_factors(m, 1, (int)rows);
  m->cb = 0; m->nc = 2 * m->q;
  run_embed(m, tokens, 1, (int)rows, m->buf.h);
  run_layers(m, m->buf.h, 0, m->cfg.n_layers, 1, (int)rows);
  run_head(m, m->buf.h, tokens, labels, 1, (int)rows, losses_out);
  m->pk = mpz_model::Packed();
  return check_device(m, "mpz_forward_perturbed_packed");
}

mpz_status mpz_forward_copies(mpz_model* m, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                              int32_t copy_begin, int32_t n_copies, float* losses_out) {
  if (const mpz_status st = validate_pass(m, "mpz_forward_copies", tokens, labels, E, S, losses_out)) return st;
  if (copy_begin < 0 || n_copies < 1 || copy_begin + n_copies > 2 * m->q) return fail(m, MPZ_ERR_SHAPE, "copy range outside [0, 2q)");
  prepare_factors(m, E, S);
  m->cb = copy_begin; m->nc = n_copies;
  float* h = m->buf.h + (size_t)copy_begin * E * S * m->cfg.d_model;
  run_embed(m, tokens, E, S, h);
  run_layers(m, h, 0, m->cfg.n_layers, E, S);
  run_head(m, h, tokens, labels, E, S, losses_out + copy_begin);
  m->cb = 0; m->nc = 2 * m->q;
  return check_device(m, "mpz_forward_copies");
}

mpz_status mpz_forward_copies_strided(mpz_model* m, const int32_t* tokens, const int32_t* labels, int32_t E, int32_t S,
                                      int32_t copy_begin, int32_t n_copies, int32_t copy_step, float* losses_out) {
  if (const mpz_status st = validate_pass(m, "mpz_forward_copies_strided", tokens, labels, E, S, losses_out)) return st;
  if (copy_begin < 0 || n_copies < 1 || copy_step < 1 || copy_begin + (int64_t)(n_copies - 1) * copy_step >= 2 * m->q ||
      copy_begin + n_copies > 2 * m->q_max)
    return fail(m, MPZ_ERR_SHAPE, "copies outside [0, 2q)");
  prepare_factors(m, E, S);
  m->cb = copy_begin; m->nc = n_copies; m->cstep = copy_step;
  float* h = m->buf.h + (size_t)copy_begin * E * S * m->cfg.d_model;
  run_embed(m, tokens, E, S, h);
  run_layers(m, h, 0, m->cfg.n_layers, E, S);
  run_head(m, h, tokens, labels, E, S, losses_out + copy_begin);
  m->cb = 0; m->nc = 2 * m->q; m->cstep = 1;
  return check_device(m, "mpz_forward_copies_strided");
}

mpz_status mpz_debug_embed(mpz_model* m, const int32_t* tokens, int32_t E, int32_t S, float* h_out) {
  if (!m || !tokens || !h_out) return fail(m, MPZ_ERR_NULL, "mpz_debug_embed: NULL argument");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "mpz_debug_embed before mpz_regen_noise");
  if (E < 1 || E > m->E_max || S < 2 || S > m->S_max) return fail(m, MPZ_ERR_SHAPE, "E or S outside what the model was initialised for");
  run_embed(m, tokens, E, S, h_out);
  return check_device(m, "mpz_debug_embed");
}

mpz_status mpz_debug_run_layers(mpz_model* m, float* h, int32_t layer_begin, int32_t layer_end, int32_t E, int32_t S) {
  if (!m || !h) return fail(m, MPZ_ERR_NULL, "mpz_debug_run_layers: NULL argument");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "mpz_debug_run_layers before mpz_regen_noise");
  if (E < 1 || E > m->E_max || S < 2 || S > m->S_max) return fail(m, MPZ_ERR_SHAPE, "E or S outside what the model was initialised for");
  if (layer_begin < 0 || layer_end > m->cfg.n_layers || layer_begin > layer_end) return fail(m, MPZ_ERR_SHAPE, "layer range outside the model");
  prepare_factors(m, E, S);
  run_layers(m, h, layer_begin, layer_end, E, S);
  return check_device(m, "mpz_debug_run_layers");
}

mpz_status mpz_debug_head_loss(mpz_model* m, const float* h, const int32_t* tokens, const int32_t* labels,
                               const int32_t* lengths, int32_t E, int32_t S, float* losses_out) {
  if (!m || !h || !tokens || !losses_out) return fail(m, MPZ_ERR_NULL, "mpz_debug_head_loss: NULL argument");
  if (m->cfg.loss_mode != MPZ_LOSS_NEXT_TOKEN_ALL_POS && !labels) return fail(m, MPZ_ERR_NULL, "this loss mode needs labels");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "mpz_debug_head_loss before mpz_regen_noise");
  if (E < 1 || E > m->E_max || S < 2 || S > m->S_max) return fail(m, MPZ_ERR_SHAPE, "E or S outside what the model was initialised for");
  m->lengths = lengths;
  run_head(m, h, tokens, labels, E, S, losses_out);
  m->lengths = nullptr;
  return check_device(m, "mpz_debug_head_loss");
}

mpz_status mpz_zo_update(mpz_model* m, const float* losses, float lr, float* proj_grads_out) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_zo_update: NULL model");
  if (!losses) return fail(m, MPZ_ERR_NULL, "mpz_zo_update: NULL losses");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "mpz_zo_update before mpz_regen_noise");
  if (!(m->eps > 0.f)) return fail(m, MPZ_ERR_CONFIG, "the last mpz_regen_noise used eps = 0: the two-point quotient is undefined");
  if (!std::isfinite(lr)) return fail(m, MPZ_ERR_CONFIG, "lr must be finite");
  ProfScope ps(m, MPZ_PROF_UPDATE, 0.0, 8.0 * m->P);
  launch_update(m->stream, m->masters, m->P, m->tab, m->seed, m->step, m->q, m->eps, lr, m->cfg.perturb_A, losses,
                proj_grads_out);
  m->have_noise = false;                       // the perturbed copies no longer match the masters
  return check_device(m, "mpz_zo_update");
}

mpz_status mpz_zo_update_regen(mpz_model* m, const float* losses, float lr, uint32_t next_step, float* proj_grads_out) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_zo_update_regen: NULL model");
  if (!losses) return fail(m, MPZ_ERR_NULL, "mpz_zo_update_regen: NULL losses");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "mpz_zo_update_regen before mpz_regen_noise");
  if (!(m->eps > 0.f)) return fail(m, MPZ_ERR_CONFIG, "the stored pairs were made with eps = 0: the two-point quotient is undefined");
  if (!std::isfinite(lr)) return fail(m, MPZ_ERR_CONFIG, "lr must be finite");
  ensure_pert(m);                               // the stored pairs in fp32 (a stateful run keeps them from here on)
  {
    ProfScope ps(m, MPZ_PROF_UPDATE, 0.0, 8.0 * m->P * (1.0 + 2.0 * m->q));
    launch_update_regen(m->stream, m->masters, m->buf.pert, m->P, m->tab, m->seed, next_step, m->q, m->eps, lr,
                        m->cfg.perturb_A, losses, proj_grads_out);
  }
  ProfScope ps_pack(m, MPZ_PROF_PACK, 0.0, m->use_mfma ? 2.0 * m->q * (4.0 * m->P + 2.0 * m->packed_per_copy) : 0.0);
  if (m->use_mfma)
    launch_pack_factors(m->stream, m->buf.pert, m->P, 2 * m->q, m->tab, m->cfg.n_layers, m->cfg.lora_rank, m->rp,
                        m->buf.packed, m->packed_per_copy);
  m->step = next_step;                          // the stored copies now belong to next_step and match the masters
  m->cb = 0; m->nc = 2 * m->q;
  return check_device(m, "mpz_zo_update_regen");
}

mpz_status mpz_debug_noise_alu_probe(int64_t n_groups, int32_t q, float* sink, void* hip_stream) {
  if (!sink) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_noise_alu_probe: NULL sink");
  if (n_groups < 1 || n_groups > ((int64_t)1 << 31) || q < 1 || q > 64) return fail(nullptr, MPZ_ERR_SHAPE, "n_groups or q out of range");
  launch_noise_alu_probe((hipStream_t)hip_stream, n_groups, q, sink);
  return check_device(nullptr, "mpz_debug_noise_alu_probe");
}

mpz_status mpz_debug_noise(mpz_model* m, uint64_t seed, uint32_t step, int32_t k, int32_t tensor_id, float* z_out) {
  if (!m || !z_out) return fail(m, MPZ_ERR_NULL, "mpz_debug_noise: NULL argument");
  if (k < 0) return fail(m, MPZ_ERR_SHAPE, "k must be non-negative");
  for (const auto& t : m->tensors)
    if (t.tensor_id == tensor_id) {
      launch_debug_noise(m->stream, z_out, (int64_t)t.rows * t.cols, seed, step, k, tensor_id);
      return check_device(m, "mpz_debug_noise");
    }
  return fail(m, MPZ_ERR_SHAPE, "no LoRA factor with this tensor_id");
}

mpz_status mpz_debug_normals_from_words(const uint32_t* words, size_t n4, float* normals_out, void* hip_stream) {
  if (!words || !normals_out) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_normals_from_words: NULL argument");
  if (n4 == 0) return MPZ_OK;
  if (n4 > ((size_t)1 << 31)) return fail(nullptr, MPZ_ERR_SHAPE, "too many groups");
  launch_normals_from_words((hipStream_t)hip_stream, words, n4, normals_out);
  return check_device(nullptr, "mpz_debug_normals_from_words");
}

mpz_status mpz_debug_perturbed_copy(mpz_model* m, int32_t c, float* out) {
  if (!m || !out) return fail(m, MPZ_ERR_NULL, "mpz_debug_perturbed_copy: NULL argument");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "no perturbed copies: call mpz_regen_noise first");
  if (c < 0 || c >= 2 * m->q) return fail(m, MPZ_ERR_SHAPE, "copy index outside [0, 2q)");
  ensure_pert(m);
  hipError_t e = hipMemcpyAsync(out, m->buf.pert + (int64_t)c * m->P, (size_t)m->P * 4, hipMemcpyDeviceToDevice, m->stream);
  if (e != hipSuccess) return fail(m, MPZ_ERR_DEVICE, hipGetErrorString(e));
  return MPZ_OK;
}

mpz_status mpz_debug_qkv_projection(mpz_model* m, const void* x, int32_t layer, int32_t E, int32_t S, float* out) {
  if (!m || !x || !out) return fail(m, MPZ_ERR_NULL, "mpz_debug_qkv_projection: NULL argument");
  if (!m->have_noise) return fail(m, MPZ_ERR_STATE, "mpz_debug_qkv_projection before mpz_regen_noise");
  if (E < 1 || E > m->E_max || S < 2 || S > m->S_max) return fail(m, MPZ_ERR_SHAPE, "E or S outside what the model was initialised for");
  if (layer < 0 || layer >= m->cfg.n_layers) return fail(m, MPZ_ERR_SHAPE, "layer outside the model");
  if (m->cfg.dtype != MPZ_DTYPE_BF16) return fail(m, MPZ_ERR_CONFIG, "mpz_debug_qkv_projection is for bf16 models");
  prepare_factors(m, E, S);
  Buffers b = m->buf;
  b.x = const_cast<void*>(x);
  run_qkv(m, b, layer, E, S, false, 1, out);
  return check_device(m, "mpz_debug_qkv_projection");
}

mpz_status mpz_debug_attention(mpz_model* m, const void* qkv, int32_t n_seq, int32_t S, void* out) {
  if (!m || !qkv || !out) return fail(m, MPZ_ERR_NULL, "mpz_debug_attention: NULL argument");
  if (n_seq < 1 || S < 2) return fail(m, MPZ_ERR_SHAPE, "n_seq < 1 or S < 2");
  const mpz_config& c = m->cfg;
  const int d = c.d_model, dh = d / c.n_heads, nqkv = d + 2 * c.n_kv_heads * dh;
  if (m->use_mfma && attention_mfma_supported(dh, nqkv, d))
    launch_attention_mfma(m->stream, qkv, nqkv, out, n_seq, S, c.n_heads, c.n_kv_heads, dh, nullptr, 1, S);
  else
    launch_attention_simple(m->stream, c.dtype, qkv, nqkv, out, n_seq, S, c.n_heads, c.n_kv_heads, dh, nullptr, 1, S);
  return check_device(m, "mpz_debug_attention");
}

mpz_status mpz_debug_gemm_bf16(int32_t M, int32_t N, int32_t K, const void* x, const void* w, const float* bias,
                               int32_t act, void* out, int32_t out_f32, int32_t tile_cfg, void* hip_stream) {
  if (!x || !w || !out) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_gemm_bf16: NULL argument");
  MfmaGemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.x = x; g.w = w; g.w_rows = N; g.bias = bias; g.rows_per_copy = M; g.act = act;
  g.out_f32 = out_f32; g.out = out; g.ldo = N; g.tile_cfg = tile_cfg;
  if (act == MPZ_ACT_SWIGLU) { g.dual = 1; g.dual_offset = N; g.w_rows = 2 * N; g.act = -1; }
  if (!mfma_gemm_supported(g)) return fail(nullptr, MPZ_ERR_SHAPE, "shape not supported by the MFMA GEMM (K % 64, N % 4)");
  const hipError_t le = launch_gemm_mfma((hipStream_t)hip_stream, g);
  if (le != hipSuccess) return fail(nullptr, MPZ_ERR_DEVICE, std::string("mpz_debug_gemm_bf16: ") + hipGetErrorString(le));
  return check_device(nullptr, "mpz_debug_gemm_bf16");
}

mpz_status mpz_debug_gemm_bf16_splitk(int32_t M, int32_t N, int32_t K, const void* x, const void* w, const float* bias,
                                      int32_t act, const float* residual, void* out, int32_t out_f32, int32_t k_splits,
                                      float* partial, size_t partial_elems, void* hip_stream) {
  if (!x || !w || !out || !partial) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_gemm_bf16_splitk: NULL argument");
  const int forced_tile = k_splits / 1000;       // measurement: k_splits + 1000 x tile configuration
  k_splits %= 1000;
  if (k_splits < 0 || k_splits > 64) return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_gemm_bf16_splitk: k_splits outside [0, 64]");
  MfmaGemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.x = x; g.w = w; g.w_rows = N; g.bias = bias; g.rows_per_copy = M; g.act = act;
  g.residual = residual; g.out_f32 = out_f32; g.out = out; g.ldo = N; g.tile_cfg = 100 * k_splits;
  if (act == MPZ_ACT_SWIGLU) { g.dual = 1; g.dual_offset = N; g.w_rows = 2 * N; g.act = -1; }
  if (K % 64 || N % 4 || M < 1 || N < 1) return fail(nullptr, MPZ_ERR_SHAPE, "shape not supported by the MFMA GEMM (K % 64, N % 4)");
  const int ks = mfma_gemm_splits(g, partial_elems);
  if (k_splits >= 2 && ks != k_splits) return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_gemm_bf16_splitk: k_splits does not fit K or the partial buffer");
  g.tile_cfg = ks > 1 ? 100 * ks + forced_tile : 0;
  if (ks > 1) { g.k_splits = ks; g.partial = partial; g.ldp = (g.dual ? 2 : 1) * N; }
  if (!mfma_gemm_supported(g)) return fail(nullptr, MPZ_ERR_SHAPE, "shape not supported by the MFMA GEMM");
  const hipError_t le = launch_gemm_mfma((hipStream_t)hip_stream, g);
  if (le != hipSuccess) return fail(nullptr, MPZ_ERR_DEVICE, std::string("mpz_debug_gemm_bf16_splitk: ") + hipGetErrorString(le));
  if (check_device(nullptr, "mpz_debug_gemm_bf16_splitk") != MPZ_OK) return MPZ_ERR_DEVICE;
  return MPZ_OK;
}

mpz_status mpz_debug_gemm_nf4_splitk(int32_t M, int32_t N, int32_t K, const void* x, const void* w_codes, const float* w_absmax,
                                     const float* bias, int32_t act, const float* residual, void* out, int32_t out_f32,
                                     int32_t k_splits, float* partial, size_t partial_elems, void* hip_stream) {
  if (!x || !w_codes || !w_absmax || !out || !partial) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_gemm_nf4_splitk: NULL argument");
  if (k_splits < 2 || k_splits > 64) return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_gemm_nf4_splitk: k_splits outside [2, 64]");
  if (K % 64 || N % 4 || M < 1 || N < 1) return fail(nullptr, MPZ_ERR_SHAPE, "shape not supported by the MFMA GEMM (K % 64, N % 4)");
  MfmaGemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.x = x; g.w = w_codes; g.w_absmax = w_absmax; g.w_rows = N; g.bias = bias; g.rows_per_copy = M; g.act = act;
  g.residual = residual; g.out_f32 = out_f32; g.out = out; g.ldo = N; g.tile_cfg = 100 * k_splits;
  if (act == MPZ_ACT_SWIGLU) { g.dual = 1; g.dual_offset = N; g.w_rows = 2 * N; g.act = -1; }
  if (mfma_gemm_splits(g, partial_elems) != k_splits)
    return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_gemm_nf4_splitk: k_splits does not fit K or the partial buffer");
  g.k_splits = k_splits; g.partial = partial; g.ldp = (g.dual ? 2 : 1) * N;
  if (!mfma_gemm_supported(g)) return fail(nullptr, MPZ_ERR_SHAPE, "shape or alignment not supported by the MFMA GEMM");
  const hipError_t le = launch_gemm_mfma((hipStream_t)hip_stream, g);
  if (le != hipSuccess) return fail(nullptr, MPZ_ERR_DEVICE, std::string("mpz_debug_gemm_nf4_splitk: ") + hipGetErrorString(le));
  return check_device(nullptr, "mpz_debug_gemm_nf4_splitk");
}

int32_t mpz_debug_gemm_splits(int32_t M, int32_t N, int32_t K, int32_t dual, size_t partial_elems) {
  MfmaGemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.dual = dual != 0; g.dual_offset = dual ? N : 0;
  return mfma_gemm_splits(g, partial_elems);
}

mpz_status mpz_debug_gemm_int8(int32_t M, int32_t N, int32_t K, const void* x, const void* w_codes, const float* w_scale,
                               const float* bias, int32_t act, void* out, int32_t out_f32, int32_t tile_cfg,
                               void* hip_stream) {
  if (!x || !w_codes || !w_scale || !out) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_gemm_int8: NULL argument");
  MfmaGemmArgs g{};
  g.M = M; g.N = N; g.K = K; g.x = x; g.w = w_codes; g.w_scale = w_scale; g.w_rows = N; g.bias = bias; g.rows_per_copy = M;
  g.act = act; g.out_f32 = out_f32; g.out = out; g.ldo = N; g.tile_cfg = tile_cfg;
  if (act == MPZ_ACT_SWIGLU) { g.dual = 1; g.dual_offset = N; g.w_rows = 2 * N; g.act = -1; }
  if (!mfma_gemm_supported(g)) return fail(nullptr, MPZ_ERR_SHAPE, "shape not supported by the MFMA GEMM (K % 64, N % 4, scale alignment)");
  const hipError_t le = launch_gemm_mfma((hipStream_t)hip_stream, g);
  if (le != hipSuccess) return fail(nullptr, MPZ_ERR_DEVICE, std::string("mpz_debug_gemm_int8: ") + hipGetErrorString(le));
  return check_device(nullptr, "mpz_debug_gemm_int8");
}

mpz_status mpz_debug_set_two_halves(mpz_model* m, int32_t enable) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_set_two_halves: NULL model");
  m->two_halves = enable != 0;
  return MPZ_OK;
}

int32_t mpz_debug_last_pass_streams(const mpz_model* m) { return m ? m->last_pass_streams : 0; }

mpz_status mpz_debug_mfma_probe(const void* operands, int32_t blocks, int32_t iters, int32_t with_lds, float* out,
                                void* hip_stream) {
  if (!operands || !out) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_mfma_probe: NULL argument");
  if (blocks < 1 || blocks > 65536 || iters < 1 || iters > (1 << 24)) return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_mfma_probe: blocks or iters out of range");
  if (((uintptr_t)operands & 15u) != 0) return fail(nullptr, MPZ_ERR_CONFIG, "mpz_debug_mfma_probe: operands must be 16-byte aligned");
  if (with_lds < 0 || with_lds > 2) return fail(nullptr, MPZ_ERR_CONFIG, "mpz_debug_mfma_probe: with_lds outside [0, 2]");
  launch_mfma_probe((hipStream_t)hip_stream, operands, blocks, iters, with_lds, out);
  return hipGetLastError() == hipSuccess ? MPZ_OK : fail(nullptr, MPZ_ERR_DEVICE, "mpz_debug_mfma_probe: launch failed");
}

mpz_status mpz_debug_hbm_read_probe(const void* buf, int64_t rows, int64_t row_bytes, int32_t rows_per_block, int32_t seg_bytes,
                                    int32_t k_splits, int32_t lds_bytes, int32_t mode, uint32_t* out, void* hip_stream) {
  if (!buf || !out) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_hbm_read_probe: NULL argument");
  if (((uintptr_t)buf & 15u) != 0) return fail(nullptr, MPZ_ERR_CONFIG, "mpz_debug_hbm_read_probe: buf must be 16-byte aligned");
  // every access of the kernel stays inside [rows][row_bytes]: whole row blocks, whole tiles, whole splits
  if (rows < 1 || row_bytes < 16 || rows_per_block < 1 || seg_bytes < 16 || seg_bytes % 16 || k_splits < 1 || k_splits > 65535 ||
      rows % rows_per_block || row_bytes % ((int64_t)seg_bytes * k_splits) || rows / rows_per_block > 0x7fffffff ||
      (int64_t)rows_per_block * seg_bytes % 4096 || lds_bytes < 0 || lds_bytes > 160 * 1024)
    return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_hbm_read_probe: rows % rows_per_block, row_bytes % (seg_bytes * k_splits), "
                                        "rows_per_block * seg_bytes % 4096 must be 0; lds_bytes in [0, 160 KiB]");
  const int64_t L = (int64_t)rows_per_block * seg_bytes / 4096;
  if (L != 1 && L != 2 && L != 4 && L != 8 && L != 16)
    return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_hbm_read_probe: rows_per_block * seg_bytes must be 4, 8, 16, 32 or 64 KiB");
  if (mode < 0 || mode > 3) return fail(nullptr, MPZ_ERR_CONFIG, "mpz_debug_hbm_read_probe: mode outside [0, 3]");
  if ((mode & 2) && (int64_t)lds_bytes < ((mode & 1) ? 2 : 1) * (int64_t)rows_per_block * seg_bytes)
    return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_hbm_read_probe: mode bit 1 needs lds_bytes >= the bytes of the tiles it stages");
  const hipError_t e = launch_hbm_read_probe((hipStream_t)hip_stream, buf, rows, row_bytes, rows_per_block, seg_bytes, k_splits,
                                             lds_bytes, mode, out);
  if (e != hipSuccess) return fail(nullptr, MPZ_ERR_DEVICE, std::string("mpz_debug_hbm_read_probe: ") + hipGetErrorString(e));
  return hipGetLastError() == hipSuccess ? MPZ_OK : fail(nullptr, MPZ_ERR_DEVICE, "mpz_debug_hbm_read_probe: launch failed");
}

mpz_status mpz_debug_dequant_nf4(const void* codes, const float* absmax, void* out, int64_t n_elems, void* hip_stream) {
  if (!codes || !absmax || !out) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_dequant_nf4: NULL argument");
  if (n_elems < 64 || n_elems % 64) return fail(nullptr, MPZ_ERR_SHAPE, "mpz_debug_dequant_nf4: n_elems must be a positive multiple of 64");
  if ((((uintptr_t)codes | (uintptr_t)absmax) & 3u) || ((uintptr_t)out & 15u))
    return fail(nullptr, MPZ_ERR_CONFIG, "mpz_debug_dequant_nf4: codes / absmax 4-byte, out 16-byte aligned");
  launch_nf4_dequant((hipStream_t)hip_stream, codes, absmax, out, n_elems);
  return hipGetLastError() == hipSuccess ? MPZ_OK : fail(nullptr, MPZ_ERR_DEVICE, "mpz_debug_dequant_nf4: launch failed");
}

mpz_status mpz_debug_set_fused_norm_lora(mpz_model* m, int32_t enable) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_set_fused_norm_lora: NULL model");
  m->fuse_norm_lora = enable != 0;
  return MPZ_OK;
}

mpz_status mpz_debug_set_split_k(mpz_model* m, int32_t enable) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_set_split_k: NULL model");
  m->split_k = enable != 0;
  return MPZ_OK;
}

mpz_status mpz_debug_set_fused_perturb_pack(mpz_model* m, int32_t enable) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_set_fused_perturb_pack: NULL model");
  m->fuse_perturb_pack = enable != 0;
  m->have_noise = false;
  return MPZ_OK;
}

mpz_status mpz_debug_set_tile_config(mpz_model* m, int32_t tile_cfg) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_set_tile_config: NULL model");
  if (!(tile_cfg == 0 || tile_cfg == 1 || tile_cfg == 6 || (tile_cfg >= 9 && tile_cfg <= 12)))
    return fail(m, MPZ_ERR_CONFIG, "tile configuration must be 0 (by shape), 1, 6, 9, 10, 11 or 12");
  m->force_tile_cfg = tile_cfg;
  return MPZ_OK;
}

mpz_status mpz_debug_set_kernel_path(mpz_model* m, int32_t simple_only) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_debug_set_kernel_path: NULL model");
  m->use_mfma = !simple_only && m->cfg.dtype == MPZ_DTYPE_BF16;
  m->have_noise = false;                       // operand layouts differ between the paths: regenerate
  return MPZ_OK;
}

mpz_status mpz_profile_begin(mpz_model* m) {
  if (!m) return fail(nullptr, MPZ_ERR_NULL, "mpz_profile_begin: NULL model");
  m->prof_on = true; m->prof_used = 0;
  for (int i = 0; i < MPZ_PROF_COUNT; ++i) m->prof_flops[i] = m->prof_bytes[i] = 0.0;
  return MPZ_OK;
}

mpz_status mpz_profile_end(mpz_model* m, mpz_profile_entry* out) {
  if (!m || !out) return fail(m, MPZ_ERR_NULL, "mpz_profile_end: NULL argument");
  if (!m->prof_on) return fail(m, MPZ_ERR_STATE, "mpz_profile_end without mpz_profile_begin");
  m->prof_on = false;
  if (hipStreamSynchronize(m->stream) != hipSuccess) return fail(m, MPZ_ERR_DEVICE, "stream synchronisation failed");
  for (int i = 0; i < MPZ_PROF_COUNT; ++i) { out[i].ms = 0.0; out[i].launches = 0; out[i].flops = m->prof_flops[i]; out[i].bytes = m->prof_bytes[i]; }
  for (size_t i = 0; i + 1 < m->prof_used; i += 2) {
    float t = 0.f;
    if (hipEventElapsedTime(&t, m->prof_ev[i], m->prof_ev[i + 1]) != hipSuccess) return fail(m, MPZ_ERR_DEVICE, "hipEventElapsedTime failed");
    const int cat = m->prof_cat[i / 2];
    out[cat].ms += t; out[cat].launches += 1;
  }
  return MPZ_OK;
}

void mpz_destroy(mpz_model* m) { delete m; }

const char* mpz_last_error(const mpz_model* m) { return m ? m->err.c_str() : g_last_error.c_str(); }

const char* mpz_status_string(mpz_status s) {
  switch (s) {
    case MPZ_OK: return "MPZ_OK";
    case MPZ_ERR_NULL: return "MPZ_ERR_NULL";
    case MPZ_ERR_CONFIG: return "MPZ_ERR_CONFIG";
    case MPZ_ERR_SHAPE: return "MPZ_ERR_SHAPE";
    case MPZ_ERR_WORKSPACE: return "MPZ_ERR_WORKSPACE";
    case MPZ_ERR_STATE: return "MPZ_ERR_STATE";
    case MPZ_ERR_DEVICE: return "MPZ_ERR_DEVICE";
  }
  return "MPZ_ERR_UNKNOWN";
}

}  // extern "C"
