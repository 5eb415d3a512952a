// Host side of the HiFT step library: parameter layout, layer units, groups and visiting
// order, the step itself (forward over all units, backward truncated at the lowest unit of
// the active group, weight gradients and optimizer update for that group only) and the
// movement of the group's optimizer state between pinned host memory and HBM on side streams.
// Implements the C ABI declared in include/hift.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/hift.h"
#include "kernels.h"

using namespace hift;

namespace {

thread_local std::string g_err;

hift_status fail(hift_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return s;
}

#define HIP_TRY(expr)                                                                         \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return fail(HIFT_EDEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

// ------------------------------------------------------------------------------------------
// layout (appendix "Implementation Details": embeddings = one unit, each hidden layer = one
// unit, all head parameters = one unit)
// ------------------------------------------------------------------------------------------
struct Tensor {
  std::string name;
  int unit, kind;
  int64_t off, rows, cols;
  // byte offsets of the copies in MFMA fragment order inside the packed-weight arena, or -1:
  // pk_fwd packs w as [rows, cols] (forward, y = x . w^T), pk_bwd packs w^T (dX = dY . w)
  int64_t pk_fwd = -1, pk_bwd = -1;
  int pk_order = PK_ORDER_PLAIN;  // block order of the forward copy (which fused epilogue it is made for)
  // index of the normalisation gain folded into the forward copy, or -1: the layer then multiplies the rows
  // as they are before the normalisation, and the kernel scales by their 1 / rms (see Gemm::rowsq)
  int pk_gain = -1;
  // position in the bf16 copy of the model (elements), or -1: a matrix that has both fragment-order copies keeps no
  // row-major bf16 copy; what would read it reads the copies (contractions) or the fp32 master (re-packing)
  int64_t wc_off = -1;
  int64_t fac_off = 0;  // Adafactor: first float of this tensor's statistics ([rows | cols], or [rows] for vectors)
  int64_t fac_count() const { return cols > 1 ? rows + cols : rows; }
  int64_t count() const { return rows * cols; }
};

struct Layout {
  std::vector<Tensor> t;
  std::vector<int64_t> unit_off, unit_cnt;
  std::vector<int> unit_first;  // first tensor index of each unit (+ sentinel)
  int64_t n_params = 0;
  int n_units = 0;
  int find(const std::string& name) const {
    for (size_t i = 0; i < t.size(); ++i)
      if (t[i].name == name) return (int)i;
    return -1;
  }
};

hift_status check_config(const hift_config* c) {
  if (!c) return fail(HIFT_EINVAL, "config is null");
  if (c->arch < 0 || c->arch > 2) return fail(HIFT_EINVAL, "arch %d unknown", c->arch);
  if (c->n_layers < 1 || c->d_model < 2 || c->n_heads < 1 || c->d_ffn < 1 || c->vocab < 1 || c->max_seq < 1)
    return fail(HIFT_EINVAL, "sizes must be positive");
  if (c->d_model % c->n_heads != 0) return fail(HIFT_EINVAL, "d_model must be a multiple of n_heads");
  if (c->arch == HIFT_ARCH_RMS_ROPE_DECODER && (c->d_model / c->n_heads) % 2 != 0)
    return fail(HIFT_EINVAL, "head width must be even for rotary positions");
  if (c->arch == HIFT_ARCH_POSTLN_ENCODER && c->n_classes < 1) return fail(HIFT_EINVAL, "n_classes must be >= 1");
  if (c->dtype != HIFT_F32 && c->dtype != HIFT_BF16) return fail(HIFT_EINVAL, "dtype unknown");
  if (c->tie_embeddings && c->arch == HIFT_ARCH_POSTLN_ENCODER)
    return fail(HIFT_EINVAL, "tie_embeddings applies to the decoders (the encoder's head is a classifier)");
  if (!(c->norm_eps >= 0.f)) return fail(HIFT_EINVAL, "norm_eps must be >= 0");
  if (c->unfused & ~(HIFT_UNFUSED_EPILOGUES | HIFT_UNFUSED_ATTENTION | HIFT_UNFUSED_NORM | HIFT_UNSHARED_LAST_ROUND))
    return fail(HIFT_EINVAL, "unfused has unknown bits set (%d)", c->unfused);
  if (c->lora_rank < 0 || (c->lora_rank > 0 && !(c->lora_alpha > 0.f))) return fail(HIFT_EINVAL, "lora_rank must be >= 0 and lora_alpha > 0");
  if (c->lora_rank > 0 && c->dtype == HIFT_BF16 && c->lora_rank % 8 != 0)
    return fail(HIFT_EINVAL, "lora_rank must be a multiple of 8 in bf16 mode (16-byte pieces of the adapter operands)");
  if (c->master_on_host && (c->dtype != HIFT_BF16 || !c->state_on_host))
    return fail(HIFT_EINVAL, "master_on_host needs dtype bf16 (the forward copy stays in HBM) and state_on_host");
  return HIFT_OK;
}

void build_layout(const hift_config& c, Layout& L) {
  const int64_t d = c.d_model, f = c.d_ffn, V = c.vocab;
  const int nl = c.n_layers;
  int64_t off = 0;
  auto add = [&](const std::string& n, int unit, int kind, int64_t r, int64_t cl) {
    L.t.push_back(Tensor{n, unit, kind, off, r, cl});
    off += r * cl;
  };
  const int M = HIFT_KIND_MATRIX, G = HIFT_KIND_GAIN, Bk = HIFT_KIND_BIAS;
  if (c.arch == HIFT_ARCH_PRELN_DECODER) {
    add("tok_emb", 0, M, V, d);
    add("pos_emb", 0, M, c.max_seq, d);
    for (int l = 0; l < nl; ++l) {
      const std::string p = "l" + std::to_string(l) + ".";
      const int u = l + 1;
      add(p + "ln1_g", u, G, d, 1); add(p + "ln1_b", u, Bk, d, 1);
      add(p + "wqkv", u, M, 3 * d, d); add(p + "bqkv", u, Bk, 3 * d, 1);
      add(p + "wo", u, M, d, d); add(p + "bo", u, Bk, d, 1);
      add(p + "ln2_g", u, G, d, 1); add(p + "ln2_b", u, Bk, d, 1);
      add(p + "w1", u, M, f, d); add(p + "b1", u, Bk, f, 1);
      add(p + "w2", u, M, d, f); add(p + "b2", u, Bk, d, 1);
    }
    add("lnf_g", nl + 1, G, d, 1); add("lnf_b", nl + 1, Bk, d, 1);
    if (!c.tie_embeddings) add("whead", nl + 1, M, V, d);
  } else if (c.arch == HIFT_ARCH_POSTLN_ENCODER) {
    add("tok_emb", 0, M, V, d);
    add("pos_emb", 0, M, c.max_seq, d);
    add("lne_g", 0, G, d, 1); add("lne_b", 0, Bk, d, 1);
    for (int l = 0; l < nl; ++l) {
      const std::string p = "l" + std::to_string(l) + ".";
      const int u = l + 1;
      add(p + "wqkv", u, M, 3 * d, d); add(p + "bqkv", u, Bk, 3 * d, 1);
      add(p + "wo", u, M, d, d); add(p + "bo", u, Bk, d, 1);
      add(p + "ln1_g", u, G, d, 1); add(p + "ln1_b", u, Bk, d, 1);
      add(p + "w1", u, M, f, d); add(p + "b1", u, Bk, f, 1);
      add(p + "w2", u, M, d, f); add(p + "b2", u, Bk, d, 1);
      add(p + "ln2_g", u, G, d, 1); add(p + "ln2_b", u, Bk, d, 1);
    }
    add("wc", nl + 1, M, c.n_classes, d);
    add("bc", nl + 1, Bk, c.n_classes, 1);
  } else {
    add("tok_emb", 0, M, V, d);
    for (int l = 0; l < nl; ++l) {
      const std::string p = "l" + std::to_string(l) + ".";
      const int u = l + 1;
      add(p + "g1", u, G, d, 1);
      add(p + "wqkv", u, M, 3 * d, d);
      add(p + "wo", u, M, d, d);
      add(p + "g2", u, G, d, 1);
      add(p + "wgu", u, M, 2 * f, d);
      add(p + "wd", u, M, d, f);
    }
    add("gf", nl + 1, G, d, 1);
    if (!c.tie_embeddings) add("whead", nl + 1, M, V, d);
  }
  L.n_units = nl + 2;
  L.n_params = off;
  L.unit_off.assign(L.n_units, 0);
  L.unit_cnt.assign(L.n_units, 0);
  L.unit_first.assign(L.n_units + 1, (int)L.t.size());
  for (int i = (int)L.t.size() - 1; i >= 0; --i) {
    L.unit_first[L.t[i].unit] = i;
    L.unit_off[L.t[i].unit] = L.t[i].off;
    L.unit_cnt[L.t[i].unit] += L.t[i].count();
  }
}

int group_count(int n, int m) { return n % m == 0 ? n / m : n / m + 1; }

uint64_t splitmix64(uint64_t& s) {
  s += 0x9E3779B97F4A7C15ull;
  uint64_t z = s;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

void make_order(int k, int strategy, uint64_t seed, int32_t* out) {
  for (int i = 0; i < k; ++i) out[i] = strategy == HIFT_TOP2DOWN ? k - 1 - i : i;
  if (strategy == HIFT_RANDOM) {
    uint64_t s = seed;
    for (int i = k - 1; i > 0; --i) {
      const int j = (int)(splitmix64(s) % (uint64_t)(i + 1));
      std::swap(out[i], out[j]);
    }
  }
}

int n_state_of(const hift_opt& o) {
  if (o.kind == HIFT_ADAMW) return 2;
  if (o.kind == HIFT_ADAGRAD) return 1;
  if (o.kind == HIFT_ADAFACTOR) return 0;  // factored statistics: a few numbers per row and column, kept in HBM
  return o.momentum > 0.0 ? 1 : 0;
}

hift_status check_opt(const hift_opt* o) {
  if (!o) return fail(HIFT_EINVAL, "optimizer is null");
  if (o->kind < 0 || o->kind > 3) return fail(HIFT_EINVAL, "optimizer kind %d unknown", o->kind);
  if (o->momentum < 0.0) return fail(HIFT_EINVAL, "momentum must be >= 0");
  return HIFT_OK;
}

inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

// Bump allocator over the caller's arena.  With base == nullptr it only measures.
// categories of device memory, for the memory report
enum { MEM_MASTER = 0, MEM_FORWARD = 1, MEM_PACKED = 2, MEM_GRAD = 3, MEM_STATE = 4, MEM_ACT = 5, MEM_WORK = 6, MEM_N = 7 };

struct Bump {
  unsigned char* base;
  size_t used = 0;
  size_t by_cat[MEM_N] = {0, 0, 0, 0, 0, 0, 0};
  int cat = MEM_WORK;
  explicit Bump(void* b) : base(reinterpret_cast<unsigned char*>(b)) {}
  void* take(size_t bytes) {
    void* p = base ? base + used : nullptr;
    used += up256(bytes);
    by_cat[cat] += up256(bytes);
    return p;
  }
};

struct LayerAct {
  void *na, *qkv, *ctx, *xmid, *nb, *fpre, *act;  // na: h1 | s1, nb: h2 | s2
  float *st1, *st2;
  float* lse;  // fused attention: log2 of each row's sum of exponentials, [B, H, S]
};

struct Prof {
  bool on = false;
  struct Rec { hipEvent_t a, b; int cat, sub; double work; };
  std::vector<Rec> pool;
  size_t used = 0;
};

// The pinned host arena as the caller hands it in: one block, or several chunks (a host may grant page-locked memory
// only in pieces smaller than the whole).  The library addresses it as one range of bytes -- [master (if it lives on
// the host)][state 0][state 1], each n_params floats -- and splits every access where a chunk ends.
struct PinnedSpace {
  struct Chunk { unsigned char* base; size_t bytes, start; };
  std::vector<Chunk> chunks;  // in address order of the logical range
  size_t total = 0;
  void add(void* p, size_t bytes) {
    chunks.push_back(Chunk{reinterpret_cast<unsigned char*>(p), bytes, total});
    total += bytes;
  }
  // fn(host pointer, bytes, offset within the request) for every piece of [off, off + bytes), in order
  template <class F>
  hift_status pieces(size_t off, size_t bytes, F fn) const {
    size_t done = 0;
    for (const Chunk& c : chunks) {
      if (done == bytes) break;
      const size_t lo = off + done;
      if (lo < c.start || lo >= c.start + c.bytes) continue;
      const size_t n = std::min(bytes - done, c.start + c.bytes - lo);
      const hift_status s = fn(c.base + (lo - c.start), n, done);
      if (s != HIFT_OK) return s;
      done += n;
    }
    return done == bytes ? HIFT_OK : fail(HIFT_ESTATE, "access outside the pinned arena");
  }
  hift_status read(void* dst, size_t off, size_t bytes) const {
    return pieces(off, bytes, [&](unsigned char* p, size_t n, size_t at) {
      memcpy(reinterpret_cast<unsigned char*>(dst) + at, p, n);
      return HIFT_OK;
    });
  }
  hift_status write(size_t off, const void* src, size_t bytes) const {
    return pieces(off, bytes, [&](unsigned char* p, size_t n, size_t at) {
      memcpy(p, reinterpret_cast<const unsigned char*>(src) + at, n);
      return HIFT_OK;
    });
  }
};

}  // namespace

constexpr int NSLOT = 3;

struct hift_model {
  hift_config cfg;
  hift_opt opt;
  Layout lay;
  int dt, es;  // element type of weights/activations, its size
  int max_batch, max_seq_len;
  int64_t maxT;
  int64_t grad_cap;  // parameters the gradient buffer and one state slot can hold
  int n_state;
  bool on_host;
  bool master_host;  // fp32 master of inactive groups in pinned memory, travelling with the state
  int n_move;        // arrays per parameter that a slot holds: optimizer state (+ master)
  // device memory
  float* master = nullptr;
  void* wc = nullptr;  // weights the forward uses: bf16 copy, or the master itself in fp32 mode
  unsigned char* wpk = nullptr;  // copies of the large bf16 matrices in MFMA fragment order
  size_t wpk_bytes = 0;
  void* gemm_ws = nullptr;
  float* rowsq = nullptr;  // [maxT, d / 64] partial sums of squares of the rows a folded normalisation takes
  float* fac = nullptr;      // Adafactor statistics of every tensor (resident: they are tiny)
  float* af_work = nullptr;  // Adafactor reduction scratch
  int64_t n_fac = 0;
  size_t af_work_floats = 0;
  float* grad = nullptr;
  float* state_full = nullptr;  // [n_state][n_params] when state stays in HBM
  // State of the active group when the rest lives on the host: [n_state][grad_cap] each.  Three slots:
  // while one is updated, the next group's state arrives in the second and the previous group's
  // drains from the third, so the two directions of the host link run at the same time.
  float* slot[NSLOT] = {nullptr, nullptr, nullptr};
  PinnedSpace pin;                      // [master (when it lives on the host)][n_state][n_params] floats
  size_t host_state_off = 0;            // byte offset of the state arrays in `pin` (the master, if there, comes first)
  float* cos_sin = nullptr;
  // low-rank adapters on the query and value projections (cfg.lora_rank > 0).  Per layer, r = rank: A_q | A_v stacked
  // [2r, d], then B_q [d, r], B_v [d, r]; all layers one after the other.  fp32 master, copy in the compute type,
  // gradient and AdamW moments, all resident (4 r d values per layer).
  int lora_r = 0;
  int64_t n_lora = 0;
  float *lora_master = nullptr, *lora_grad = nullptr, *lora_m = nullptr, *lora_v = nullptr;
  void* lora_wc = nullptr;
  std::vector<void*> lora_u;  // per layer: s (h A_q^T | h A_v^T), [T, 2r], kept for the backward pass
  void* lora_du = nullptr;    // [T, 2r]
  int64_t lora_t = 0;         // adapter updates so far
  std::vector<void*> xs;  // residual stream: xs[l] enters layer l, xs[L] enters the head
  std::vector<LayerAct> la;
  void *e0 = nullptr, *xf = nullptr, *xcls = nullptr, *logits = nullptr;
  float *st_e = nullptr, *st_f = nullptr, *row_loss = nullptr, *loss_dev = nullptr, *part = nullptr;
  void *D[3] = {nullptr, nullptr, nullptr}, *dqkv = nullptr, *prob = nullptr, *dprob = nullptr, *attn_dsum = nullptr, *dact = nullptr, *dffn = nullptr,
       *dcls = nullptr;
  // streams and events
  hipStream_t cs, hs, ds;
  hipEvent_t ev_h2d[NSLOT], ev_opt[NSLOT], ev_d2h[NSLOT], ev_t0, ev_t1, ev_w0, ev_w1;
  bool d2h_pending[NSLOT] = {false, false, false};
  int h2d_last = -1;            // slot of the most recent host-to-device transfer
  int d2h_group[NSLOT] = {-1, -1, -1};  // group whose state the pending write-back of a slot carries
  int slot_group[NSLOT] = {-1, -1, -1};  // group whose state a slot holds (arrived or in flight)
  int cur_slot = 0;
  // schedule
  int m = 0, k = 0;
  std::vector<int32_t> order;
  // updates each unit has had; drives AdamW's bias correction, Adafactor's decay and SGD's first-buffer rule.
  // Kept per unit, not per group, so that it stays right when the grouping changes while the state is kept.
  std::vector<int64_t> unit_steps;
  int64_t t = 0;
  // learning-rate schedule evaluated at the cycle index (used by hift_train)
  int lr_kind = -1;  // -1: none set, the rate is whatever hift_set_lr left
  double lr_base = 0.0;
  int64_t lr_warmup = 0, lr_total = 0;
  uint64_t h2d_bytes = 0, d2h_bytes = 0;
  bool timed = false;
  int copy_engine = 0;   // 0: hipMemcpyAsync, 1: small-grid copy kernel
  int copy_blocks = 16;
  Prof prof;

  int64_t wc_count = 0;  // elements of the bf16 copy
  const Tensor& T_(const std::string& n) const { return lay.t[lay.find(n)]; }
  // the tensor as the forward pass reads it (null for a matrix that lives only in its fragment-order copies)
  void* W(const Tensor& t) const {
    if (dt != DT_BF16) return reinterpret_cast<unsigned char*>(wc) + t.off * es;
    return t.wc_off >= 0 ? reinterpret_cast<unsigned char*>(wc) + t.wc_off * 2 : nullptr;
  }
  void* W(const std::string& n) const { return W(T_(n)); }
};

namespace {

// Carves every buffer of a model out of the arenas (or only measures them when arena == null).
void carve(hift_model* mm, void* dev, size_t* dev_bytes, size_t* pinned_bytes, size_t* by_cat = nullptr) {
  hift_model& M = *mm;
  const hift_config& c = M.cfg;
  const int64_t d = c.d_model, f = c.d_ffn, V = c.vocab, H = c.n_heads;
  const int64_t T = M.maxT, B = M.max_batch, S = M.max_seq_len;
  const int64_t np = M.lay.n_params;
  const size_t es = M.es;
  const bool enc = c.arch == HIFT_ARCH_POSTLN_ENCODER, rms = c.arch == HIFT_ARCH_RMS_ROPE_DECODER;
  const int64_t fw = rms ? 2 * f : f;
  Bump b(dev);
  b.cat = MEM_MASTER;
  M.master = M.master_host ? nullptr : (float*)b.take(np * 4);
  b.cat = MEM_FORWARD;
  M.wc = M.dt == DT_BF16 ? b.take((size_t)M.wc_count * 2) : (void*)M.master;
  b.cat = MEM_PACKED;
  M.wpk = M.wpk_bytes ? (unsigned char*)b.take(M.wpk_bytes) : nullptr;
  b.cat = MEM_GRAD;
  M.grad = (float*)b.take(M.grad_cap * 4);
  if (M.n_move > 0 && M.on_host) {
    // a slot holds [master (if it travels)][state 0][state 1] of one group
    for (auto& sl : M.slot) {
      b.cat = MEM_MASTER;
      sl = M.master_host ? (float*)b.take((size_t)M.grad_cap * 4) : nullptr;
      b.cat = MEM_STATE;
      float* st = M.n_state > 0 ? (float*)b.take((size_t)M.n_state * M.grad_cap * 4) : nullptr;
      if (!sl) sl = st;
    }
  } else if (M.n_state > 0) {
    b.cat = MEM_STATE;
    M.state_full = (float*)b.take((size_t)M.n_state * np * 4);
  }
  if (M.n_fac > 0) {
    b.cat = MEM_STATE;
    M.fac = (float*)b.take((size_t)M.n_fac * 4);
    b.cat = MEM_WORK;
    M.af_work = (float*)b.take(M.af_work_floats * 4);
  }
  if (M.lora_r > 0) {
    const size_t nl = (size_t)M.n_lora;
    b.cat = MEM_MASTER;
    M.lora_master = (float*)b.take(nl * 4);
    b.cat = MEM_FORWARD;
    M.lora_wc = M.dt == DT_BF16 ? b.take(nl * 2) : (void*)M.lora_master;
    b.cat = MEM_GRAD;
    M.lora_grad = (float*)b.take(nl * 4);
    b.cat = MEM_STATE;
    M.lora_m = (float*)b.take(nl * 4);
    M.lora_v = (float*)b.take(nl * 4);
    b.cat = MEM_ACT;
    M.lora_u.assign(c.n_layers, nullptr);
    for (auto& u : M.lora_u) u = b.take(T * 2 * M.lora_r * es);
    b.cat = MEM_WORK;
    M.lora_du = b.take(T * 2 * M.lora_r * es);
  }
  b.cat = MEM_WORK;
  if (rms) M.cos_sin = (float*)b.take((size_t)c.max_seq * (d / H / 2) * 2 * 4);
  b.cat = MEM_ACT;
  M.xs.assign(c.n_layers + 1, nullptr);
  for (auto& x : M.xs) x = b.take(T * d * es);
  M.la.assign(c.n_layers, LayerAct{});
  for (auto& a : M.la) {
    a.na = b.take(T * d * es);
    a.qkv = b.take(T * 3 * d * es);
    a.ctx = b.take(T * d * es);
    a.xmid = b.take(T * d * es);
    a.nb = b.take(T * d * es);
    a.fpre = b.take(T * fw * es);
    a.act = b.take(T * f * es);
    a.st1 = (float*)b.take(T * 2 * 4);
    a.st2 = (float*)b.take(T * 2 * 4);
    a.lse = (float*)b.take(B * H * S * 4);
  }
  if (enc) {
    M.e0 = b.take(T * d * es);
    M.st_e = (float*)b.take(T * 2 * 4);
    M.xcls = b.take(B * d * es);
    M.dcls = b.take(B * d * es);
    M.logits = b.take(B * (int64_t)c.n_classes * es);
  } else {
    M.xf = b.take(T * d * es);
    M.st_f = (float*)b.take(T * 2 * 4);
    M.logits = b.take(T * V * es);
  }
  b.cat = MEM_WORK;
  M.row_loss = (float*)b.take((T + 1) * 4);
  M.loss_dev = (float*)b.take(256);
  const int64_t wmax = std::max<int64_t>(std::max<int64_t>(3 * d, fw), std::max<int64_t>(d, c.n_classes));
  M.part = (float*)b.take((size_t)2 * ((T + 63) / 64) * wmax * 4);
  for (auto& x : M.D) x = b.take(T * d * es);
  M.dqkv = b.take(T * 3 * d * es);
  // one probability matrix and its gradient for the attention that runs as separate contractions and softmax
  // kernels (fp32, head widths other than 64 and 128, odd sequence lengths): the backward pass forms a layer's
  // probabilities again from its q and k instead of keeping them per layer
  M.prob = b.take(B * H * S * S * es);
  M.dprob = b.take(B * H * S * S * es);
  M.attn_dsum = b.take(B * H * S * 4);
  M.dact = b.take(T * f * es);
  M.dffn = b.take(T * fw * es);
  M.gemm_ws = M.wpk_bytes ? b.take(PACKED_WS_BYTES) : nullptr;  // shared tiles of the packed-operand contraction
  M.rowsq = M.wpk_bytes ? (float*)b.take((size_t)M.maxT * ((M.cfg.d_model + 63) / 64) * 4) : nullptr;
  if (dev_bytes) *dev_bytes = b.used;
  if (pinned_bytes) *pinned_bytes = M.on_host ? (size_t)M.n_move * np * 4 : 0;
  if (by_cat)
    for (int i = 0; i < MEM_N; ++i) by_cat[i] = b.by_cat[i];
}

int64_t largest_group(const Layout& L, int m) {
  const int k = group_count(L.n_units, m);
  int64_t best = 0;
  for (int j = 0; j < k; ++j) {
    int64_t c = 0;
    for (int u = j * m; u < std::min((j + 1) * m, L.n_units); ++u) c += L.unit_cnt[u];
    best = std::max(best, c);
  }
  return best;
}

hift_status init_model_shape(hift_model* M, const hift_config* cfg, const hift_opt* opt, int m, int max_batch,
                             int max_seq) {
  hift_status s = check_config(cfg);
  if (s != HIFT_OK) return s;
  s = check_opt(opt);
  if (s != HIFT_OK) return s;
  if (m < 1) return fail(HIFT_EINVAL, "m must be >= 1");
  if (max_batch < 1 || max_seq < 1) return fail(HIFT_EINVAL, "max_batch and max_seq must be >= 1");
  if (max_seq > cfg->max_seq) return fail(HIFT_EINVAL, "max_seq %d exceeds the position range %d", max_seq, cfg->max_seq);
  M->cfg = *cfg;
  M->opt = *opt;
  M->dt = cfg->dtype == HIFT_BF16 ? DT_BF16 : DT_F32;
  M->es = (int)dt_size(M->dt);
  M->max_batch = max_batch;
  M->max_seq_len = max_seq;
  M->maxT = (int64_t)max_batch * max_seq;
  build_layout(*cfg, M->lay);
  M->grad_cap = (largest_group(M->lay, m) + 63) & ~(int64_t)63;
  M->n_state = cfg->lora_rank > 0 ? 0 : n_state_of(*opt);  // with adapters the base model is never updated: no state for it
  M->on_host = cfg->state_on_host != 0;
  M->master_host = cfg->master_on_host != 0;
  M->n_move = M->n_state + (M->master_host ? 1 : 0);
  M->unit_steps.assign(M->lay.n_units, 0);
  M->lora_r = cfg->lora_rank;
  M->n_lora = (int64_t)cfg->n_layers * 4 * cfg->lora_rank * cfg->d_model;
  M->n_fac = 0;
  M->af_work_floats = 0;
  if (opt->kind == HIFT_ADAFACTOR)
    for (Tensor& t : M->lay.t) {
      t.fac_off = M->n_fac;
      M->n_fac += t.fac_count();
      M->af_work_floats = std::max(M->af_work_floats, adafactor_work_floats(t.rows, t.cols));
    }
  // Which matrices get copies in fragment order: those whose contraction, at the largest batch,
  // is one the packed-operand kernel takes.
  M->wpk_bytes = 0;
  for (Tensor& t : M->lay.t) {
    // of the embeddings unit only a token table that doubles as output matrix multiplies anything
    const bool contracts = t.unit != 0 || (cfg->tie_embeddings && t.name == "tok_emb");
    if (t.kind != HIFT_KIND_MATRIX || !contracts || M->dt != DT_BF16 || cfg->no_packed_copies) continue;
    const int64_t rows = (cfg->arch == HIFT_ARCH_POSTLN_ENCODER && t.unit == M->lay.n_units - 1) ? max_batch : M->maxT;
    Gemm g;
    g.dtype = DT_BF16;
    g.M = rows; g.N = t.rows; g.K = t.cols; g.lda = t.cols; g.ldc = t.rows; g.ldr = t.rows;
    if (packed_gemm_applies(g)) {
      t.pk_fwd = (int64_t)M->wpk_bytes;
      M->wpk_bytes += (packed_b_bytes(t.rows, t.cols) + 255) & ~(size_t)255;
      // forward copies of the RMSNorm/RoPE/SwiGLU decoder whose epilogue applies the rotation or the gated
      // activation (cfg->unfused & HIFT_UNFUSED_EPILOGUES keeps the separate kernels)
      const bool epi_on = !(cfg->unfused & HIFT_UNFUSED_EPILOGUES);
      const bool layer_t = t.unit >= 1 && t.unit <= cfg->n_layers;
      const std::string leaf = t.name.substr(t.name.find('.') + 1);
      if (epi_on && layer_t && cfg->arch == HIFT_ARCH_RMS_ROPE_DECODER && t.rows % 256 == 0) {
        // (with adapters the rotation stays a kernel of its own: the adapters' part is added to q before it)
        if (leaf == "wqkv" && cfg->d_model / cfg->n_heads == 128 && cfg->lora_rank == 0) t.pk_order = PK_ORDER_PAIR64;
        if (leaf == "wgu") t.pk_order = PK_ORDER_HALVES;
        // The normalisation in front of either goes into the contraction (Gemm::rowsq), unless
        // cfg->unfused & HIFT_UNFUSED_NORM keeps the normalisation kernels
        const bool fold_on = !(cfg->unfused & HIFT_UNFUSED_NORM);
        if (fold_on && t.cols % 512 == 0 && t.cols <= 6144 && t.pk_order != PK_ORDER_PLAIN)
          t.pk_gain = M->lay.find(t.name.substr(0, t.name.find('.') + 1) + (leaf == "wqkv" ? "g1" : "g2"));
      }
    }
    g.N = t.cols; g.K = t.rows; g.lda = t.rows; g.ldc = t.cols; g.ldr = t.cols;
    if (packed_gemm_applies(g)) {
      t.pk_bwd = (int64_t)M->wpk_bytes;
      M->wpk_bytes += (packed_b_bytes(t.cols, t.rows) + 255) & ~(size_t)255;
    }
  }
  // The bf16 copy of the model: every tensor, except matrices that have both fragment-order copies (7B shape: 13.5 GB
  // less).  Kept for all when the master lives on the host (its pieces pass through a slot tensor by tensor boundaries
  // unknown to them) and for a token table that is also the output matrix (the embedding lookup reads its rows).
  M->wc_count = 0;
  for (Tensor& t : M->lay.t) {
    if (M->master_host) {  // the copy mirrors the parameter order exactly
      t.wc_off = t.off;
      M->wc_count = t.off + t.count();
      continue;
    }
    const bool packed_only = t.pk_fwd >= 0 && t.pk_bwd >= 0 && t.unit != 0;
    t.wc_off = packed_only ? -1 : M->wc_count;
    if (!packed_only) M->wc_count += (t.count() + 7) & ~(int64_t)7;  // 16-byte aligned starts
  }
  return HIFT_OK;
}

// bf16 copy of the tensors of units [ulo, uhi) from the fp32 master in HBM (tensors that keep one)
hipError_t cast_units(hift_model* M, int ulo, int uhi) {
  if (M->dt != DT_BF16) return hipSuccess;
  for (int i = M->lay.unit_first[ulo]; i < M->lay.unit_first[uhi]; ++i) {
    const Tensor& t = M->lay.t[i];
    if (t.wc_off < 0) continue;
    hipError_t e = cast_f32_to(DT_BF16, t.count(), M->master + t.off, M->W(t), M->cs);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Rebuilds the fragment-order copies of the matrices of units [ulo, uhi) from the bf16 weights.
hipError_t repack_units(hift_model* M, int ulo, int uhi) {
  if (!M->wpk) return hipSuccess;
  for (int i = M->lay.unit_first[ulo]; i < M->lay.unit_first[uhi]; ++i) {
    const Tensor& t = M->lay.t[i];
    // source: the row-major bf16 copy, or, where none is kept, the fp32 master (rounded on the way: the same values)
    const bool f32src = M->dt == DT_BF16 && t.wc_off < 0;
    const void* src = f32src ? (const void*)(M->master + t.off) : (const void*)M->W(t);
    if (t.pk_fwd >= 0) {
      hipError_t e = pack_b(src, t.cols, t.rows, t.cols, true, M->wpk + t.pk_fwd, M->cs, t.pk_order,
                            t.pk_gain >= 0 ? M->W(M->lay.t[t.pk_gain]) : nullptr, f32src);
      if (e != hipSuccess) return e;
    }
    if (t.pk_bwd >= 0) {
      hipError_t e = pack_b(src, t.cols, t.cols, t.rows, false, M->wpk + t.pk_bwd, M->cs, PK_ORDER_PLAIN, nullptr, f32src);
      if (e != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

// ---- profiling of kernel classes (events around launches) ---------------------------------
// CAT_GEMM: linear layers (forward and dX) on the packed-operand kernel (the dominant kernel);
// CAT_GEMM_REST: every other linear-layer contraction (dW, small shapes, fp32)
enum { CAT_GEMM = 0, CAT_ATTN = 1, CAT_ELEM = 2, CAT_OPT = 3, CAT_GEMM_REST = 4, CAT_PACK = 5, CAT_N = 6 };
// Kinds of row-wise / elementwise kernel inside CAT_ELEM, each timed with its algorithmic bytes: every element the
// kernel has to read once plus every element it has to write once (gains, statistics and labels are not counted).
enum { RW_EMBED_FWD = 0, RW_NORM_FWD, RW_ROW_SUMSQ, RW_ROPE, RW_ACT_FWD, RW_ACT_BWD, RW_SOFTMAX_FWD, RW_SOFTMAX_BWD,
       RW_CROSS_ENTROPY, RW_NORM_BWD_DX, RW_NORM_BWD_PARAMS, RW_COL_SUM, RW_EMBED_BWD, RW_FIRST_ROWS, RW_LOSS_MEAN, RW_N };
const char* const RW_NAMES[RW_N] = {
    "embedding lookup", "normalisation forward", "row sums of squares", "rotary embedding", "activation forward",
    "activation backward", "softmax forward", "softmax backward", "cross-entropy with gradient", "normalisation backward dX",
    "normalisation backward gain/shift", "column sums (bias gradient)", "embedding gradient (clear + scatter)",
    "first-token gather / scatter", "loss bookkeeping (count of targets, mean of row losses; one workgroup each)"};

struct Scope {
  hift_model* M;
  Prof::Rec* r = nullptr;
  Scope(hift_model* m, int cat, double work, int sub = 0) : M(m) {
    if (!M->prof.on) return;
    if (M->prof.used == M->prof.pool.size()) {
      Prof::Rec n{};
      if (hipEventCreate(&n.a) != hipSuccess || hipEventCreate(&n.b) != hipSuccess) return;
      M->prof.pool.push_back(n);
    }
    r = &M->prof.pool[M->prof.used++];
    r->cat = cat;
    r->sub = sub;
    r->work = work;
    (void)hipEventRecord(r->a, M->cs);
  }
  ~Scope() {
    if (r) (void)hipEventRecord(r->b, M->cs);
  }
};

#define K_TRY(expr) HIP_TRY(expr)

// A row-wise kernel launch (a launcher returning hipError_t) under its own timing scope
#define RW(kind, bytes, call)                                                                      \
  do {                                                                                             \
    Scope rw_sc_(M, CAT_ELEM, (bytes), (kind));                                                    \
    hipError_t rw_e_ = (call);                                                                     \
    if (rw_e_ != hipSuccess) return fail(HIFT_EDEVICE, "kernel launch failed: %s", hipGetErrorString(rw_e_)); \
  } while (0)

#define ST_TRY(expr)                 \
  do {                               \
    hift_status s_ = (expr);         \
    if (s_ != HIFT_OK) return s_;    \
  } while (0)


// What a linear layer's epilogue may take over when the weight's packed copy is ordered for it:
// the rotary embedding of q and k (S = sequence length), or the gated activation (act [rows, out/2];
// keep_pre = false: the pre-activations are not needed later and y is not written).  fused reports
// whether it did; if not, y holds the plain product and the caller runs the separate kernel.
struct LinEpi {
  int S = 0;
  void* act = nullptr;
  bool keep_pre = true;
  bool fused = false;
  float* norm_stats = nullptr;  // weights with a folded normalisation: where (0, 1 / rms) per row goes, or null
  bool gelu = false;            // plain block order: bias and GELU in the epilogue (act [rows, out]; keep_pre as above)
};

// Whether a linear layer with this weight applies the normalisation in front of it itself: x is then the rows
// before the normalisation, and M->rowsq must hold their sums of squares.
bool folds_norm(const hift_model* M, const Tensor& w, int64_t rows) {
  if (w.pk_gain < 0 || w.pk_fwd < 0) return false;
  Gemm g;
  g.dtype = M->dt;
  g.M = rows; g.N = w.rows; g.K = w.cols; g.lda = w.cols; g.ldc = g.ldr = w.rows;
  // the same question linear() asks (alignment aside, which the arenas guarantee): a weight without a row-major copy
  // goes through the packed-operand kernel at any batch, also one of too few tiles to fill the chip
  const bool only_packed = M->dt == DT_BF16 && w.wc_off < 0;
  return packed_gemm_applies(g, only_packed);
}

// rowsq (optional): in, whether the sums of squares of y's rows are wanted in M->rowsq (y feeds a weight that
// folds its normalisation); out, whether the kernel that ran left them there.
hift_status linear(hift_model* M, const void* x, int64_t rows, const Tensor& w, const Tensor* bias, const void* R,
                   void* y, LinEpi* epi = nullptr, bool* rowsq = nullptr) {
  // y[rows, out] = x[rows, in] . w[out, in]^T (+ bias) (+ R)
  Gemm g;
  g.dtype = M->dt;
  g.M = rows; g.N = w.rows; g.K = w.cols;
  g.A = x; g.lda = w.cols;
  g.B = M->W(w); g.ldb = w.cols;
  g.C = y; g.ldc = w.rows;
  g.bias = bias ? M->W(*bias) : nullptr;
  g.R = R; g.ldr = w.rows;
  Scope sc(M, CAT_GEMM, 2.0 * rows * w.rows * w.cols);
  const bool only_packed = M->dt == DT_BF16 && w.wc_off < 0;  // no row-major copy to fall back on: any batch goes here
  if (w.pk_fwd >= 0 && packed_gemm_applies(g, only_packed)) {
    if (w.pk_order != PK_ORDER_PLAIN) {
      // the copy's block order is undone only by the epilogue it was made for
      if (!epi || bias || R) return fail(HIFT_ESTATE, "packed copy ordered for a fused epilogue used without one");
      if (w.pk_order == PK_ORDER_HALVES) {
        g.epi = EPI_SWIGLU;
        g.C2 = epi->act; g.ldc2 = w.rows / 2;
        if (!epi->keep_pre) g.C = nullptr;
      } else {
        g.epi = EPI_ROPE;
        g.cos_sin = M->cos_sin; g.S = epi->S; g.rot_cols = 2 * (int64_t)M->cfg.d_model;
      }
      epi->fused = true;
      if (w.pk_gain >= 0) {
        g.rowsq = M->rowsq; g.norm_eps = M->cfg.norm_eps; g.norm_stats = epi->norm_stats;
      }
    } else if (epi && epi->gelu && epi->act && !R && w.rows % 8 == 0) {
      if (!(M->cfg.unfused & HIFT_UNFUSED_EPILOGUES)) {
        g.epi = EPI_GELU;
        g.C2 = epi->act; g.ldc2 = w.rows;
        if (!epi->keep_pre) g.C = nullptr;
        epi->fused = true;
      }
    }
    if (rowsq) {
      *rowsq = *rowsq && g.epi == EPI_NONE && w.rows % 256 == 0;
      if (*rowsq) g.rowsq_out = M->rowsq;
    }
    g.ws = (M->cfg.unfused & HIFT_UNSHARED_LAST_ROUND) ? nullptr : M->gemm_ws;
    K_TRY(gemm_packed(g, M->wpk + w.pk_fwd, M->cs));
    return HIFT_OK;
  }
  if (rowsq) *rowsq = false;
  if (only_packed) return fail(HIFT_ESTATE, "%s has no row-major copy and the packed-operand kernel refused the problem", w.name.c_str());
  if (sc.r) sc.r->cat = CAT_GEMM_REST;
  K_TRY(gemm(g, M->cs));
  return HIFT_OK;
}

// gate_pre / dgu: if given and the packed kernel takes the problem, dx (the gradient of the gated activation,
// [rows, in]) is not stored; the epilogue turns it into the gradient of gate | up ([rows, 2 in]) with the forward's
// pre-activations and *fused is set.  Otherwise dx is written and the caller runs the separate kernel.
// gelu: the activation was GELU: gate_pre is [rows, in] and dgu [rows, in] receives d act * gelu'(pre).
hift_status linear_dx(hift_model* M, const void* dy, int64_t rows, const Tensor& w, const void* R, void* dx,
                      const void* gate_pre = nullptr, void* dgu = nullptr, bool* fused = nullptr, bool gelu = false) {
  // dx[rows, in] = dy[rows, out] . w[out, in] (+ R)
  Gemm g;
  g.dtype = M->dt;
  g.M = rows; g.N = w.cols; g.K = w.rows;
  g.A = dy; g.lda = w.rows;
  g.B = M->W(w); g.ldb = w.cols; g.b_kmajor = false;
  g.C = dx; g.ldc = w.cols;
  g.R = R; g.ldr = w.cols;
  Scope sc(M, CAT_GEMM, 2.0 * rows * w.rows * w.cols);
  const bool only_packed = M->dt == DT_BF16 && w.wc_off < 0;
  if (w.pk_bwd >= 0 && packed_gemm_applies(g, only_packed)) {
    const bool epi_on = !(M->cfg.unfused & HIFT_UNFUSED_EPILOGUES);
    if (epi_on && gate_pre && dgu && fused && !R && w.cols % 8 == 0 && (reinterpret_cast<uintptr_t>(dgu) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(gate_pre) & 15) == 0) {
      const int64_t width = gelu ? w.cols : 2 * w.cols;
      g.epi = gelu ? EPI_GELU_BWD : EPI_SWIGLU_BWD;
      g.C2 = const_cast<void*>(gate_pre); g.ldc2 = width;
      g.C = dgu; g.ldc = width;
      *fused = true;
    }
    g.ws = (M->cfg.unfused & HIFT_UNSHARED_LAST_ROUND) ? nullptr : M->gemm_ws;
    K_TRY(gemm_packed(g, M->wpk + w.pk_bwd, M->cs));
    return HIFT_OK;
  }
  if (only_packed) return fail(HIFT_ESTATE, "%s has no row-major copy and the packed-operand kernel refused the problem", w.name.c_str());
  if (sc.r) sc.r->cat = CAT_GEMM_REST;
  K_TRY(gemm(g, M->cs));
  return HIFT_OK;
}

hift_status linear_dw(hift_model* M, const void* dy, const void* x, int64_t rows, const Tensor& w, int64_t glo) {
  // grad_w[out, in] = dy[rows, out]^T . x[rows, in], fp32, into the group-local gradient buffer
  Gemm g;
  g.dtype = M->dt;
  g.out_f32 = true;
  g.M = w.rows; g.N = w.cols; g.K = rows;
  g.A = dy; g.lda = w.rows; g.a_kmajor = false;
  g.B = x; g.ldb = w.cols; g.b_kmajor = false;
  g.C = M->grad + (w.off - glo); g.ldc = w.cols;
  Scope sc(M, CAT_GEMM_REST, 2.0 * rows * w.rows * w.cols);
  K_TRY(gemm(g, M->cs));
  return HIFT_OK;
}

hift_status bias_grad(hift_model* M, const void* dy, int64_t rows, const Tensor& b, int64_t glo) {
  RW(RW_COL_SUM, (double)rows * b.rows * M->es, col_sum(M->dt, rows, b.rows, dy, b.rows, M->part, M->grad + (b.off - glo), M->cs));
  return HIFT_OK;
}

// Whether a layer's attention runs on the fused kernels, forward and backward alike (the backward needs what
// only the fused forward leaves, and the other way round).  Never with cfg.unfused & HIFT_UNFUSED_ATTENTION.
bool attention_is_fused(const hift_model* M, const LayerAct& a, int S) {
  const bool fused_on = !(M->cfg.unfused & HIFT_UNFUSED_ATTENTION);
  const int64_t d = M->cfg.d_model, hd = d / M->cfg.n_heads;
  return fused_on && attention_fwd_fused_applies(M->dt, S, (int)hd, 3 * d, d, a.qkv, nullptr, a.ctx) &&
         attention_bwd_fused_applies(M->dt, S, (int)hd, 3 * d, d, a.qkv, a.ctx, M->D[2], M->dqkv);
}

// Probabilities of one layer into M->prob, for the unfused attention: scores q . k^T, then the softmax in place.
hift_status attention_probs(hift_model* M, LayerAct& a, int B, int S) {
  const hift_config& c = M->cfg;
  const int64_t d = c.d_model, H = c.n_heads, hd = d / H;
  const size_t es = M->es;
  unsigned char* qkv = (unsigned char*)a.qkv;
  const bool causal = c.arch != HIFT_ARCH_POSTLN_ENCODER;
  {
    Gemm g;  // scores = q . k^T
    g.dtype = M->dt;
    g.M = S; g.N = S; g.K = hd;
    g.A = qkv; g.lda = 3 * d;
    g.B = qkv + d * es; g.ldb = 3 * d;
    g.C = M->prob; g.ldc = S;
    g.nb = B; g.nh = (int)H;
    g.sa1 = (int64_t)S * 3 * d; g.sa2 = hd; g.sb1 = g.sa1; g.sb2 = hd;
    g.sc1 = H * (int64_t)S * S; g.sc2 = (int64_t)S * S;
    if (causal) g.band = BAND_SKIP_UPPER;  // the softmax never reads scores above the diagonal
    Scope sc(M, CAT_ATTN, 2.0 * B * H * S * S * hd);
    K_TRY(gemm(g, M->cs));
  }
  RW(RW_SOFTMAX_FWD, 2.0 * B * H * S * S * es, softmax_fwd(M->dt, (int64_t)B * H, S, 1.0f / sqrtf((float)hd), causal, M->prob, M->cs));
  return HIFT_OK;
}

// keep = false: no backward pass will come through this layer; the fused kernel then stores nothing but the context
hift_status attention_fwd(hift_model* M, LayerAct& a, int B, int S, bool keep) {
  const hift_config& c = M->cfg;
  const int64_t d = c.d_model, H = c.n_heads, hd = d / H;
  const size_t es = M->es;
  unsigned char* qkv = (unsigned char*)a.qkv;
  const bool causal = c.arch != HIFT_ARCH_POSTLN_ENCODER;
  if (attention_is_fused(M, a, S)) {
    // scores, softmax and P.V in one kernel; of the softmax only each row's log-sum is kept for the backward pass
    Scope sc(M, CAT_ATTN, 4.0 * B * H * S * S * hd);
    K_TRY(attention_fwd_fused(B, (int)H, S, (int)hd, causal, a.qkv, 3 * d, nullptr, a.ctx, d, keep ? a.lse : nullptr, M->cs));
    return HIFT_OK;
  }
  ST_TRY(attention_probs(M, a, B, S));
  {
    Gemm g;  // ctx = p . v
    g.dtype = M->dt;
    g.M = S; g.N = hd; g.K = S;
    g.A = M->prob; g.lda = S;
    g.B = qkv + 2 * d * es; g.ldb = 3 * d; g.b_kmajor = false;
    g.C = a.ctx; g.ldc = d;
    g.nb = B; g.nh = (int)H;
    g.sa1 = H * (int64_t)S * S; g.sa2 = (int64_t)S * S;
    g.sb1 = (int64_t)S * 3 * d; g.sb2 = hd;
    g.sc1 = (int64_t)S * d; g.sc2 = hd;
    if (causal) g.band = BAND_K_UPTO_ROW;  // probabilities above the diagonal are exact zeros
    Scope sc(M, CAT_ATTN, 2.0 * B * H * S * S * hd);
    K_TRY(gemm(g, M->cs));
  }
  return HIFT_OK;
}

hift_status attention_bwd(hift_model* M, LayerAct& a, const void* dctx, int B, int S, bool* unrotated) {
  // dctx [T, d] -> M->dqkv [T, 3d]: gradients with respect to v and to the rotated q, k -- or, with *unrotated set
  // (fused kernels on a rotary architecture), to q and k as projected
  const hift_config& c = M->cfg;
  const int64_t d = c.d_model, H = c.n_heads, hd = d / H;
  const size_t es = M->es;
  unsigned char* qkv = (unsigned char*)a.qkv;
  unsigned char* dqkv = (unsigned char*)M->dqkv;
  const double fl = 2.0 * B * H * S * S * hd;
  const bool causal = c.arch != HIFT_ARCH_POSTLN_ENCODER;
  auto batch = [&](Gemm& g) { g.dtype = M->dt; g.nb = B; g.nh = (int)H; };
  const int64_t sP1 = H * (int64_t)S * S, sP2 = (int64_t)S * S, sQ1 = (int64_t)S * 3 * d, sX1 = (int64_t)S * d;
  *unrotated = false;
  if (attention_is_fused(M, a, S)) {
    // two kernels, query-major (dq) and key-major (dk, dv); both form the probabilities again from q, k and the
    // stored log-sums and undo the rotary embedding on the way out
    if (dctx != M->D[2]) return fail(HIFT_ESTATE, "attention backward expects its input in the third gradient buffer");
    const float* cs = c.arch == HIFT_ARCH_RMS_ROPE_DECODER ? M->cos_sin : nullptr;
    *unrotated = cs != nullptr;
    Scope sc(M, CAT_ATTN, 7 * fl);  // S and dP twice, dQ, dV, dK
    K_TRY(attention_bwd_fused(B, (int)H, S, (int)hd, causal, a.qkv, 3 * d, a.ctx, a.lse, dctx, d, (float*)M->attn_dsum, M->dqkv, cs,
                              M->cs));
    return HIFT_OK;
  }
  ST_TRY(attention_probs(M, a, B, S));  // the forward pass kept q and k, not the probabilities
  {
    Gemm g;  // dv[j,e] = sum_i p[i,j] dctx[i,e]
    batch(g);
    g.M = S; g.N = hd; g.K = S;
    g.A = M->prob; g.lda = S; g.a_kmajor = false; g.sa1 = sP1; g.sa2 = sP2;
    g.B = dctx; g.ldb = d; g.b_kmajor = false; g.sb1 = sX1; g.sb2 = hd;
    g.C = dqkv + 2 * d * es; g.ldc = 3 * d; g.sc1 = sQ1; g.sc2 = hd;
    if (causal) g.band = BAND_K_FROM_ROW;  // p[i,j] = 0 for i < j
    Scope sc(M, CAT_ATTN, fl);
    K_TRY(gemm(g, M->cs));
  }
  {
    Gemm g;  // dp[i,j] = sum_e dctx[i,e] v[j,e]
    batch(g);
    g.M = S; g.N = S; g.K = hd;
    g.A = dctx; g.lda = d; g.sa1 = sX1; g.sa2 = hd;
    g.B = qkv + 2 * d * es; g.ldb = 3 * d; g.sb1 = sQ1; g.sb2 = hd;
    g.C = M->dprob; g.ldc = S; g.sc1 = sP1; g.sc2 = sP2;
    if (causal) g.band = BAND_SKIP_UPPER;  // the softmax backward never reads dp above the diagonal
    Scope sc(M, CAT_ATTN, fl);
    K_TRY(gemm(g, M->cs));
  }
  RW(RW_SOFTMAX_BWD, 3.0 * B * H * S * S * es, softmax_bwd(M->dt, (int64_t)B * H, S, 1.0f / sqrtf((float)hd), causal, M->prob, M->dprob, M->cs));
  {
    Gemm g;  // dq[i,e] = sum_j ds[i,j] k[j,e]
    batch(g);
    g.M = S; g.N = hd; g.K = S;
    g.A = M->dprob; g.lda = S; g.sa1 = sP1; g.sa2 = sP2;
    g.B = qkv + d * es; g.ldb = 3 * d; g.b_kmajor = false; g.sb1 = sQ1; g.sb2 = hd;
    g.C = dqkv; g.ldc = 3 * d; g.sc1 = sQ1; g.sc2 = hd;
    if (causal) g.band = BAND_K_UPTO_ROW;  // ds[i,j] = 0 for j > i
    Scope sc(M, CAT_ATTN, fl);
    K_TRY(gemm(g, M->cs));
  }
  {
    Gemm g;  // dk[j,e] = sum_i ds[i,j] q[i,e]
    batch(g);
    g.M = S; g.N = hd; g.K = S;
    g.A = M->dprob; g.lda = S; g.a_kmajor = false; g.sa1 = sP1; g.sa2 = sP2;
    g.B = qkv; g.ldb = 3 * d; g.b_kmajor = false; g.sb1 = sQ1; g.sb2 = hd;
    g.C = dqkv + d * es; g.ldc = 3 * d; g.sc1 = sQ1; g.sc2 = hd;
    if (causal) g.band = BAND_K_FROM_ROW;  // ds[i,j] = 0 for i < j
    Scope sc(M, CAT_ATTN, fl);
    K_TRY(gemm(g, M->cs));
  }
  return HIFT_OK;
}

// ---- low-rank adapters (the LoRA baseline of section 4.3) ---------------------------------------------------
// q = h Wq^T + s (h A_q^T) B_q^T, v likewise, s = alpha / r.  The scale is applied to the small intermediate
// u = s (h A^T) in the forward pass and to its gradient in the backward pass, so that no weight is kept scaled.
struct LoraPtrs {
  unsigned char *acat, *bq, *bv;  // compute-type copies: A_q | A_v [2r, d], B_q [d, r], B_v [d, r]
  float *g_acat, *g_bq, *g_bv;    // their gradients
};
LoraPtrs lora_ptrs(const hift_model* M, int l) {
  const int64_t r = M->lora_r, d = M->cfg.d_model, per = 4 * r * d, es = M->es;
  unsigned char* w = reinterpret_cast<unsigned char*>(M->lora_wc) + (int64_t)l * per * es;
  float* g = M->lora_grad + (int64_t)l * per;
  return LoraPtrs{w, w + 2 * r * d * es, w + 3 * r * d * es, g, g + 2 * r * d, g + 3 * r * d};
}

hift_status small_gemm(hift_model* M, const Gemm& g) {
  Scope sc(M, CAT_GEMM_REST, 2.0 * g.M * g.N * g.K);
  K_TRY(gemm(g, M->cs));
  return HIFT_OK;
}

// Adds the adapters' part to the q and v columns of qkv [T, 3d] (before any rotation); h: the layer's input [T, d]
hift_status lora_fwd(hift_model* M, int l, const void* h, int64_t T, void* qkv) {
  const int64_t r = M->lora_r, d = M->cfg.d_model, es = M->es;
  const LoraPtrs P = lora_ptrs(M, l);
  unsigned char* u = reinterpret_cast<unsigned char*>(M->lora_u[l]);
  Gemm g;  // u = h . (A_q | A_v)^T
  g.dtype = M->dt;
  g.M = T; g.N = 2 * r; g.K = d;
  g.A = h; g.lda = d; g.B = P.acat; g.ldb = d; g.C = u; g.ldc = 2 * r;
  ST_TRY(small_gemm(M, g));
  RW(RW_ACT_FWD, 2.0 * T * 2 * r * es, scale_inplace(M->dt, T * 2 * r, M->cfg.lora_alpha / (float)r, u, M->cs));
  for (int part = 0; part < 2; ++part) {  // q += u_q . B_q^T ; v += u_v . B_v^T, in place
    Gemm a;
    a.dtype = M->dt;
    a.M = T; a.N = d; a.K = r;
    a.A = u + part * r * es; a.lda = 2 * r;
    a.B = part ? P.bv : P.bq; a.ldb = r;
    a.C = reinterpret_cast<unsigned char*>(qkv) + part * 2 * d * es; a.ldc = 3 * d;
    a.R = a.C; a.ldr = 3 * d;
    ST_TRY(small_gemm(M, a));
  }
  return HIFT_OK;
}

// dqkv [T, 3d]: gradients of the projections as computed (before rotation).  Leaves the adapters' gradients of
// layer l in M->lora_grad and, if dh is given, adds the adapters' part to the gradient of the layer's input.
hift_status lora_bwd(hift_model* M, int l, const void* h, int64_t T, const void* dqkv, void* dh) {
  const int64_t r = M->lora_r, d = M->cfg.d_model, es = M->es;
  const LoraPtrs P = lora_ptrs(M, l);
  const unsigned char* dq = reinterpret_cast<const unsigned char*>(dqkv);
  unsigned char* u = reinterpret_cast<unsigned char*>(M->lora_u[l]);
  unsigned char* du = reinterpret_cast<unsigned char*>(M->lora_du);
  for (int part = 0; part < 2; ++part) {
    const unsigned char* dy = dq + part * 2 * d * es;
    Gemm a;  // d u_part = d y . B  [T, r]
    a.dtype = M->dt;
    a.M = T; a.N = r; a.K = d;
    a.A = dy; a.lda = 3 * d;
    a.B = part ? P.bv : P.bq; a.ldb = r; a.b_kmajor = false;
    a.C = du + part * r * es; a.ldc = 2 * r;
    ST_TRY(small_gemm(M, a));
    Gemm b;  // d B = d y^T . u_part  [d, r]  (u carries the scale)
    b.dtype = M->dt; b.out_f32 = true;
    b.M = d; b.N = r; b.K = T;
    b.A = dy; b.lda = 3 * d; b.a_kmajor = false;
    b.B = u + part * r * es; b.ldb = 2 * r; b.b_kmajor = false;
    b.C = part ? P.g_bv : P.g_bq; b.ldc = r;
    ST_TRY(small_gemm(M, b));
  }
  RW(RW_ACT_BWD, 2.0 * T * 2 * r * es, scale_inplace(M->dt, T * 2 * r, M->cfg.lora_alpha / (float)r, du, M->cs));
  {
    Gemm c;  // d (A_q | A_v) = d u^T . h  [2r, d]
    c.dtype = M->dt; c.out_f32 = true;
    c.M = 2 * r; c.N = d; c.K = T;
    c.A = du; c.lda = 2 * r; c.a_kmajor = false;
    c.B = h; c.ldb = d; c.b_kmajor = false;
    c.C = P.g_acat; c.ldc = d;
    ST_TRY(small_gemm(M, c));
  }
  if (dh) {
    Gemm e;  // d h += d u . (A_q | A_v)
    e.dtype = M->dt;
    e.M = T; e.N = d; e.K = 2 * r;
    e.A = du; e.lda = 2 * r;
    e.B = P.acat; e.ldb = d; e.b_kmajor = false;
    e.C = dh; e.ldc = d; e.R = dh; e.ldr = d;
    ST_TRY(small_gemm(M, e));
  }
  return HIFT_OK;
}

struct Names {
  const Tensor *n1g, *n1b, *wqkv, *bqkv, *wo, *bo, *n2g, *n2b, *w1, *b1, *w2, *b2;
};

Names layer_names(const hift_model* M, int l) {
  const std::string p = "l" + std::to_string(l) + ".";
  auto get = [&](const char* n) -> const Tensor* {
    const int i = M->lay.find(p + n);
    return i < 0 ? nullptr : &M->lay.t[i];
  };
  Names n{};
  if (M->cfg.arch == HIFT_ARCH_RMS_ROPE_DECODER) {
    n.n1g = get("g1"); n.wqkv = get("wqkv"); n.wo = get("wo"); n.n2g = get("g2"); n.w1 = get("wgu"); n.w2 = get("wd");
  } else {
    n.n1g = get("ln1_g"); n.n1b = get("ln1_b"); n.wqkv = get("wqkv"); n.bqkv = get("bqkv"); n.wo = get("wo");
    n.bo = get("bo"); n.n2g = get("ln2_g"); n.n2b = get("ln2_b"); n.w1 = get("w1"); n.b1 = get("b1");
    n.w2 = get("w2"); n.b2 = get("b2");
  }
  return n;
}

// keep_from: lowest unit the backward pass will reach; layers below it keep no pre-activations
hift_status forward(hift_model* M, const hift_batch* bt, int keep_from) {
  const hift_config& c = M->cfg;
  const int B = bt->batch, S = bt->seq;
  const int64_t T = (int64_t)B * S;
  const int d = c.d_model, f = c.d_ffn, H = c.n_heads, hd = d / H;
  const int dt = M->dt;
  const double es = M->es;
  const bool enc = c.arch == HIFT_ARCH_POSTLN_ENCODER, rms = c.arch == HIFT_ARCH_RMS_ROPE_DECODER;
  hipStream_t st = M->cs;
  {
    const void* pos = rms ? nullptr : M->W("pos_emb");
    void* dst = enc ? M->e0 : M->xs[0];
    RW(RW_EMBED_FWD, (double)T * d * es * (pos ? 3 : 2), embed_fwd(dt, bt->tokens, T, S, d, c.vocab, M->W("tok_emb"), pos, dst, st));
    if (enc) RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, false, T, d, c.norm_eps, M->e0, M->W("lne_g"), M->W("lne_b"), M->xs[0], M->st_e, st));
  }
  bool have_sq = false;  // M->rowsq holds the sums of squares of the rows the next normalisation takes
  for (int l = 0; l < c.n_layers; ++l) {
    LayerAct& a = M->la[l];
    const Names n = layer_names(M, l);
    const void* x = M->xs[l];
    const void* h1 = x;
    if (folds_norm(M, *n.wqkv, T)) {
      if (!have_sq) {
        RW(RW_ROW_SUMSQ, 1.0 * T * d * es, row_sumsq(T, d, x, d / 64, M->rowsq, st));
      }
    } else if (!enc) {
      RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, rms, T, d, c.norm_eps, x, M->W(*n.n1g), n.n1b ? M->W(*n.n1b) : nullptr, a.na, a.st1, st));
      h1 = a.na;
    }
    LinEpi rot;
    rot.S = S;
    rot.norm_stats = a.st1;
    ST_TRY(linear(M, h1, T, *n.wqkv, n.bqkv, nullptr, a.qkv, &rot));
    if (M->lora_r > 0) {
      if (rot.fused) return fail(HIFT_ESTATE, "adapters need the projections before their rotation");
      ST_TRY(lora_fwd(M, l, h1, T, a.qkv));
    }
    if (rms && !rot.fused) {
      RW(RW_ROPE, 4.0 * T * d * es, rope(dt, a.qkv, T, S, H, hd, M->cos_sin, +1, st));
    }
    ST_TRY(attention_fwd(M, a, B, S, l + 1 >= keep_from));
    if (enc) {
      ST_TRY(linear(M, a.ctx, T, *n.wo, n.bo, x, a.na));  // s1 = x + attn
      RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, false, T, d, c.norm_eps, a.na, M->W(*n.n1g), M->W(*n.n1b), a.xmid, a.st1, st));
    } else {
      have_sq = folds_norm(M, *n.w1, T);
      ST_TRY(linear(M, a.ctx, T, *n.wo, n.bo, x, a.xmid, nullptr, &have_sq));
    }
    const void* h2 = a.xmid;
    if (folds_norm(M, *n.w1, T)) {
      if (!have_sq) {
        RW(RW_ROW_SUMSQ, 1.0 * T * d * es, row_sumsq(T, d, a.xmid, d / 64, M->rowsq, st));
      }
    } else if (!enc) {
      RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, rms, T, d, c.norm_eps, a.xmid, M->W(*n.n2g), n.n2b ? M->W(*n.n2b) : nullptr, a.nb, a.st2, st));
      h2 = a.nb;
    }
    LinEpi gate;
    gate.act = a.act;
    gate.keep_pre = l + 1 >= keep_from;
    gate.norm_stats = a.st2;
    gate.gelu = !rms;
    ST_TRY(linear(M, h2, T, *n.w1, n.b1, nullptr, a.fpre, &gate));
    if (!gate.fused) {
      if (rms) RW(RW_ACT_FWD, 3.0 * T * f * es, swiglu_fwd(dt, T, f, a.fpre, a.act, st));
      else RW(RW_ACT_FWD, 2.0 * T * f * es, gelu_fwd(dt, T * f, a.fpre, a.act, st));
    }
    if (enc) {
      ST_TRY(linear(M, a.act, T, *n.w2, n.b2, a.xmid, a.nb));  // s2 = xmid + ffn
      RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, false, T, d, c.norm_eps, a.nb, M->W(*n.n2g), M->W(*n.n2b), M->xs[l + 1], a.st2, st));
    } else {
      have_sq = l + 1 < c.n_layers && folds_norm(M, *layer_names(M, l + 1).wqkv, T);
      ST_TRY(linear(M, a.act, T, *n.w2, n.b2, a.xmid, M->xs[l + 1], nullptr, &have_sq));
    }
  }
  void* xl = M->xs[c.n_layers];
  if (enc) {
    {
      RW(RW_FIRST_ROWS, 2.0 * B * d * es, gather_first(dt, B, S, d, xl, M->xcls, st));
    }
    ST_TRY(linear(M, M->xcls, B, M->T_("wc"), &M->T_("bc"), nullptr, M->logits));
    RW(RW_LOSS_MEAN, 4.0 * (B), cross_entropy_count(B, bt->labels, M->row_loss, st));
    RW(RW_CROSS_ENTROPY, 2.0 * (B) * (c.n_classes) * es, cross_entropy_rows(dt, B, c.n_classes, M->logits, bt->labels, M->row_loss, st));
    RW(RW_LOSS_MEAN, 4.0 * (B), cross_entropy_mean(B, M->row_loss, M->loss_dev, st));
  } else {
    {
      if (rms) RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, true, T, d, c.norm_eps, xl, M->W("gf"), nullptr, M->xf, M->st_f, st));
      else RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, false, T, d, c.norm_eps, xl, M->W("lnf_g"), M->W("lnf_b"), M->xf, M->st_f, st));
    }
    ST_TRY(linear(M, M->xf, T, M->T_(c.tie_embeddings ? "tok_emb" : "whead"), nullptr, nullptr, M->logits));
    RW(RW_LOSS_MEAN, 4.0 * (T), cross_entropy_count(T, bt->labels, M->row_loss, st));
    RW(RW_CROSS_ENTROPY, 2.0 * (T) * (c.vocab) * es, cross_entropy_rows(dt, T, c.vocab, M->logits, bt->labels, M->row_loss, st));
    RW(RW_LOSS_MEAN, 4.0 * (T), cross_entropy_mean(T, M->row_loss, M->loss_dev, st));
  }
  return HIFT_OK;
}

// Backward from the loss down to unit `lo`; weight gradients for units in [ulo, uhi) only.
hift_status backward(hift_model* M, const hift_batch* bt, int ulo, int uhi, int64_t glo) {
  const hift_config& c = M->cfg;
  const int B = bt->batch, S = bt->seq;
  const int64_t T = (int64_t)B * S;
  const int d = c.d_model, f = c.d_ffn, H = c.n_heads, hd = d / H;
  const int dt = M->dt, L = c.n_layers;
  const double es = M->es;
  const bool enc = c.arch == HIFT_ARCH_POSTLN_ENCODER, rms = c.arch == HIFT_ARCH_RMS_ROPE_DECODER;
  hipStream_t st = M->cs;
  auto active = [&](int u) { return u >= ulo && u < uhi; };
  auto G = [&](const Tensor& t) { return M->grad + (t.off - glo); };
  void *Dc = M->D[0], *D1 = M->D[1], *D2 = M->D[2];

  // ---- head unit (L+1) ----
  const bool head_on = active(L + 1);
  if (enc) {
    const Tensor &wc = M->T_("wc"), &bc = M->T_("bc");
    if (head_on) {
      ST_TRY(linear_dw(M, M->logits, M->xcls, B, wc, glo));
      ST_TRY(bias_grad(M, M->logits, B, bc, glo));
    }
    if (ulo == L + 1) return HIFT_OK;
    ST_TRY(linear_dx(M, M->logits, B, wc, nullptr, M->dcls));
    RW(RW_FIRST_ROWS, (double)T * d * es + 1.0 * B * d * es, scatter_first(dt, B, S, d, M->dcls, Dc, st));
  } else {
    // tied embeddings: the output matrix is the token table of unit 0; its gradient starts here and the
    // embedding part is added at the bottom of the backward pass
    const Tensor& wh = M->T_(c.tie_embeddings ? "tok_emb" : "whead");
    if (c.tie_embeddings ? active(0) : head_on) ST_TRY(linear_dw(M, M->logits, M->xf, T, wh, glo));
    ST_TRY(linear_dx(M, M->logits, T, wh, nullptr, D2));  // d xf
    const Tensor& g = M->T_(rms ? "gf" : "lnf_g");
    if (head_on)
      RW(RW_NORM_BWD_PARAMS, 2.0 * T * d * es, norm_bwd_params(dt, rms, T, d, D2, M->xs[L], M->st_f, M->part, G(g),
                                   rms ? nullptr : G(M->T_("lnf_b")), st));
    if (ulo == L + 1) return HIFT_OK;
    RW(RW_NORM_BWD_DX, 3.0 * T * d * es, norm_bwd_dx(dt, rms, T, d, D2, M->xs[L], M->W(g), M->st_f, nullptr, Dc, st));
  }

  // ---- hidden layers, top down; Dc holds d loss / d xs[l+1] ----
  for (int l = L - 1; l >= 0; --l) {
    const int u = l + 1;
    if (u < ulo) break;
    const bool on = active(u), need_dx = u > ulo;
    LayerAct& a = M->la[l];
    const Names n = layer_names(M, l);
    const void* x = M->xs[l];
    if (!enc) {
      // x_out = xmid + W2 act(W1 h2),  h2 = norm2(xmid)
      if (on) {
        ST_TRY(linear_dw(M, Dc, a.act, T, *n.w2, glo));
        if (n.b2) ST_TRY(bias_grad(M, Dc, T, *n.b2, glo));
      }
      bool gate_done = false;
      if (rms) ST_TRY(linear_dx(M, Dc, T, *n.w2, nullptr, M->dact, a.fpre, M->dffn, &gate_done));
      else ST_TRY(linear_dx(M, Dc, T, *n.w2, nullptr, M->dact, a.fpre, M->dffn, &gate_done, true));
      if (!gate_done) {
        if (rms) RW(RW_ACT_BWD, 5.0 * T * f * es, swiglu_bwd(dt, T, f, M->dact, a.fpre, M->dffn, st));
        else RW(RW_ACT_BWD, 3.0 * T * f * es, gelu_bwd(dt, T * f, M->dact, a.fpre, M->dffn, st));
      }
      if (on) {
        if (folds_norm(M, *n.w1, T)) {  // the forward pass never wrote the normalised rows
          RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, rms, T, d, c.norm_eps, a.xmid, M->W(*n.n2g), nullptr, a.nb, a.st2, st));
        }
        ST_TRY(linear_dw(M, M->dffn, a.nb, T, *n.w1, glo));
        if (n.b1) ST_TRY(bias_grad(M, M->dffn, T, *n.b1, glo));
      }
      ST_TRY(linear_dx(M, M->dffn, T, *n.w1, nullptr, D2));  // d h2
      {
        if (on)
          RW(RW_NORM_BWD_PARAMS, 2.0 * T * d * es, norm_bwd_params(dt, rms, T, d, D2, a.xmid, a.st2, M->part, G(*n.n2g),
                                       n.n2b ? G(*n.n2b) : nullptr, st));
        RW(RW_NORM_BWD_DX, 4.0 * T * d * es, norm_bwd_dx(dt, rms, T, d, D2, a.xmid, M->W(*n.n2g), a.st2, Dc, D1, st));  // d xmid
      }
      // xmid = x + Wo ctx
      if (on) {
        ST_TRY(linear_dw(M, D1, a.ctx, T, *n.wo, glo));
        if (n.bo) ST_TRY(bias_grad(M, D1, T, *n.bo, glo));
      }
      ST_TRY(linear_dx(M, D1, T, *n.wo, nullptr, D2));  // d ctx
      bool unrotated = false;
      ST_TRY(attention_bwd(M, a, D2, B, S, &unrotated));
      if (rms && !unrotated) {
        RW(RW_ROPE, 4.0 * T * d * es, rope(dt, M->dqkv, T, S, H, hd, M->cos_sin, -1, st));
      }
      if (on) {
        if (folds_norm(M, *n.wqkv, T)) {
          RW(RW_NORM_FWD, 2.0 * T * d * es, norm_fwd(dt, rms, T, d, c.norm_eps, x, M->W(*n.n1g), nullptr, a.na, a.st1, st));
        }
        ST_TRY(linear_dw(M, M->dqkv, a.na, T, *n.wqkv, glo));
        if (n.bqkv) ST_TRY(bias_grad(M, M->dqkv, T, *n.bqkv, glo));
      }
      if (M->lora_r > 0) {  // the adapters' gradients; with need_dx their part of d h1 is added below
        if (folds_norm(M, *n.wqkv, T)) return fail(HIFT_ESTATE, "adapters need the normalised rows");
        if (on || need_dx) ST_TRY(linear_dx(M, M->dqkv, T, *n.wqkv, nullptr, D2));  // d h1, base part
        ST_TRY(lora_bwd(M, l, a.na, T, M->dqkv, (on || need_dx) ? D2 : nullptr));
      }
      if (on || need_dx) {
        if (M->lora_r == 0) ST_TRY(linear_dx(M, M->dqkv, T, *n.wqkv, nullptr, D2));  // d h1
        if (on)
          RW(RW_NORM_BWD_PARAMS, 2.0 * T * d * es, norm_bwd_params(dt, rms, T, d, D2, x, a.st1, M->part, G(*n.n1g),
                                       n.n1b ? G(*n.n1b) : nullptr, st));
        if (need_dx) RW(RW_NORM_BWD_DX, 4.0 * T * d * es, norm_bwd_dx(dt, rms, T, d, D2, x, M->W(*n.n1g), a.st1, D1, Dc, st));
      }
    } else {
      // x_out = LN2(s2), s2 = xmid + W2 gelu(W1 xmid);  xmid = LN1(s1), s1 = x + Wo ctx
      {
        if (on) RW(RW_NORM_BWD_PARAMS, 2.0 * T * d * es, norm_bwd_params(dt, false, T, d, Dc, a.nb, a.st2, M->part, G(*n.n2g), G(*n.n2b), st));
        RW(RW_NORM_BWD_DX, 3.0 * T * d * es, norm_bwd_dx(dt, false, T, d, Dc, a.nb, M->W(*n.n2g), a.st2, nullptr, D1, st));  // d s2
      }
      if (on) {
        ST_TRY(linear_dw(M, D1, a.act, T, *n.w2, glo));
        ST_TRY(bias_grad(M, D1, T, *n.b2, glo));
      }
      bool gelu_done = false;
      ST_TRY(linear_dx(M, D1, T, *n.w2, nullptr, M->dact, a.fpre, M->dffn, &gelu_done, true));
      if (!gelu_done) {
        RW(RW_ACT_BWD, 3.0 * T * f * es, gelu_bwd(dt, T * f, M->dact, a.fpre, M->dffn, st));
      }
      if (on) {
        ST_TRY(linear_dw(M, M->dffn, a.xmid, T, *n.w1, glo));
        ST_TRY(bias_grad(M, M->dffn, T, *n.b1, glo));
      }
      ST_TRY(linear_dx(M, M->dffn, T, *n.w1, D1, D2));  // d xmid = d s2 + dffn . W1
      {
        if (on) RW(RW_NORM_BWD_PARAMS, 2.0 * T * d * es, norm_bwd_params(dt, false, T, d, D2, a.na, a.st1, M->part, G(*n.n1g), G(*n.n1b), st));
        RW(RW_NORM_BWD_DX, 3.0 * T * d * es, norm_bwd_dx(dt, false, T, d, D2, a.na, M->W(*n.n1g), a.st1, nullptr, D1, st));  // d s1
      }
      if (on) {
        ST_TRY(linear_dw(M, D1, a.ctx, T, *n.wo, glo));
        ST_TRY(bias_grad(M, D1, T, *n.bo, glo));
      }
      ST_TRY(linear_dx(M, D1, T, *n.wo, nullptr, D2));  // d ctx
      bool unrotated = false;  // no rotary embedding in this architecture
      ST_TRY(attention_bwd(M, a, D2, B, S, &unrotated));
      if (on) {
        ST_TRY(linear_dw(M, M->dqkv, x, T, *n.wqkv, glo));
        ST_TRY(bias_grad(M, M->dqkv, T, *n.bqkv, glo));
      }
      if (need_dx) ST_TRY(linear_dx(M, M->dqkv, T, *n.wqkv, D1, Dc));  // d x = d s1 + dqkv . Wqkv
      if (M->lora_r > 0) ST_TRY(lora_bwd(M, l, x, T, M->dqkv, need_dx ? Dc : nullptr));
    }
  }

  // ---- embeddings unit (0) ----
  if (ulo == 0) {
    const Tensor& te = M->T_("tok_emb");
    const void* dx = Dc;
    if (enc) {
      RW(RW_NORM_BWD_PARAMS, 2.0 * T * d * es, norm_bwd_params(dt, false, T, d, Dc, M->e0, M->st_e, M->part, G(M->T_("lne_g")), G(M->T_("lne_b")), st));
      RW(RW_NORM_BWD_DX, 3.0 * T * d * es, norm_bwd_dx(dt, false, T, d, Dc, M->e0, M->W("lne_g"), M->st_e, nullptr, D1, st));
      dx = D1;
    }
    float* gpos = nullptr;
    const bool tied = c.tie_embeddings != 0;  // the table's gradient already holds its part as output matrix
    int64_t zero_cnt = tied ? 0 : te.count();
    if (!rms) {
      const Tensor& pe = M->T_("pos_emb");
      gpos = G(pe);
      zero_cnt += pe.count();  // pos_emb follows tok_emb in the layout
    }
    if (zero_cnt) RW(RW_EMBED_BWD, 1.0 * ((size_t)zero_cnt * 4), fill_zero(tied ? gpos : G(te), (size_t)zero_cnt * 4, st));
    RW(RW_EMBED_BWD, (double)T * d * (es + 4.0), embed_bwd(dt, bt->tokens, T, S, d, c.vocab, dx, G(te), gpos, tied, st));
  }
  return HIFT_OK;
}

void group_range(const hift_model* M, int gid, int* ulo, int* uhi, int64_t* plo, int64_t* pcnt) {
  const int lo = gid * M->m, hi = std::min((gid + 1) * M->m, M->lay.n_units);
  *ulo = lo;
  *uhi = hi;
  *plo = M->lay.unit_off[lo];
  int64_t c = 0;
  for (int u = lo; u < hi; ++u) c += M->lay.unit_cnt[u];
  *pcnt = c;
}

// One leg of the optimizer-state movement, on the host-to-device or device-to-host stream:
// hipMemcpyAsync (DMA engines) by default, or a copy kernel with a small fixed grid.  Any
// kernel that reads or writes host memory while the step runs slows the step's own kernels
// severely (measured: 4x on the contractions even with 16 workgroups), so the DMA path is the
// one to use; fetch_state keeps it on the DMA engines.
hift_status state_copy(hift_model* M, void* dst, const void* src, size_t bytes, bool to_device) {
  hipStream_t st = to_device ? M->hs : M->ds;
  if (M->copy_engine == 1 && bytes % 16 == 0 && (reinterpret_cast<uintptr_t>(dst) & 15) == 0 &&
      (reinterpret_cast<uintptr_t>(src) & 15) == 0) {
    HIP_TRY(copy_stream(dst, src, bytes, M->copy_blocks, st));
  } else {
    HIP_TRY(hipMemcpyAsync(dst, src, bytes, to_device ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost, st));
  }
  return HIFT_OK;
}

// Queue the host-to-device copy of a group's state into a slot (Algorithm 1 step i).
hift_status fetch_state(hift_model* M, int gid, int s) {
  int ulo, uhi;
  int64_t plo, cnt;
  group_range(M, gid, &ulo, &uhi, &plo, &cnt);
  // order the copy after the write-backs it depends on, and only those: the one that last
  // drained this slot, and one that carries this group's own state to the host
  for (int q = 0; q < NSLOT; ++q)
    if (M->d2h_pending[q] && (q == s || M->d2h_group[q] == gid)) HIP_TRY(hipStreamWaitEvent(M->hs, M->ev_d2h[q], 0));
  // keep one host-to-device transfer outstanding at the moment the next is submitted: the host
  // runs up to a step ahead of the GPU, and a copy submitted while the copy engine still has
  // a backlog is executed by a full-grid copy kernel instead, which starves the step's kernels
  if (M->copy_engine == 0 && M->h2d_last >= 0) HIP_TRY(hipEventSynchronize(M->ev_h2d[M->h2d_last]));
  for (int j = 0; j < M->n_move; ++j) {  // array j of the pinned range: the master first when it travels, then the state
    unsigned char* dst = reinterpret_cast<unsigned char*>(M->slot[s] + (size_t)j * M->grad_cap);
    ST_TRY(M->pin.pieces(((size_t)j * M->lay.n_params + plo) * 4, (size_t)cnt * 4, [&](unsigned char* h, size_t n, size_t at) {
      return state_copy(M, dst + at, h, n, true);
    }));
    M->h2d_bytes += (uint64_t)cnt * 4;
  }
  HIP_TRY(hipEventRecord(M->ev_h2d[s], M->hs));
  M->h2d_last = s;
  M->slot_group[s] = gid;
  return HIFT_OK;
}

hift_status sync_all(hift_model* M);

// Master on the host: rebuilds the bf16 forward copy of parameters [off, off+cnt) from the pinned
// master, one slot-sized piece at a time through the first slot (the streams must be idle).
hift_status load_forward_copy(hift_model* M, int64_t off, int64_t cnt) {
  for (int64_t done = 0; done < cnt; done += M->grad_cap) {
    const int64_t n = std::min<int64_t>(M->grad_cap, cnt - done);
    ST_TRY(M->pin.pieces((size_t)(off + done) * 4, (size_t)n * 4, [&](unsigned char* h, size_t nb, size_t at) {
      HIP_TRY(hipMemcpyAsync(reinterpret_cast<unsigned char*>(M->slot[0]) + at, h, nb, hipMemcpyHostToDevice, M->cs));
      return HIFT_OK;
    }));
    HIP_TRY(cast_f32_to(DT_BF16, n, M->slot[0], (unsigned char*)M->wc + (off + done) * 2, M->cs));
    HIP_TRY(hipStreamSynchronize(M->cs));
  }
  for (int& g : M->slot_group) g = -1;  // slot 0 no longer holds a group's state
  return HIFT_OK;
}

hift_status sync_all(hift_model* M) {
  HIP_TRY(hipStreamSynchronize(M->cs));
  HIP_TRY(hipStreamSynchronize(M->hs));
  HIP_TRY(hipStreamSynchronize(M->ds));
  for (bool& b : M->d2h_pending) b = false;
  return HIFT_OK;
}

hift_status unit_span(const hift_model* M, int ulo, int uhi, int64_t* off, int64_t* cnt) {
  if (ulo < 0 || uhi > M->lay.n_units || ulo >= uhi) return fail(HIFT_EINVAL, "unit range [%d,%d) invalid", ulo, uhi);
  *off = M->lay.unit_off[ulo];
  int64_t c = 0;
  for (int u = ulo; u < uhi; ++u) c += M->lay.unit_cnt[u];
  *cnt = c;
  return HIFT_OK;
}

}  // namespace

// ==========================================================================================
// C ABI
// ==========================================================================================
extern "C" {

const char* hift_last_error(void) { return g_err.c_str(); }

hift_status hift_group_count(int32_t n_units, int32_t m, int32_t* k_out) {
  if (n_units < 1 || m < 1 || !k_out) return fail(HIFT_EINVAL, "n_units and m must be >= 1");
  *k_out = group_count(n_units, m);
  return HIFT_OK;
}

hift_status hift_group_order(int32_t k, hift_strategy s, uint64_t seed, int32_t* order_out) {
  if (k < 1 || !order_out || (int)s < 0 || (int)s > 2) return fail(HIFT_EINVAL, "bad k, strategy or output");
  make_order(k, (int)s, seed, order_out);
  return HIFT_OK;
}

hift_status hift_tensor_count(const hift_config* cfg, int32_t* n_tensors, int64_t* n_params) {
  hift_status s = check_config(cfg);
  if (s != HIFT_OK) return s;
  Layout L;
  build_layout(*cfg, L);
  if (n_tensors) *n_tensors = (int32_t)L.t.size();
  if (n_params) *n_params = L.n_params;
  return HIFT_OK;
}

hift_status hift_tensor_at(const hift_config* cfg, int32_t index, hift_tensor_info* out) {
  hift_status s = check_config(cfg);
  if (s != HIFT_OK) return s;
  if (!out) return fail(HIFT_EINVAL, "out is null");
  Layout L;
  build_layout(*cfg, L);
  if (index < 0 || index >= (int)L.t.size()) return fail(HIFT_EINVAL, "tensor index %d out of range", index);
  const Tensor& t = L.t[index];
  memset(out, 0, sizeof *out);
  snprintf(out->name, sizeof out->name, "%s", t.name.c_str());
  out->unit = t.unit;
  out->kind = t.kind;
  out->offset = t.off;
  out->rows = t.rows;
  out->cols = t.cols;
  return HIFT_OK;
}

hift_status hift_query_bytes(const hift_config* cfg, const hift_opt* opt, int32_t m, int32_t max_batch,
                             int32_t max_seq, size_t* device_bytes, size_t* pinned_host_bytes) {
  hift_model M;
  hift_status s = init_model_shape(&M, cfg, opt, m, max_batch, max_seq);
  if (s != HIFT_OK) return s;
  carve(&M, nullptr, device_bytes, pinned_host_bytes);
  return HIFT_OK;
}

hift_status hift_memory_report(const hift_config* cfg, const hift_opt* opt, int32_t m, int32_t max_batch,
                               int32_t max_seq, hift_memory* out) {
  if (!out) return fail(HIFT_EINVAL, "out is null");
  hift_model M;
  hift_status s = init_model_shape(&M, cfg, opt, m, max_batch, max_seq);
  if (s != HIFT_OK) return s;
  size_t dev = 0, pin = 0, cat[MEM_N];
  carve(&M, nullptr, &dev, &pin, cat);
  memset(out, 0, sizeof(*out));
  out->device_master = cat[MEM_MASTER];
  out->device_forward = cat[MEM_FORWARD];
  out->device_packed = cat[MEM_PACKED];
  out->device_grad = cat[MEM_GRAD];
  out->device_state = cat[MEM_STATE];
  out->device_activations = cat[MEM_ACT];
  out->device_workspace = cat[MEM_WORK];
  out->device_total = dev;
  out->pinned_total = pin;
  out->para = out->device_master + out->device_forward + out->device_packed;
  out->gra = out->device_grad;
  out->sta = out->device_state;
  out->pgs = out->para + out->gra + out->sta;
  out->residual = out->device_activations + out->device_workspace;
  out->total = out->pgs + out->residual;
  out->n_params = (uint64_t)M.lay.n_params;
  out->peak_trainable = (uint64_t)largest_group(M.lay, m);
  out->k = group_count(M.lay.n_units, m);
  out->zeta1 = 4.0 * (double)M.lay.n_params;
  out->zeta_fpft = 4.0 * out->zeta1;
  out->zeta_hift = (out->k + 3.0) / out->k * out->zeta1;
  out->zeta_hift_peak = out->zeta1 + 12.0 * (double)out->peak_trainable;
  return HIFT_OK;
}

hift_status hift_model_create(const hift_config* cfg, const hift_opt* opt, int32_t m, int32_t max_batch,
                              int32_t max_seq, const float* init_params_host, void* device_arena,
                              size_t device_bytes, void* pinned_arena, size_t pinned_bytes, void* compute_stream,
                              void* h2d_stream, void* d2h_stream, hift_model** out) {
  void* chunks[1] = {pinned_arena};
  size_t sizes[1] = {pinned_bytes};
  return hift_model_create_chunked(cfg, opt, m, max_batch, max_seq, init_params_host, device_arena, device_bytes, chunks,
                                   sizes, pinned_arena ? 1 : 0, compute_stream, h2d_stream, d2h_stream, out);
}

hift_status hift_model_create_chunked(const hift_config* cfg, const hift_opt* opt, int32_t m, int32_t max_batch,
                                      int32_t max_seq, const float* init_params_host, void* device_arena,
                                      size_t device_bytes, void* const* pinned_chunks, const size_t* pinned_chunk_bytes,
                                      int32_t n_chunks, void* compute_stream, void* h2d_stream, void* d2h_stream,
                                      hift_model** out) {
  if (!out) return fail(HIFT_EINVAL, "out is null");
  *out = nullptr;
  hift_model* M = new hift_model();
  hift_status s = init_model_shape(M, cfg, opt, m, max_batch, max_seq);
  if (s != HIFT_OK) { delete M; return s; }
  size_t need_dev = 0, need_pin = 0;
  carve(M, nullptr, &need_dev, &need_pin);
  if (!device_arena || (reinterpret_cast<uintptr_t>(device_arena) & 255)) {
    delete M;
    return fail(HIFT_EINVAL, "device arena must be non-null and 256-byte aligned");
  }
  if (n_chunks < 0 || (n_chunks > 0 && (!pinned_chunks || !pinned_chunk_bytes))) {
    delete M;
    return fail(HIFT_EINVAL, "pinned chunks: negative count or null arrays");
  }
  for (int i = 0; i < n_chunks && M->pin.total < need_pin; ++i) {
    if (!pinned_chunks[i] || pinned_chunk_bytes[i] % 16 != 0 || (reinterpret_cast<uintptr_t>(pinned_chunks[i]) & 15)) {
      delete M;
      return fail(HIFT_EINVAL, "pinned chunk %d is null, not 16-byte aligned or not a multiple of 16 bytes long", i);
    }
    M->pin.add(pinned_chunks[i], std::min(pinned_chunk_bytes[i], need_pin - M->pin.total));
  }
  if (device_bytes < need_dev || M->pin.total < need_pin) {
    delete M;
    return fail(HIFT_ENOMEM, "arenas too small: need %zu device and %zu pinned bytes", need_dev, need_pin);
  }
  carve(M, device_arena, nullptr, nullptr);
  M->host_state_off = M->master_host ? (size_t)M->lay.n_params * 4 : 0;
  M->cs = (hipStream_t)compute_stream;
  M->hs = (hipStream_t)h2d_stream;
  M->ds = (hipStream_t)d2h_stream;
  auto bail = [&](hift_status st) { hift_model_destroy(M); return st; };
#define CR_TRY(expr)                                                                                  \
  do {                                                                                                \
    hipError_t e_ = (expr);                                                                           \
    if (e_ != hipSuccess) {                                                                           \
      fail(HIFT_EDEVICE, "%s failed: %s", #expr, hipGetErrorString(e_));                              \
      return bail(HIFT_EDEVICE);                                                                      \
    }                                                                                                 \
  } while (0)
  std::vector<hipEvent_t*> evs;
  for (int q = 0; q < NSLOT; ++q) { evs.push_back(&M->ev_h2d[q]); evs.push_back(&M->ev_opt[q]); evs.push_back(&M->ev_d2h[q]); }
  for (auto e : evs) *e = nullptr;
  M->ev_t0 = M->ev_t1 = M->ev_w0 = M->ev_w1 = nullptr;
  for (auto e : evs) CR_TRY(hipEventCreateWithFlags(e, hipEventDisableTiming));
  CR_TRY(hipEventCreate(&M->ev_t0));
  CR_TRY(hipEventCreate(&M->ev_t1));
  CR_TRY(hipEventCreate(&M->ev_w0));
  CR_TRY(hipEventCreate(&M->ev_w1));
  for (const PinnedSpace::Chunk& ch : M->pin.chunks) memset(ch.base, 0, ch.bytes);
  // state and gradient buffers start at zero
  if (M->state_full) CR_TRY(fill_zero(M->state_full, (size_t)M->n_state * M->lay.n_params * 4, M->cs));
  for (int q = 0; q < NSLOT; ++q)
    if (M->slot[q]) CR_TRY(fill_zero(M->slot[q], (size_t)M->n_move * M->grad_cap * 4, M->cs));
  CR_TRY(fill_zero(M->grad, (size_t)M->grad_cap * 4, M->cs));
  if (M->gemm_ws) CR_TRY(fill_zero(M->gemm_ws, 1024, M->cs));  // the counters; every launch leaves them at zero
  if (M->fac) CR_TRY(fill_zero(M->fac, (size_t)M->n_fac * 4, M->cs));
  if (M->lora_r > 0) {  // adapters start at zero (the model is the base model) until hift_lora_write; so do their moments
    CR_TRY(fill_zero(M->lora_master, (size_t)M->n_lora * 4, M->cs));
    if (M->dt == DT_BF16) CR_TRY(fill_zero(M->lora_wc, (size_t)M->n_lora * 2, M->cs));
    CR_TRY(fill_zero(M->lora_grad, (size_t)M->n_lora * 4, M->cs));
    CR_TRY(fill_zero(M->lora_m, (size_t)M->n_lora * 4, M->cs));
    CR_TRY(fill_zero(M->lora_v, (size_t)M->n_lora * 4, M->cs));
  }
  if (M->cos_sin) {
    const int hd2 = cfg->d_model / cfg->n_heads / 2;
    std::vector<float> tab((size_t)cfg->max_seq * hd2 * 2);
    for (int p = 0; p < cfg->max_seq; ++p)
      for (int i = 0; i < hd2; ++i) {
        const double ang = (double)p * pow((double)cfg->rope_base, -2.0 * i / (2.0 * hd2));
        tab[((size_t)p * hd2 + i) * 2] = (float)cos(ang);
        tab[((size_t)p * hd2 + i) * 2 + 1] = (float)sin(ang);
      }
    CR_TRY(hipMemcpyAsync(M->cos_sin, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, M->cs));
    CR_TRY(hipStreamSynchronize(M->cs));
  }
  if (M->master_host) {
    if (init_params_host && M->pin.write(0, init_params_host, (size_t)M->lay.n_params * 4) != HIFT_OK) return bail(HIFT_ESTATE);
    if (load_forward_copy(M, 0, M->lay.n_params) != HIFT_OK) return bail(HIFT_EDEVICE);
  } else {
    if (init_params_host) {
      CR_TRY(hipMemcpyAsync(M->master, init_params_host, (size_t)M->lay.n_params * 4, hipMemcpyHostToDevice, M->cs));
    } else {
      CR_TRY(fill_zero(M->master, (size_t)M->lay.n_params * 4, M->cs));
    }
    CR_TRY(cast_units(M, 0, M->lay.n_units));
  }
  CR_TRY(repack_units(M, 0, M->lay.n_units));
  CR_TRY(hipStreamSynchronize(M->cs));
#undef CR_TRY
  *out = M;
  return HIFT_OK;
}

void hift_model_destroy(hift_model* M) {
  if (!M) return;
  if (M->cs) (void)hipStreamSynchronize(M->cs);
  if (M->hs) (void)hipStreamSynchronize(M->hs);
  if (M->ds) (void)hipStreamSynchronize(M->ds);
  hipEvent_t evs[] = {M->ev_h2d[0], M->ev_h2d[1], M->ev_h2d[2], M->ev_opt[0], M->ev_opt[1], M->ev_opt[2], M->ev_d2h[0], M->ev_d2h[1], M->ev_d2h[2],
                      M->ev_t0, M->ev_t1, M->ev_w0, M->ev_w1};
  for (auto e : evs)
    if (e) (void)hipEventDestroy(e);
  for (auto& r : M->prof.pool) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  delete M;
}

hift_status hift_set_group_schedule(hift_model* M, hift_strategy s, int32_t m, uint64_t seed, int32_t* k_out) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (m < 1 || (int)s < 0 || (int)s > 2) return fail(HIFT_EINVAL, "bad m or strategy");
  const int64_t need = largest_group(M->lay, m);
  if (need > M->grad_cap) return fail(HIFT_ENOMEM, "largest group (%lld parameters) exceeds the buffers sized at creation (%lld)",
                                      (long long)need, (long long)M->grad_cap);
  hift_status st = sync_all(M);
  if (st != HIFT_OK) return st;
  // state held in a slot is already mirrored on the host (every step writes it back)
  for (int& g : M->slot_group) g = -1;
  M->m = m;
  M->k = group_count(M->lay.n_units, m);
  M->order.resize(M->k);
  make_order(M->k, (int)s, seed, M->order.data());
  M->t = 0;
  if (k_out) *k_out = M->k;
  return HIFT_OK;
}

hift_status hift_schedule_group_at(const hift_model* M, int64_t t, int32_t* gid) {
  if (!M || !gid) return fail(HIFT_EINVAL, "null argument");
  if (M->k == 0) return fail(HIFT_ESTATE, "no schedule set");
  if (t < 1) return fail(HIFT_EINVAL, "steps are numbered from 1");
  *gid = M->order[(t - 1) % M->k];
  return HIFT_OK;
}

hift_status hift_group_units(const hift_model* M, int32_t gid, int32_t* unit_lo, int32_t* unit_hi) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (M->k == 0) return fail(HIFT_ESTATE, "no schedule set");
  if (gid < 0 || gid >= M->k) return fail(HIFT_EINVAL, "group %d outside [0,%d)", gid, M->k);
  if (unit_lo) *unit_lo = gid * M->m;
  if (unit_hi) *unit_hi = std::min((gid + 1) * M->m, M->lay.n_units);
  return HIFT_OK;
}

hift_status hift_set_lr(hift_model* M, double lr) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  M->opt.lr = lr;
  return HIFT_OK;
}

hift_status hift_lr_at_cycle(int32_t kind, double base_lr, int64_t warmup, int64_t total, int64_t cycle, double* lr_out) {
  if (!lr_out) return fail(HIFT_EINVAL, "lr_out is null");
  if (kind != HIFT_LR_CONSTANT && kind != HIFT_LR_LINEAR) return fail(HIFT_EINVAL, "schedule kind %d unknown", kind);
  if (warmup < 0 || total < 0 || cycle < 0) return fail(HIFT_EINVAL, "warm-up, total and cycle must be >= 0");
  if (kind == HIFT_LR_CONSTANT) {
    *lr_out = base_lr;
  } else if (cycle < warmup) {
    *lr_out = base_lr * (double)cycle / (double)std::max<int64_t>(1, warmup);
  } else {
    *lr_out = base_lr * std::max(0.0, (double)(total - cycle) / (double)std::max<int64_t>(1, total - warmup));
  }
  return HIFT_OK;
}

hift_status hift_set_lr_schedule(hift_model* M, int32_t kind, double base_lr, int64_t warmup_cycles, int64_t total_cycles) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  double probe;
  ST_TRY(hift_lr_at_cycle(kind, base_lr, warmup_cycles, total_cycles, 0, &probe));
  M->lr_kind = kind;
  M->lr_base = base_lr;
  M->lr_warmup = warmup_cycles;
  M->lr_total = total_cycles;
  return HIFT_OK;
}

hift_status hift_train(hift_model* M, const hift_batch* batches, int32_t n_batches, int64_t n_steps, float* losses_out) {
  if (!M || !batches) return fail(HIFT_EINVAL, "null argument");
  if (M->k == 0) return fail(HIFT_ESTATE, "no schedule set");
  if (n_batches < 1 || n_steps < 0) return fail(HIFT_EINVAL, "n_batches must be >= 1 and n_steps >= 0");
  for (int64_t i = 0; i < n_steps; ++i) {
    if (M->lr_kind >= 0) {  // the rate moves only when a sweep over all groups is complete
      double lr;
      ST_TRY(hift_lr_at_cycle(M->lr_kind, M->lr_base, M->lr_warmup, M->lr_total, M->t / M->k, &lr));
      M->opt.lr = lr;
    }
    const int32_t gid = M->order[M->t % M->k];
    ST_TRY(hift_step(M, &batches[i % n_batches], gid, losses_out ? losses_out + i : nullptr));
  }
  return HIFT_OK;
}

// ---- checkpoint: everything a run needs to continue as if it had not stopped ----
namespace {
struct CkptHeader {
  char magic[8];
  int64_t n_params, n_fac, t;
  int32_t version, n_state, k, m, lr_kind, opt_kind;
  double lr, lr_base;
  int64_t lr_warmup, lr_total;
};
constexpr char CKPT_MAGIC[8] = {'H', 'I', 'F', 'T', 'C', 'K', 'P', '2'};

size_t ckpt_bytes(const hift_model* M) {
  return sizeof(CkptHeader) + (size_t)M->k * 4 + (size_t)M->lay.n_units * 8 +
         ((size_t)M->lay.n_params * (1 + M->n_state) + (size_t)M->n_fac) * 4;
}
}  // namespace

hift_status hift_checkpoint_bytes(const hift_model* M, size_t* bytes) {
  if (!M || !bytes) return fail(HIFT_EINVAL, "null argument");
  if (M->k == 0) return fail(HIFT_ESTATE, "no schedule set");
  *bytes = ckpt_bytes(M);
  return HIFT_OK;
}

hift_status hift_checkpoint_save(hift_model* M, void* host_buffer, size_t bytes) {
  if (!M || !host_buffer) return fail(HIFT_EINVAL, "null argument");
  if (M->k == 0) return fail(HIFT_ESTATE, "no schedule set");
  if (bytes < ckpt_bytes(M)) return fail(HIFT_ENOMEM, "buffer holds %zu bytes, the checkpoint needs %zu", bytes, ckpt_bytes(M));
  ST_TRY(sync_all(M));  // every write-back has landed: the host copies of state (and master) are current
  unsigned char* p = reinterpret_cast<unsigned char*>(host_buffer);
  CkptHeader h{};
  memcpy(h.magic, CKPT_MAGIC, 8);
  h.n_params = M->lay.n_params; h.n_fac = M->n_fac; h.t = M->t;
  h.version = 2; h.n_state = M->n_state; h.k = M->k; h.m = M->m; h.lr_kind = M->lr_kind; h.opt_kind = M->opt.kind;
  h.lr = M->opt.lr; h.lr_base = M->lr_base; h.lr_warmup = M->lr_warmup; h.lr_total = M->lr_total;
  memcpy(p, &h, sizeof(h)); p += sizeof(h);
  memcpy(p, M->order.data(), (size_t)M->k * 4); p += (size_t)M->k * 4;
  memcpy(p, M->unit_steps.data(), (size_t)M->lay.n_units * 8); p += (size_t)M->lay.n_units * 8;
  const size_t np4 = (size_t)M->lay.n_params * 4;
  if (M->master_host) ST_TRY(M->pin.read(p, 0, np4));
  else HIP_TRY(hipMemcpy(p, M->master, np4, hipMemcpyDeviceToHost));
  p += np4;
  for (int j = 0; j < M->n_state; ++j, p += np4) {
    if (M->on_host) ST_TRY(M->pin.read(p, M->host_state_off + (size_t)j * np4, np4));
    else HIP_TRY(hipMemcpy(p, M->state_full + (size_t)j * M->lay.n_params, np4, hipMemcpyDeviceToHost));
  }
  if (M->n_fac) HIP_TRY(hipMemcpy(p, M->fac, (size_t)M->n_fac * 4, hipMemcpyDeviceToHost));
  return HIFT_OK;
}

hift_status hift_checkpoint_load(hift_model* M, const void* host_buffer, size_t bytes) {
  if (!M || !host_buffer) return fail(HIFT_EINVAL, "null argument");
  if (bytes < sizeof(CkptHeader)) return fail(HIFT_EINVAL, "buffer too small for a checkpoint header");
  const unsigned char* p = reinterpret_cast<const unsigned char*>(host_buffer);
  CkptHeader h;
  memcpy(&h, p, sizeof(h)); p += sizeof(h);
  if (memcmp(h.magic, CKPT_MAGIC, 8) != 0 || h.version != 2) return fail(HIFT_EINVAL, "not a checkpoint of this library");
  if (h.n_params != M->lay.n_params || h.n_state != M->n_state || h.n_fac != M->n_fac || h.opt_kind != M->opt.kind)
    return fail(HIFT_EINVAL, "checkpoint is of another model or optimizer (%lld parameters, %d state arrays)",
                (long long)h.n_params, h.n_state);
  if (h.k < 1 || h.m < 1 || h.k != group_count(M->lay.n_units, h.m) || largest_group(M->lay, h.m) > M->grad_cap)
    return fail(HIFT_EINVAL, "checkpoint grouping (m = %d, k = %d) does not fit this model's buffers", h.m, h.k);
  const size_t np4 = (size_t)M->lay.n_params * 4;
  const size_t nu = (size_t)M->lay.n_units;
  const size_t need = sizeof(CkptHeader) + (size_t)h.k * 4 + nu * 8 + np4 * (1 + (size_t)M->n_state) + (size_t)M->n_fac * 4;
  if (bytes < need) return fail(HIFT_EINVAL, "buffer holds %zu bytes, the checkpoint has %zu", bytes, need);
  // everything is checked before the model is touched: a damaged checkpoint leaves it as it was
  std::vector<int32_t> order(h.k);
  memcpy(order.data(), p, (size_t)h.k * 4); p += (size_t)h.k * 4;
  std::vector<int64_t> usteps(nu);
  memcpy(usteps.data(), p, nu * 8); p += nu * 8;
  std::vector<char> seen(h.k, 0);
  for (int i = 0; i < h.k; ++i) {
    if (order[i] < 0 || order[i] >= h.k || seen[order[i]]) return fail(HIFT_EINVAL, "checkpoint order is damaged");
    seen[order[i]] = 1;
  }
  for (size_t u = 0; u < nu; ++u)
    if (usteps[u] < 0) return fail(HIFT_EINVAL, "checkpoint update counts are damaged");
  if (h.t < 0 || h.lr_kind < -1 || h.lr_kind > HIFT_LR_LINEAR) return fail(HIFT_EINVAL, "checkpoint header is damaged");
  ST_TRY(sync_all(M));
  M->m = h.m; M->k = h.k; M->t = h.t;
  M->order = order;
  M->unit_steps = usteps;
  M->opt.lr = h.lr; M->lr_kind = h.lr_kind; M->lr_base = h.lr_base; M->lr_warmup = h.lr_warmup; M->lr_total = h.lr_total;
  ST_TRY(hift_write_params(M, 0, M->lay.n_units, reinterpret_cast<const float*>(p), (size_t)M->lay.n_params));
  p += np4;
  for (int j = 0; j < M->n_state; ++j, p += np4) {
    if (M->on_host) ST_TRY(M->pin.write(M->host_state_off + (size_t)j * np4, p, np4));
    else HIP_TRY(hipMemcpy(M->state_full + (size_t)j * M->lay.n_params, p, np4, hipMemcpyHostToDevice));
  }
  if (M->n_fac) HIP_TRY(hipMemcpy(M->fac, p, (size_t)M->n_fac * 4, hipMemcpyHostToDevice));
  for (int& g : M->slot_group) g = -1;  // whatever the slots hold is stale
  return HIFT_OK;
}

hift_status hift_cycle_index(const hift_model* M, int64_t* steps_done, int64_t* cycles_done) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (M->k == 0) return fail(HIFT_ESTATE, "no schedule set");
  if (steps_done) *steps_done = M->t;
  if (cycles_done) *cycles_done = M->t / M->k;
  return HIFT_OK;
}

hift_status hift_step(hift_model* M, const hift_batch* bt, int32_t gid, float* loss_out) {
  if (!M || !bt) return fail(HIFT_EINVAL, "null argument");
  if (M->k == 0) return fail(HIFT_ESTATE, "no schedule set");
  if (gid < 0 || gid >= M->k) return fail(HIFT_EINVAL, "group %d outside [0,%d)", gid, M->k);
  if (bt->batch < 1 || bt->seq < 1 || bt->batch > M->max_batch || bt->seq > M->max_seq_len)
    return fail(HIFT_EINVAL, "batch %d x seq %d outside the maxima %d x %d", bt->batch, bt->seq, M->max_batch,
                M->max_seq_len);
  if (!bt->tokens || !bt->labels) return fail(HIFT_EINVAL, "tokens or labels null");
  if (M->lora_r > 0) return fail(HIFT_ESTATE, "a model with adapters trains its adapters: use hift_lora_step");
  int ulo, uhi;
  int64_t plo, cnt;
  group_range(M, gid, &ulo, &uhi, &plo, &cnt);
  const bool moving = M->on_host && M->n_move > 0;
  HIP_TRY(hipEventRecord(M->ev_t0, M->cs));

  // ---- state movement, queued ahead of the compute (Algorithm 1 step i, issued early) ----
  int s = 0;
  if (moving) {
    s = -1;
    for (int q = 0; q < NSLOT; ++q)
      if (M->slot_group[q] == gid) s = q;
    if (s < 0) {
      s = M->cur_slot;
      ST_TRY(fetch_state(M, gid, s));
    }
    // a slot reused without a new fetch may still be draining to the host from its last update
    if (M->d2h_pending[s]) HIP_TRY(hipStreamWaitEvent(M->cs, M->ev_d2h[s], 0));
    M->cur_slot = s;
    // prefetch the state of the group the schedule visits next into the slot after this one (the
    // one after that is still draining the previous group's state); the write-back that last used
    // the slot is ordered before the copy inside fetch_state
    const int next = M->order[(M->t + 1) % M->k];
    const bool on_schedule = M->order[M->t % M->k] == gid;
    bool resident = false;
    for (int q = 0; q < NSLOT; ++q) resident = resident || M->slot_group[q] == next;
    if (on_schedule && !resident) ST_TRY(fetch_state(M, next, (s + 1) % NSLOT));
  }

  ST_TRY(forward(M, bt, ulo));
  ST_TRY(backward(M, bt, ulo, uhi, plo));

  // ---- optimizer on the group (its update number drives AdamW's bias correction) ----
  HIP_TRY(hipEventRecord(M->ev_w0, M->cs));
  if (moving) HIP_TRY(hipStreamWaitEvent(M->cs, M->ev_h2d[s], 0));
  HIP_TRY(hipEventRecord(M->ev_w1, M->cs));
  for (int u = ulo; u < uhi; ++u) M->unit_steps[u] += 1;
  OptArgs oa{M->opt.kind, M->opt.lr, M->opt.beta1, M->opt.beta2, M->opt.eps, M->opt.weight_decay, M->opt.momentum};
  float *s1b = nullptr, *s2b = nullptr;
  int64_t sbase = plo;  // state index = parameter offset - sbase
  float* mbase = M->master_host ? M->slot[s] - plo : M->master;  // master of parameter i at mbase[i]
  if (M->n_state > 0) {
    if (moving) {
      s1b = M->slot[s] + (size_t)(M->master_host ? 1 : 0) * M->grad_cap;
      s2b = s1b + M->grad_cap;
    } else {
      s1b = M->state_full;
      s2b = M->state_full + M->lay.n_params;
      sbase = 0;
    }
  }
  {
    double bytes_per = M->n_state == 2 ? 28.0 : (M->n_state == 1 ? 20.0 : 12.0);
    if (M->opt.kind == HIFT_ADAFACTOR) bytes_per = 24.0;  // the gradient is read four times (row, column, clipping, update)
    if (M->dt == DT_BF16) bytes_per += 2.0;
    Scope sc(M, CAT_OPT, bytes_per * cnt);
    for (int i = M->lay.unit_first[ulo]; i < M->lay.unit_first[uhi]; ++i) {
      const Tensor& t = M->lay.t[i];
      const int64_t tg = M->unit_steps[t.unit];
      void* cc = M->dt == DT_BF16 ? M->W(t) : nullptr;  // null also for a matrix kept only in fragment order
      if (M->opt.kind == HIFT_ADAFACTOR) {
        K_TRY(adafactor_update(M->opt.lr, M->opt.weight_decay, t.kind == HIFT_KIND_MATRIX, tg, t.rows, t.cols,
                               mbase + t.off, M->grad + (t.off - plo), M->fac + t.fac_off, M->af_work, cc, M->cs));
        continue;
      }
      K_TRY(optimizer_update(oa, t.count(), t.kind == HIFT_KIND_MATRIX, tg, mbase + t.off,
                             M->grad + (t.off - plo), s1b ? s1b + (t.off - sbase) : nullptr,
                             (s2b && M->n_state == 2) ? s2b + (t.off - sbase) : nullptr, cc, M->cs));
    }
  }
  if (moving) HIP_TRY(hipEventRecord(M->ev_opt[s], M->cs));
  if (M->wpk) {  // the updated matrices in fragment order, for the next forward and dX
    double bytes = 0;
    for (int i = M->lay.unit_first[ulo]; i < M->lay.unit_first[uhi]; ++i)
      // per copy: the source read once (fp32 master, or the bf16 copy where one is kept) and the copy written once
      bytes += ((M->lay.t[i].wc_off < 0 ? 4.0 : 2.0) + 2.0) * M->lay.t[i].count() *
               ((M->lay.t[i].pk_fwd >= 0) + (M->lay.t[i].pk_bwd >= 0));
    Scope sc(M, CAT_PACK, bytes);
    K_TRY(repack_units(M, ulo, uhi));
  }
  HIP_TRY(hipEventRecord(M->ev_t1, M->cs));
  M->timed = true;

  // ---- state back to the host (Algorithm 1 step k) ----
  if (moving) {
    HIP_TRY(hipStreamWaitEvent(M->ds, M->ev_opt[s], 0));
    for (int j = 0; j < M->n_move; ++j) {
      const unsigned char* src = reinterpret_cast<const unsigned char*>(M->slot[s] + (size_t)j * M->grad_cap);
      ST_TRY(M->pin.pieces(((size_t)j * M->lay.n_params + plo) * 4, (size_t)cnt * 4, [&](unsigned char* h, size_t n, size_t at) {
        return state_copy(M, h, src + at, n, false);
      }));
      M->d2h_bytes += (uint64_t)cnt * 4;
    }
    HIP_TRY(hipEventRecord(M->ev_d2h[s], M->ds));
    M->d2h_pending[s] = true;
    M->d2h_group[s] = gid;
    M->cur_slot = (s + 1) % NSLOT;
  }
  M->t += 1;
  if (loss_out) {
    HIP_TRY(hipMemcpyAsync(loss_out, M->loss_dev, 4, hipMemcpyDeviceToHost, M->cs));
    HIP_TRY(hipStreamSynchronize(M->cs));
  }
  return HIFT_OK;
}

// ---- low-rank adapters -------------------------------------------------------------------------------------
hift_status hift_lora_param_count(const hift_config* cfg, int64_t* n) {
  hift_status s = check_config(cfg);
  if (s != HIFT_OK) return s;
  if (!n) return fail(HIFT_EINVAL, "n is null");
  *n = (int64_t)cfg->n_layers * 4 * cfg->lora_rank * cfg->d_model;
  return HIFT_OK;
}

hift_status hift_lora_write(hift_model* M, const float* src, size_t count) {
  if (!M || !src) return fail(HIFT_EINVAL, "null argument");
  if (M->lora_r == 0) return fail(HIFT_ESTATE, "the model has no adapters");
  if ((int64_t)count != M->n_lora) return fail(HIFT_EINVAL, "buffer holds %zu floats, the adapters hold %lld", count, (long long)M->n_lora);
  ST_TRY(sync_all(M));
  HIP_TRY(hipMemcpy(M->lora_master, src, count * 4, hipMemcpyHostToDevice));
  if (M->dt == DT_BF16) HIP_TRY(cast_f32_to(DT_BF16, M->n_lora, M->lora_master, M->lora_wc, M->cs));
  HIP_TRY(hipStreamSynchronize(M->cs));
  return HIFT_OK;
}

hift_status hift_lora_read(hift_model* M, int32_t which, float* dst, size_t count) {
  if (!M || !dst) return fail(HIFT_EINVAL, "null argument");
  if (M->lora_r == 0) return fail(HIFT_ESTATE, "the model has no adapters");
  if ((int64_t)count != M->n_lora) return fail(HIFT_EINVAL, "buffer holds %zu floats, the adapters hold %lld", count, (long long)M->n_lora);
  if (which < 0 || which > 3) return fail(HIFT_EINVAL, "which must be 0 (master), 1 (compute copy), 2 or 3 (AdamW moments)");
  ST_TRY(sync_all(M));
  if (which == 1 && M->dt == DT_BF16) {
    std::vector<uint16_t> tmp(count);
    HIP_TRY(hipMemcpy(tmp.data(), M->lora_wc, count * 2, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < count; ++i) {
      const uint32_t u = (uint32_t)tmp[i] << 16;
      memcpy(dst + i, &u, 4);
    }
    return HIFT_OK;
  }
  const float* src = which <= 1 ? M->lora_master : (which == 2 ? M->lora_m : M->lora_v);
  HIP_TRY(hipMemcpy(dst, src, count * 4, hipMemcpyDeviceToHost));
  return HIFT_OK;
}

hift_status hift_lora_step(hift_model* M, const hift_batch* bt, float* loss_out) {
  if (!M || !bt) return fail(HIFT_EINVAL, "null argument");
  if (M->lora_r == 0) return fail(HIFT_ESTATE, "the model has no adapters");
  if (M->opt.kind != HIFT_ADAMW) return fail(HIFT_ESTATE, "adapters are trained with AdamW");
  if (bt->batch < 1 || bt->seq < 1 || bt->batch > M->max_batch || bt->seq > M->max_seq_len)
    return fail(HIFT_EINVAL, "batch %d x seq %d outside the maxima %d x %d", bt->batch, bt->seq, M->max_batch, M->max_seq_len);
  if (!bt->tokens || !bt->labels) return fail(HIFT_EINVAL, "tokens or labels null");
  HIP_TRY(hipEventRecord(M->ev_t0, M->cs));
  // forward over everything; backward down to the first hidden layer (no unit of the base model is active: no
  // weight gradient of the base is formed, and the first layer's input needs no gradient)
  ST_TRY(forward(M, bt, 1));
  ST_TRY(backward(M, bt, 1, 1, 0));
  M->lora_t += 1;
  {
    const double bytes_per = 28.0 + (M->dt == DT_BF16 ? 2.0 : 0.0);
    Scope sc(M, CAT_OPT, bytes_per * M->n_lora);
    OptArgs oa{M->opt.kind, M->opt.lr, M->opt.beta1, M->opt.beta2, M->opt.eps, M->opt.weight_decay, M->opt.momentum};
    K_TRY(optimizer_update(oa, M->n_lora, true, M->lora_t, M->lora_master, M->lora_grad, M->lora_m, M->lora_v,
                           M->dt == DT_BF16 ? M->lora_wc : nullptr, M->cs));
  }
  HIP_TRY(hipEventRecord(M->ev_w0, M->cs));
  HIP_TRY(hipEventRecord(M->ev_w1, M->cs));
  HIP_TRY(hipEventRecord(M->ev_t1, M->cs));
  M->timed = true;
  if (loss_out) {
    HIP_TRY(hipMemcpyAsync(loss_out, M->loss_dev, 4, hipMemcpyDeviceToHost, M->cs));
    HIP_TRY(hipStreamSynchronize(M->cs));
  }
  return HIFT_OK;
}

hift_status hift_read_params(hift_model* M, int32_t ulo, int32_t uhi, int32_t which, float* dst, size_t dst_count) {
  if (!M || !dst) return fail(HIFT_EINVAL, "null argument");
  int64_t off, cnt;
  ST_TRY(unit_span(M, ulo, uhi, &off, &cnt));
  if ((int64_t)dst_count != cnt) return fail(HIFT_EINVAL, "buffer holds %zu floats, units hold %lld", dst_count, (long long)cnt);
  if (which != 0 && which != 1) return fail(HIFT_EINVAL, "which must be 0 or 1");
  ST_TRY(sync_all(M));
  if (which == 0 && M->master_host) {
    ST_TRY(M->pin.read(dst, (size_t)off * 4, (size_t)cnt * 4));  // every write-back has landed
  } else if (which == 0 || M->dt == DT_F32) {
    HIP_TRY(hipMemcpy(dst, M->master + off, (size_t)cnt * 4, hipMemcpyDeviceToHost));
  } else {
    // tensor by tensor: from the bf16 copy, or, for a matrix kept only in fragment order, the master rounded to
    // nearest even, which is what its copies hold
    std::vector<uint16_t> tmp;
    for (int i = M->lay.unit_first[ulo]; i < M->lay.unit_first[uhi]; ++i) {
      const Tensor& t = M->lay.t[i];
      float* out = dst + (t.off - off);
      if (t.wc_off >= 0) {
        tmp.resize((size_t)t.count());
        HIP_TRY(hipMemcpy(tmp.data(), M->W(t), (size_t)t.count() * 2, hipMemcpyDeviceToHost));
        for (int64_t e = 0; e < t.count(); ++e) {
          const uint32_t u = (uint32_t)tmp[e] << 16;
          memcpy(out + e, &u, 4);
        }
      } else {
        HIP_TRY(hipMemcpy(out, M->master + t.off, (size_t)t.count() * 4, hipMemcpyDeviceToHost));
        for (int64_t e = 0; e < t.count(); ++e) {
          uint32_t u;
          memcpy(&u, out + e, 4);
          if ((u & 0x7F800000u) != 0x7F800000u) u += 0x7FFFu + ((u >> 16) & 1u);  // nearest even; inf / nan stay
          u &= 0xFFFF0000u;
          memcpy(out + e, &u, 4);
        }
      }
    }
  }
  return HIFT_OK;
}

namespace {
hift_status write_params_from(hift_model* M, int32_t ulo, int32_t uhi, const float* src, size_t src_count, bool src_on_device) {
  if (!M || !src) return fail(HIFT_EINVAL, "null argument");
  int64_t off, cnt;
  ST_TRY(unit_span(M, ulo, uhi, &off, &cnt));
  if ((int64_t)src_count != cnt) return fail(HIFT_EINVAL, "buffer holds %zu floats, units hold %lld", src_count, (long long)cnt);
  ST_TRY(sync_all(M));
  if (M->master_host) {
    if (src_on_device) {
      ST_TRY(M->pin.pieces((size_t)off * 4, (size_t)cnt * 4, [&](unsigned char* h, size_t n, size_t at) {
        HIP_TRY(hipMemcpy(h, reinterpret_cast<const unsigned char*>(src) + at, n, hipMemcpyDeviceToHost));
        return HIFT_OK;
      }));
    } else {
      ST_TRY(M->pin.write((size_t)off * 4, src, (size_t)cnt * 4));
    }
    ST_TRY(load_forward_copy(M, off, cnt));
    HIP_TRY(repack_units(M, ulo, uhi));
    HIP_TRY(hipStreamSynchronize(M->cs));
    return HIFT_OK;
  }
  // a device-to-device copy does not wait on the host: it goes on the compute stream, in front of the cast that reads it
  if (src_on_device) HIP_TRY(hipMemcpyAsync(M->master + off, src, (size_t)cnt * 4, hipMemcpyDeviceToDevice, M->cs));
  else HIP_TRY(hipMemcpy(M->master + off, src, (size_t)cnt * 4, hipMemcpyHostToDevice));
  if (M->dt != DT_BF16) HIP_TRY(hipStreamSynchronize(M->cs));
  if (M->dt == DT_BF16) {
    HIP_TRY(cast_units(M, ulo, uhi));
    HIP_TRY(repack_units(M, ulo, uhi));
    HIP_TRY(hipStreamSynchronize(M->cs));
  }
  return HIFT_OK;
}
}  // namespace

hift_status hift_write_params(hift_model* M, int32_t ulo, int32_t uhi, const float* src, size_t src_count) {
  return write_params_from(M, ulo, uhi, src, src_count, false);
}

hift_status hift_write_params_device(hift_model* M, int32_t ulo, int32_t uhi, const float* src_device, size_t src_count) {
  return write_params_from(M, ulo, uhi, src_device, src_count, true);
}

hift_status hift_read_state(hift_model* M, int32_t ulo, int32_t uhi, int32_t slot, float* dst, size_t dst_count) {
  if (!M || !dst) return fail(HIFT_EINVAL, "null argument");
  int64_t off, cnt;
  ST_TRY(unit_span(M, ulo, uhi, &off, &cnt));
  if ((int64_t)dst_count != cnt) return fail(HIFT_EINVAL, "buffer holds %zu floats, units hold %lld", dst_count, (long long)cnt);
  if (slot < 0 || slot >= M->n_state) return fail(HIFT_EINVAL, "state slot %d outside [0,%d)", slot, M->n_state);
  ST_TRY(sync_all(M));
  if (M->on_host) {
    ST_TRY(M->pin.read(dst, M->host_state_off + ((size_t)slot * M->lay.n_params + off) * 4, (size_t)cnt * 4));  // write-back has landed
  } else {
    HIP_TRY(hipMemcpy(dst, M->state_full + (size_t)slot * M->lay.n_params + off, (size_t)cnt * 4, hipMemcpyDeviceToHost));
  }
  return HIFT_OK;
}

hift_status hift_read_factored_state(hift_model* M, int32_t tensor_index, float* dst, size_t dst_count) {
  if (!M || !dst) return fail(HIFT_EINVAL, "null argument");
  if (!M->fac) return fail(HIFT_ESTATE, "the optimizer keeps no factored statistics");
  if (tensor_index < 0 || tensor_index >= (int)M->lay.t.size()) return fail(HIFT_EINVAL, "tensor %d outside [0,%zu)", tensor_index, M->lay.t.size());
  const Tensor& t = M->lay.t[tensor_index];
  if ((int64_t)dst_count != t.fac_count()) return fail(HIFT_EINVAL, "buffer holds %zu floats, the tensor has %lld statistics", dst_count, (long long)t.fac_count());
  ST_TRY(sync_all(M));
  HIP_TRY(hipMemcpy(dst, M->fac + t.fac_off, (size_t)t.fac_count() * 4, hipMemcpyDeviceToHost));
  return HIFT_OK;
}

hift_status hift_transfer_stats(hift_model* M, uint64_t* h2d, uint64_t* d2h) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (h2d) *h2d = M->h2d_bytes;
  if (d2h) *d2h = M->d2h_bytes;
  return HIFT_OK;
}

hift_status hift_last_step_ms(hift_model* M, float* step_ms, float* exposed_copy_ms) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (!M->timed) return fail(HIFT_ESTATE, "no step taken yet");
  ST_TRY(sync_all(M));
  if (step_ms) HIP_TRY(hipEventElapsedTime(step_ms, M->ev_t0, M->ev_t1));
  if (exposed_copy_ms) HIP_TRY(hipEventElapsedTime(exposed_copy_ms, M->ev_w0, M->ev_w1));
  return HIFT_OK;
}

hift_status hift_set_state_copy_engine(hift_model* M, int32_t engine, int32_t blocks) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (engine < 0 || engine > 1 || blocks < 1 || blocks > 1024) return fail(HIFT_EINVAL, "engine must be 0 or 1, blocks in [1,1024]");
  ST_TRY(sync_all(M));
  M->copy_engine = engine;
  M->copy_blocks = blocks;
  return HIFT_OK;
}

hift_status hift_profile_enable(hift_model* M, int32_t on) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  ST_TRY(sync_all(M));
  M->prof.on = on != 0;
  M->prof.used = 0;
  return HIFT_OK;
}

hift_status hift_profile_read(hift_model* M, int32_t category, int64_t* launches, double* total_ms, double* work) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (category < 0 || category >= CAT_N) return fail(HIFT_EINVAL, "category outside [0,%d)", CAT_N);
  ST_TRY(sync_all(M));
  int64_t n = 0;
  double ms = 0, w = 0;
  for (size_t i = 0; i < M->prof.used; ++i) {
    const Prof::Rec& r = M->prof.pool[i];
    if (r.cat != category) continue;
    float e = 0.f;
    HIP_TRY(hipEventElapsedTime(&e, r.a, r.b));
    ms += e;
    w += r.work;
    ++n;
  }
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  if (work) *work = w;
  return HIFT_OK;
}

hift_status hift_profile_read_rowwise(hift_model* M, int32_t kind, const char** name, int64_t* launches, double* total_ms,
                                      double* bytes) {
  if (!M) return fail(HIFT_EINVAL, "model is null");
  if (kind < 0 || kind >= RW_N) return fail(HIFT_EINVAL, "kind outside [0,%d)", RW_N);
  ST_TRY(sync_all(M));
  int64_t n = 0;
  double ms = 0, w = 0;
  for (size_t i = 0; i < M->prof.used; ++i) {
    const Prof::Rec& r = M->prof.pool[i];
    if (r.cat != CAT_ELEM || r.sub != kind) continue;
    float e = 0.f;
    HIP_TRY(hipEventElapsedTime(&e, r.a, r.b));
    ms += e;
    w += r.work;
    ++n;
  }
  if (name) *name = RW_NAMES[kind];
  if (launches) *launches = n;
  if (total_ms) *total_ms = ms;
  if (bytes) *bytes = w;
  return HIFT_OK;
}

// ---- single kernels ------------------------------------------------------------------------
hift_status hift_kernel_gemm(int32_t dtype, int32_t a_kmajor, int32_t b_kmajor, int32_t out_f32, int64_t Mm,
                             int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                             int64_t ldc, const void* bias, const void* R, int32_t batch, int64_t sa, int64_t sb,
                             int64_t sc, void* stream) {
  if (dtype != HIFT_F32 && dtype != HIFT_BF16) return fail(HIFT_EINVAL, "dtype unknown");
  if (Mm < 0 || N < 0 || K < 0 || batch < 0) return fail(HIFT_EINVAL, "negative size");
  if ((Mm > 0 && N > 0) && (!A || !B || !C) && K > 0) return fail(HIFT_EINVAL, "null operand");
  if (lda < (a_kmajor ? K : Mm) || ldb < (b_kmajor ? K : N) || ldc < N)
    return fail(HIFT_EINVAL, "a leading dimension is shorter than the rows it strides over");
  Gemm g;
  g.dtype = dtype == HIFT_BF16 ? DT_BF16 : DT_F32;
  g.a_kmajor = a_kmajor != 0; g.b_kmajor = b_kmajor != 0; g.out_f32 = out_f32 != 0 || dtype == HIFT_F32;
  g.M = Mm; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.bias = bias; g.R = R; g.ldr = ldc;
  g.nb = batch; g.nh = 1; g.sa1 = sa; g.sb1 = sb; g.sc1 = sc;
  HIP_TRY(gemm(g, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_packed_bytes(int64_t N, int64_t K, size_t* bytes) {
  if (!bytes || N < 0 || K < 0) return fail(HIFT_EINVAL, "bad argument");
  *bytes = packed_b_bytes(N, K);
  return HIFT_OK;
}

hift_status hift_kernel_pack_b(int32_t b_kmajor, int64_t N, int64_t K, const void* B, int64_t ldb, void* Bp,
                               void* stream) {
  if (!B || !Bp) return fail(HIFT_EINVAL, "null operand");
  if (packed_b_bytes(N, K) == 0) return fail(HIFT_EINVAL, "shape cannot be packed (N >= 256, K a multiple of 32)");
  if (ldb < (b_kmajor ? K : N)) return fail(HIFT_EINVAL, "ldb is shorter than a row of B in the layout named");
  HIP_TRY(pack_b(B, ldb, N, K, b_kmajor != 0, Bp, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_gemm_packed(int32_t out_f32, int64_t Mm, int64_t N, int64_t K, const void* A, int64_t lda,
                                    const void* Bp, void* C, int64_t ldc, const void* bias, const void* R,
                                    void* stream) {
  if (!A || !Bp || !C) return fail(HIFT_EINVAL, "null operand");
  Gemm g;
  g.dtype = DT_BF16;
  g.out_f32 = out_f32 != 0;
  g.M = Mm; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.C = C; g.ldc = ldc; g.bias = bias; g.R = R; g.ldr = ldc;
  if (!packed_gemm_applies(g)) return fail(HIFT_EINVAL, "problem is not one the packed-operand kernel takes");
  HIP_TRY(gemm_packed(g, Bp, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_packed_workspace_bytes(size_t* bytes) {
  if (!bytes) return fail(HIFT_EINVAL, "bytes is null");
  *bytes = PACKED_WS_BYTES;
  return HIFT_OK;
}

hift_status hift_kernel_gemm_packed_ws(int32_t out_f32, int64_t Mm, int64_t N, int64_t K, const void* A, int64_t lda,
                                       const void* Bp, void* C, int64_t ldc, const void* bias, const void* R,
                                       void* workspace, size_t workspace_bytes, void* stream) {
  if (!A || !Bp || !C || !workspace) return fail(HIFT_EINVAL, "null operand");
  if (workspace_bytes < PACKED_WS_BYTES || (reinterpret_cast<uintptr_t>(workspace) & 15) != 0)
    return fail(HIFT_EINVAL, "work space too small or not 16-byte aligned");
  Gemm g;
  g.dtype = DT_BF16;
  g.out_f32 = out_f32 != 0;
  g.M = Mm; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.C = C; g.ldc = ldc; g.bias = bias; g.R = R; g.ldr = ldc;
  g.ws = workspace;
  if (!packed_gemm_applies(g)) return fail(HIFT_EINVAL, "problem is not one the packed-operand kernel takes");
  HIP_TRY(gemm_packed(g, Bp, (hipStream_t)stream));
  return HIFT_OK;
}

// Work space of hift_kernel_gemm_packed_static: one array per GPU, held from the moment the library is loaded.
// In host code the name is only a handle for hipGetSymbolAddress; kernels are given the address it returns.
static __device__ __align__(256) unsigned char scratch[PACKED_WS_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
void* g_scratch_ptr[MAX_DEVICES];  // device address of `scratch` on each GPU, once asked for
}  // namespace

hift_status hift_kernel_gemm_packed_static(int32_t out_f32, int64_t Mm, int64_t N, int64_t K, const void* A, int64_t lda,
                                           const void* Bp, void* C, int64_t ldc, const void* bias, const void* R,
                                           void* stream) {
  if (!A || !Bp || !C) return fail(HIFT_EINVAL, "null operand");
  Gemm g;
  g.dtype = DT_BF16;
  g.out_f32 = out_f32 != 0;
  g.M = Mm; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.C = C; g.ldc = ldc; g.bias = bias; g.R = R; g.ldr = ldc;
  if (!packed_gemm_applies(g)) return fail(HIFT_EINVAL, "problem is not one the packed-operand kernel takes");
  const size_t need = packed_ws_needed(g);
  if (need > sizeof(scratch))
    return fail(HIFT_EINVAL, "the shared last round of this problem needs %zu bytes of work space, the built-in one holds %zu",
                need, sizeof(scratch));
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(HIFT_EDEVICE, "device index %d outside [0,%d)", dev, MAX_DEVICES);
  void* ws = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!ws) {  // first call on this GPU (two threads racing here both store the same address)
    HIP_TRY(hipGetSymbolAddress(&ws, HIP_SYMBOL(scratch)));
    if (!ws) return fail(HIFT_EDEVICE, "hipGetSymbolAddress returned a null address");
    __atomic_store_n(&g_scratch_ptr[dev], ws, __ATOMIC_RELEASE);
  }
  hipStream_t st = (hipStream_t)stream;
  // the counters must be zero at the start; a launch leaves them so, but the array outlives a call that failed half-way
  if (need) HIP_TRY(fill_zero(ws, 1024, st));
  g.ws = ws;
  HIP_TRY(gemm_packed(g, Bp, st));
  return HIFT_OK;
}

hift_status hift_kernel_gemm_packed_rowsq(int64_t Mm, int64_t N, int64_t K, const void* A, int64_t lda, const void* Bp,
                                          void* C, int64_t ldc, const void* R, float* rowsq, void* workspace,
                                          void* stream) {
  if (!A || !Bp || !C || !rowsq) return fail(HIFT_EINVAL, "null operand");
  if (N % 256 != 0) return fail(HIFT_EINVAL, "N must be a multiple of 256");
  if (reinterpret_cast<uintptr_t>(workspace) & 15) return fail(HIFT_EINVAL, "work space not 16-byte aligned");
  Gemm g;
  g.dtype = DT_BF16;
  g.M = Mm; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.C = C; g.ldc = ldc; g.R = R; g.ldr = ldc;
  g.rowsq_out = rowsq;
  g.ws = workspace;
  if (!packed_gemm_applies(g)) return fail(HIFT_EINVAL, "problem is not one the packed-operand kernel takes");
  HIP_TRY(gemm_packed(g, Bp, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_row_sumsq(int64_t rows, int32_t d, const void* x, int32_t n, float* out, void* stream) {
  if (rows < 0 || d < 1 || n < 1) return fail(HIFT_EINVAL, "bad argument");
  if (rows == 0) return HIFT_OK;
  if (!x || !out) return fail(HIFT_EINVAL, "null operand");
  HIP_TRY(row_sumsq(rows, d, x, n, out, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_linear_fused(int32_t epilogue, int64_t Mm, int64_t N, int64_t K, const void* A, int64_t lda,
                                     const void* W, void* packed_scratch, void* C, void* aux, const float* cos_sin,
                                     int32_t seq, int64_t rot_cols, void* stream) {
  return hift_kernel_linear_norm_fused(epilogue, Mm, N, K, A, lda, W, nullptr, packed_scratch, C, aux, cos_sin, seq,
                                       rot_cols, nullptr, 0.f, nullptr, nullptr, stream);
}

hift_status hift_kernel_linear_norm_fused(int32_t epilogue, int64_t Mm, int64_t N, int64_t K, const void* A, int64_t lda,
                                          const void* W, const void* gain, void* packed_scratch, void* C, void* aux,
                                          const float* cos_sin, int32_t seq, int64_t rot_cols, const float* rowsq,
                                          float norm_eps, float* stats, void* workspace, void* stream) {
  if (!A || !W || !packed_scratch) return fail(HIFT_EINVAL, "null operand");
  if (reinterpret_cast<uintptr_t>(workspace) & 15) return fail(HIFT_EINVAL, "work space not 16-byte aligned");
  if ((gain == nullptr) != (rowsq == nullptr)) return fail(HIFT_EINVAL, "gain and rowsq go together");
  if (gain && (epilogue == HIFT_EPILOGUE_SWIGLU_BWD || K % 512 != 0 || K > 6144 || (reinterpret_cast<uintptr_t>(rowsq) & 15) != 0))
    return fail(HIFT_EINVAL, "folded normalisation: forward epilogues only, K a multiple of 512 up to 6144, rowsq 16-byte aligned");
  if (epilogue != HIFT_EPILOGUE_SWIGLU && epilogue != HIFT_EPILOGUE_ROPE && epilogue != HIFT_EPILOGUE_SWIGLU_BWD)
    return fail(HIFT_EINVAL, "epilogue unknown");
  const bool bwd = epilogue == HIFT_EPILOGUE_SWIGLU_BWD;
  if (packed_b_bytes(N, K) == 0 || (!bwd && N % 256 != 0) || (bwd && N % 8 != 0))
    return fail(HIFT_EINVAL, "shape cannot be packed (N a multiple of 256, or of 8 for the backward epilogue; K of 32)");
  Gemm g;
  g.dtype = DT_BF16;
  g.M = Mm; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.C = C; g.ldc = bwd ? 2 * N : N;
  int order = PK_ORDER_PLAIN;
  if (epilogue == HIFT_EPILOGUE_SWIGLU) {
    if (!aux) return fail(HIFT_EINVAL, "act is null");
    g.epi = EPI_SWIGLU; g.C2 = aux; g.ldc2 = N / 2;
    order = PK_ORDER_HALVES;
  } else if (bwd) {
    if (!aux || !C) return fail(HIFT_EINVAL, "the backward epilogue needs the pre-activations and C");
    g.epi = EPI_SWIGLU_BWD; g.C2 = aux; g.ldc2 = 2 * N;
  } else {
    if (!C || !cos_sin || seq < 1 || rot_cols < 0 || rot_cols > N || rot_cols % 128 != 0)
      return fail(HIFT_EINVAL, "rotation needs C, the table, seq >= 1 and rot_cols a multiple of 128 within N");
    g.epi = EPI_ROPE; g.cos_sin = cos_sin; g.S = seq; g.rot_cols = rot_cols;
    order = PK_ORDER_PAIR64;
  }
  if (!packed_gemm_applies(g)) return fail(HIFT_EINVAL, "problem is not one the packed-operand kernel takes");
  hipStream_t st = (hipStream_t)stream;
  if (gain) {
    g.rowsq = rowsq; g.norm_eps = norm_eps; g.norm_stats = stats;
  }
  g.ws = workspace;
  HIP_TRY(pack_b(W, K, N, K, true, packed_scratch, st, order, gain));
  HIP_TRY(gemm_packed(g, packed_scratch, st));
  return HIFT_OK;
}

hift_status hift_kernel_linear_gelu(int32_t backward, int64_t Mm, int64_t N, int64_t K, const void* A, int64_t lda,
                                    const void* W, const void* bias, void* packed_scratch, void* C, void* aux,
                                    void* stream) {
  if (!A || !W || !packed_scratch || !aux) return fail(HIFT_EINVAL, "null operand");
  if (backward && (!C || bias)) return fail(HIFT_EINVAL, "the backward epilogue needs C and takes no bias");
  if (packed_b_bytes(N, K) == 0 || N % 8 != 0) return fail(HIFT_EINVAL, "shape cannot be packed (N a multiple of 8, K of 32)");
  Gemm g;
  g.dtype = DT_BF16;
  g.M = Mm; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.C = C; g.ldc = N; g.bias = bias;
  g.epi = backward ? EPI_GELU_BWD : EPI_GELU;
  g.C2 = aux; g.ldc2 = N;
  if (!packed_gemm_applies(g)) return fail(HIFT_EINVAL, "problem is not one the packed-operand kernel takes");
  hipStream_t st = (hipStream_t)stream;
  HIP_TRY(pack_b(W, K, N, K, true, packed_scratch, st));
  HIP_TRY(gemm_packed(g, packed_scratch, st));
  return HIFT_OK;
}

hift_status hift_kernel_optimizer(const hift_opt* opt, int64_t count, int32_t decay, int64_t t, float* master,
                                  const float* grad, float* state1, float* state2, void* compute_copy, void* stream) {
  hift_status s = check_opt(opt);
  if (s != HIFT_OK) return s;
  if (count < 0 || t < 1) return fail(HIFT_EINVAL, "count must be >= 0 and t >= 1");
  if (opt->kind == HIFT_ADAFACTOR) return fail(HIFT_EINVAL, "Adafactor works on whole tensors; it has no element-wise kernel entry");
  OptArgs oa{opt->kind, opt->lr, opt->beta1, opt->beta2, opt->eps, opt->weight_decay, opt->momentum};
  HIP_TRY(optimizer_update(oa, count, decay != 0, t, master, grad, state1, state2, compute_copy, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_attention_fwd(int32_t batch, int32_t heads, int32_t seq, int32_t head_dim, int32_t causal,
                                      const void* qkv, void* prob, void* ctx, float* lse, void* stream) {
  const int64_t d = (int64_t)heads * head_dim;
  if (batch < 0 || heads < 1 || seq < 0 || !qkv || !ctx) return fail(HIFT_EINVAL, "bad argument");
  if (!attention_fwd_fused_applies(DT_BF16, seq, head_dim, 3 * d, d, qkv, prob, ctx))
    return fail(HIFT_EINVAL, "the fused kernel takes bf16, head widths 64 and 128 and 16-byte aligned buffers");
  HIP_TRY(attention_fwd_fused(batch, heads, seq, head_dim, causal != 0, qkv, 3 * d, prob, ctx, d, lse, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_attention_bwd(int32_t batch, int32_t heads, int32_t seq, int32_t head_dim, int32_t causal,
                                      const void* qkv, const void* ctx, const float* lse, const void* dctx, float* dsum,
                                      void* dqkv, const float* cos_sin, void* stream) {
  const int64_t d = (int64_t)heads * head_dim;
  if (batch < 0 || heads < 1 || seq < 0 || !qkv || !ctx || !lse || !dctx || !dsum || !dqkv) return fail(HIFT_EINVAL, "bad argument");
  if (!attention_bwd_fused_applies(DT_BF16, seq, head_dim, 3 * d, d, qkv, ctx, dctx, dqkv) ||
      (reinterpret_cast<uintptr_t>(cos_sin) & 7) != 0)
    return fail(HIFT_EINVAL, "the fused kernels take bf16, head widths 64 and 128 and 16-byte aligned buffers");
  HIP_TRY(attention_bwd_fused(batch, heads, seq, head_dim, causal != 0, qkv, 3 * d, ctx, lse, dctx, d, dsum, dqkv, cos_sin,
                              (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_norm_fwd(int32_t dtype, int32_t rms, int64_t rows, int32_t d, float eps, const void* x,
                                 const void* g, const void* b, void* y, float* stats, void* stream) {
  if (dtype != HIFT_F32 && dtype != HIFT_BF16) return fail(HIFT_EINVAL, "dtype unknown");
  if (rows < 0 || d < 1) return fail(HIFT_EINVAL, "bad shape");
  HIP_TRY(norm_fwd(dtype == HIFT_BF16 ? DT_BF16 : DT_F32, rms != 0, rows, d, eps, x, g, b, y, stats, (hipStream_t)stream));
  return HIFT_OK;
}

hift_status hift_kernel_cross_entropy(int32_t dtype, int64_t rows, int32_t V, void* logits, const int32_t* labels,
                                      float* row_loss_scratch, float* loss_out, void* stream) {
  if (dtype != HIFT_F32 && dtype != HIFT_BF16) return fail(HIFT_EINVAL, "dtype unknown");
  if (rows < 0 || V < 1) return fail(HIFT_EINVAL, "bad shape");
  HIP_TRY(cross_entropy(dtype == HIFT_BF16 ? DT_BF16 : DT_F32, rows, V, logits, labels, row_loss_scratch, loss_out,
                        (hipStream_t)stream));
  return HIFT_OK;
}

}  // extern "C"
