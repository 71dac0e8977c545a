// C ABI of the verification library: argument validation, workspace lay-out, and the fixed kernel
// sequence of one verification forward (Sec. 2.4) on the caller's stream.
#include "../../include/ded_verify.h"
#include "ded_kernels.h"

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

using namespace ded;

namespace {

constexpr int kMaskWords = 4;   // ancestor bitmask words per row (max_nodes <= 256)
constexpr int kMaxNodes = 256;
constexpr int64_t kAttnPartRows = 1 << 17;  // split-KV partial rows the workspace reserves at least
constexpr int kGemmCounters = 1 << 16;      // split-K arrival tickets (a GEMM with more output tiles runs unsplit)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int round_up(int v, int a) { return (v + a - 1) / a * a; }

enum KClass {
  KC_META = 0, KC_ROPE_TABLE, KC_EMBED, KC_RMSNORM, KC_GEMM_QKV, KC_QKV_EPILOGUE, KC_TREE_ATTN, KC_ATTN_MERGE,
  KC_GEMM_O, KC_GEMM_GATE_UP, KC_SILU_MUL, KC_GEMM_DOWN, KC_GEMM_LM_HEAD, KC_ARGMAX, KC_EXPORT, KC_WALK,
  KC_COMPACT, KC_LAYOUT, KC_SAMPLE, KC_TOP2_REDUCE, KC_COUNT
};
const char* const kClassNames[KC_COUNT] = {
    "meta_upload", "rope_table", "embed", "add_rmsnorm", "gemm_qkv", "qkv_rope_epilogue", "tree_attention",
    "attention_merge", "gemm_o", "gemm_gate_up", "silu_mul", "gemm_down", "gemm_lm_head", "argmax",
    "export_logits", "accept_walk", "kv_compact", "layout_convert", "sample_top_p", "top2_reduce"};

struct Carve {  // bump allocator over the workspace (base may be null when only sizing)
  char* base;
  size_t off = 0;
  explicit Carve(char* b) : base(b) {}
  template <typename T>
  T* take(size_t count) {
    off = align_up(off, 256);
    T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

}  // namespace

// Scratch of ded_tree_attention_static: device memory that belongs to the library itself, for callers that
// cannot allocate and bring no workspace region of their own for it.  One copy per GPU, held until the
// process ends.  In host code the array's name is only a handle: its device address is resolved once per
// device (resolve_static_scratch) and that pointer is what kernels, copies and memsets receive.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static unsigned char* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// With `device` current: the address of this device's copy of `scratch` (null if the runtime refuses).
static unsigned char* resolve_static_scratch(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[device] = static_cast<unsigned char*>(p);
  }
  return g_scratch_ptr[device];
}

struct ded_ctx {
  ded_config cfg;
  ModelDims md;
  bool bf16 = false;
  hipStream_t stream = nullptr;
  int device = -1;                          // the device that was current at ded_verify_init
  unsigned char* static_scratch = nullptr;  // this device's copy of the library's own scratch array
  int max_n_pad = 0;    // max_nodes rounded up to 16
  int max_rows = 0;     // max_batch * max_n_pad
  int max_rows_pad = 0; // rounded up to 64

  // weights inside the workspace
  void* emb = nullptr;
  void* lm_head = nullptr;
  float* final_norm = nullptr;
  std::vector<void*> wqkv, wo, wgu, wdown;
  std::vector<float*> norm_attn, norm_ffn;
  // caches
  std::vector<void*> kc, vc;
  void** d_kc = nullptr;
  void** d_vc = nullptr;
  // activations
  float* x = nullptr;
  float* logits = nullptr;
  float2* rope_tab = nullptr;
  // fp32 path
  float *f_y = nullptr, *f_qkv = nullptr, *f_o = nullptr, *f_gu = nullptr, *f_h = nullptr;
  // bf16 path
  bf16_t *y_p = nullptr, *o_p = nullptr, *h_p = nullptr, *q_p = nullptr;
  float* part = nullptr;
  int64_t part_elems = 0;
  float* ssq = nullptr;     // [rows_pad][d / 64] sum of squares of the residual stream per feature group
  int* counters = nullptr;  // split-K arrival tickets, one per output tile (kept at zero between launches)
  float* attn_part_o = nullptr;
  float2* attn_part_ml = nullptr;
  int64_t attn_part_rows = 0;
  void* top2_part = nullptr;  // [rows_pad][ceil(V / 64)] x 16 B: per-group candidates of the fused LM-head argmax
  // step meta (device + pinned host mirror, one contiguous block)
  char* d_meta = nullptr;
  char* h_meta = nullptr;
  size_t meta_bytes = 0;
  hipEvent_t meta_ev = nullptr;  // completion of the last upload from h_meta
  bool meta_inflight = false;
  size_t off_token = 0, off_parent = 0, off_depth = 0, off_pos = 0, off_mask = 0, off_p = 0, off_n = 0;
  // results
  int32_t* d_amax = nullptr;
  float* d_margin = nullptr;
  int32_t* d_rowflag = nullptr;  // [rows] != 0: the row's logits hold a NaN or an infinity
  int32_t* d_seqflag = nullptr;  // [max_batch] the same per sequence (real nodes only), written by the walk
  float* d_uniform = nullptr;  // [rows] uniform numbers of ded_sample
  int32_t *d_nacc = nullptr, *d_path = nullptr, *d_acctok = nullptr;
  char* h_res = nullptr;  // pinned: amax | margin | row flags, or nacc | seqflag | path | acctok
  size_t res_bytes = 0;
  // state of the pending step
  bool pending = false;
  bool have_argmax = false;
  bool have_logits = false;    // the workspace holds the fp32 logits of the last step
  bool poisoned = false;       // the last step's tree slots may hold NaN / infinite K/V: cleared before they can be read
  bool sampling_seen = false;  // ded_sample has been used on this context: steps keep their logits from then on
  int batch = 0, n_step = 0;
  int max_p = 0;
  std::vector<int32_t> s_p, s_n, s_parent;
  // profiling
  bool prof_on = false;
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;
  struct Span { int cls; size_t e0, e1; };
  std::vector<Span> spans;
  double prof_ms[KC_COUNT] = {};
  int64_t prof_n[KC_COUNT] = {};

  StepMeta meta() const { return meta_at(d_meta); }
  // the step description inside a device copy of the meta block that starts at `base`
  StepMeta meta_at(const char* base) const {
    StepMeta m;
    m.token = reinterpret_cast<const int32_t*>(base + off_token);
    m.parent = reinterpret_cast<const int32_t*>(base + off_parent);
    m.depth = reinterpret_cast<const int32_t*>(base + off_depth);
    m.pos = reinterpret_cast<const int32_t*>(base + off_pos);
    m.mask = reinterpret_cast<const uint64_t*>(base + off_mask);
    m.seq_p = reinterpret_cast<const int32_t*>(base + off_p);
    m.seq_n = reinterpret_cast<const int32_t*>(base + off_n);
    m.batch = batch;
    m.n_step = n_step;
    m.rows = batch * n_step;
    return m;
  }
};

namespace {

// ---------------------------------------------------------------------------------------------
bool config_ok(const ded_config* c) {
  if (!c) return false;
  if (c->n_layers < 0 || c->d_model <= 0 || c->n_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
      c->vocab <= 0 || c->max_batch <= 0 || c->kv_capacity <= 0 || c->max_nodes <= 0)
    return false;
  if (c->n_layers > 0 && c->d_ffn <= 0) return false;
  if (c->n_heads % c->n_kv_heads) return false;
  if (c->max_nodes > kMaxNodes) return false;
  if (c->head_dim % 2) return false;
  if (!(c->rope_base > 0.f) || !(c->rms_eps >= 0.f)) return false;
  if ((int64_t)c->max_batch * round_up(c->max_nodes, 16) > (1 << 20)) return false;
  if (c->dtype == DED_F32) {
    if (c->head_dim > 256 || 256 % c->head_dim) return false;
    return true;
  }
  if (c->dtype == DED_BF16) {
    if (c->head_dim != 128) return false;
    if (c->d_model % 128 || c->vocab % 16 || c->kv_capacity % 64) return false;
    if (c->n_layers > 0 && c->d_ffn % 128) return false;
    return true;
  }
  return false;
}

struct Sizes {
  int max_n_pad, max_rows, max_rows_pad;
  size_t elem;  // bytes per stored element
};

Sizes sizes_of(const ded_config& c) {
  Sizes s;
  s.max_n_pad = round_up(c.max_nodes, 16);
  s.max_rows = c.max_batch * s.max_n_pad;
  s.max_rows_pad = round_up(s.max_rows, 64);
  s.elem = c.dtype == DED_BF16 ? 2 : 4;
  return s;
}

// Single description of the workspace; used for sizing (ctx == nullptr members untouched) and for init.
size_t carve_workspace(const ded_config& c, char* base, ded_ctx* ctx) {
  Sizes z = sizes_of(c);
  Carve w(base);
  const int64_t d = c.d_model, V = c.vocab, F = c.d_ffn;
  const int64_t qd = (int64_t)c.n_heads * c.head_dim, kvd = (int64_t)c.n_kv_heads * c.head_dim;
  const int64_t qkv_n = qd + 2 * kvd;
  const int L = c.n_layers;
  auto bytes = [&](int64_t n) { return (size_t)n * z.elem; };

  // bf16 matrices are re-laid-out with the feature count padded to a multiple of 64
  auto wbytes = [&](int64_t n_out, int64_t k_in) {
    return bytes((c.dtype == DED_BF16 ? (n_out + 63) / 64 * 64 : n_out) * k_in);
  };
  char* emb = w.take<char>(bytes(V * d));
  char* lm = w.take<char>(wbytes(V, d));
  float* fn = w.take<float>(d);
  if (ctx) {
    ctx->emb = emb;
    ctx->lm_head = lm;
    ctx->final_norm = fn;
    ctx->wqkv.assign(L, nullptr);
    ctx->wo.assign(L, nullptr);
    ctx->wgu.assign(L, nullptr);
    ctx->wdown.assign(L, nullptr);
    ctx->norm_attn.assign(L, nullptr);
    ctx->norm_ffn.assign(L, nullptr);
  }
  for (int l = 0; l < L; ++l) {
    char* a = w.take<char>(wbytes(qkv_n, d));
    char* b = w.take<char>(wbytes(d, qd));
    char* g = w.take<char>(wbytes(2 * F, d));
    char* dn = w.take<char>(wbytes(d, F));
    float* na = w.take<float>(d);
    float* nf = w.take<float>(d);
    if (ctx) {
      ctx->wqkv[l] = a;
      ctx->wo[l] = b;
      ctx->wgu[l] = g;
      ctx->wdown[l] = dn;
      ctx->norm_attn[l] = na;
      ctx->norm_ffn[l] = nf;
    }
  }
  void** dkc = w.take<void*>(std::max(L, 1));
  void** dvc = w.take<void*>(std::max(L, 1));
  float* x = w.take<float>((int64_t)z.max_rows_pad * d);
  float* logits = w.take<float>((int64_t)z.max_rows_pad * V);
  float2* tab = w.take<float2>((int64_t)z.max_rows * (c.head_dim / 2));
  if (ctx) {
    ctx->d_kc = dkc;
    ctx->d_vc = dvc;
    ctx->x = x;
    ctx->logits = logits;
    ctx->rope_tab = tab;
  }
  if (c.dtype == DED_F32) {
    float* y = w.take<float>((int64_t)z.max_rows_pad * d);
    float* qkv = w.take<float>((int64_t)z.max_rows_pad * qkv_n);
    float* o = w.take<float>((int64_t)z.max_rows_pad * qd);
    float* gu = w.take<float>((int64_t)z.max_rows_pad * 2 * F);
    float* h = w.take<float>((int64_t)z.max_rows_pad * F);
    if (ctx) {
      ctx->f_y = y;
      ctx->f_qkv = qkv;
      ctx->f_o = o;
      ctx->f_gu = gu;
      ctx->f_h = h;
    }
  } else {
    // GEMM inputs and queries are kept as hi/lo pairs of f16: two planes each
    bf16_t* y = w.take<bf16_t>((int64_t)z.max_rows_pad * d * 2);
    bf16_t* o = w.take<bf16_t>((int64_t)z.max_rows_pad * qd * 2);
    bf16_t* h = w.take<bf16_t>((int64_t)z.max_rows_pad * std::max<int64_t>(F, 1) * 2);
    bf16_t* q = w.take<bf16_t>((int64_t)z.max_rows_pad * qd * 2);
    // split-K partials: at most 8 slices of 64 rows, or one slice of every row
    int64_t widest = std::max<int64_t>(std::max<int64_t>(qkv_n, 2 * F), std::max<int64_t>(d, round_up((int)V, 64)));
    int64_t part_elems = widest * std::max<int64_t>(8 * 64, z.max_rows_pad);
    float* part = w.take<float>(part_elems);
    float* ssq = w.take<float>((int64_t)z.max_rows_pad * (d / 64));
    int* counters = w.take<int>(kGemmCounters);
    int64_t arows = std::max<int64_t>(kAttnPartRows, (int64_t)z.max_rows * c.n_heads);
    float* apo = w.take<float>(arows * c.head_dim);
    float2* apm = w.take<float2>(arows);
    char* t2 = w.take<char>((size_t)z.max_rows_pad * ((V + 63) / 64) * 16);
    if (ctx) {
      ctx->top2_part = t2;
      ctx->y_p = y;
      ctx->o_p = o;
      ctx->h_p = h;
      ctx->q_p = q;
      ctx->part = part;
      ctx->part_elems = part_elems;
      ctx->ssq = ssq;
      ctx->counters = counters;
      ctx->attn_part_o = apo;
      ctx->attn_part_ml = apm;
      ctx->attn_part_rows = arows;
    }
  }
  // step meta block
  size_t m = 0;
  auto mtake = [&](size_t n) {
    m = align_up(m, 256);
    size_t o = m;
    m += n;
    return o;
  };
  size_t o_token = mtake((size_t)z.max_rows * 4), o_parent = mtake((size_t)z.max_rows * 4),
         o_depth = mtake((size_t)z.max_rows * 4), o_pos = mtake((size_t)z.max_rows * 4),
         o_mask = mtake((size_t)z.max_rows * 8 * kMaskWords), o_p = mtake((size_t)c.max_batch * 4),
         o_n = mtake((size_t)c.max_batch * 4);
  m = align_up(m, 256);
  char* dmeta = w.take<char>(m);
  int stride = c.max_nodes + 1;
  int32_t* amax = w.take<int32_t>(z.max_rows_pad);
  float* margin = w.take<float>(z.max_rows_pad);
  float* uniform = w.take<float>(z.max_rows_pad);
  int32_t* rowflag = w.take<int32_t>(z.max_rows_pad);
  // one block, so that a single copy brings a step's verdict to the host: nacc | seqflag | path | acctok
  int32_t* nacc = w.take<int32_t>((int64_t)c.max_batch * (2 + 2 * stride));
  // (no arithmetic on the null pointers of a sizing pass)
  int32_t* seqflag = nacc ? nacc + c.max_batch : nullptr;
  int32_t* path = nacc ? seqflag + c.max_batch : nullptr;
  int32_t* acct = nacc ? path + (int64_t)c.max_batch * stride : nullptr;
  if (ctx) {
    ctx->d_meta = dmeta;
    ctx->meta_bytes = m;
    ctx->off_token = o_token;
    ctx->off_parent = o_parent;
    ctx->off_depth = o_depth;
    ctx->off_pos = o_pos;
    ctx->off_mask = o_mask;
    ctx->off_p = o_p;
    ctx->off_n = o_n;
    ctx->d_amax = amax;
    ctx->d_margin = margin;
    ctx->d_uniform = uniform;
    ctx->d_rowflag = rowflag;
    ctx->d_seqflag = seqflag;
    ctx->d_nacc = nacc;
    ctx->d_path = path;
    ctx->d_acctok = acct;
  }
  return align_up(w.off, 256);
}

#define HIP_TRY(expr)                     \
  do {                                    \
    if ((expr) != hipSuccess) {           \
      (void)hipGetLastError();            \
      return DED_EHIP;                    \
    }                                     \
  } while (0)

// Profiling bracket around one launcher call.
struct ProfScope {
  ded_ctx* c;
  int cls;
  size_t e0 = 0;
  bool on;
  ProfScope(ded_ctx* ctx, int k) : c(ctx), cls(k), on(ctx->prof_on) {
    if (!on) return;
    e0 = next();
    (void)hipEventRecord(c->ev_pool[e0], c->stream);
  }
  ~ProfScope() {
    if (!on) return;
    size_t e1 = next();
    (void)hipEventRecord(c->ev_pool[e1], c->stream);
    c->spans.push_back({cls, e0, e1});
  }
  size_t next() {
    if (c->ev_used == c->ev_pool.size()) {
      hipEvent_t e;
      (void)hipEventCreate(&e);
      c->ev_pool.push_back(e);
    }
    return c->ev_used++;
  }
};

int prof_drain(ded_ctx* c) {
  if (c->spans.empty()) return DED_OK;
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (auto& s : c->spans) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, c->ev_pool[s.e0], c->ev_pool[s.e1]) == hipSuccess) {
      c->prof_ms[s.cls] += ms;
      c->prof_n[s.cls] += 1;
    }
  }
  c->spans.clear();
  c->ev_used = 0;
  return DED_OK;
}

// ---------------------------------------------------------------------------------------------
// Host-side tree ingest: validation, depth, position, ancestor bitmask (mask[i] = mask[parent] | bit i).
int validate_step(const ded_config& cfg, int32_t batch, const int32_t* prefix_len, const int32_t* n_nodes,
                  const int32_t* parent, const int32_t* token, bool need_token) {
  if (batch < 1 || batch > cfg.max_batch) return DED_EINVAL;
  if (!prefix_len || !n_nodes || !parent || (need_token && !token)) return DED_EINVAL;
  for (int b = 0; b < batch; ++b) {
    int n = n_nodes[b], p = prefix_len[b];
    if (n < 1 || n > cfg.max_nodes || p < 0) return DED_EINVAL;
    if ((int64_t)p + n > cfg.kv_capacity) return DED_ECAP;
    const int32_t* par = parent + (int64_t)b * cfg.max_nodes;
    if (par[0] != -1) return DED_ETREE;
    for (int i = 1; i < n; ++i)
      if (par[i] < 0 || par[i] >= i) return DED_ETREE;
    if (need_token) {
      const int32_t* tok = token + (int64_t)b * cfg.max_nodes;
      for (int i = 0; i < n; ++i)
        if (tok[i] < 0 || tok[i] >= cfg.vocab) return DED_ETOKEN;
    }
  }
  return DED_OK;
}

int ingest_and_upload(ded_ctx* c, int32_t batch, const int32_t* prefix_len, const int32_t* n_nodes,
                      const int32_t* parent, const int32_t* token, char* d_meta_dst = nullptr) {
  const ded_config& cfg = c->cfg;
  int nmax = 0, pmax = 0;
  for (int b = 0; b < batch; ++b) {
    nmax = std::max(nmax, n_nodes[b]);
    pmax = std::max(pmax, prefix_len[b]);
  }
  int n_step = round_up(nmax, 16);
  if (c->meta_inflight) {  // the pinned mirror may still be feeding the previous upload
    HIP_TRY(hipEventSynchronize(c->meta_ev));
    c->meta_inflight = false;
  }
  c->batch = batch;
  c->n_step = n_step;
  c->max_p = pmax;
  c->s_p.assign(prefix_len, prefix_len + batch);
  c->s_n.assign(n_nodes, n_nodes + batch);
  c->s_parent.assign((size_t)batch * cfg.max_nodes, -1);
  int32_t* h_token = reinterpret_cast<int32_t*>(c->h_meta + c->off_token);
  int32_t* h_parent = reinterpret_cast<int32_t*>(c->h_meta + c->off_parent);
  int32_t* h_depth = reinterpret_cast<int32_t*>(c->h_meta + c->off_depth);
  int32_t* h_pos = reinterpret_cast<int32_t*>(c->h_meta + c->off_pos);
  uint64_t* h_mask = reinterpret_cast<uint64_t*>(c->h_meta + c->off_mask);
  int32_t* h_p = reinterpret_cast<int32_t*>(c->h_meta + c->off_p);
  int32_t* h_n = reinterpret_cast<int32_t*>(c->h_meta + c->off_n);
  for (int b = 0; b < batch; ++b) {
    const int32_t* par = parent + (int64_t)b * cfg.max_nodes;
    const int32_t* tok = token ? token + (int64_t)b * cfg.max_nodes : nullptr;
    int n = n_nodes[b], P = prefix_len[b];
    h_p[b] = P;
    h_n[b] = n;
    for (int i = 0; i < n_step; ++i) {
      int r = b * n_step + i;
      uint64_t* mr = h_mask + (size_t)r * kMaskWords;
      if (i < n) {
        c->s_parent[(size_t)b * cfg.max_nodes + i] = par[i];
        h_parent[r] = par[i];
        h_token[r] = tok ? tok[i] : 0;
        if (i == 0) {
          h_depth[r] = 0;
          for (int w = 0; w < kMaskWords; ++w) mr[w] = 0;
        } else {
          int pr = b * n_step + par[i];
          h_depth[r] = h_depth[pr] + 1;
          const uint64_t* mp = h_mask + (size_t)pr * kMaskWords;
          for (int w = 0; w < kMaskWords; ++w) mr[w] = mp[w];
        }
        mr[i >> 6] |= 1ull << (i & 63);
      } else {  // padding row: behaves like a copy of the root, never read back
        h_parent[r] = -1;
        h_token[r] = tok ? tok[0] : 0;
        h_depth[r] = 0;
        for (int w = 0; w < kMaskWords; ++w) mr[w] = 0;
        mr[0] = 1ull;
      }
      h_pos[r] = P + h_depth[r];
    }
  }
  {
    ProfScope ps(c, KC_META);
    HIP_TRY(hipMemcpyAsync(d_meta_dst ? d_meta_dst : c->d_meta, c->h_meta, c->meta_bytes, hipMemcpyHostToDevice,
                           c->stream));
  }
  HIP_TRY(hipEventRecord(c->meta_ev, c->stream));
  c->meta_inflight = true;
  return DED_OK;
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? DED_OK : DED_EHIP; }

// ---------------------------------------------------------------------------------------------
int forward_f32(ded_ctx* c) {
  const ModelDims& md = c->md;
  StepMeta m = c->meta();
  hipStream_t s = c->stream;
  const int d = md.d, qd = md.H * md.hd, kvd = md.Hkv * md.hd, qkv_n = qd + 2 * kvd, F = md.F;
  { ProfScope p(c, KC_ROPE_TABLE); launch_rope_table(c->rope_tab, m.pos, m.rows, md.hd, md.rope_base, s); }
  { ProfScope p(c, KC_EMBED); f32_embed(c->x, (const float*)c->emb, m, d, s); }
  for (int l = 0; l < md.n_layers; ++l) {
    { ProfScope p(c, KC_RMSNORM); f32_rmsnorm(c->f_y, c->x, c->norm_attn[l], m.rows, d, md.eps, s); }
    { ProfScope p(c, KC_GEMM_QKV); f32_gemm(c->f_qkv, c->f_y, (const float*)c->wqkv[l], m.rows, qkv_n, d, false, s); }
    { ProfScope p(c, KC_QKV_EPILOGUE); f32_rope_kv(c->f_qkv, (float*)c->kc[l], (float*)c->vc[l], c->rope_tab, m, md, s); }
    { ProfScope p(c, KC_TREE_ATTN); f32_tree_attention(c->f_o, c->f_qkv, qkv_n, (const float*)c->kc[l], (const float*)c->vc[l], m, md, s); }
    { ProfScope p(c, KC_GEMM_O); f32_gemm(c->x, c->f_o, (const float*)c->wo[l], m.rows, d, qd, true, s); }
    { ProfScope p(c, KC_RMSNORM); f32_rmsnorm(c->f_y, c->x, c->norm_ffn[l], m.rows, d, md.eps, s); }
    { ProfScope p(c, KC_GEMM_GATE_UP); f32_gemm(c->f_gu, c->f_y, (const float*)c->wgu[l], m.rows, 2 * F, d, false, s); }
    { ProfScope p(c, KC_SILU_MUL); f32_silu_mul(c->f_h, c->f_gu, m.rows, F, s); }
    { ProfScope p(c, KC_GEMM_DOWN); f32_gemm(c->x, c->f_h, (const float*)c->wdown[l], m.rows, d, F, true, s); }
  }
  { ProfScope p(c, KC_RMSNORM); f32_rmsnorm(c->f_y, c->x, c->final_norm, m.rows, d, md.eps, s); }
  { ProfScope p(c, KC_GEMM_LM_HEAD); f32_gemm(c->logits, c->f_y, (const float*)c->lm_head, m.rows, md.V, d, false, s); }
  return launch_status();
}

// After a step whose logits were not finite the K/V it appended (slots prefix_len .. prefix_len + n_nodes of every
// sequence, every layer) may be NaN or infinite.  Dead slots are still fetched by whole-tile loads (and multiplied
// by a zero weight), so they are zeroed before any later step can fetch them.
int clear_step_slots(ded_ctx* c) {
  for (int l = 0; l < c->md.n_layers; ++l)
    for (int b = 0; b < c->batch; ++b) {
      if (c->bf16) bf16_kv_clear((bf16_t*)c->kc[l], (bf16_t*)c->vc[l], b, c->s_p[b], c->s_n[b], c->md, c->stream);
      else f32_kv_clear((float*)c->kc[l], (float*)c->vc[l], b, c->s_p[b], c->s_n[b], c->md, c->stream);
    }
  c->poisoned = false;
  return launch_status();
}

// LM head of the 16-bit path on the final residual stream (c->y_p / c->ssq as the last layer left them).  With
// want_logits the fp32 logits are written to the workspace; without, only the per-group top-2 candidates that the
// per-node argmax needs (the logits never reach memory).
bool lm_head_bf16(ded_ctx* c, bool want_logits) {
  const ModelDims& md = c->md;
  const int rows = c->batch * c->n_step, rows_pad = round_up(rows, 64), d = md.d;
  GemmEpilogue e = {};
  e.rows = rows;
  e.rb_total = rows_pad / 16;
  e.eps = md.eps;
  e.ssq_in = c->ssq;
  e.ssq_groups = d / 64;
  e.inv_k = 1.0f / (float)d;
  if (want_logits) {
    e.kind = EPI_LOGITS;
    e.out = c->logits;
    e.out_stride = md.V;
  } else {
    e.kind = EPI_TOP2;
    e.top2_part = c->top2_part;
    e.top2_groups = (md.V + 63) / 64;
  }
  const int64_t slice = (int64_t)rows_pad * round_up(md.V, 64);
  int cap = (int)std::min<int64_t>(8, c->part_elems / slice);
  // From 256 rows on the projection is bound by the matrix cores and reads the hi plane of its input alone: the lo
  // plane matters for what is carried through the layers, not here, where one rounding of the final normalised input
  // (2^-12 relative) moves a logit by ~2e-4.  Below, the weight stream bounds it and the lo product is free.
  const int planes = rows_pad >= 256 ? 1 : 2;
  GemmPlan plan = bf16_gemm_plan(rows_pad, md.V, d, planes, std::max(cap, 1));
  if (bf16_gemm_tiles(rows_pad, md.V, plan) > kGemmCounters) plan.splits = 1;
  ProfScope p(c, KC_GEMM_LM_HEAD);
  return bf16_gemm(c->part, slice, c->y_p, (const bf16_t*)c->lm_head, rows_pad, md.V, d, planes, plan, c->counters, e,
                   c->stream);
}

int forward_bf16(ded_ctx* c, bool want_logits) {
  const ModelDims& md = c->md;
  StepMeta m = c->meta();
  hipStream_t s = c->stream;
  const int d = md.d, qd = md.H * md.hd, kvd = md.Hkv * md.hd, qkv_n = qd + 2 * kvd, F = md.F, L = md.n_layers;
  const int rows_pad = round_up(m.rows, 64);
  bool ok = true;
  GemmEpilogue base = {};
  base.rows = m.rows;
  base.rb_total = rows_pad / 16;
  base.eps = md.eps;
  // planes: 2 = the input is consumed as hi + lo, 1 = hi only (enough for the O and down projections)
  auto gemm = [&](int cls, const bf16_t* xp, const void* w, int N, int K, int planes, const GemmEpilogue& epi) {
    const int64_t slice = (int64_t)rows_pad * round_up(N, 64);
    int cap = (int)std::min<int64_t>(8, c->part_elems / slice);
    GemmPlan plan = bf16_gemm_plan(rows_pad, N, K, planes, std::max(cap, 1));
    if (bf16_gemm_tiles(rows_pad, N, plan) > kGemmCounters) plan.splits = 1;
    ProfScope p(c, cls);
    ok = bf16_gemm(c->part, slice, xp, (const bf16_t*)w, rows_pad, N, K, planes, plan, c->counters,
                   epi, s) && ok;
  };
  // RMSNorm is deferred: whoever produces the residual stream also writes x * gain(next norm) as the next
  // GEMM input and sum(x^2) per 64 features; the consuming GEMM multiplies its output rows by 1/rms.
  auto normed_input = [&](GemmEpilogue& e) {
    e.ssq_in = c->ssq;
    e.ssq_groups = d / 64;
    e.inv_k = 1.0f / (float)d;
  };
  auto next_gain = [&](int l) { return l < L ? c->norm_attn[l] : c->final_norm; };
  { ProfScope p(c, KC_ROPE_TABLE); launch_rope_table(c->rope_tab, m.pos, m.rows, md.hd, md.rope_base, s); }
  { ProfScope p(c, KC_EMBED); bf16_embed(c->x, c->y_p, c->ssq, (const bf16_t*)c->emb, next_gain(0), m, rows_pad, d, s); }
  for (int l = 0; l < L; ++l) {
    {
      GemmEpilogue e = base;
      e.kind = EPI_QKV;
      normed_input(e);
      e.q_packed = c->q_p;
      e.k_cache = (bf16_t*)c->kc[l];
      e.v_cache = (bf16_t*)c->vc[l];
      e.rope_tab = c->rope_tab;
      e.seq_p = m.seq_p;
      e.seq_n = m.seq_n;
      e.n_step = m.n_step;
      e.H = md.H;
      e.Hkv = md.Hkv;
      e.cap = md.cap;
      gemm(KC_GEMM_QKV, c->y_p, c->wqkv[l], qkv_n, d, 2, e);
    }
    int ns = bf16_attn_pick_splits(m, md, c->max_p, c->attn_part_rows);
    { ProfScope p(c, KC_TREE_ATTN);
      bf16_tree_attention(c->o_p, rows_pad, c->q_p, (const bf16_t*)c->kc[l], (const bf16_t*)c->vc[l], c->attn_part_o,
                          c->attn_part_ml, ns, bf16_attn_query_planes(m, md), m, md, s); }
    {
      GemmEpilogue e = base;
      e.kind = EPI_RESIDUAL;
      e.x = c->x;
      e.gain = c->norm_ffn[l];
      e.y_packed = c->y_p;
      e.ssq_out = c->ssq;
      gemm(KC_GEMM_O, c->o_p, c->wo[l], d, qd, 1, e);
    }
    {
      GemmEpilogue e = base;
      e.kind = EPI_SILU;
      normed_input(e);
      e.y_packed = c->h_p;
      gemm(KC_GEMM_GATE_UP, c->y_p, c->wgu[l], 2 * F, d, 2, e);
    }
    {
      GemmEpilogue e = base;
      e.kind = EPI_RESIDUAL;
      e.x = c->x;
      e.gain = next_gain(l + 1);
      e.y_packed = c->y_p;
      e.ssq_out = c->ssq;
      gemm(KC_GEMM_DOWN, c->h_p, c->wdown[l], d, F, 1, e);
    }
  }
  ok = lm_head_bf16(c, want_logits) && ok;
  if (!ok) return DED_EINVAL;
  return launch_status();
}

}  // namespace

// =============================================================================================
extern "C" {

const char* ded_strerror(int code) {
  switch (code) {
    case DED_OK: return "ok";
    case DED_EINVAL: return "invalid argument or unsupported configuration";
    case DED_ETREE: return "malformed draft tree (parent[0] must be -1 and 0 <= parent[i] < i)";
    case DED_ETOKEN: return "token id outside the vocabulary";
    case DED_ECAP: return "prefix_len + n_nodes exceeds kv_capacity";
    case DED_ESTATE: return "call out of order";
    case DED_EHIP: return "HIP runtime failure";
    case DED_ENOMEM: return "workspace too small or host allocation failed";
    case DED_ENONFINITE: return "NaN or infinity in the logits of a tree node (weights or activations outside the half-precision operand range?)";
    default: return "unknown error";
  }
}

size_t ded_workspace_bytes(const ded_config* cfg) {
  if (!config_ok(cfg)) return 0;
  return carve_workspace(*cfg, nullptr, nullptr);
}

size_t ded_kv_layer_bytes(const ded_config* cfg) {
  if (!config_ok(cfg)) return 0;
  size_t elem = cfg->dtype == DED_BF16 ? 2 : 4;
  return (size_t)cfg->max_batch * cfg->n_kv_heads * cfg->kv_capacity * cfg->head_dim * elem;
}

int ded_validate_tree(const ded_config* cfg, int32_t batch, const int32_t* prefix_len, const int32_t* n_nodes,
                      const int32_t* parent, const int32_t* token) {
  if (!config_ok(cfg)) return DED_EINVAL;
  return validate_step(*cfg, batch, prefix_len, n_nodes, parent, token, true);
}

int ded_verify_init(const ded_config* cfg, const ded_weights* w, const ded_kv* kv, void* workspace,
                    size_t workspace_bytes, void* hip_stream, ded_ctx** out) {
  if (!out) return DED_EINVAL;
  *out = nullptr;
  if (!config_ok(cfg) || !w || !kv || !workspace) return DED_EINVAL;
  const int L = cfg->n_layers;
  if (!w->emb || !w->lm_head || !w->final_norm) return DED_EINVAL;
  if (L > 0 && (!w->wqkv || !w->wo || !w->wgate_up || !w->wdown || !w->norm_attn || !w->norm_ffn || !kv->k || !kv->v))
    return DED_EINVAL;
  for (int l = 0; l < L; ++l)
    if (!w->wqkv[l] || !w->wo[l] || !w->wgate_up[l] || !w->wdown[l] || !w->norm_attn[l] || !w->norm_ffn[l] ||
        !kv->k[l] || !kv->v[l])
      return DED_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return DED_EINVAL;
  size_t need = carve_workspace(*cfg, nullptr, nullptr);
  if (workspace_bytes < need) return DED_ENOMEM;

  ded_ctx* c = new (std::nothrow) ded_ctx();
  if (!c) return DED_ENOMEM;
  c->cfg = *cfg;
  c->bf16 = cfg->dtype == DED_BF16;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  // set-up of the library's own scratch array: resolved here, once per device, with the context's device current
  if (hipGetDevice(&c->device) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return DED_EHIP;
  }
  c->static_scratch = resolve_static_scratch(c->device);
  if (!c->static_scratch) {
    delete c;
    return DED_EHIP;
  }
  c->md = ModelDims{cfg->n_layers, cfg->d_model, cfg->n_heads, cfg->n_kv_heads, cfg->head_dim,
                    cfg->d_ffn,    cfg->vocab,   cfg->kv_capacity, cfg->rope_base, cfg->rms_eps};
  Sizes z = sizes_of(*cfg);
  c->max_n_pad = z.max_n_pad;
  c->max_rows = z.max_rows;
  c->max_rows_pad = z.max_rows_pad;
  carve_workspace(*cfg, static_cast<char*>(workspace), c);
  c->kc.assign(kv->k, kv->k + L);
  c->vc.assign(kv->v, kv->v + L);

  auto fail = [&](int code) {
    ded_verify_free(c);
    return code;
  };
  int stride = cfg->max_nodes + 1;
  c->res_bytes = align_up((size_t)z.max_rows_pad * 12 + (size_t)cfg->max_batch * 4 * (2 + 2 * stride), 256);
  if (hipHostMalloc(reinterpret_cast<void**>(&c->h_meta), c->meta_bytes, hipHostMallocDefault) != hipSuccess ||
      hipHostMalloc(reinterpret_cast<void**>(&c->h_res), c->res_bytes, hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    return fail(DED_EHIP);
  }
  memset(c->h_meta, 0, c->meta_bytes);
  if (hipEventCreateWithFlags(&c->meta_ev, hipEventDisableTiming) != hipSuccess) {
    (void)hipGetLastError();
    return fail(DED_EHIP);
  }
  hipStream_t s = c->stream;
  const int64_t d = cfg->d_model, V = cfg->vocab, F = cfg->d_ffn;
  const int64_t qd = (int64_t)cfg->n_heads * cfg->head_dim, kvd = (int64_t)cfg->n_kv_heads * cfg->head_dim;
  const int64_t qkv_n = qd + 2 * kvd;
#define INIT_TRY(expr)                  \
  do {                                  \
    if ((expr) != hipSuccess) {         \
      (void)hipGetLastError();          \
      return fail(DED_EHIP);            \
    }                                   \
  } while (0)
  // activations start from zero so that padding rows hold finite values
  {
    char* act0 = reinterpret_cast<char*>(c->d_kc);
    size_t act_bytes = need - (size_t)(act0 - static_cast<char*>(workspace));
    INIT_TRY(hipMemsetAsync(act0, 0, act_bytes, s));
  }
  // cache slots beyond the live range are read (and masked) by whole-tile loads: keep them finite
  for (int l = 0; l < L; ++l) {
    INIT_TRY(hipMemsetAsync(c->kc[l], 0, ded_kv_layer_bytes(cfg), s));
    INIT_TRY(hipMemsetAsync(c->vc[l], 0, ded_kv_layer_bytes(cfg), s));
  }
  if (L > 0) {
    INIT_TRY(hipMemcpyAsync(c->d_kc, c->kc.data(), sizeof(void*) * L, hipMemcpyHostToDevice, s));
    INIT_TRY(hipMemcpyAsync(c->d_vc, c->vc.data(), sizeof(void*) * L, hipMemcpyHostToDevice, s));
  }
  auto copy_gain = [&](float* dst, const float* src) {
    return hipMemcpyAsync(dst, src, sizeof(float) * d, hipMemcpyDeviceToDevice, s);
  };
  INIT_TRY(copy_gain(c->final_norm, w->final_norm));
  INIT_TRY(hipMemcpyAsync(c->emb, w->emb, (size_t)V * d * z.elem, hipMemcpyDeviceToDevice, s));
  if (!c->bf16) {
    INIT_TRY(hipMemcpyAsync(c->lm_head, w->lm_head, (size_t)V * d * 4, hipMemcpyDeviceToDevice, s));
    for (int l = 0; l < L; ++l) {
      INIT_TRY(hipMemcpyAsync(c->wqkv[l], w->wqkv[l], (size_t)qkv_n * d * 4, hipMemcpyDeviceToDevice, s));
      INIT_TRY(hipMemcpyAsync(c->wo[l], w->wo[l], (size_t)d * qd * 4, hipMemcpyDeviceToDevice, s));
      INIT_TRY(hipMemcpyAsync(c->wgu[l], w->wgate_up[l], (size_t)2 * F * d * 4, hipMemcpyDeviceToDevice, s));
      INIT_TRY(hipMemcpyAsync(c->wdown[l], w->wdown[l], (size_t)d * F * 4, hipMemcpyDeviceToDevice, s));
      INIT_TRY(copy_gain(c->norm_attn[l], w->norm_attn[l]));
      INIT_TRY(copy_gain(c->norm_ffn[l], w->norm_ffn[l]));
    }
  } else {
    bf16_pack_weight((bf16_t*)c->lm_head, (const bf16_t*)w->lm_head, (int)V, (int)d, PERM_NONE, s);
    for (int l = 0; l < L; ++l) {
      bf16_pack_weight((bf16_t*)c->wqkv[l], (const bf16_t*)w->wqkv[l], (int)qkv_n, (int)d, PERM_ROPE, s);
      bf16_pack_weight((bf16_t*)c->wo[l], (const bf16_t*)w->wo[l], (int)d, (int)qd, PERM_NONE, s);
      bf16_pack_weight((bf16_t*)c->wgu[l], (const bf16_t*)w->wgate_up[l], (int)(2 * F), (int)d, PERM_GATE_UP, s);
      bf16_pack_weight((bf16_t*)c->wdown[l], (const bf16_t*)w->wdown[l], (int)d, (int)F, PERM_NONE, s);
      INIT_TRY(copy_gain(c->norm_attn[l], w->norm_attn[l]));
      INIT_TRY(copy_gain(c->norm_ffn[l], w->norm_ffn[l]));
    }
    INIT_TRY(hipGetLastError());
  }
  INIT_TRY(hipStreamSynchronize(s));
#undef INIT_TRY
  *out = c;
  return DED_OK;
}

void ded_verify_free(ded_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->stream);
  for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
  if (c->meta_ev) (void)hipEventDestroy(c->meta_ev);
  if (c->h_meta) (void)hipHostFree(c->h_meta);
  if (c->h_res) (void)hipHostFree(c->h_res);
  delete c;
}

int ded_verify_step(ded_ctx* c, int32_t batch, const int32_t* prefix_len, const int32_t* n_nodes,
                    const int32_t* parent, const int32_t* token, float* logits_out) {
  if (!c) return DED_EINVAL;
  int rc = validate_step(c->cfg, batch, prefix_len, n_nodes, parent, token, true);
  if (rc != DED_OK) return rc;
  if (c->poisoned && (rc = clear_step_slots(c)) != DED_OK) return rc;
  rc = ingest_and_upload(c, batch, prefix_len, n_nodes, parent, token);
  if (rc != DED_OK) return rc;
  c->pending = false;
  c->have_argmax = false;
  // the fp32 logits are materialised only for a caller that asks for them or samples from them
  const bool want_logits = !c->bf16 || logits_out != nullptr || c->sampling_seen;
  c->have_logits = false;
  rc = c->bf16 ? forward_bf16(c, want_logits) : forward_f32(c);
  if (rc != DED_OK) return rc;
  StepMeta m = c->meta();
  if (want_logits) {
    ProfScope p(c, KC_ARGMAX);
    launch_argmax(c->logits, c->md.V, m.rows, c->md.V, c->d_amax, c->d_margin, c->d_rowflag, c->stream);
  } else {
    ProfScope p(c, KC_TOP2_REDUCE);
    launch_top2_reduce(c->top2_part, (c->md.V + 63) / 64, m.rows, c->d_amax, c->d_margin, c->d_rowflag, c->stream);
  }
  c->have_logits = want_logits;
  if (logits_out) {
    ProfScope p(c, KC_EXPORT);
    launch_export_logits(logits_out, c->logits, c->md.V, m, c->cfg.max_nodes, c->md.V, c->stream);
  }
  rc = launch_status();
  if (rc != DED_OK) return rc;
  c->pending = true;
  c->have_argmax = true;
  return DED_OK;
}

int ded_accept(ded_ctx* c, int32_t mode, int32_t* accepted_tokens, int32_t* n_accepted,
               int32_t* compaction_idx, int32_t* new_prefix_len) {
  if (!c || !accepted_tokens || !n_accepted || !compaction_idx || !new_prefix_len) return DED_EINVAL;
  if (mode != 0 && mode != 1) return DED_EINVAL;
  if (!c->pending) return DED_ESTATE;
  const int mn = c->cfg.max_nodes, stride = mn + 1, B = c->batch;
  if (mode == 1) {
    for (int b = 0; b < B; ++b)
      for (int i = 1; i < c->s_n[b]; ++i)
        if (c->s_parent[(size_t)b * mn + i] != i - 1) return DED_ETREE;
  }
  StepMeta m = c->meta();
  hipStream_t s = c->stream;
  { ProfScope p(c, KC_WALK);
    launch_accept_walk(m, c->d_amax, c->d_rowflag, mode, c->d_nacc, c->d_seqflag, c->d_path, c->d_acctok, stride, s); }
  if (c->md.n_layers > 0 && mode == 0) {
    ProfScope p(c, KC_COMPACT);
    if (c->bf16)
      bf16_kv_compact((bf16_t* const*)c->d_kc, (bf16_t* const*)c->d_vc, c->d_path, c->d_nacc, m, c->md, stride, s);
    else
      f32_kv_compact((float* const*)c->d_kc, (float* const*)c->d_vc, c->d_path, c->d_nacc, m, c->md, stride, s);
  }
  if (launch_status() != DED_OK) return DED_EHIP;
  int32_t* h_n = reinterpret_cast<int32_t*>(c->h_res);
  const int MB = c->cfg.max_batch;
  int32_t* h_flag = h_n + MB;
  int32_t* h_path = h_flag + MB;
  int32_t* h_tok = h_path + (size_t)MB * stride;
  // nacc | seqflag | path | acctok are one device block with the same layout: path and acctok of the live
  // sequences end before (2 MB + (MB + B) * stride) words
  HIP_TRY(hipMemcpyAsync(h_n, c->d_nacc, sizeof(int32_t) * (2 * (size_t)MB + (size_t)(MB + B) * stride),
                         hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  c->pending = false;
  for (int b = 0; b < B; ++b)
    if (h_flag[b]) {  // the walk kept nothing: every sequence's cache is as it was before the step
      int rc = clear_step_slots(c);
      return rc != DED_OK ? rc : DED_ENONFINITE;
    }
  for (int b = 0; b < B; ++b) {
    int len = h_n[b];
    if (len < 1 || len > c->s_n[b]) return DED_EHIP;
    n_accepted[b] = len;
    new_prefix_len[b] = c->s_p[b] + len;
    memcpy(accepted_tokens + (size_t)b * stride, h_tok + (size_t)b * stride, sizeof(int32_t) * len);
    memcpy(compaction_idx + (size_t)b * stride, h_path + (size_t)b * stride, sizeof(int32_t) * len);
  }
  return DED_OK;
}

int ded_sample(ded_ctx* c, float temperature, float top_p, const float* uniform) {
  if (!c || !uniform) return DED_EINVAL;
  if (!(temperature > 0.f) || !(top_p > 0.f) || !(top_p <= 1.f)) return DED_EINVAL;
  if (!c->pending || !c->have_argmax) return DED_ESTATE;
  const int mn = c->cfg.max_nodes, rows = c->batch * c->n_step;
  float* h_u = reinterpret_cast<float*>(c->h_res);  // nothing else is in flight on the pinned result block
  for (int b = 0; b < c->batch; ++b)
    for (int i = 0; i < c->n_step; ++i) {
      float u = i < c->s_n[b] ? uniform[(size_t)b * mn + i] : 0.f;
      if (!(u >= 0.f) || !(u < 1.f)) return DED_EINVAL;
      h_u[b * c->n_step + i] = u;
    }
  HIP_TRY(hipMemcpyAsync(c->d_uniform, h_u, sizeof(float) * rows, hipMemcpyHostToDevice, c->stream));
  // A step keeps its logits only if the caller asked for them or the context has sampled before; the first
  // sampled step of a context recomputes them from the final residual stream, which is still in place.
  c->sampling_seen = true;
  if (!c->have_logits) {
    if (!lm_head_bf16(c, true)) return DED_EINVAL;
    c->have_logits = true;
  }
  { ProfScope p(c, KC_SAMPLE);
    launch_sample_top_p(c->logits, c->md.V, rows, c->md.V, temperature, top_p, c->d_uniform, c->d_amax, c->stream); }
  if (launch_status() != DED_OK) return DED_EHIP;
  int32_t* h_f = reinterpret_cast<int32_t*>(c->h_res) + c->max_rows_pad;
  HIP_TRY(hipMemcpyAsync(h_f, c->d_rowflag, sizeof(int32_t) * rows, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));  // h_res is free again
  for (int b = 0; b < c->batch; ++b)
    for (int i = 0; i < c->s_n[b]; ++i)
      if (h_f[b * c->n_step + i]) {
        c->poisoned = true;
        return DED_ENONFINITE;
      }
  return DED_OK;
}

int ded_get_argmax(ded_ctx* c, int32_t* argmax, float* margin) {
  if (!c || !argmax) return DED_EINVAL;
  if (!c->have_argmax) return DED_ESTATE;
  const int rows = c->batch * c->n_step, mn = c->cfg.max_nodes;
  int32_t* h_a = reinterpret_cast<int32_t*>(c->h_res);
  float* h_m = reinterpret_cast<float*>(c->h_res) + c->max_rows_pad;
  HIP_TRY(hipMemcpyAsync(h_a, c->d_amax, sizeof(int32_t) * rows, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipMemcpyAsync(h_m, c->d_margin, sizeof(float) * rows, hipMemcpyDeviceToHost, c->stream));
  int32_t* h_f = reinterpret_cast<int32_t*>(c->h_res) + 2 * (size_t)c->max_rows_pad;
  HIP_TRY(hipMemcpyAsync(h_f, c->d_rowflag, sizeof(int32_t) * rows, hipMemcpyDeviceToHost, c->stream));
  HIP_TRY(hipStreamSynchronize(c->stream));
  for (int b = 0; b < c->batch; ++b)
    for (int i = 0; i < c->s_n[b]; ++i)
      if (h_f[b * c->n_step + i]) {
        c->poisoned = true;
        return DED_ENONFINITE;
      }
  for (int b = 0; b < c->batch; ++b)
    for (int i = 0; i < c->s_n[b]; ++i) {
      argmax[(size_t)b * mn + i] = h_a[b * c->n_step + i];
      if (margin) margin[(size_t)b * mn + i] = h_m[b * c->n_step + i];
    }
  return DED_OK;
}

static int kv_copy_common(ded_ctx* c, int32_t layer, int32_t seq, int32_t first, int32_t n, void* kp, void* vp,
                          bool to_cache) {
  if (!c || layer < 0 || layer >= c->md.n_layers || seq < 0 || seq >= c->cfg.max_batch || first < 0 || n < 0)
    return DED_EINVAL;
  if ((int64_t)first + n > c->cfg.kv_capacity) return DED_ECAP;
  if (n == 0 || (!kp && !vp)) return DED_OK;
  ProfScope p(c, KC_LAYOUT);
  if (c->bf16) {
    bf16_kv_copy((bf16_t*)c->kc[layer], (bf16_t*)c->vc[layer], (bf16_t*)kp, (bf16_t*)vp, to_cache, seq, first, n,
                 c->md, c->stream);
  } else {
    if (kp) f32_kv_copy((float*)c->kc[layer], (float*)kp, to_cache, seq, first, n, c->md, c->stream);
    if (vp) f32_kv_copy((float*)c->vc[layer], (float*)vp, to_cache, seq, first, n, c->md, c->stream);
  }
  return launch_status();
}

int ded_kv_store(ded_ctx* c, int32_t layer, int32_t seq, int32_t first_slot, int32_t n, const void* k_plain,
                 const void* v_plain) {
  return kv_copy_common(c, layer, seq, first_slot, n, const_cast<void*>(k_plain), const_cast<void*>(v_plain), true);
}

int ded_kv_load(ded_ctx* c, int32_t layer, int32_t seq, int32_t first_slot, int32_t n, void* k_plain,
                void* v_plain) {
  return kv_copy_common(c, layer, seq, first_slot, n, k_plain, v_plain, false);
}

// Transient device buffers of one stand-alone attention call: the step description, the queries and the output
// in operand-fragment form, and the split-KV partials.
struct AttnScratch {
  char* d_meta;
  bf16_t *q_p, *o_p;
  float* part_o;
  float2* part_ml;
  int64_t part_rows;
};

static int tree_attention_common(ded_ctx* c, int32_t layer, int32_t batch, const int32_t* prefix_len,
                                 const int32_t* n_nodes, const int32_t* parent, const void* q, const void* k_tree,
                                 const void* v_tree, void* out, bool st) {
  if (!c || !q || !k_tree || !v_tree || !out) return DED_EINVAL;
  if (layer < 0 || layer >= c->md.n_layers) return DED_EINVAL;
  int rc = validate_step(c->cfg, batch, prefix_len, n_nodes, parent, nullptr, false);
  if (rc != DED_OK) return rc;
  if (c->poisoned && (rc = clear_step_slots(c)) != DED_OK) return rc;
  const ModelDims& md = c->md;
  AttnScratch ws = {c->d_meta, c->q_p, c->o_p, c->attn_part_o, c->attn_part_ml, c->attn_part_rows};
  int ns = 1;
  if (c->bf16) {
    // the key-range count is the workspace path's in both variants, so both give the same bits
    int nmax = 0, pmax = 0;
    for (int b = 0; b < batch; ++b) {
      nmax = std::max(nmax, n_nodes[b]);
      pmax = std::max(pmax, prefix_len[b]);
    }
    StepMeta shape = {};
    shape.batch = batch;
    shape.n_step = round_up(nmax, 16);
    shape.rows = batch * shape.n_step;
    ns = bf16_attn_pick_splits(shape, md, pmax, c->attn_part_rows);
    if (st) {  // carve the library's own array; a call that does not fit is refused before anything is enqueued
      const int64_t rows_pad = round_up(shape.rows, 64), qd = (int64_t)md.H * md.hd;
      const int64_t part_rows = (int64_t)batch * md.H * ns * shape.n_step;
      Carve w(reinterpret_cast<char*>(c->static_scratch));
      ws.d_meta = w.take<char>(c->meta_bytes);
      ws.q_p = w.take<bf16_t>(rows_pad * qd * 2);
      ws.o_p = w.take<bf16_t>(rows_pad * qd * 2);
      ws.part_o = w.take<float>(part_rows * md.hd);
      ws.part_ml = w.take<float2>(part_rows);
      ws.part_rows = part_rows;
      if (w.off > kStaticScratchBytes) return DED_ECAP;
    }
  } else if (st) {
    return DED_EINVAL;  // the fp32 path has no transient buffers of this kind
  }
  rc = ingest_and_upload(c, batch, prefix_len, n_nodes, parent, nullptr, ws.d_meta);
  if (rc != DED_OK) return rc;
  c->pending = false;
  c->have_argmax = false;
  StepMeta m = c->meta_at(ws.d_meta);
  hipStream_t s = c->stream;
  const int mn = c->cfg.max_nodes, qd = md.H * md.hd;
  if (c->bf16) {
    const int rows_pad = round_up(m.rows, 64);
    { ProfScope p(c, KC_LAYOUT);
      bf16_scatter_tree_kv((bf16_t*)c->kc[layer], (bf16_t*)c->vc[layer], (const bf16_t*)k_tree, (const bf16_t*)v_tree, m, md, mn, s);
      bf16_pack_q(ws.q_p, (const bf16_t*)q, m, md, mn, s); }
    { ProfScope p(c, KC_TREE_ATTN);
      bf16_tree_attention(ws.o_p, rows_pad, ws.q_p, (const bf16_t*)c->kc[layer], (const bf16_t*)c->vc[layer], ws.part_o,
                          ws.part_ml, ns, 1, m, md, s); }
    { ProfScope p(c, KC_LAYOUT); bf16_unpack_o((bf16_t*)out, ws.o_p, rows_pad, m, md, mn, s); }
  } else {
    { ProfScope p(c, KC_LAYOUT);
      f32_scatter_tree_kv((float*)c->kc[layer], (float*)c->vc[layer], (const float*)k_tree, (const float*)v_tree, m, md, mn, s);
      f32_gather_rows(c->f_qkv, (const float*)q, m, mn, qd, true, s); }
    { ProfScope p(c, KC_TREE_ATTN);
      f32_tree_attention(c->f_o, c->f_qkv, qd, (const float*)c->kc[layer], (const float*)c->vc[layer], m, md, s); }
    { ProfScope p(c, KC_LAYOUT); f32_gather_rows((float*)out, c->f_o, m, mn, qd, false, s); }
  }
  return launch_status();
}

int ded_tree_attention(ded_ctx* c, int32_t layer, int32_t batch, const int32_t* prefix_len,
                       const int32_t* n_nodes, const int32_t* parent, const void* q, const void* k_tree,
                       const void* v_tree, void* out) {
  return tree_attention_common(c, layer, batch, prefix_len, n_nodes, parent, q, k_tree, v_tree, out, false);
}

int ded_tree_attention_static(ded_ctx* c, int32_t layer, int32_t batch, const int32_t* prefix_len,
                              const int32_t* n_nodes, const int32_t* parent, const void* q, const void* k_tree,
                              const void* v_tree, void* out) {
  if (!c) return DED_EINVAL;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return DED_EHIP;
  }
  if (dev != c->device || !c->static_scratch) return DED_EINVAL;  // the array's address belongs to the context's device
  return tree_attention_common(c, layer, batch, prefix_len, n_nodes, parent, q, k_tree, v_tree, out, true);
}

size_t ded_static_scratch_bytes(void) { return kStaticScratchBytes; }

int ded_probe_stream_read(const void* device_buffer, size_t bytes, void* sink4, void* hip_stream) {
  if (!device_buffer || !sink4 || bytes < 16 || reinterpret_cast<uintptr_t>(device_buffer) % 16) return DED_EINVAL;
  launch_stream_read(device_buffer, bytes / 16 * 16, static_cast<uint32_t*>(sink4), reinterpret_cast<hipStream_t>(hip_stream));
  return launch_status();
}

int ded_profile_enable(ded_ctx* c, int32_t on) {
  if (!c) return DED_EINVAL;
  int rc = prof_drain(c);
  if (rc != DED_OK) return rc;
  if (on) {
    for (int i = 0; i < KC_COUNT; ++i) {
      c->prof_ms[i] = 0;
      c->prof_n[i] = 0;
    }
  }
  c->prof_on = on != 0;
  return DED_OK;
}

int ded_profile_read(ded_ctx* c, int32_t cap, const char** names, double* total_ms, int64_t* launches) {
  if (!c || cap < 0 || (cap > 0 && (!names || !total_ms || !launches))) return DED_EINVAL;
  int rc = prof_drain(c);
  if (rc != DED_OK) return rc;
  for (int i = 0; i < KC_COUNT && i < cap; ++i) {
    names[i] = kClassNames[i];
    total_ms[i] = c->prof_ms[i];
    launches[i] = c->prof_n[i];
  }
  return KC_COUNT;
}

}  // extern "C"
