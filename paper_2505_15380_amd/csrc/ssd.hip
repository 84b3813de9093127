// libssd: host side of the C ABI declared in include/ssd.h.  Validates arguments, carves the caller's
// workspaces, and enqueues the kernels of one forward / acceptance step on the caller's stream.
#include "../../include/ssd.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <type_traits>
#include <vector>

#include "attention.h"
#include "common.h"
#include "gemm.h"
#include "gemm_rows.h"
#include "persistent.h"
#include "dataflow.h"
#include "sample.h"

using namespace ssd;

// ------------------------------------------------------------------------------------------------ errors
static thread_local std::string g_err;
static int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}
#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) return fail(SSD_EHIP, "%s: %s", #expr, hipGetErrorString(e_));   \
  } while (0)
#define LAUNCH_CHECK() HIP_TRY(hipGetLastError())

extern "C" const char* ssd_strerror(int code) {
  switch (code) {
    case SSD_OK: return "ok";
    case SSD_EINVAL: return "invalid argument";
    case SSD_ENOMEM: return "out of pool or buffer space";
    case SSD_EHIP: return "HIP error";
    case SSD_ENOSUP: return "unsupported shape";
    default: return "unknown error";
  }
}
extern "C" const char* ssd_last_error(void) { return g_err.c_str(); }

// ------------------------------------------------------------------------------------------------ profiling
static int g_prof_kind = -1;
static std::vector<std::pair<hipEvent_t, hipEvent_t>> g_prof_events;
struct ProfScope {                   // brackets the launches of one kernel family with a pair of events
  hipEvent_t stop = nullptr;
  hipStream_t st;
  ProfScope(int kind, hipStream_t s) : st(s) {
    if (kind != g_prof_kind) return;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return; }
    (void)hipEventRecord(a, st);
    g_prof_events.emplace_back(a, b);
    stop = b;
  }
  ~ProfScope() { if (stop) (void)hipEventRecord(stop, st); }
};
enum { PROF_QKV = 0, PROF_ATTN = 1, PROF_O = 2, PROF_GATEUP = 3, PROF_DOWN = 4, PROF_HEAD = 5, PROF_PERSISTENT = 6 };

extern "C" int ssd_profile_begin(int kind) {
  if (kind < 0 || kind > 6) return fail(SSD_EINVAL, "profile kind %d out of range", kind);
  if (g_prof_kind >= 0) return fail(SSD_EINVAL, "a profile is already running");
  g_prof_kind = kind;
  return SSD_OK;
}
extern "C" int ssd_profile_end(double* total_ms, int* launches) {
  if (g_prof_kind < 0) return fail(SSD_EINVAL, "no profile is running");
  g_prof_kind = -1;
  double sum = 0;
  int n = 0;
  int rc = SSD_OK;
  for (auto& ev : g_prof_events) {
    float ms = 0;
    hipError_t e = hipEventSynchronize(ev.second);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.first, ev.second);
    if (e != hipSuccess) rc = fail(SSD_EHIP, "profile events: %s", hipGetErrorString(e));
    else { sum += ms; ++n; }
    (void)hipEventDestroy(ev.first);
    (void)hipEventDestroy(ev.second);
  }
  g_prof_events.clear();
  if (total_ms) *total_ms = sum;
  if (launches) *launches = n;
  return rc;
}

// ------------------------------------------------------------------------------------------------ carving
struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <typename T>
  T* take(size_t n) {
    off = (off + 255) & ~(size_t)255;
    T* p = base ? (T*)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
  size_t size() const { return (off + 255) & ~(size_t)255; }
};

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

// ------------------------------------------------------------------------------------------------ model
struct LayerW {
  const float *ln1, *bqkv, *ln2;
  const void *wqkv, *wo, *wgate, *wup, *wdown;
};
struct ssd_model {
  ssd_model_config c;
  int max_positions;
  const void* embed;
  const float* final_norm;
  const void* head;
  std::vector<LayerW> layers;
  const float2* rope;
  PLayer* dev_layers;
  std::vector<PLayer> host_layers;    // per-layer pointers; the persistent kernel needs them equally spaced
  size_t layer_stride = 0;            // bytes between consecutive layers' tensors (0: not equally spaced)
  size_t esize() const { return c.dtype == SSD_DTYPE_BF16 ? 2 : 4; }
  int n_qkv() const { return (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim; }
};

static size_t mat_elems(const ssd_model_config& c, int N, int K) {   // elements a matrix takes in the model workspace
  return c.dtype == SSD_DTYPE_BF16 ? (size_t)cdiv(N, 16) * 16 * K : (size_t)N * K;
}

static int check_config(const ssd_model_config* c, int max_positions) {
  if (!c) return fail(SSD_EINVAL, "null config");
  if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 || c->vocab < 1 ||
      c->n_embed < c->vocab || max_positions < 1 || !(c->rope_base > 1.0f) || !(c->rms_eps >= 0.0f))
    return fail(SSD_EINVAL, "bad model dimensions");
  if (c->dtype != SSD_DTYPE_FP32 && c->dtype != SSD_DTYPE_BF16) return fail(SSD_EINVAL, "bad dtype %d", c->dtype);
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) return fail(SSD_ENOSUP, "head_dim must be 32, 64 or 128");
  if (c->n_q_heads % c->n_kv_heads) return fail(SSD_ENOSUP, "n_q_heads must be a multiple of n_kv_heads");
  if (c->d_model % 32 || (c->n_q_heads * c->head_dim) % 32 || c->d_ffn % 32)
    return fail(SSD_ENOSUP, "d_model, n_q_heads*head_dim and d_ffn must be multiples of 32");
  if (c->vocab > 16384) return fail(SSD_ENOSUP, "vocab > 16384");
  return SSD_OK;
}

// Lays the model workspace out; with base == nullptr only measures it.
static size_t model_layout(const ssd_model_config& c, int max_positions, void* base, ssd_model* m) {
  Carver cv(base);
  const size_t es = c.dtype == SSD_DTYPE_BF16 ? 2 : 4;
  const int d = c.d_model, nqkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, nqd = c.n_q_heads * c.head_dim;
  auto mat = [&](int N, int K) { return (const void*)cv.take<char>(mat_elems(c, N, K) * es); };
  const void* embed = cv.take<char>((size_t)c.n_embed * d * es);
  const float* fn = cv.take<float>(d);
  const void* head = mat(c.vocab, d);
  const float2* rope = cv.take<float2>((size_t)max_positions * (c.head_dim / 2));
  PLayer* dev_layers = cv.take<PLayer>(c.n_layers);
  if (m) { m->embed = embed; m->final_norm = fn; m->head = head; m->rope = rope; m->dev_layers = dev_layers; m->layers.resize(c.n_layers); }
  for (int l = 0; l < c.n_layers; ++l) {
    LayerW w;
    w.ln1 = cv.take<float>(d);
    w.wqkv = mat(nqkv, d);
    w.bqkv = cv.take<float>(nqkv);
    w.wo = mat(d, nqd);
    w.ln2 = cv.take<float>(d);
    w.wgate = mat(c.d_ffn, d);
    w.wup = mat(c.d_ffn, d);
    w.wdown = mat(d, c.d_ffn);
    if (!c.qkv_bias) w.bqkv = nullptr;
    if (m) m->layers[l] = w;
  }
  return cv.size();
}

extern "C" size_t ssd_model_workspace_bytes(const ssd_model_config* cfg, int max_positions) {
  if (check_config(cfg, max_positions) != SSD_OK) return 0;
  return model_layout(*cfg, max_positions, nullptr, nullptr);
}

static int put_matrix(const ssd_model_config& c, const void* src, const void* dst, int N, int K, hipStream_t st) {
  if (c.dtype == SSD_DTYPE_BF16) {
    const int ntiles = cdiv(N, 16);
    const size_t pieces = (size_t)ntiles * (K / 32) * 64;
    const int blocks = (int)std::min<size_t>((pieces + 255) / 256, 65535);
    hipLaunchKernelGGL(k_pack_bf16, dim3(blocks), dim3(256), 0, st, (const bf16_t*)src, (uint4*)dst, N, K, ntiles);
    LAUNCH_CHECK();
  } else {
    HIP_TRY(hipMemcpyAsync((void*)dst, src, (size_t)N * K * 4, hipMemcpyDeviceToDevice, st));
  }
  return SSD_OK;
}

extern "C" int ssd_model_create(const ssd_model_config* cfg, const void* const* dev_weights, int n_weights,
                                int max_positions, void* dev_model_ws, size_t ws_bytes, void* stream, ssd_model** out) {
  int rc = check_config(cfg, max_positions);
  if (rc) return rc;
  if (!dev_weights || !dev_model_ws || !out) return fail(SSD_EINVAL, "null argument");
  if (n_weights != 3 + 8 * cfg->n_layers) return fail(SSD_EINVAL, "expected %d weight pointers, got %d", 3 + 8 * cfg->n_layers, n_weights);
  for (int i = 0; i < n_weights; ++i) {
    const bool is_bias = i >= 3 && (i - 3) % 8 == 2;
    if (!dev_weights[i] && !(is_bias && !cfg->qkv_bias)) return fail(SSD_EINVAL, "weight pointer %d is null", i);
  }
  if ((uintptr_t)dev_model_ws & 255) return fail(SSD_EINVAL, "model workspace must be 256-byte aligned");
  const size_t need = model_layout(*cfg, max_positions, nullptr, nullptr);
  if (ws_bytes < need) return fail(SSD_ENOMEM, "model workspace: need %zu bytes, got %zu", need, ws_bytes);
  ssd_model* m = new (std::nothrow) ssd_model();
  if (!m) return fail(SSD_ENOMEM, "host allocation failed");
  m->c = *cfg;
  m->max_positions = max_positions;
  model_layout(*cfg, max_positions, dev_model_ws, m);
  hipStream_t st = (hipStream_t)stream;
  const ssd_model_config& c = *cfg;
  const size_t es = m->esize();
  const int d = c.d_model, nqkv = m->n_qkv(), nqd = c.n_q_heads * c.head_dim;
#define TRY_RC(x) do { rc = (x); if (rc) { delete m; return rc; } } while (0)
#define COPY(dst, src, bytes) do { hipError_t e_ = hipMemcpyAsync((void*)(dst), (src), (bytes), hipMemcpyDeviceToDevice, st); \
    if (e_ != hipSuccess) { delete m; return fail(SSD_EHIP, "copy of weights: %s", hipGetErrorString(e_)); } } while (0)
  COPY(m->embed, dev_weights[0], (size_t)c.n_embed * d * es);
  COPY(m->final_norm, dev_weights[1], (size_t)d * 4);
  TRY_RC(put_matrix(c, dev_weights[2], m->head, c.vocab, d, st));
  for (int l = 0; l < c.n_layers; ++l) {
    const void* const* w = dev_weights + 3 + 8 * l;
    const LayerW& L = m->layers[l];
    COPY(L.ln1, w[0], (size_t)d * 4);
    TRY_RC(put_matrix(c, w[1], L.wqkv, nqkv, d, st));
    if (c.qkv_bias) COPY(L.bqkv, w[2], (size_t)nqkv * 4);
    TRY_RC(put_matrix(c, w[3], L.wo, d, nqd, st));
    COPY(L.ln2, w[4], (size_t)d * 4);
    TRY_RC(put_matrix(c, w[5], L.wgate, c.d_ffn, d, st));
    TRY_RC(put_matrix(c, w[6], L.wup, c.d_ffn, d, st));
    TRY_RC(put_matrix(c, w[7], L.wdown, d, c.d_ffn, st));
  }
  {
    const int half = c.head_dim / 2, total = max_positions * half;
    hipLaunchKernelGGL(k_rope_table, dim3(cdiv(total, 256)), dim3(256), 0, st, (float2*)m->rope, max_positions, half,
                       (double)c.rope_base);
    hipError_t e_ = hipGetLastError();
    if (e_ != hipSuccess) { delete m; return fail(SSD_EHIP, "rope table: %s", hipGetErrorString(e_)); }
  }
  m->host_layers.resize(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerW& L = m->layers[l];
    m->host_layers[l] = PLayer{L.wqkv, L.wo, L.wgate, L.wup, L.wdown, L.ln1, L.ln2, L.bqkv};
  }
  m->layer_stride = 1;
  if (c.n_layers > 1) {
    const size_t st = (const char*)m->host_layers[1].wqkv - (const char*)m->host_layers[0].wqkv;
    bool uniform = true;
    for (int l = 1; l < c.n_layers; ++l) {
      const PLayer &x = m->host_layers[l - 1], &y = m->host_layers[l];
      auto gap = [&](const void* p, const void* q) { return (size_t)((const char*)q - (const char*)p); };
      uniform = uniform && gap(x.wqkv, y.wqkv) == st && gap(x.wo, y.wo) == st && gap(x.wgate, y.wgate) == st &&
                gap(x.wup, y.wup) == st && gap(x.wdown, y.wdown) == st && gap(x.ln1, y.ln1) == st && gap(x.ln2, y.ln2) == st &&
                (!c.qkv_bias || gap(x.bqkv, y.bqkv) == st);
    }
    m->layer_stride = uniform ? st : 0;
  }
  {
    hipError_t e_ = hipMemcpyAsync(m->dev_layers, m->host_layers.data(), sizeof(PLayer) * c.n_layers, hipMemcpyHostToDevice, st);
    if (e_ == hipSuccess) e_ = hipStreamSynchronize(st);
    if (e_ != hipSuccess) { delete m; return fail(SSD_EHIP, "layer table: %s", hipGetErrorString(e_)); }
  }
#undef COPY
#undef TRY_RC
  *out = m;
  return SSD_OK;
}

extern "C" int ssd_model_destroy(ssd_model* m) {
  delete m;
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ kv
constexpr int MAX_SPLITS = 16;   // capacity of the k-split partial buffer
constexpr int MAX_ROWS = 1024;

struct ssd_kv {
  const ssd_model* m;
  KvView v;
  int max_seqs, max_rows, NC;
  // workspace
  Rows rows;
  float *h, *q, *o_part, *ml_part, *part, *logits, *probs;
  void *xn, *attn, *act;
  int32_t* scratch_i;              // [2 * max_seqs]: n_accepted / next_token when the caller passes none
  // persistent-kernel buffers (one instance per layer, see persistent.h)
  float *p_h, *p_sumsq, *p_part, *p_att_o, *p_att_ml;
  bf16_t *p_hg, *p_q, *p_attn, *p_act;        // split operand rows: 2 bf16 per value
  int32_t* tickets;
  uint32_t* bar;
  unsigned long long* trace;       // [256][512] clock samples of the persistent kernel's barriers
  bool trace_on = false;
  int NP, p_rows;
  uint32_t bar_epoch = 0;          // grid barriers executed so far by the kernel with barriers (compared wrap-safe)
  uint32_t launch_no = 1;          // host's copy of ctl[3]: the number the next forward on this cache will read
  int persistent_wgs = 0;          // 0: the persistent kernel is not usable for this cache
  int cus = 0;                     // compute units of the device
  // tagged workspace of the barrier-free forward (see dataflow.h); null when that kernel is not usable
  u64 *t_base = nullptr, *t_h, *t_hg, *t_sq, *t_q, *t_kvn, *t_attn, *t_att_p, *t_part2, *t_rowblk;
  size_t t_words = 0;
  bool dataflow = false;
  bool attn_whole = false;   // barrier-free kernel: attention of short prefixes without parts.  Default: caches with two
                             // pending slots (draft caches: one-row steps gain 10 %); SSD_ATTN_WHOLE=0 never, 1 every cache
  bool gemm_wide = true;     // per-operator path, many rows: the LDS-shared GEMM kernel (SSD_GEMM=narrow: the generic one)
  bool attn_mfma = true;     // per-operator path: matrix-core attention where it applies (SSD_ATTN=valu: the scalar kernel)
  int32_t* ticket_alt = nullptr;   // ssd_verify_noalloc: the commit's arrival counter in the library's static scratch
  bool capturing = false;          // a cycle is being captured on this cache: no synchronisation, no fallback kernels
  int last_path = 0;               // 1 per-operator launches, 2 barrier kernel, 3 barrier-free kernel, 4 the same with attention without parts
  bool last_whole = false;
  int df_sb = 0;             // SSD_DF_FLIGHT=2|4|10|12: words in flight per thread of the operand staging (0: chosen per launch)
  // host
  int32_t* mirror_host;
  std::vector<int> len_ub, npend_ub;
};

static size_t kv_layout(const ssd_model* m, int max_seqs, int max_rows, int n_blocks, int mbps, void* base, ssd_kv* kv) {
  const ssd_model_config& c = m->c;
  Carver cv(base);
  const int Mmax = max_seqs * max_rows;
  const int NC = cdiv(m->max_positions, ATT_CHUNK);
  const int nqd = c.n_q_heads * c.head_dim;
  int32_t* len = cv.take<int32_t>(max_seqs);
  int32_t* n_pend = cv.take<int32_t>(max_seqs);
  int32_t* pend = cv.take<int32_t>(2 * max_seqs);
  int32_t* owned = cv.take<int32_t>(max_seqs);
  int32_t* table = cv.take<int32_t>((size_t)max_seqs * mbps);
  int32_t* free_stack = cv.take<int32_t>(n_blocks);
  int32_t* ctl = cv.take<int32_t>(8);
  int32_t* rpos = cv.take<int32_t>(Mmax);
  int32_t* ract = cv.take<int32_t>(Mmax);
  int32_t* scratch_i = cv.take<int32_t>(2 * max_seqs);
  const int Mpad = cdiv(Mmax, 16) * 16;                    // operand buffers also serve as split rows: whole row tiles
  float* h = cv.take<float>((size_t)Mmax * c.d_model);
  void* xn = cv.take<float>((size_t)Mpad * c.d_model);
  float* q = cv.take<float>((size_t)Mmax * nqd);
  float* o_part = cv.take<float>((size_t)Mmax * c.n_q_heads * NC * c.head_dim);
  float* ml_part = cv.take<float>((size_t)Mmax * c.n_q_heads * NC * 2);
  void* attn = cv.take<float>((size_t)Mpad * nqd);
  float* part = cv.take<float>((size_t)MAX_SPLITS * Mmax * c.d_model);
  void* act = cv.take<float>((size_t)Mpad * c.d_ffn);
  float* logits = cv.take<float>((size_t)Mmax * c.vocab);
  float* probs = cv.take<float>((size_t)Mmax * c.vocab);
  const int NP = cdiv(m->max_positions, ATT_PART);
  const bool p_ok = c.dtype == SSD_DTYPE_BF16 && c.head_dim == 64;
  const int PR = p_ok ? std::min(Mmax, 16) : 0, L = c.n_layers;      // rows the persistent kernel can take
  float* p_h = cv.take<float>((size_t)(2 * L + 1) * PR * c.d_model);
  bf16_t* p_hg = cv.take<bf16_t>((size_t)(2 * L + 1) * PR * c.d_model * 2);
  float* p_sumsq = cv.take<float>((size_t)(2 * L + 1) * PR * (c.d_model / 32 + 1));
  bf16_t* p_q = cv.take<bf16_t>((size_t)L * PR * nqd * 2);
  bf16_t* p_attn = cv.take<bf16_t>((size_t)L * PR * nqd * 2);
  bf16_t* p_act = cv.take<bf16_t>((size_t)L * PR * c.d_ffn * 2);
  float* p_part = cv.take<float>((size_t)2 * L * P_MAX_SPLITS * PR * c.d_model);
  float* p_att_o = cv.take<float>((size_t)L * PR * c.n_q_heads * NP * 64);
  float* p_att_ml = cv.take<float>((size_t)L * PR * c.n_q_heads * NP * 2);
  int32_t* tickets = cv.take<int32_t>(std::max(c.d_model / 32 + 1, Mmax * c.n_kv_heads));
  uint32_t* bar = cv.take<uint32_t>(128);
  unsigned long long* trace = cv.take<unsigned long long>(p_ok ? 256 * 512 : 0);
  // tagged words of the barrier-free forward: one block, zeroed at creation
  const size_t TR = PR;
  const size_t w_h = (size_t)(2 * L + 1) * TR * c.d_model, w_sq = (size_t)(2 * L + 1) * TR * (c.d_model / 32);
  const size_t w_q = (size_t)L * TR * nqd, w_kvn = (size_t)L * TR * 2 * c.n_kv_heads * 64;
  const size_t w_attp = (size_t)L * TR * c.n_q_heads * NP * 96;
  const size_t w_part2 = (size_t)2 * (c.d_ffn / 32) * TR * c.d_model;
  const size_t t_words = w_h * 2 + w_sq + w_q * 2 + w_kvn + w_attp + w_part2 + 16;
  u64* t_base = cv.take<u64>(t_words);
  if (kv) {
    u64* t = t_base;
    kv->t_base = t_base; kv->t_words = t_words;
    kv->t_h = t; t += w_h; kv->t_hg = t; t += w_h; kv->t_sq = t; t += w_sq; kv->t_q = t; t += w_q; kv->t_attn = t; t += w_q;
    kv->t_kvn = t; t += w_kvn; kv->t_att_p = t; t += w_attp; kv->t_part2 = t; t += w_part2;
    kv->t_rowblk = t;

    kv->trace = trace;
    kv->p_h = p_h; kv->p_hg = p_hg; kv->p_sumsq = p_sumsq; kv->p_q = p_q; kv->p_attn = p_attn; kv->p_act = p_act; kv->p_part = p_part; kv->p_att_o = p_att_o;
    kv->p_att_ml = p_att_ml; kv->tickets = tickets; kv->bar = bar; kv->NP = NP; kv->p_rows = PR;
    kv->v.len = len; kv->v.n_pend = n_pend; kv->v.pend = pend; kv->v.owned = owned; kv->v.table = table;
    kv->v.free_stack = free_stack; kv->v.ctl = ctl;
    kv->rows.pos = rpos; kv->rows.active = ract;
    kv->scratch_i = scratch_i;
    kv->h = h; kv->xn = xn; kv->q = q; kv->o_part = o_part; kv->ml_part = ml_part; kv->attn = attn; kv->part = part;
    kv->act = act; kv->logits = logits; kv->probs = probs;
    kv->NC = NC;
  }
  return cv.size();
}

extern "C" size_t ssd_kv_pool_bytes(const ssd_model* m, int n_blocks, int block_tokens) {
  if (!m || n_blocks < 1 || block_tokens < 1) return 0;
  return (size_t)m->c.n_layers * 2 * n_blocks * m->c.n_kv_heads * block_tokens * m->c.head_dim * m->esize();
}

extern "C" size_t ssd_kv_workspace_bytes(const ssd_model* m, int max_seqs, int max_rows, int n_blocks, int mbps) {
  if (!m || max_seqs < 1 || max_rows < 1 || n_blocks < 1 || mbps < 1) return 0;
  return kv_layout(m, max_seqs, max_rows, n_blocks, mbps, nullptr, nullptr);
}

extern "C" int ssd_kv_create(const ssd_model* m, int max_seqs, int max_rows, int n_blocks, int block_tokens, int mbps,
                             int pending_cap, void* dev_pool, size_t pool_bytes, void* dev_ws, size_t ws_bytes,
                             void* stream, ssd_kv** out) {
  if (!m || !dev_pool || !dev_ws || !out) return fail(SSD_EINVAL, "null argument");
  if (max_seqs < 1 || max_rows < 1 || n_blocks < 1 || block_tokens < 1 || mbps < 1)
    return fail(SSD_EINVAL, "bad cache dimensions");
  if (max_seqs * max_rows > MAX_ROWS) return fail(SSD_ENOSUP, "max_seqs*max_rows = %d exceeds %d", max_seqs * max_rows, MAX_ROWS);
  if (pending_cap != 1 && pending_cap != 2) return fail(SSD_EINVAL, "pending_cap must be 1 or 2");
  if (max_rows < pending_cap) return fail(SSD_EINVAL, "max_rows < pending_cap");
  if (((uintptr_t)dev_pool & 255) || ((uintptr_t)dev_ws & 255)) return fail(SSD_EINVAL, "buffers must be 256-byte aligned");
  const size_t need_pool = ssd_kv_pool_bytes(m, n_blocks, block_tokens);
  if (pool_bytes < need_pool) return fail(SSD_ENOMEM, "KV pool: need %zu bytes, got %zu", need_pool, pool_bytes);
  const size_t need_ws = kv_layout(m, max_seqs, max_rows, n_blocks, mbps, nullptr, nullptr);
  if (ws_bytes < need_ws) return fail(SSD_ENOMEM, "KV workspace: need %zu bytes, got %zu", need_ws, ws_bytes);
  ssd_kv* kv = new (std::nothrow) ssd_kv();
  if (!kv) return fail(SSD_ENOMEM, "host allocation failed");
  kv->m = m;
  kv->max_seqs = max_seqs;
  kv->max_rows = max_rows;
  kv_layout(m, max_seqs, max_rows, n_blocks, mbps, dev_ws, kv);
  KvView& v = kv->v;
  v.pool = dev_pool;
  v.n_blocks = n_blocks; v.bt = block_tokens; v.mbps = mbps; v.max_seqs = max_seqs; v.pcap = pending_cap;
  v.n_layers = m->c.n_layers; v.nkv = m->c.n_kv_heads; v.hd = m->c.head_dim;
  v.err = kv->bar + 64;
  hipError_t e = hipHostMalloc((void**)&kv->mirror_host, (2 * max_seqs + 2) * sizeof(int32_t), hipHostMallocMapped);
  if (e != hipSuccess) { delete kv; return fail(SSD_EHIP, "hipHostMalloc: %s", hipGetErrorString(e)); }
  memset(kv->mirror_host, 0, (2 * max_seqs + 2) * sizeof(int32_t));
  e = hipHostGetDevicePointer((void**)&v.mirror, kv->mirror_host, 0);
  if (e != hipSuccess) { (void)hipHostFree(kv->mirror_host); delete kv; return fail(SSD_EHIP, "hipHostGetDevicePointer: %s", hipGetErrorString(e)); }
  kv->len_ub.assign(max_seqs, 0);
  kv->npend_ub.assign(max_seqs, 0);
  const int n = std::max(std::max(n_blocks, max_seqs * mbps), max_seqs);
  hipLaunchKernelGGL(k_kv_init, dim3(cdiv(n, 256)), dim3(256), 0, (hipStream_t)stream, v);
  e = hipGetLastError();
  if (e == hipSuccess) e = hipMemsetAsync(kv->bar, 0, 128 * sizeof(uint32_t), (hipStream_t)stream);
  if (e == hipSuccess)
    e = hipMemsetAsync(kv->tickets, 0, sizeof(int32_t) * std::max(m->c.d_model / 32 + 1, max_seqs * max_rows * m->c.n_kv_heads),
                       (hipStream_t)stream);
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess)
      kv->cus = cus;                                       // (every path sizes its k-splits by it)
  }
  // The persistent forward needs: bf16 storage, head_dim 64, 16-token blocks, <= 16 query heads per kv head.
  kv->persistent_wgs = 0;
  if (e == hipSuccess && m->c.dtype == SSD_DTYPE_BF16 && m->c.head_dim == 64 && block_tokens == 16 && m->layer_stride &&
      m->c.n_q_heads / m->c.n_kv_heads <= 16 &&
      (size_t)n_blocks * m->c.n_kv_heads * 1024 < ((size_t)1 << 31)) {   // lane offsets into a K/V plane are 32-bit
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus >= 16) {
      const int want = std::max(32, cdiv(m->c.d_ffn / 16, 2));      // two gate/up tile pairs per workgroup
      kv->persistent_wgs = std::max(0, std::min(want, cus));        // one workgroup per CU at most: all co-resident
      kv->cus = cus;
    }
  }
  // The barrier-free forward additionally needs its word offsets to fit 32 bits; its words start untagged (zero).
  kv->dataflow = false;
  if (e == hipSuccess && kv->persistent_wgs > 0 && kv->t_words > 0 && kv->t_words < ((size_t)1 << 32)) {
    e = hipMemsetAsync(kv->t_base, 0, kv->t_words * sizeof(u64), (hipStream_t)stream);
    const char* env = getenv("SSD_FORWARD");
    kv->dataflow = !(env && strcmp(env, "barrier") == 0);
  }
  {
    const char* env = getenv("SSD_ATTN");
    kv->attn_mfma = !(env && strcmp(env, "valu") == 0);
    env = getenv("SSD_ATTN_WHOLE");
    kv->attn_whole = env ? (env[0] == '1' || (env[0] == '2' && pending_cap == 2)) : (pending_cap == 2);
    env = getenv("SSD_DF_FLIGHT");
    kv->df_sb = env ? atoi(env) : 0;
    if (kv->df_sb != 2 && kv->df_sb != 4 && kv->df_sb != 10 && kv->df_sb != 12) kv->df_sb = 0;
    env = getenv("SSD_GEMM");
    kv->gemm_wide = !(env && strcmp(env, "narrow") == 0);
  }
  if (e != hipSuccess) { (void)hipHostFree(kv->mirror_host); delete kv; return fail(SSD_EHIP, "k_kv_init: %s", hipGetErrorString(e)); }
  *out = kv;
  return SSD_OK;
}

extern "C" int ssd_kv_destroy(ssd_kv* kv) {
  if (!kv) return SSD_OK;
  if (kv->mirror_host) (void)hipHostFree(kv->mirror_host);
  delete kv;
  return SSD_OK;
}

// Error words that device code left in the host-mapped mirror (no synchronisation: what has been published so far).
// They are sticky until ssd_kv_clear_error.
static int kv_check_flags(const ssd_kv* kv) {
  const volatile int32_t* mh = kv->mirror_host;
  const int dev_err = mh[2 * kv->max_seqs + 1], st_err = mh[2 * kv->max_seqs];
  if (dev_err & (int)DEV_ERR_TIMEOUT)
    return fail(SSD_EHIP, "a bounded wait inside a persistent forward kernel timed out: results since then are void and "
                          "nothing was committed; call ssd_kv_clear_error before using this cache again");
  if (dev_err & (int)DEV_ERR_TAGS)
    return fail(SSD_EHIP, "the launch numbering of this cache is exhausted; call ssd_kv_clear_error");
  if (st_err & KV_ERR_ROLLBACK)
    return fail(SSD_EINVAL, "a rollback asked for more positions than the sequence held and was refused");
  if (st_err & KV_ERR_POOL) return fail(SSD_ENOMEM, "device allocator reported pool exhaustion");
  return SSD_OK;
}

// Bring the host's length bounds up to date with the device (synchronises the stream).
static int kv_refresh(ssd_kv* kv, hipStream_t st) {
  HIP_TRY(hipStreamSynchronize(st));
  for (int s = 0; s < kv->max_seqs; ++s) {
    kv->len_ub[s] = kv->mirror_host[2 * s];
    kv->npend_ub[s] = kv->mirror_host[2 * s + 1];
  }
  return kv_check_flags(kv);
}

// Re-zero everything the persistent kernels synchronise through and restart the launch numbering (stream-ordered).
static int kv_clear_sync_state(ssd_kv* kv, hipStream_t st) {
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  HIP_TRY(hipStreamIsCapturing(st, &cs));
  if (cs != hipStreamCaptureStatusNone) return fail(SSD_EINVAL, "the cache's launch numbering cannot be cleared inside a stream capture");
  HIP_TRY(hipMemsetAsync(kv->bar, 0, 128 * sizeof(uint32_t), st));
  HIP_TRY(hipMemsetAsync(kv->tickets, 0, sizeof(int32_t) * std::max(kv->m->c.d_model / 32 + 1, kv->max_seqs * kv->max_rows * kv->m->c.n_kv_heads), st));
  if (kv->t_base && kv->t_words) HIP_TRY(hipMemsetAsync(kv->t_base, 0, kv->t_words * sizeof(u64), st));
  hipLaunchKernelGGL(k_kv_clear_error, dim3(1), dim3(1), 0, st, kv->v);
  LAUNCH_CHECK();
  kv->launch_no = 1;
  kv->bar_epoch = 0;
  return SSD_OK;
}

// Before enqueuing `n` more forwards on the cache: the launch numbers they will read must stay below the limit.
static int kv_launch_guard(ssd_kv* kv, hipStream_t st, uint32_t n) {
  if (kv->launch_no + n < TAG_LIMIT) return SSD_OK;
  return kv_clear_sync_state(kv, st);
}

// Can sequences [seq0, seq0+B) each take R more positions?  Uses the host's upper bounds; refreshes once
// from the device before giving up.
static int kv_check_room(ssd_kv* kv, int seq0, int B, int R, hipStream_t st) {
  for (int attempt = 0; attempt < 2; ++attempt) {
    long blocks = 0;
    bool ok = true;
    for (int s = 0; s < kv->max_seqs; ++s) {
      const bool in = s >= seq0 && s < seq0 + B;
      const int tokens = kv->len_ub[s] + (in ? R : 0);
      const int nb = cdiv(tokens, kv->v.bt);
      if (in && (nb > kv->v.mbps || tokens > kv->m->max_positions)) ok = false;
      blocks += nb;
    }
    if (ok && blocks <= kv->v.n_blocks) return SSD_OK;
    if (attempt == 0) {
      int rc = kv_refresh(kv, st);
      if (rc) return rc;
    }
  }
  return fail(SSD_ENOMEM, "KV cache cannot hold %d more positions for sequences %d..%d", R, seq0, seq0 + B - 1);
}

// ------------------------------------------------------------------------------------------------ forward
template <typename DT, int EPI>
static int launch_gemm(const ssd_model* m, GemmArgs g, int items, hipStream_t st) {
  if (m->c.dtype == SSD_DTYPE_BF16) {
    const int MT = cdiv(g.M, 16);
    if (MT <= 1) hipLaunchKernelGGL((k_gemm_bf16<1, EPI, BF16>), dim3(items), dim3(BLOCK), 0, st, g);
    else if (MT <= 2) hipLaunchKernelGGL((k_gemm_bf16<2, EPI, BF16>), dim3(items), dim3(BLOCK), 0, st, g);
    else hipLaunchKernelGGL((k_gemm_bf16<2, EPI, BF16>), dim3(items, cdiv(MT, 2)), dim3(BLOCK), 0, st, g);
  } else {
    hipLaunchKernelGGL((k_gemm_f32<EPI, F32>), dim3(items), dim3(BLOCK), 0, st, g);
  }
  LAUNCH_CHECK();
  return SSD_OK;
}

// Launch shape of k_gemm_wide (see gemm.h) for M rows: fewest row groups of at most 4 tiles, the largest staged chunk
// that fits the LDS budget, and for k-split outputs one slice per chunk up to the partial buffer's capacity.
struct WidePlan {
  int mtw, grid, waves;
  size_t lds;
  WideArgs wa;
};
static WidePlan plan_wide(int M, int N, int K, bool partial, int mtw_forced, int max_slices) {
  WidePlan p;
  const int MT = cdiv(M, 16), KT = K / 32;
  p.waves = WIDE_WAVES;
  int n_rowg = cdiv(MT, 4);
  p.mtw = cdiv(MT, n_rowg);
  if (mtw_forced >= 1 && mtw_forced <= WIDE_MAX_MTW) p.mtw = mtw_forced;
  if (p.mtw == 5) p.mtw = 6;                              // instantiated: 1, 2, 3, 4, 6, 8
  if (p.mtw == 7) p.mtw = 8;
  n_rowg = cdiv(MT, p.mtw);
  const int lds_budget = WIDE_LDS_BYTES;
  const int kc_slice = (lds_budget / 2048 / p.mtw) & ~3;                 // k-tiles per slice of a k-split output
  const int kc_max = (WIDE_SG * p.waves / p.mtw) & ~3;                   // k-tiles per staged chunk (two buffers of it)
  const int n_pairs = partial ? cdiv(cdiv(N, 16), 2) : cdiv(N, 16);
  p.wa.n_colg = cdiv(n_pairs, p.waves);
  p.wa.n_rowg = n_rowg;
  p.wa.n_slices = partial ? std::min(max_slices, std::max(1, cdiv(KT, kc_slice))) : 1;
  p.wa.slice_kt = (cdiv(KT, p.wa.n_slices) + 3) & ~3;
  p.wa.n_slices = cdiv(KT, p.wa.slice_kt);
  p.wa.KC = std::min(kc_max, p.wa.slice_kt);
  p.grid = 8 * cdiv(p.wa.n_colg, 8) * n_rowg * p.wa.n_slices;          // see the kernel's index map
  p.lds = (size_t)2 * p.mtw * p.wa.KC * 2048;
  return p;
}

template <int EPI>
static int launch_wide(const GemmArgs& g, const WidePlan& p, hipStream_t st) {
  static const hipError_t lds_ok = [] {                   // more than 64 KB of dynamic LDS is opt-in, once per process
    const void* fns[] = {(const void*)k_gemm_wide<1, EPI, 8, 1>, (const void*)k_gemm_wide<2, EPI, 8, 1>,
                         (const void*)k_gemm_wide<3, EPI, 8, 1>, (const void*)k_gemm_wide<4, EPI, 8, 1>,
                         (const void*)k_gemm_wide<6, EPI, 8, 1>, (const void*)k_gemm_wide<8, EPI, 8, 1>};
    for (const void* f : fns) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, WIDE_LDS_BYTES);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }();
  if (lds_ok != hipSuccess) return fail(SSD_EHIP, "hipFuncSetAttribute: %s", hipGetErrorString(lds_ok));
  const dim3 grid(p.grid), block(p.waves * 64);
  switch (p.mtw) {
    case 1: hipLaunchKernelGGL((k_gemm_wide<1, EPI, 8, 1>), grid, block, p.lds, st, g, p.wa); break;
    case 2: hipLaunchKernelGGL((k_gemm_wide<2, EPI, 8, 1>), grid, block, p.lds, st, g, p.wa); break;
    case 3: hipLaunchKernelGGL((k_gemm_wide<3, EPI, 8, 1>), grid, block, p.lds, st, g, p.wa); break;
    case 4: hipLaunchKernelGGL((k_gemm_wide<4, EPI, 8, 1>), grid, block, p.lds, st, g, p.wa); break;
    case 6: hipLaunchKernelGGL((k_gemm_wide<6, EPI, 8, 1>), grid, block, p.lds, st, g, p.wa); break;
    case 8: hipLaunchKernelGGL((k_gemm_wide<8, EPI, 8, 1>), grid, block, p.lds, st, g, p.wa); break;
    default: return fail(SSD_EINVAL, "no wide GEMM for %d row tiles per workgroup", p.mtw);
  }
  LAUNCH_CHECK();
  return SSD_OK;
}

// Launch of k_gemm_rows (gemm_rows.h), from 256 rows on.  The tile a workgroup owns is chosen for the fewest bytes per
// workgroup at a workgroup per CU or fewer: 8 waves take 64, 128 or 256 rows (by the launch's rows) x 12 weight tiles
// of gate and up or 8 of a k-split output; the QKV projection, whose epilogue wants a whole head in one wave, 4 waves
// x 64 or 128 rows x one head.  k-split outputs get 8 slices, one per XCD (16 where that still leaves few workgroups).
// Returns the number of slices (> 0).
template <int EPI>
static int launch_rows(const GemmArgs& g, int cus, int hd, bool partial, int max_slices, hipStream_t st) {
  const int KT = g.K / 32, MT = cdiv(g.M, 16);
  const int n_wt = EPI == EPI_SWIGLU ? 2 * cdiv(g.N, 16) : cdiv(g.N, 16);     // weight tiles in all (gate and up both count)
  RowsPlan p;
  auto slices = [&](int n_wg) {                            // a multiple of 8 slices (one XCD each), about a workgroup per CU
    int ns = 1;
    if (partial && KT >= 16 && max_slices >= 8) ns = (n_wg * 12 <= cus && KT >= 64 && max_slices >= 16) ? 16 : 8;
    p.slice_kt = cdiv(KT, ns);
    p.n_slices = cdiv(KT, p.slice_kt);
  };
  if constexpr (EPI == EPI_QKV) {
    const int tm = MT >= 48 ? 2 : 1;                       // 64 rows x one head per workgroup, 128 rows from 768 rows on
    p.n_rowb = cdiv(MT, 4 * tm);
    p.n_colb = cdiv(n_wt, hd / 16);
    slices(1);
    const dim3 grid(8 * cdiv(p.n_colb, 8) * p.n_rowb), block(256);
    if (hd == 64 && tm == 1) hipLaunchKernelGGL((k_gemm_rows<EPI, 1, 4, 4, 1, 6, 1>), grid, block, 0, st, g, p);
    else if (hd == 64) hipLaunchKernelGGL((k_gemm_rows<EPI, 2, 4, 4, 1, 6, 1>), grid, block, 0, st, g, p);
    else if (hd == 128 && tm == 1) hipLaunchKernelGGL((k_gemm_rows<EPI, 1, 8, 4, 1, 6, 1>), grid, block, 0, st, g, p);
    else if (hd == 128) hipLaunchKernelGGL((k_gemm_rows<EPI, 2, 8, 4, 1, 4, 1>), grid, block, 0, st, g, p);
    else return fail(SSD_ENOSUP, "no many-row QKV kernel for head_dim %d", hd);
  } else {
    constexpr int TN = EPI == EPI_SWIGLU ? 6 : 4;
    // rows per workgroup: 64 below 384 rows, 128 up to 767, 256 from there on (the tile grows with the rows as long as
    // about 200 workgroups remain: a workgroup's bytes per output fall, the number of busy CUs does not)
    const int tm = MT >= 48 ? 4 : MT >= 24 ? 2 : 1;
    p.n_rowb = cdiv(MT, 4 * tm);
    p.n_colb = cdiv(n_wt, 2 * TN);
    slices(p.n_colb * p.n_rowb);
    const dim3 grid(p.n_slices > 1 ? 8 * cdiv(p.n_slices, 8) * p.n_colb * p.n_rowb : 8 * cdiv(p.n_colb, 8) * p.n_rowb), block(512);
    if (tm == 4) hipLaunchKernelGGL((k_gemm_rows<EPI, 4, TN, 4, 2, 2, 1>), grid, block, 0, st, g, p);
    else if (tm == 2) hipLaunchKernelGGL((k_gemm_rows<EPI, 2, TN, 4, 2, 6, 1>), grid, block, 0, st, g, p);
    else hipLaunchKernelGGL((k_gemm_rows<EPI, 1, TN, 4, 2, 6, 1>), grid, block, 0, st, g, p);
  }
  LAUNCH_CHECK();
  return p.n_slices;
}

static int pick_splits(int K, int npairs) {
  const int KT = K / 32;
  int gs = std::max(1, 256 / std::max(1, npairs));
  gs = std::min(gs, std::max(1, KT / 8));
  return std::min(gs, MAX_SPLITS);
}

template <typename DT, int HD>
static int launch_attn(AttnArgs a, int nchunks, int nkv, int B, int M, bool mfma, hipStream_t st) {
  if constexpr (std::is_same<DT, BF16>::value && (HD == 64 || HD == 128)) {
    if (mfma && a.kv.bt == 16) {                          // keys and values as matrix-core fragments, 256-key parts
      const int nparts = cdiv(nchunks * ATT_CHUNK, ATT_PART_KEYS);
      // many query rows per sequence (prefill chunks): groups of row tiles get workgroups of their own
      const int ntiles = cdiv(a.rows.R * (a.nq / nkv), 16);
      // (about two workgroups per CU: a group that stages a part's keys for more row tiles re-reads them less)
      const int groups = std::max(1, std::min(cdiv(ntiles, 4), cdiv(512, nparts * nkv * B)));
      a.nparts = nparts;
      a.tiles_per_wg = (cdiv(ntiles, groups) + 3) & ~3;
      hipLaunchKernelGGL((k_attn_part_mfma<HD>), dim3(nparts * cdiv(ntiles, a.tiles_per_wg), nkv, B), dim3(BLOCK), 0, st, a);
      LAUNCH_CHECK();
      hipLaunchKernelGGL((k_attn_combine_parts<HD, F32>), dim3(M * a.nq), dim3(WAVE), 0, st, a);
      LAUNCH_CHECK();
      return SSD_OK;
    }
  }
  hipLaunchKernelGGL((k_attn_chunk<HD, DT>), dim3(nchunks, nkv, B), dim3(BLOCK), 0, st, a);
  LAUNCH_CHECK();
  hipLaunchKernelGGL((k_attn_combine<HD, F32>), dim3(M * a.nq), dim3(WAVE), 0, st, a);
  LAUNCH_CHECK();
  return SSD_OK;
}

// The same forward as one persistent kernel (see persistent.h).
static int forward_persistent(const ssd_model* m, ssd_kv* kv, Rows rows, int B, int pcap, const int32_t* dev_tokens,
                              int tok_stride, bool with_head, hipStream_t st) {
  const ssd_model_config& c = m->c;
  PArgs a;
  memset(&a, 0, sizeof a);
  a.n_layers = c.n_layers; a.d = c.d_model; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads; a.ffn = c.d_ffn; a.vocab = c.vocab;
  a.n_embed = c.n_embed; a.eps = c.rms_eps; a.scale = 1.0f / sqrtf((float)c.head_dim);
  a.embed = (const bf16_t*)m->embed; a.final_norm = m->final_norm; a.head = m->head; a.rope = m->rope;
  a.layer0 = m->host_layers[0];
  a.layer_stride = m->layer_stride;
  a.kv = kv->v; a.rows = rows; a.pcap = pcap; a.n_seqs = B; a.tok_stride = tok_stride; a.with_head = with_head ? 1 : 0;
  a.tokens = dev_tokens;
  const size_t PR = kv->p_rows;
  a.h = kv->p_h; a.hg = kv->p_hg; a.sumsq = kv->p_sumsq; a.q = kv->p_q; a.attn = kv->p_attn; a.act = kv->p_act;
  a.part = kv->p_part; a.att_o = kv->p_att_o; a.att_ml = kv->p_att_ml; a.logits = kv->logits; a.NP = kv->NP;
  a.st_h = PR * c.d_model; a.st_hg = 2 * PR * c.d_model; a.st_sq = PR * (c.d_model / 32);
  a.st_q = 2 * PR * c.n_q_heads * c.head_dim; a.st_act = 2 * PR * c.d_ffn;
  a.st_part = (size_t)P_MAX_SPLITS * PR * c.d_model; a.part_stride = PR * c.d_model;
  a.st_att_o = PR * c.n_q_heads * kv->NP * 64; a.st_att_ml = PR * c.n_q_heads * kv->NP * 2;
  int max_len = 0;
  for (int s = rows.seq0; s < rows.seq0 + B; ++s) max_len = std::max(max_len, kv->len_ub[s]);
  a.n_parts = std::min(kv->NP, cdiv(max_len + rows.R, ATT_PART));
  a.tickets = kv->tickets; a.bar = kv->bar; a.epoch_base = kv->bar_epoch;
  a.trace = (kv->trace_on && 2 * (1 + 5 * c.n_layers) <= 512) ? kv->trace : nullptr;
  const int G = kv->persistent_wgs, NU = 2 * G, npairs = c.d_model / 32;
  auto splits = [&](int K) { return std::max(1, std::min(std::min(NU / npairs, (K / 32) / 4), P_MAX_SPLITS)); };
  a.gs_o = (c.n_q_heads * c.head_dim) / 32 <= 4 * PF_K ? 1 : splits(c.n_q_heads * c.head_dim);   // <= PF_K k-tiles per wave: all prefetched
  a.gs_d = splits(c.d_ffn);
  kv->bar_epoch += (with_head ? 1u : 0u) + 5u * (uint32_t)c.n_layers;  // barriers this launch executes
  ProfScope ps(PROF_PERSISTENT, st);
  hipLaunchKernelGGL(k_forward_persistent, dim3(G), dim3(PBLOCK), 0, st, a);
  LAUNCH_CHECK();
  return SSD_OK;
}

// The same forward without grid barriers between phases (see dataflow.h).  Returns -1 when the launch does not
// fit that kernel's limits, so that the caller takes the barrier kernel instead.
static int forward_dataflow(const ssd_model* m, ssd_kv* kv, Rows rows, int B, int pcap, const int32_t* dev_tokens,
                            int tok_stride, bool with_head, hipStream_t st) {
  const ssd_model_config& c = m->c;
  const int npairs = c.d_model / 32, M = rows.M;
  const int nqd = c.n_q_heads * c.head_dim, grp = c.n_q_heads / c.n_kv_heads;
  int max_len = 0;
  for (int s = rows.seq0; s < rows.seq0 + B; ++s) max_len = std::max(max_len, kv->len_ub[s]);
  const int n_parts = std::min(kv->NP, cdiv(max_len + rows.R, ATT_PART));
  // Workgroups [0, g_mlp) take the MLP items (two 16-column items each); the phases with few items (QKV, attention,
  // output projection) get workgroups of their own after them, as far as the device has compute units.
  const int g_mlp = std::min(kv->persistent_wgs, cdiv(c.d_ffn / 16, 2));
  // short prefixes: attention without parts (decided from the host's bound of the cached lengths alone, so that every
  // forward from one cache state takes the same path whatever its row count)
  const int att_tiles = B * c.n_kv_heads * cdiv(rows.R * grp, 16);
  const bool whole = kv->attn_whole && max_len + 16 <= DF_WHOLE_CHUNKS * 64 &&
                     g_mlp + (c.n_q_heads + 2 * c.n_kv_heads) * 2 + att_tiles + npairs <= kv->cus;
  const int n_att_items = whole ? att_tiles : att_tiles * n_parts;
  const int n_small = (c.n_q_heads + 2 * c.n_kv_heads) * 2 + n_att_items + npairs;
  // with compute units to spare every small-phase item gets a workgroup of its own (its waves then do not share their
  // SIMDs with a second item), else two items share one
  const int small_stride = g_mlp + n_small <= kv->cus ? 2 : 1;
  const int G = std::min(kv->cus, g_mlp + cdiv(small_stride * n_small, 2)), NU = 2 * G;
  // limits: one round of attention (its units wait for each other's parts), query rows of an item, LDS staging capacity
  const bool fits = M <= 16 && rows.R * grp <= DF_ATT_ROWS && small_stride * n_att_items <= NU &&
                    M * (c.d_model + 4) <= DF_AW && M * (nqd + 4) <= DF_AW && M * (c.d_model / 32) <= DF_SQ_WORDS &&
                    c.n_layers <= 128 && 2 + 10 * c.n_layers + 2 <= 512;
  if (!fits) return -1;
  DArgs a;
  memset(&a, 0, sizeof a);
  a.n_layers = c.n_layers; a.d = c.d_model; a.nq = c.n_q_heads; a.nkv = c.n_kv_heads; a.ffn = c.d_ffn; a.vocab = c.vocab;
  a.n_embed = c.n_embed; a.eps = c.rms_eps; a.scale = 1.0f / sqrtf((float)c.head_dim);
  a.embed = (const bf16_t*)m->embed; a.final_norm = m->final_norm; a.head = m->head; a.rope = m->rope;
  a.layer0 = m->host_layers[0];
  a.layer_stride = m->layer_stride;
  a.kv = kv->v; a.rows = rows; a.pcap = pcap; a.n_seqs = B; a.tok_stride = tok_stride; a.with_head = with_head ? 1 : 0;
  a.tokens = dev_tokens;
  const size_t PR = kv->p_rows;
  a.tw = kv->t_base; a.h = kv->t_h; a.hg = kv->t_hg; a.sq = kv->t_sq; a.q = kv->t_q; a.kvn = kv->t_kvn; a.attn = kv->t_attn;
  a.att_p = kv->t_att_p; a.logits = kv->logits;
  a.st_h = PR * c.d_model; a.st_sq = PR * (c.d_model / 32); a.st_q = PR * nqd; a.st_kvn = PR * 2 * c.n_kv_heads * 64;
  a.st_att_p = PR * c.n_q_heads * kv->NP * 96;
  a.rowblk = kv->t_rowblk;
  a.part2 = kv->t_part2; a.st_part2 = (size_t)(c.d_ffn / 32) * PR * c.d_model;
  a.NP = kv->NP; a.n_parts = n_parts; a.g_mlp = g_mlp; a.small_stride = small_stride;
  a.bar = kv->bar;
  a.trace = kv->trace_on ? kv->trace : nullptr;
  ProfScope ps(PROF_PERSISTENT, st);
  kv->last_whole = whole;
  // words of one operand staging: the rows' operand words and their sums of squares; one flight holds 512 x SB
  const int stage_words = M * (std::max(c.d_model, nqd) + c.d_model / 32);
  const int sb = kv->df_sb ? kv->df_sb : stage_words <= 2 * PBLOCK ? 2 : stage_words <= 4 * PBLOCK ? 4 : stage_words <= 10 * PBLOCK ? 10 : 12;
#define DF_LAUNCH(W, S) hipLaunchKernelGGL((k_forward_dataflow<W, S>), dim3(G), dim3(PBLOCK), 0, st, a)
  if (whole) { if (sb == 2) DF_LAUNCH(true, 2); else if (sb == 4) DF_LAUNCH(true, 4); else DF_LAUNCH(true, 12); }
  else { if (sb == 2) DF_LAUNCH(false, 2); else if (sb == 4) DF_LAUNCH(false, 4); else if (sb == 10) DF_LAUNCH(false, 10); else DF_LAUNCH(false, 12); }
#undef DF_LAUNCH
  LAUNCH_CHECK();
  return SSD_OK;
}

// One decoder forward for sequences [seq0, seq0+B), R rows each.  pcap = pending slots at the head of each
// sequence's rows (0: all rows take explicit tokens).  Leaves logits [B*R][vocab] in the workspace when
// with_head.  The caller has checked room.
template <typename DT>
static int forward(const ssd_model* m, ssd_kv* kv, int seq0, int B, int R, int pcap, const int32_t* dev_tokens,
                   int tok_stride, bool with_head, hipStream_t st) {
  const ssd_model_config& c = m->c;
  const int M = B * R, d = c.d_model, hd = c.head_dim, nq = c.n_q_heads, nkv = c.n_kv_heads;
  const int nqd = nq * hd, nqkv = m->n_qkv();
  Rows rows = kv->rows;
  rows.M = M; rows.R = R; rows.seq0 = seq0;
  {                                     // every forward is followed by a kernel that advances the cache's launch number
    const int rc = kv_launch_guard(kv, st, 1);
    if (rc) return rc;
    ++kv->launch_no;
  }
  if (kv->capturing && !(kv->persistent_wgs > 0 && M <= kv->p_rows && kv->dataflow))
    return fail(SSD_ENOSUP, "this launch does not fit the barrier-free forward kernel: it cannot be captured");
  if (kv->persistent_wgs > 0 && M <= kv->p_rows) {
    if (kv->dataflow) {
      const int rc = forward_dataflow(m, kv, rows, B, pcap, dev_tokens, tok_stride, with_head, st);
      if (rc >= 0) { kv->last_path = kv->last_whole ? 4 : 3; return rc; }
    }
    if (kv->capturing) return fail(SSD_ENOSUP, "this launch does not fit the barrier-free forward kernel: it cannot be captured");
    kv->last_path = 2;
    return forward_persistent(m, kv, rows, B, pcap, dev_tokens, tok_stride, with_head, st);
  }
  kv->last_path = 1;

  EmbedArgs e;
  e.kv = kv->v; e.rows = rows; e.pcap = pcap; e.n_seqs = B; e.tokens = dev_tokens; e.tok_stride = tok_stride;
  e.embed = m->embed; e.n_embed = c.n_embed; e.d = d; e.h = kv->h;
  hipLaunchKernelGGL((k_embed<DT>), dim3(M), dim3(BLOCK), 0, st, e);
  LAUNCH_CHECK();

  int max_len = 0;
  for (int s = seq0; s < seq0 + B; ++s) max_len = std::max(max_len, kv->len_ub[s]);
  const int nchunks = cdiv(max_len + R, ATT_CHUNK);

  GemmArgs g0;
  memset(&g0, 0, sizeof g0);
  g0.M = M; g0.kv = kv->v; g0.rows = rows; g0.nq = nq; g0.rope = m->rope;
  const size_t part_stride = (size_t)M * d;
  // k-splits fill the machine: about two workgroups per CU over (column pairs x row groups x splits), at least 8
  // k-tiles per workgroup
  const int row_groups = m->c.dtype == SSD_DTYPE_BF16 && M > 32 ? cdiv(cdiv(M, 16), 2) : 1;
  const int npairs_d = cdiv(cdiv(d, 16), 2);
  auto splits_for = [&](int Kd) {
    if (row_groups == 1) return pick_splits(Kd, npairs_d);
    const int want = std::max(1, 2 * kv->cus / (npairs_d * row_groups));
    return std::max(1, std::min(std::min(want, (Kd / 32) / 8), (int)MAX_SPLITS));
  };
  const int gs_o = splits_for(nqd);
  const bool wide = m->c.dtype == SSD_DTYPE_BF16 && M > 32 && kv->gemm_wide;
  // down projection: slices of the long k range per workgroup, if that still gives half the CUs a workgroup
  // (measured: 18.7 vs 44.6 us per launch on the 1.5B shape at 72 rows, 168 workgroups; 18.7 vs 17.5 us on the 0.5B
  // shape at 112 rows, where it has 80)
  const WidePlan down_plan = plan_wide(M, d, c.d_ffn, true, 0, MAX_SPLITS);
  const bool wide_down = wide &&
                         2 * down_plan.wa.n_colg * down_plan.wa.n_rowg * down_plan.wa.n_slices >= kv->cus;
  const int gs_d = wide_down ? down_plan.wa.n_slices : splits_for(c.d_ffn);
  // from 256 rows on (prefill chunks): the kernels whose waves each own row tiles x weight tiles (gemm_rows.h); every GEMM
  // operand (normalised rows, attention output, SwiGLU output) is then kept as split rows
  const bool rowsk = wide && M >= 256 && d <= 4096 && (hd == 64 || hd == 128);
  auto add_norm = [&](int n_part_, const float* gain) -> int {
    if (rowsk) hipLaunchKernelGGL(k_add_norm_split, dim3(M), dim3(BLOCK), 0, st, kv->h, kv->part, n_part_, part_stride, gain,
                                  c.rms_eps, (bf16_t*)kv->xn, d);
    else hipLaunchKernelGGL((k_add_norm<F32>), dim3(M), dim3(BLOCK), 0, st, kv->h, kv->part, n_part_, part_stride, gain,
                            c.rms_eps, kv->xn, d);
    LAUNCH_CHECK();
    return SSD_OK;
  };
  int n_part = 0;
  int rc;
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerW& L = m->layers[l];
    if ((rc = add_norm(n_part, L.ln1))) return rc;
    GemmArgs g = g0;                                       // QKV + bias + rotary + cache write
    g.A = kv->xn; g.lda = d; g.W0 = L.wqkv; g.W1 = L.wqkv; g.N = nqkv; g.K = d; g.gs = 1;
    g.bias = L.bqkv; g.q = kv->q; g.layer = l;
    {
      ProfScope ps(PROF_QKV, st);
      if (rowsk) rc = std::min(0, launch_rows<EPI_QKV>(g, kv->cus, hd, false, 1, st));
      else rc = launch_gemm<DT, EPI_QKV>(m, g, (nq + 2 * nkv) * (hd / 32), st);
    }
    if (rc) return rc;

    AttnArgs a;
    a.q = kv->q; a.kv = kv->v; a.rows = rows; a.layer = l; a.nq = nq; a.scale = 1.0f / sqrtf((float)hd);
    a.o_part = kv->o_part; a.ml_part = kv->ml_part; a.NC = kv->NC; a.out = kv->attn;
    a.split_kt = rowsk ? nqd / 32 : 0;
    {
      ProfScope ps(PROF_ATTN, st);
      if (hd == 32) rc = launch_attn<DT, 32>(a, nchunks, nkv, B, M, kv->attn_mfma, st);
      else if (hd == 64) rc = launch_attn<DT, 64>(a, nchunks, nkv, B, M, kv->attn_mfma, st);
      else rc = launch_attn<DT, 128>(a, nchunks, nkv, B, M, kv->attn_mfma, st);
    }
    if (rc) return rc;

    g = g0;                                                // output projection -> k-split partials
    g.A = kv->attn; g.lda = nqd; g.W0 = L.wo; g.W1 = L.wo; g.N = d; g.K = nqd; g.gs = gs_o;
    g.out = kv->part; g.out_split_stride = part_stride; g.ldo = d;
    int np_o = gs_o;
    {
      ProfScope ps(PROF_O, st);
      if (rowsk) { np_o = launch_rows<EPI_PARTIAL>(g, kv->cus, hd, true, MAX_SPLITS, st); rc = std::min(0, np_o); }
      else rc = launch_gemm<DT, EPI_PARTIAL>(m, g, cdiv(cdiv(d, 16), 2) * gs_o, st);
    }
    if (rc) return rc;

    if ((rc = add_norm(np_o, L.ln2))) return rc;

    g = g0;                                                // gate / up + SwiGLU
    g.A = kv->xn; g.lda = d; g.W0 = L.wgate; g.W1 = L.wup; g.N = c.d_ffn; g.K = d; g.gs = 1; g.act = kv->act;
    g.act_split_kt = rowsk ? c.d_ffn / 32 : 0;
    {
      ProfScope ps(PROF_GATEUP, st);
      if (rowsk) {
        rc = std::min(0, launch_rows<EPI_SWIGLU>(g, kv->cus, hd, false, 1, st));
      } else if (wide) {                                          // many rows: activations shared through LDS (see gemm.h)
        // two row tiles per workgroup: measured best on both shapes (more workgroups beat fewer weight re-reads)
        rc = launch_wide<EPI_SWIGLU>(g, plan_wide(M, c.d_ffn, d, false, 2, 1), st);
      } else {
        rc = launch_gemm<DT, EPI_SWIGLU>(m, g, cdiv(c.d_ffn, 16), st);
      }
    }
    if (rc) return rc;

    g = g0;                                                // down projection -> k-split partials
    g.A = kv->act; g.lda = c.d_ffn; g.W0 = L.wdown; g.W1 = L.wdown; g.N = d; g.K = c.d_ffn; g.gs = gs_d;
    g.out = kv->part; g.out_split_stride = part_stride; g.ldo = d;
    n_part = gs_d;
    {
      ProfScope ps(PROF_DOWN, st);
      if (rowsk) { n_part = launch_rows<EPI_PARTIAL>(g, kv->cus, hd, true, MAX_SPLITS, st); rc = std::min(0, n_part); }
      else if (wide_down) rc = launch_wide<EPI_PARTIAL>(g, down_plan, st);
      else rc = launch_gemm<DT, EPI_PARTIAL>(m, g, cdiv(cdiv(d, 16), 2) * gs_d, st);
    }
    if (rc) return rc;
  }
  if (!with_head) return SSD_OK;
  if ((rc = add_norm(n_part, m->final_norm))) return rc;
  GemmArgs g = g0;
  g.A = kv->xn; g.lda = d; g.W0 = m->head; g.W1 = m->head; g.N = c.vocab; g.K = d; g.gs = 1;
  g.out = kv->logits; g.out_split_stride = 0; g.ldo = c.vocab;
  ProfScope ps(PROF_HEAD, st);
  if (rowsk) return std::min(0, launch_rows<EPI_PARTIAL>(g, kv->cus, hd, false, 1, st));
  return launch_gemm<DT, EPI_PARTIAL>(m, g, cdiv(cdiv(c.vocab, 16), 2), st);
}

static int forward_any(const ssd_model* m, ssd_kv* kv, int seq0, int B, int R, int pcap, const int32_t* dev_tokens,
                       int tok_stride, bool with_head, hipStream_t st) {
  return m->c.dtype == SSD_DTYPE_BF16 ? forward<BF16>(m, kv, seq0, B, R, pcap, dev_tokens, tok_stride, with_head, st)
                                      : forward<F32>(m, kv, seq0, B, R, pcap, dev_tokens, tok_stride, with_head, st);
}

static int check_pair(const ssd_model* m, const ssd_kv* kv) {
  if (!m || !kv) return fail(SSD_EINVAL, "null handle");
  if (kv->m != m) return fail(SSD_EINVAL, "the cache was created for another model");
  return SSD_OK;
}

static int check_sample(const ssd_sample_config* s) {
  if (!s) return fail(SSD_EINVAL, "null sample config");
  if (!(s->beta >= 0.0f)) return fail(SSD_EINVAL, "beta must be >= 0");
  if (!s->greedy && !(s->temperature > 0.0f)) return fail(SSD_EINVAL, "temperature must be > 0");
  if (s->top_k < 0) return fail(SSD_EINVAL, "top_k must be >= 0");
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ prefill
extern "C" int ssd_prefill(ssd_model* m, ssd_kv* kv, int seq, const int32_t* dev_tokens, int n, void* stream) {
  int rc = check_pair(m, kv);
  if (rc) return rc;
  if (!dev_tokens || n < 1) return fail(SSD_EINVAL, "prefill needs at least one token");
  if (seq < 0 || seq >= kv->max_seqs) return fail(SSD_EINVAL, "sequence %d out of range", seq);
  if ((rc = kv_check_flags(kv))) return rc;
  hipStream_t st = (hipStream_t)stream;
  hipLaunchKernelGGL(k_kv_set, dim3(1), dim3(1), 0, st, kv->v, seq, 0, 0, 0, 0, (const int32_t*)nullptr, 0);
  LAUNCH_CHECK();
  kv->len_ub[seq] = 0;
  kv->npend_ub[seq] = 0;
  if ((rc = kv_check_room(kv, seq, 1, n - 1, st))) return rc;
  const int chunk = std::min(kv->max_rows, MAX_ROWS);
  for (int i = 0; i < n - 1; i += chunk) {
    const int R = std::min(chunk, n - 1 - i);
    if ((rc = forward_any(m, kv, seq, 1, R, 0, dev_tokens + i, 0, false, st))) return rc;
    hipLaunchKernelGGL(k_kv_set, dim3(1), dim3(1), 0, st, kv->v, seq, -1, R, 0, 0, (const int32_t*)nullptr, 1);
    LAUNCH_CHECK();
    kv->len_ub[seq] += R;
  }
  hipLaunchKernelGGL(k_kv_set, dim3(1), dim3(1), 0, st, kv->v, seq, -1, 0, 1, 0, dev_tokens + (n - 1), 0);
  LAUNCH_CHECK();
  kv->npend_ub[seq] = 1;
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ step
// Forward + warp + acceptance + commit for sequences 0..B-1.
// `step_dev`: when set, the cycle counter on the device is added to step_ctr (captured cycles); `bump_step`: this
// step's sampling kernel is the last of its cycle and advances that counter.
static int step(ssd_model* m, ssd_kv* kv, int B, int K, const int32_t* dev_x, const float* dev_pd,
                const ssd_sample_config* cfg, uint64_t step_ctr, int slot_base, int32_t* dev_n, int32_t* dev_next,
                int next_stride, float* probs_out, size_t probs_seq_stride, bool probs_last_row_only,
                float* logits_out, hipStream_t st, const int32_t* step_dev = nullptr, bool bump_step = false,
                bool full_pcap = false) {
  const ssd_model_config& c = m->c;
  // Rows per sequence that carry pending tokens: the cache's capacity, or less when the host knows that no sequence of
  // the launch holds that many (a draft cache owes two tokens only right after a fully accepted cycle; at 16 sequences
  // one row each instead of two keeps the draft steps on the persistent kernel).
  int pcap = 1;
  for (int s = 0; s < B; ++s) pcap = std::max(pcap, kv->npend_ub[s]);
  pcap = std::min(pcap, kv->v.pcap);
  if (full_pcap) pcap = kv->v.pcap;     // a captured step must hold whatever the sequences owe at any replay
  const int R = pcap + K, M = B * R, V = c.vocab;
  int rc;
  if (!kv->capturing && (rc = kv_check_room(kv, 0, B, R, st))) return rc;      // (a captured cycle checks before each replay)
  if ((rc = forward_any(m, kv, 0, B, R, pcap, dev_x, K, true, st))) return rc;
  if (logits_out) HIP_TRY(hipMemcpyAsync(logits_out, kv->logits, (size_t)M * V * 4, hipMemcpyDeviceToDevice, st));

  // rows that need a distribution: all K+1 of a verification, or the last row of a draft step
  WarpArgs w;
  w.ld = V; w.V = V; w.temperature = cfg->temperature; w.top_k = cfg->top_k; w.greedy = cfg->greedy;
  AcceptArgs a;
  memset(&a, 0, sizeof a);
  if (probs_last_row_only) {
    w.logits = kv->logits + (size_t)(R - 1) * V;
    w.ld = R * V;                       // one row per sequence
    w.probs = probs_out ? probs_out : kv->probs;
    w.probs_stride = probs_out ? probs_seq_stride : (size_t)V;
    a.pt = w.probs; a.pt_seq_stride = w.probs_stride;
  } else {
    w.logits = kv->logits + (size_t)(pcap - 1) * V;   // row of the last pending token, then the K drafts
    // rows pcap-1 .. R-1 of every sequence are consecutive only when pcap == 1 (a target cache)
    w.probs = probs_out ? probs_out : kv->probs;
    w.probs_stride = V;
    a.pt = w.probs; a.pt_seq_stride = (size_t)(K + 1) * V;
  }
  const bool one_row = probs_last_row_only || (K == 0 && pcap == 1);     // one row per sequence: fused with the sampling
  if (!one_row) {
    if (w.V <= 8 * SBLOCK) hipLaunchKernelGGL(k_warp_softmax<8>, dim3(M), dim3(SBLOCK), 0, st, w);
    else hipLaunchKernelGGL(k_warp_softmax<16>, dim3(M), dim3(SBLOCK), 0, st, w);
    LAUNCH_CHECK();
  }
  a.pd = dev_pd; a.x = dev_x; a.uniforms = nullptr; a.seed = cfg->seed; a.step = step_ctr;
  a.step_dev = step_dev; a.bump_step = bump_step ? 1 : 0; a.bump_launch = 1;
  a.B = B; a.K = K; a.V = V; a.beta = cfg->beta;
  a.n_acc = dev_n; a.next_tok = dev_next; a.tok_stride = next_stride; a.flags = nullptr;
  a.kv = kv->v; a.seq0 = 0;
  a.ticket = kv->ticket_alt ? kv->ticket_alt : kv->v.ctl + 2;
  a.slot_base = slot_base;
  const bool sp8 = a.V <= 8 * SBLOCK;
  if (one_row) {
    if (sp8) hipLaunchKernelGGL(k_warp_accept<8>, dim3(B), dim3(SBLOCK), 0, st, w, a);
    else hipLaunchKernelGGL(k_warp_accept<16>, dim3(B), dim3(SBLOCK), 0, st, w, a);
  } else {
    if (sp8) hipLaunchKernelGGL(k_accept<8>, dim3(B), dim3(SBLOCK), 0, st, a);
    else hipLaunchKernelGGL(k_accept<16>, dim3(B), dim3(SBLOCK), 0, st, a);
  }
  LAUNCH_CHECK();
  return SSD_OK;
}

extern "C" int ssd_verify(ssd_model* target, ssd_kv* kv, int n_seqs, const int32_t* prefix_len,
                          const int32_t* dev_draft_tokens, const float* dev_draft_probs, int K,
                          const ssd_sample_config* cfg, uint64_t step_ctr, int32_t* dev_n_accepted,
                          int32_t* dev_next_token, float* dev_target_probs_opt, float* dev_logits_opt, void* stream) {
  int rc = check_pair(target, kv);
  if (rc) return rc;
  if ((rc = check_sample(cfg))) return rc;
  if (kv->v.pcap != 1) return fail(SSD_EINVAL, "ssd_verify needs a target cache (pending_cap 1)");
  if (n_seqs < 1 || n_seqs > kv->max_seqs) return fail(SSD_EINVAL, "n_seqs %d out of range", n_seqs);
  if (K < 0 || K > SSD_MAX_K || K + 1 > kv->max_rows) return fail(SSD_EINVAL, "K = %d out of range (max_rows %d)", K, kv->max_rows);
  if (K > 0 && (!dev_draft_tokens || !dev_draft_probs)) return fail(SSD_EINVAL, "draft tokens / probabilities are null");
  if (!dev_n_accepted || !dev_next_token) return fail(SSD_EINVAL, "output pointers are null");
  if ((rc = kv_check_flags(kv))) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (prefix_len) {
    if ((rc = kv_refresh(kv, st))) return rc;
    for (int s = 0; s < n_seqs; ++s)
      if (prefix_len[s] != kv->len_ub[s] || kv->npend_ub[s] != 1)
        return fail(SSD_EINVAL, "sequence %d: prefix_len %d but the cache holds %d positions (%d pending)", s,
                    prefix_len[s], kv->len_ub[s], kv->npend_ub[s]);
  }
  rc = step(target, kv, n_seqs, K, dev_draft_tokens, dev_draft_probs, cfg, step_ctr, 0, dev_n_accepted, dev_next_token,
            1, dev_target_probs_opt, 0, false, dev_logits_opt, st);
  if (rc) return rc;
  for (int s = 0; s < n_seqs; ++s) { kv->len_ub[s] += K + 1; kv->npend_ub[s] = 1; }
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ no-allocation variant
// Staging of ssd_verify_noalloc: [0, 256) the commit's arrival counter, then the logits rows, then the probability rows.
// One copy per GPU for the life of the process; every call on a GPU uses that GPU's copy.
constexpr size_t NOALLOC_MAX_ELEMS = SSD_NOALLOC_MAX_ELEMS;
static __device__ __align__(256) unsigned char scratch[256 + 2 * NOALLOC_MAX_ELEMS * sizeof(float)];
constexpr int NOALLOC_MAX_DEVICES = 64;
static unsigned char* g_scratch_dev[NOALLOC_MAX_DEVICES];      // device address of `scratch` on each GPU (0: not asked yet)

// The device address of this GPU's copy of `scratch` (the array's name is only a host-side handle of the symbol).
static int noalloc_scratch(unsigned char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return fail(SSD_ENOSUP, "device ordinal %d not supported", dev);
  if (!g_scratch_dev[dev]) {
    unsigned char* p = nullptr;
    HIP_TRY(hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(SSD_EHIP, "hipGetSymbolAddress returned a null address");
    g_scratch_dev[dev] = p;
  }
  *out = g_scratch_dev[dev];
  return SSD_OK;
}

extern "C" int ssd_verify_noalloc(ssd_model* target, ssd_kv* kv, int n_seqs, const int32_t* dev_draft_tokens,
                                  const float* dev_draft_probs, int K, const ssd_sample_config* cfg, uint64_t step_ctr,
                                  int32_t* dev_n_accepted, int32_t* dev_next_token, void* stream) {
  int rc = check_pair(target, kv);
  if (rc) return rc;
  if ((rc = check_sample(cfg))) return rc;
  if (kv->v.pcap != 1) return fail(SSD_EINVAL, "ssd_verify_noalloc needs a target cache (pending_cap 1)");
  if (n_seqs < 1 || n_seqs > kv->max_seqs) return fail(SSD_EINVAL, "n_seqs %d out of range", n_seqs);
  if (K < 0 || K > SSD_MAX_K || K + 1 > kv->max_rows) return fail(SSD_EINVAL, "K = %d out of range (max_rows %d)", K, kv->max_rows);
  if (K > 0 && (!dev_draft_tokens || !dev_draft_probs)) return fail(SSD_EINVAL, "draft tokens / probabilities are null");
  if (!dev_n_accepted || !dev_next_token) return fail(SSD_EINVAL, "output pointers are null");
  const size_t elems = (size_t)n_seqs * (K + 1) * target->c.vocab;
  if (elems > NOALLOC_MAX_ELEMS)
    return fail(SSD_ENOMEM, "ssd_verify_noalloc: n_seqs * (K+1) * vocab = %zu exceeds the static staging of %zu elements", elems,
                (size_t)NOALLOC_MAX_ELEMS);
  if ((rc = kv_check_flags(kv))) return rc;
  unsigned char* sp = nullptr;
  if ((rc = noalloc_scratch(&sp))) return rc;
  hipStream_t st = (hipStream_t)stream;
  // the arrival counter must start at zero whatever an earlier (possibly failed) call on this GPU left; the logits and
  // probability rows are written in full before they are read
  hipLaunchKernelGGL(k_zero_words, dim3(1), dim3(64), 0, st, (int32_t*)sp, 64);
  LAUNCH_CHECK();
  float* const ws_logits = kv->logits;
  float* const ws_probs = kv->probs;
  kv->logits = (float*)(sp + 256);
  kv->probs = (float*)(sp + 256) + NOALLOC_MAX_ELEMS;
  kv->ticket_alt = (int32_t*)sp;
  rc = step(target, kv, n_seqs, K, dev_draft_tokens, dev_draft_probs, cfg, step_ctr, 0, dev_n_accepted, dev_next_token, 1,
            nullptr, 0, false, nullptr, st);
  kv->logits = ws_logits;
  kv->probs = ws_probs;
  kv->ticket_alt = nullptr;
  if (rc) return rc;
  for (int s = 0; s < n_seqs; ++s) { kv->len_ub[s] += K + 1; kv->npend_ub[s] = 1; }
  return SSD_OK;
}

extern "C" int ssd_draft_step(ssd_model* draft, ssd_kv* kv_d, int n_seqs, const ssd_sample_config* cfg,
                              uint64_t step_ctr, int draft_idx, int32_t* dev_token_out, int token_stride,
                              float* dev_probs_out, size_t probs_stride, void* stream) {
  int rc = check_pair(draft, kv_d);
  if (rc) return rc;
  if ((rc = check_sample(cfg))) return rc;
  if (n_seqs < 1 || n_seqs > kv_d->max_seqs) return fail(SSD_EINVAL, "n_seqs %d out of range", n_seqs);
  if (draft_idx < 0 || draft_idx > SSD_MAX_K) return fail(SSD_EINVAL, "draft_idx out of range");
  if (!dev_token_out || token_stride < 1) return fail(SSD_EINVAL, "token output is null");
  if (dev_probs_out && probs_stride < (size_t)draft->c.vocab) return fail(SSD_EINVAL, "probs_stride < vocab");
  if (kv_d->max_rows < kv_d->v.pcap) return fail(SSD_EINVAL, "cache rows too small");
  if ((rc = kv_check_flags(kv_d))) return rc;
  hipStream_t st = (hipStream_t)stream;
  // the token is drawn with the uniform of slot SSD_DRAFT_SLOT0 + draft_idx of this cycle: the step's only slot
  ssd_sample_config c2 = *cfg;
  c2.beta = 0.0f;
  rc = step(draft, kv_d, n_seqs, 0, nullptr, nullptr, &c2, step_ctr, SSD_DRAFT_SLOT0 + draft_idx, nullptr, dev_token_out, token_stride,
            dev_probs_out, probs_stride, true, nullptr, st);
  if (rc) return rc;
  for (int s = 0; s < n_seqs; ++s) { kv_d->len_ub[s] += kv_d->npend_ub[s]; kv_d->npend_ub[s] = 1; }
  return SSD_OK;
}

extern "C" int ssd_kv_rollback(ssd_kv* kv, int seq, int new_len, int pending_token, void* stream) {
  if (!kv) return fail(SSD_EINVAL, "null handle");
  if (seq < 0 || seq >= kv->max_seqs) return fail(SSD_EINVAL, "sequence %d out of range", seq);
  hipStream_t st = (hipStream_t)stream;
  int rc = kv_check_flags(kv);
  if (rc) return rc;
  // The host knows an upper bound of the length only; beyond it the request is refused here.  Between the device's length
  // and that bound the kernel refuses it: the state stays as it is and the next call on this cache reports the error.
  if (new_len < 0 || new_len > kv->len_ub[seq]) {
    if ((rc = kv_refresh(kv, st))) return rc;
    if (new_len < 0 || new_len > kv->len_ub[seq])
      return fail(SSD_EINVAL, "rollback to %d but sequence %d holds %d positions", new_len, seq, kv->len_ub[seq]);
  }
  hipLaunchKernelGGL(k_kv_set, dim3(1), dim3(1), 0, st, kv->v, seq, new_len, 0, 1, pending_token, (const int32_t*)nullptr, 0);
  LAUNCH_CHECK();
  kv->len_ub[seq] = new_len;
  kv->npend_ub[seq] = 1;
  return SSD_OK;
}

extern "C" int ssd_kv_follow(ssd_kv* kv_d, int n_seqs, int K, const int32_t* dev_n_accepted,
                             const int32_t* dev_next_token, const int32_t* dev_draft_tokens, void* stream) {
  if (!kv_d || !dev_n_accepted || !dev_next_token || !dev_draft_tokens) return fail(SSD_EINVAL, "null argument");
  if (kv_d->v.pcap != 2) return fail(SSD_EINVAL, "ssd_kv_follow needs a draft cache (pending_cap 2)");
  if (n_seqs < 1 || n_seqs > kv_d->max_seqs || K < 1 || K > SSD_MAX_K) return fail(SSD_EINVAL, "bad n_seqs / K");
  {
    const int rc = kv_check_flags(kv_d);
    if (rc) return rc;
  }
  hipLaunchKernelGGL(k_kv_follow, dim3(1), dim3(1), 0, (hipStream_t)stream, kv_d->v, n_seqs, K, dev_n_accepted,
                     dev_next_token, dev_draft_tokens, (int32_t*)nullptr);
  LAUNCH_CHECK();
  for (int s = 0; s < n_seqs; ++s) kv_d->npend_ub[s] = 2;       // the length can only have shrunk
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ pieces
extern "C" int ssd_verify_from_probs(const float* dev_pt, const float* dev_pd, const int32_t* dev_tokens,
                                     const float* dev_uniforms, int B, int K, int V, float beta,
                                     int32_t* dev_n_accepted, int32_t* dev_next_token, int32_t* dev_flags, void* stream) {
  if (!dev_pt || !dev_uniforms || !dev_n_accepted || !dev_next_token) return fail(SSD_EINVAL, "null argument");
  if (B < 1 || K < 0 || K > SSD_MAX_K || V < 1 || V > 16384) return fail(SSD_EINVAL, "bad B / K / V");
  if (K > 0 && (!dev_pd || !dev_tokens)) return fail(SSD_EINVAL, "draft tokens / probabilities are null");
  if (!(beta >= 0.0f)) return fail(SSD_EINVAL, "beta must be >= 0");
  AcceptArgs a;
  memset(&a, 0, sizeof a);
  a.pt = dev_pt; a.pt_seq_stride = (size_t)(K + 1) * V; a.pd = dev_pd; a.x = dev_tokens; a.uniforms = dev_uniforms;
  a.B = B; a.K = K; a.V = V; a.beta = beta; a.n_acc = dev_n_accepted; a.next_tok = dev_next_token; a.tok_stride = 1;
  a.flags = dev_flags;
  if (a.V <= 8 * SBLOCK) hipLaunchKernelGGL(k_accept<8>, dim3(B), dim3(SBLOCK), 0, (hipStream_t)stream, a);
  else hipLaunchKernelGGL(k_accept<16>, dim3(B), dim3(SBLOCK), 0, (hipStream_t)stream, a);
  LAUNCH_CHECK();
  return SSD_OK;
}

extern "C" int ssd_warp_probs(const float* dev_logits, int rows, int V, const ssd_sample_config* cfg, float* dev_probs,
                              void* stream) {
  int rc = check_sample(cfg);
  if (rc) return rc;
  if (!dev_logits || !dev_probs || rows < 1 || V < 1 || V > 16384) return fail(SSD_EINVAL, "bad argument");
  WarpArgs w;
  w.logits = dev_logits; w.ld = V; w.V = V; w.temperature = cfg->temperature; w.top_k = cfg->top_k; w.greedy = cfg->greedy;
  w.probs = dev_probs; w.probs_stride = V;
  if (w.V <= 8 * SBLOCK) hipLaunchKernelGGL(k_warp_softmax<8>, dim3(rows), dim3(SBLOCK), 0, (hipStream_t)stream, w);
  else hipLaunchKernelGGL(k_warp_softmax<16>, dim3(rows), dim3(SBLOCK), 0, (hipStream_t)stream, w);
  LAUNCH_CHECK();
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ state
extern "C" int ssd_kv_state(ssd_kv* kv, int seq, void* stream, int32_t* len, int32_t* n_pending, int32_t pending[2],
                            int32_t* n_owned, int32_t* block_table, int block_table_cap) {
  if (!kv) return fail(SSD_EINVAL, "null handle");
  if (seq < 0 || seq >= kv->max_seqs) return fail(SSD_EINVAL, "sequence %d out of range", seq);
  hipStream_t st = (hipStream_t)stream;
  int rc = kv_refresh(kv, st);
  if (rc && rc != SSD_ENOMEM) return rc;
  int32_t own = 0;
  HIP_TRY(hipMemcpy(&own, kv->v.owned + seq, 4, hipMemcpyDeviceToHost));
  if (len) *len = kv->len_ub[seq];
  if (n_pending) *n_pending = kv->npend_ub[seq];
  if (pending) HIP_TRY(hipMemcpy(pending, kv->v.pend + 2 * seq, 8, hipMemcpyDeviceToHost));
  if (n_owned) *n_owned = own;
  if (block_table) {
    if (block_table_cap < own) return fail(SSD_ENOMEM, "block_table_cap %d < %d owned blocks", block_table_cap, own);
    if (own) HIP_TRY(hipMemcpy(block_table, kv->v.table + (size_t)seq * kv->v.mbps, (size_t)own * 4, hipMemcpyDeviceToHost));
  }
  return SSD_OK;
}

extern "C" int ssd_kv_free_stack(ssd_kv* kv, void* stream, int32_t* free_stack, int cap, int32_t* n_free,
                                 int32_t* dev_error_flag) {
  if (!kv) return fail(SSD_EINVAL, "null handle");
  HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
  int32_t ctl[4];
  HIP_TRY(hipMemcpy(ctl, kv->v.ctl, sizeof ctl, hipMemcpyDeviceToHost));
  if (n_free) *n_free = ctl[0];
  uint32_t bar_err = 0;
  HIP_TRY(hipMemcpy(&bar_err, kv->bar + 64, 4, hipMemcpyDeviceToHost));
  if (dev_error_flag) *dev_error_flag = (ctl[1] & KV_ERR_POOL) | (bar_err ? 2 : 0) | (ctl[1] & KV_ERR_ROLLBACK);
  if (free_stack) {
    if (cap < ctl[0]) return fail(SSD_ENOMEM, "cap %d < %d free blocks", cap, ctl[0]);
    if (ctl[0]) HIP_TRY(hipMemcpy(free_stack, kv->v.free_stack, (size_t)ctl[0] * 4, hipMemcpyDeviceToHost));
  }
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ errors on the device
extern "C" int ssd_kv_clear_error(ssd_kv* kv, void* stream) {
  if (!kv) return fail(SSD_EINVAL, "null handle");
  return kv_clear_sync_state(kv, (hipStream_t)stream);
}

extern "C" int ssd_kv_test_hook(ssd_kv* kv, int what, long long value, void* stream) {
  if (!kv) return fail(SSD_EINVAL, "null handle");
  hipStream_t st = (hipStream_t)stream;
  if (what == SSD_HOOK_TIMEOUT) {
    hipLaunchKernelGGL(k_kv_poke, dim3(1), dim3(1), 0, st, kv->v, DEV_ERR_TIMEOUT, 0);
  } else if (what == SSD_HOOK_LAUNCH_NUMBER) {
    if (value < 1 || value >= (long long)TAG_LIMIT) return fail(SSD_EINVAL, "launch number out of range");
    hipLaunchKernelGGL(k_kv_poke, dim3(1), dim3(1), 0, st, kv->v, 0u, (int)value);
    kv->launch_no = (uint32_t)value;
  } else if (what == SSD_HOOK_LAUNCH_NUMBER_DEVICE_ONLY) {
    if (value < 1 || value > (long long)TAG_LIMIT) return fail(SSD_EINVAL, "launch number out of range");
    hipLaunchKernelGGL(k_kv_poke, dim3(1), dim3(1), 0, st, kv->v, 0u, (int)value);
  } else {
    return fail(SSD_EINVAL, "unknown hook %d", what);
  }
  LAUNCH_CHECK();
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ captured cycle
struct ssd_cycle {
  ssd_model *target, *draft;
  ssd_kv *kv, *kv_d;
  int n_seqs, K;
  ssd_sample_config cfg, dcfg;
  int32_t* x;
  float* pd;
  int32_t *n_acc, *next;
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
  int cap_len_t = -1, cap_len_d = -1;     // the captured launch shapes hold while every length bound stays at or below these
  int captures = 0;
};

static void cycle_drop(ssd_cycle* c) {
  if (c->exec) (void)hipGraphExecDestroy(c->exec);
  if (c->graph) (void)hipGraphDestroy(c->graph);
  c->exec = nullptr; c->graph = nullptr;
}

// Host bookkeeping of one cycle's calls (the bounds the eager calls would have left).
static void cycle_advance_bounds(ssd_cycle* c) {
  for (int s = 0; s < c->n_seqs; ++s) {
    c->kv_d->len_ub[s] += c->kv_d->npend_ub[s] + (c->K - 1);
    c->kv_d->npend_ub[s] = 2;
    c->kv->len_ub[s] += c->K + 1;
    c->kv->npend_ub[s] = 1;
  }
}

static int cycle_capture(ssd_cycle* c, hipStream_t st) {
  cycle_drop(c);
  int rc;
  // exact lengths, room for the replays this capture will serve, numbering that cannot run out inside them
  if ((rc = kv_refresh(c->kv, st)) || (rc = kv_refresh(c->kv_d, st))) return rc;
  const int K = c->K, V = c->target->c.vocab;
  int max_t = 0, max_d = 0;
  for (int s = 0; s < c->n_seqs; ++s) { max_t = std::max(max_t, c->kv->len_ub[s]); max_d = std::max(max_d, c->kv_d->len_ub[s]); }
  // launch shapes (attention parts, workgroups) are those of a prefix up to 256 positions longer than today's
  const int ahead = 256;
  const int lim_t = std::min(c->target->max_positions, c->kv->v.mbps * c->kv->v.bt) - (K + 1);
  const int lim_d = std::min(c->draft->max_positions, c->kv_d->v.mbps * c->kv_d->v.bt) - (K + 2);
  c->cap_len_t = std::min(max_t + ahead, lim_t);
  c->cap_len_d = std::min(max_d + ahead, lim_d);
  if (c->cap_len_t < max_t || c->cap_len_d < max_d + K + 1) return fail(SSD_ENOMEM, "no room for another cycle");
  if ((rc = kv_check_room(c->kv, 0, c->n_seqs, K + 1, st)) || (rc = kv_check_room(c->kv_d, 0, c->n_seqs, K + 1, st))) return rc;
  std::vector<int> lt = c->kv->len_ub, ld = c->kv_d->len_ub, nt = c->kv->npend_ub, nd = c->kv_d->npend_ub;
  const uint32_t ln_t = c->kv->launch_no, ln_d = c->kv_d->launch_no;
  for (int s = 0; s < c->n_seqs; ++s) {
    c->kv->len_ub[s] = c->cap_len_t; c->kv_d->len_ub[s] = c->cap_len_d;
    c->kv->npend_ub[s] = 1; c->kv_d->npend_ub[s] = 2;      // the first draft step of a cycle may owe two tokens
  }
  c->kv->capturing = c->kv_d->capturing = true;
  auto restore = [&]() { c->kv->len_ub = lt; c->kv_d->len_ub = ld; c->kv->npend_ub = nt; c->kv_d->npend_ub = nd;
                         c->kv->launch_no = ln_t; c->kv_d->launch_no = ln_d; c->kv->capturing = c->kv_d->capturing = false; };
  hipError_t e = hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal);
  if (e != hipSuccess) { restore(); return fail(SSD_EHIP, "hipStreamBeginCapture: %s", hipGetErrorString(e)); }
  const int32_t* step_dev = c->kv->v.ctl + 4;
  ssd_sample_config dc = c->dcfg;
  dc.beta = 0.0f;
  rc = SSD_OK;
  for (int i = 0; i < K && !rc; ++i) {
    rc = step(c->draft, c->kv_d, c->n_seqs, 0, nullptr, nullptr, &dc, 0, SSD_DRAFT_SLOT0 + i, nullptr, c->x + i, K,
              c->pd + (size_t)i * V, (size_t)K * V, true, nullptr, st, step_dev, false, i == 0);
    for (int s = 0; s < c->n_seqs; ++s) c->kv_d->npend_ub[s] = 1;        // after a draft step exactly one token is pending
  }
  if (!rc) rc = step(c->target, c->kv, c->n_seqs, K, c->x, c->pd, &c->cfg, 0, 0, c->n_acc, c->next, 1, nullptr, 0, false,
                     nullptr, st, step_dev, false, true);
  if (!rc) {
    hipLaunchKernelGGL(k_kv_follow, dim3(1), dim3(1), 0, st, c->kv_d->v, c->n_seqs, K, c->n_acc, c->next, c->x,
                       c->kv->v.ctl + 4);
    if (hipGetLastError() != hipSuccess) rc = fail(SSD_EHIP, "k_kv_follow launch failed");
  }
  hipGraph_t g = nullptr;
  e = hipStreamEndCapture(st, &g);
  restore();
  if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
  if (e != hipSuccess) return fail(SSD_EHIP, "hipStreamEndCapture: %s", hipGetErrorString(e));
  c->graph = g;
  e = hipGraphInstantiate(&c->exec, g, nullptr, nullptr, 0);
  if (e != hipSuccess) { cycle_drop(c); return fail(SSD_EHIP, "hipGraphInstantiate: %s", hipGetErrorString(e)); }
  ++c->captures;
  return SSD_OK;
}

extern "C" int ssd_cycle_create(ssd_model* target, ssd_kv* kv, ssd_model* draft, ssd_kv* kv_d, int n_seqs, int K,
                                const ssd_sample_config* cfg, const ssd_sample_config* dcfg, int32_t* dev_draft_tokens,
                                float* dev_draft_probs, int32_t* dev_n_accepted, int32_t* dev_next_token,
                                uint64_t first_step, void* stream, ssd_cycle** out) {
  int rc = check_pair(target, kv);
  if (rc || (rc = check_pair(draft, kv_d)) || (rc = check_sample(cfg)) || (rc = check_sample(dcfg))) return rc;
  if (!out || !dev_draft_tokens || !dev_draft_probs || !dev_n_accepted || !dev_next_token) return fail(SSD_EINVAL, "null argument");
  if (kv->v.pcap != 1 || kv_d->v.pcap != 2) return fail(SSD_EINVAL, "needs a target cache (pending_cap 1) and a draft cache (pending_cap 2)");
  if (n_seqs < 1 || n_seqs > kv->max_seqs || n_seqs > kv_d->max_seqs) return fail(SSD_EINVAL, "n_seqs %d out of range", n_seqs);
  if (K < 1 || K > SSD_MAX_K || K + 1 > kv->max_rows || kv_d->max_rows < 2) return fail(SSD_EINVAL, "K = %d out of range", K);
  if (target->c.vocab != draft->c.vocab) return fail(SSD_EINVAL, "target and draft vocabularies differ");
  if (!kv->dataflow || !kv_d->dataflow) return fail(SSD_ENOSUP, "a cycle can be captured only on the barrier-free forward kernel");
  ssd_cycle* c = new (std::nothrow) ssd_cycle();
  if (!c) return fail(SSD_ENOMEM, "host allocation failed");
  c->target = target; c->draft = draft; c->kv = kv; c->kv_d = kv_d; c->n_seqs = n_seqs; c->K = K;
  c->cfg = *cfg; c->dcfg = *dcfg; c->x = dev_draft_tokens; c->pd = dev_draft_probs; c->n_acc = dev_n_accepted;
  c->next = dev_next_token;
  const int32_t words[2] = {(int32_t)(uint32_t)first_step, (int32_t)(uint32_t)(first_step >> 32)};
  hipError_t e = hipMemcpyAsync(kv->v.ctl + 4, words, sizeof words, hipMemcpyHostToDevice, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);       // `words` is on this stack frame
  if (e != hipSuccess) { delete c; return fail(SSD_EHIP, "cycle counter: %s", hipGetErrorString(e)); }
  *out = c;
  return SSD_OK;
}

extern "C" int ssd_cycle_launch(ssd_cycle* c, void* stream) {
  if (!c) return fail(SSD_EINVAL, "null handle");
  if (!stream) return fail(SSD_EINVAL, "a cycle cannot be captured on the default (NULL) stream: pass a stream of its own");
  hipStream_t st = (hipStream_t)stream;
  int rc;
  if ((rc = kv_check_flags(c->kv)) || (rc = kv_check_flags(c->kv_d))) return rc;
  const int K = c->K;
  if ((rc = kv_launch_guard(c->kv, st, 1)) || (rc = kv_launch_guard(c->kv_d, st, (uint32_t)K))) return rc;
  bool fits = c->exec != nullptr;
  for (int s = 0; s < c->n_seqs && fits; ++s)
    fits = c->kv->len_ub[s] <= c->cap_len_t && c->kv_d->len_ub[s] + K + 1 <= c->cap_len_d;
  if (fits) {                                              // pool room for this cycle, from the bounds alone
    long bt = 0, bd = 0;
    for (int s = 0; s < c->kv->max_seqs; ++s) bt += cdiv(c->kv->len_ub[s] + (s < c->n_seqs ? K + 1 : 0), c->kv->v.bt);
    for (int s = 0; s < c->kv_d->max_seqs; ++s) bd += cdiv(c->kv_d->len_ub[s] + (s < c->n_seqs ? K + 1 : 0), c->kv_d->v.bt);
    fits = bt <= c->kv->v.n_blocks && bd <= c->kv_d->v.n_blocks;
  }
  if (!fits && (rc = cycle_capture(c, st))) return rc;
  HIP_TRY(hipGraphLaunch(c->exec, st));
  c->kv->launch_no += 1;
  c->kv_d->launch_no += (uint32_t)K;
  c->kv->last_path = 3;
  cycle_advance_bounds(c);
  return SSD_OK;
}

extern "C" int ssd_cycle_captures(const ssd_cycle* c) { return c ? c->captures : 0; }

extern "C" int ssd_cycle_destroy(ssd_cycle* c) {
  if (!c) return SSD_OK;
  cycle_drop(c);
  delete c;
  return SSD_OK;
}

// ------------------------------------------------------------------------------------------------ barrier trace
extern "C" int ssd_kv_last_forward_path(const ssd_kv* kv) { return kv ? kv->last_path : 0; }

extern "C" int ssd_trace_barriers(ssd_kv* kv, int enable, void* stream, unsigned long long* out, int cap, int* n_wgs,
                                  int* n_samples) {
  if (!kv) return fail(SSD_EINVAL, "null handle");
#ifndef SSD_TRACE
  (void)enable; (void)stream; (void)out; (void)cap; (void)n_wgs; (void)n_samples;
  return fail(SSD_ENOSUP, "this build records no phase trace (build with -DSSD_TRACE)");
#else
  if (out) {
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    const int G = kv->persistent_wgs > 0 ? (kv->dataflow ? std::min(kv->cus, 256) : kv->persistent_wgs) : 0, S = 2 * (1 + 5 * kv->m->c.n_layers);
    if (G <= 0 || S > 512) return fail(SSD_ENOSUP, "no persistent kernel trace for this cache");
    if (cap < G * 512) return fail(SSD_ENOMEM, "cap %d < %d samples", cap, G * 512);
    HIP_TRY(hipMemcpy(out, kv->trace, sizeof(unsigned long long) * 512 * G, hipMemcpyDeviceToHost));
    if (n_wgs) *n_wgs = G;
    if (n_samples) *n_samples = S;
  }
  kv->trace_on = enable != 0;
  return SSD_OK;
#endif
}
