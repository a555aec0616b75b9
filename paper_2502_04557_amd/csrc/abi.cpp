// C-ABI layer of the SPRINTER decode library: validation, workspace carving,
// weight intake and the launch sequence of prefill / step / generate.
// All device work is issued through the launchers in the k_*.hip files.
#include "../../include/sprinter.h"
#include "internal.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <unordered_map>
#include <algorithm>
#include <chrono>
#include <mutex>
#include <vector>

using namespace sprinter;

namespace {

thread_local char g_err[512] = "";

// The workspace of contexts made by sprinter_create_static: callers that must not allocate device memory get it from
// here.  In host code the array's name is only a stand-in; its device address comes from hipGetSymbolAddress (per
// device, see sprinter_create_static) and only that address is ever handed to kernels.
constexpr size_t STATIC_WORKSPACE_BYTES = SPRINTER_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[STATIC_WORKSPACE_BYTES];
constexpr int MAX_STATIC_DEVICES = 64;
struct StaticSlot { void* base = nullptr; bool in_use = false; };
StaticSlot g_static[MAX_STATIC_DEVICES];
std::mutex g_static_mu;

struct Bump {   // 256-byte aligned bump allocator; base == nullptr only measures
  char* base; size_t off;
  explicit Bump(void* b) : base((char*)b), off(0) {}
  void* take(size_t bytes) {
    off = (off + 255) & ~(size_t)255;
    void* p = base ? base + off : nullptr;
    off += bytes;
    return p;
  }
};

struct Expected {      // one tensor the model needs
  std::string name;
  int64_t rows, cols;  // cols == 0: 1-D
  bool pack;           // bf16 matrix that is repacked into operand tiles
  const void** slot;   // where the usable device pointer is stored
  void* packed;        // destination of the packed copy
  const void** slot2;  // second consumer (tied LM head)
  void* packed2;
  bool seen;
};

struct Model {
  sprinter_model_cfg cfg;
  ModelDims md;
  const void *tok_emb = nullptr, *pos_emb = nullptr, *lm_head = nullptr;
  const void *normf_g = nullptr, *normf_b = nullptr;
  std::vector<LayerW> layers;
  std::vector<Expected> expected;
  std::unordered_map<std::string, int> index;
  void *kcache = nullptr, *vcache = nullptr;
  size_t layer_stride = 0;   // elements per layer in a cache
  ModelScratch sc;
  int *rd_n = nullptr, *rd_b = nullptr, *rd_tok = nullptr, *rd_pos = nullptr, *rd_slot = nullptr;
  bool loaded = false;
  RowDesc rd() const { return RowDesc{rd_n, rd_b, rd_tok, rd_pos, rd_slot}; }
};

}  // namespace

struct sprinter_ctx {
  sprinter_cfg cfg;
  hipStream_t stream;
  Model draft, target;
  // verifier
  const void *v_w1 = nullptr, *v_b1 = nullptr, *v_w2 = nullptr, *v_b2 = nullptr;
  std::vector<Expected> v_expected;
  std::unordered_map<std::string, int> v_index;
  bool v_loaded = false;
  float* ver_part = nullptr;
  int ver_chunks = 1;
  // state
  State st;
  float* tau_dev = nullptr;
  int *draft_tok = nullptr, *rej_idx = nullptr, *n_rej = nullptr, *committed = nullptr;
  float* score = nullptr;
  unsigned char* accept = nullptr;
  int rows_alloc = 0;
  unsigned long long* host_counts = nullptr;   // what the host reads: [0] (ticket << 32) | rejected rows, [1] work-list entries, [2] draft entries
  unsigned long long* kernel_word = nullptr;   // where the kernels store those words: host_counts itself (pinned memory), or, for a
                                               // context of sprinter_create_static, four words of the workspace that wait_ticket copies
  unsigned long long* dev_counts = nullptr;    // those four words of the workspace
  unsigned long long static_words[4] = {0, 0, 0, 0};
  int static_dev = -1;                         // >= 0: the workspace is the library's static array on that device
  unsigned ticket = 0;
  int *ent_off = nullptr, *t_last = nullptr;   // full-prefix mode: work-list prefix sums, last-entry flags of a chunk
  int* coin_kept = nullptr;                    // reject_mode 1: counter, and the step's logits of both models
  float *dl = nullptr, *tl = nullptr;
  // speculative-decoding baseline (cfg.sd_gamma > 0): device state, the second set of draft row descriptors
  SdBase sd;
  RowDescW sd_rd2{nullptr, nullptr, nullptr, nullptr, nullptr};
  int sd_next_entries = 0;       // entries of the next round's first draft pass, once known
  unsigned sd_wait_ticket = 0;   // != 0: the last round's finish kernel will report them under this ticket
  int run_kind = 0;              // since the last prefill: 0 nothing, 1 decode steps, 2 speculative-decoding rounds
  // host bookkeeping
  int B = 0, max_prompt_len = 0;
  long long steps_done = 0;
  bool prefilled = false;
  char err[512];
};

namespace {

int fail(sprinter_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) snprintf(ctx->err, sizeof ctx->err, "%s", buf);
  snprintf(g_err, sizeof g_err, "%s", buf);
  return code;
}

int rows_alloc_for(int max_batch) {
  if (max_batch <= 16) return 16;
  if (max_batch <= 32) return 32;
  if (max_batch <= 64) return 64;
  return round_up(max_batch, 128);
}

size_t esize(int dtype) { return dtype == SPRINTER_F32 ? 4 : 2; }
// elements of an activation buffer [rows, K] in the activation layout (bf16 mode: float16 operand tiles)
size_t act_elems(int dtype, int rows, int K) { return (size_t)rows * (dtype == SPRINTER_F32 ? K : round_up(K, 32)); }
size_t packed_elems(int N, int K) { return (size_t)round_up(N, 16) * round_up(K, 32); }

constexpr int DEFAULT_CHUNK_ROWS = 4096;

const char* check_model(const sprinter_model_cfg& m, const char* who, char* buf, size_t n) {
#define BAD(...) do { snprintf(buf, n, __VA_ARGS__); return buf; } while (0)
  if (m.arch != SPRINTER_ARCH_GPT && m.arch != SPRINTER_ARCH_LLAMA) BAD("%s: unknown arch %d", who, m.arch);
  if (m.n_layer < 1 || m.d_model < 8 || m.n_head < 1 || m.n_kv_head < 1 || m.d_ff < 8 || m.vocab < 2 || m.max_pos < 2)
    BAD("%s: non-positive dimension", who);
  if (m.d_model % m.n_head) BAD("%s: d_model %d not divisible by n_head %d", who, m.d_model, m.n_head);
  int dh = m.d_model / m.n_head;
  if (dh != 64 && dh != 128) BAD("%s: head dimension %d is not 64 or 128", who, dh);
  if (m.n_head % m.n_kv_head) BAD("%s: n_head %d not divisible by n_kv_head %d", who, m.n_head, m.n_kv_head);
  int G = m.n_head / m.n_kv_head;
  if (G != 1 && G != 2 && G != 4 && G != 8) BAD("%s: %d query heads per KV head unsupported (1, 2, 4, 8)", who, G);
  if (m.d_model % 8 || m.d_ff % 8) BAD("%s: d_model and d_ff must be multiples of 8", who);
  if (m.d_model > 8192) BAD("%s: d_model %d > 8192", who, m.d_model);
  if (!(m.norm_eps >= 0.f)) BAD("%s: norm_eps", who);
  if (m.arch == SPRINTER_ARCH_LLAMA && !(m.rope_theta > 1.f)) BAD("%s: rope_theta", who);
  return nullptr;
#undef BAD
}

int validate_cfg(const sprinter_cfg* c, char* buf, size_t n) {
  const char* e;
  if ((e = check_model(c->draft, "draft", buf, n))) return SPRINTER_E_CONFIG;
  if ((e = check_model(c->target, "target", buf, n))) return SPRINTER_E_CONFIG;
#define BAD(...) do { snprintf(buf, n, __VA_ARGS__); return SPRINTER_E_CONFIG; } while (0)
  if (c->draft.vocab != c->target.vocab) BAD("draft and target vocabularies differ (%d vs %d)", c->draft.vocab, c->target.vocab);
  if (c->ver_d_in != c->draft.d_model) BAD("verifier input width %d != draft d_model %d", c->ver_d_in, c->draft.d_model);
  if (c->ver_d_hidden < 0 || c->ver_d_hidden > 65536) BAD("verifier hidden width %d", c->ver_d_hidden);
  if (c->dtype != SPRINTER_F32 && c->dtype != SPRINTER_BF16) BAD("unknown dtype %d", c->dtype);
  if (c->max_batch < 1 || c->max_batch > 1024) BAD("max_batch %d outside [1, 1024]", c->max_batch);
  if (c->max_seq < 2) BAD("max_seq %d < 2", c->max_seq);
  if (c->draft.arch == SPRINTER_ARCH_GPT && c->max_seq > c->draft.max_pos) BAD("max_seq %d > draft max_pos %d", c->max_seq, c->draft.max_pos);
  if (c->target.arch == SPRINTER_ARCH_GPT && c->max_seq > c->target.max_pos) BAD("max_seq %d > target max_pos %d", c->max_seq, c->target.max_pos);
  if (!(c->temperature >= 0.f)) BAD("temperature must be >= 0");
  if (!(c->tau == c->tau)) BAD("tau is NaN");
  if (c->target_ctx_mode != 0 && c->target_ctx_mode != 1)
    BAD("target_ctx_mode %d is not one of 0 (own history), 1 (full prefix)", c->target_ctx_mode);
  if (c->reject_mode != 0 && c->reject_mode != 1) BAD("reject_mode %d is not one of 0 (replace), 1 (p/q correction)", c->reject_mode);
  if (c->reject_mode == 1 && !(c->temperature > 0.f)) BAD("reject_mode 1 needs a temperature > 0");
  if (c->sd_gamma < 0 || c->sd_gamma > 16) BAD("sd_gamma %d outside [0, 16]", c->sd_gamma);
  if (c->chunk_rows != 0 && (c->chunk_rows < 64 || c->chunk_rows > 4096 || c->chunk_rows % 64 != 0))
    BAD("chunk_rows %d is not 0 or a multiple of 64 in [64, 4096]", c->chunk_rows);
  // the float32 attention kernel keeps one score per cached key in LDS; the bf16 kernels keep none
  if (c->dtype == SPRINTER_F32) for (const sprinter_model_cfg* m : {&c->draft, &c->target}) {
    int dh = m->d_model / m->n_head, G = m->n_head / m->n_kv_head;
    size_t lds = (size_t)(G * dh + 2 * dh + 4 * G * dh + G * c->max_seq) * 4;
    if (lds > 64 * 1024) BAD("attention needs %zu bytes of LDS for max_seq %d (limit 65536)", lds, c->max_seq);
  }
  return SPRINTER_OK;
#undef BAD
}

ModelDims dims_of(const sprinter_model_cfg& m) {
  ModelDims d;
  d.arch = m.arch; d.n_layer = m.n_layer; d.d = m.d_model; d.H = m.n_head; d.KVH = m.n_kv_head;
  d.dh = m.d_model / m.n_head; d.ff = m.d_ff; d.V = m.vocab; d.max_pos = m.max_pos;
  d.dqkv = (m.n_head + 2 * m.n_kv_head) * d.dh; d.eps = m.norm_eps; d.theta = m.rope_theta;
  return d;
}

// Slots per (row, KV head) of a cache: the bf16 value cache is kept in blocks of 32 slots (tiles of V^T).
int kv_slots(const sprinter_cfg& c) { return c.dtype == SPRINTER_BF16 ? round_up(c.max_seq, 32) : c.max_seq; }

// Lays one model out in the workspace (or only measures when bump.base == nullptr).
void carve_model(Bump& bump, const sprinter_cfg& c, const sprinter_model_cfg& mc, Model* m, int rows) {
  ModelDims md = dims_of(mc);
  const size_t es = esize(c.dtype);
  const bool bf = c.dtype == SPRINTER_BF16;
  size_t layer_stride = (size_t)c.max_batch * md.KVH * kv_slots(c) * md.dh;
  void* kc = bump.take(layer_stride * md.n_layer * es);
  void* vc = bump.take(layer_stride * md.n_layer * es);
  ModelScratch sc;
  sc.h = (float*)bump.take((size_t)rows * md.d * 4);
  sc.xn = bump.take(act_elems(c.dtype, rows, md.d) * es);
  sc.y = (float*)bump.take((size_t)rows * md.dqkv * 4);
  sc.ao = bump.take(act_elems(c.dtype, rows, md.H * md.dh) * es);
  sc.mid = bump.take(act_elems(c.dtype, rows, md.ff) * es);
  sc.hf = (float*)bump.take((size_t)rows * md.d * 4);
  sc.hfn = bump.take(act_elems(c.dtype, rows, md.d) * es);
  sc.rope = (float*)bump.take((size_t)rows * md.dh * 4);
  sc.part = (float*)bump.take((size_t)PART_SHARES * rows * md.d * 4);
  sc.n_lm_wg = lmhead_num_wg(c.dtype, md.V);
  sc.am_part = (unsigned long long*)bump.take((size_t)sc.n_lm_wg * rows * 8);
  int* rd_n = (int*)bump.take(4);
  int* rd_b = (int*)bump.take((size_t)rows * 4);
  int* rd_tok = (int*)bump.take((size_t)rows * 4);
  int* rd_pos = (int*)bump.take((size_t)rows * 4);
  int* rd_slot = (int*)bump.take((size_t)rows * 4);
  if (m) {
    m->cfg = mc; m->md = md; m->kcache = kc; m->vcache = vc; m->layer_stride = layer_stride; m->sc = sc;
    m->rd_n = rd_n; m->rd_b = rd_b; m->rd_tok = rd_tok; m->rd_pos = rd_pos; m->rd_slot = rd_slot;
    m->layers.assign(md.n_layer, LayerW{});
    m->expected.clear();
  }
  auto want = [&](const std::string& name, int64_t r, int64_t cl, bool is_matrix, bool gathered, const void** slot,
                  const void** slot2 = nullptr) {
    bool pack = bf && is_matrix && !gathered;
    void* dst = pack ? bump.take(packed_elems((int)r, (int)cl) * 2) : nullptr;
    void* dst2 = (bf && slot2) ? bump.take(packed_elems((int)r, (int)cl) * 2) : nullptr;
    if (m) m->expected.push_back(Expected{name, r, cl, pack, slot, dst, slot2, dst2, false});
  };
  const int d = md.d, ff = md.ff, V = md.V;
  const bool gpt = md.arch == SPRINTER_ARCH_GPT;
  Model dummy;
  Model* t = m ? m : &dummy;
  if (!m) dummy.layers.assign(md.n_layer, LayerW{});
  want("tok_emb", V, d, true, true, &t->tok_emb, gpt ? &t->lm_head : nullptr);
  if (gpt) want("pos_emb", md.max_pos, d, true, true, &t->pos_emb);
  for (int i = 0; i < md.n_layer; ++i) {
    std::string p = "l" + std::to_string(i) + ".";
    LayerW& L = t->layers[i];
    want(p + "norm1.g", d, 0, false, false, (const void**)&L.n1g);
    if (gpt) want(p + "norm1.b", d, 0, false, false, (const void**)&L.n1b);
    want(p + "wqkv", md.dqkv, d, true, false, &L.wqkv);
    if (gpt) want(p + "bqkv", md.dqkv, 0, false, false, (const void**)&L.bqkv);
    want(p + "wo", d, md.H * md.dh, true, false, &L.wo);
    if (gpt) want(p + "bo", d, 0, false, false, (const void**)&L.bo);
    want(p + "norm2.g", d, 0, false, false, (const void**)&L.n2g);
    if (gpt) {
      want(p + "norm2.b", d, 0, false, false, (const void**)&L.n2b);
      want(p + "w1", ff, d, true, false, &L.w1);
      want(p + "b1", ff, 0, false, false, (const void**)&L.b1);
      want(p + "w2", d, ff, true, false, &L.w2);
      want(p + "b2", d, 0, false, false, (const void**)&L.b2);
    } else {
      want(p + "wg", ff, d, true, false, &L.wg);
      want(p + "wu", ff, d, true, false, &L.wu);
      want(p + "w2", d, ff, true, false, &L.w2);
    }
  }
  want("normf.g", d, 0, false, false, &t->normf_g);
  if (gpt) want("normf.b", d, 0, false, false, &t->normf_b);
  else want("lm_head", V, d, true, false, &t->lm_head);
  if (m) {
    m->index.clear();
    for (size_t i = 0; i < m->expected.size(); ++i) m->index[m->expected[i].name] = (int)i;
  }
}

// Rows the activation buffers hold = entries one pass of a multi-entry forward takes (prefill chunks, full-prefix
// work lists, speculative-decoding windows).
int chunk_rows_of(const sprinter_cfg& c) {
  const int batch_rows = rows_alloc_for(c.target_ctx_mode == 1 ? std::min(2 * c.max_batch, 1024) : c.max_batch);
  const int want = c.chunk_rows > 0 ? c.chunk_rows : (c.dtype == SPRINTER_BF16 ? DEFAULT_CHUNK_ROWS : 16);
  return std::max(want, batch_rows);
}

// Lays the whole workspace out; ctx == nullptr only measures.  Returns total bytes.
size_t carve(const sprinter_cfg& c, void* base, sprinter_ctx* ctx, size_t* scratch_begin, size_t* scratch_end) {
  Bump bump(base);
  // full-prefix mode: every committed token reaches the target once, so a step's work list averages one entry
  // per batch row with wide swings; buffers for twice the batch keep most steps to a single pass.
  // bf16: a prefill pass takes DEFAULT_CHUNK_ROWS prompt tokens per pass over the weights unless cfg.chunk_rows says otherwise
  const int rows = chunk_rows_of(c);
  carve_model(bump, c, c.draft, ctx ? &ctx->draft : nullptr, rows);
  carve_model(bump, c, c.target, ctx ? &ctx->target : nullptr, rows);
  int chunks = verifier_num_chunks(c.ver_d_hidden);
  float* ver_part = (float*)bump.take((size_t)chunks * c.max_batch * 4);
  State st;
  st.last_tok = (int*)bump.take((size_t)c.max_batch * 4);
  st.len_q = (int*)bump.take((size_t)c.max_batch * 4);
  st.len_p = (int*)bump.take((size_t)c.max_batch * 4);
  st.prompt_len = (int*)bump.take((size_t)c.max_batch * 4);
  st.n_target_calls = (long long*)bump.take((size_t)c.max_batch * 8);
  st.counters = (long long*)bump.take(4 * 8);
  st.hist_stride = c.max_seq + 1;
  st.hist = (int*)bump.take((size_t)c.max_batch * st.hist_stride * 4);
  int* ent_off = (int*)bump.take((size_t)(c.max_batch + 1) * 4);
  int* t_last = (int*)bump.take((size_t)rows * 4);
  int* coin_kept = (int*)bump.take(4);
  float *dl = nullptr, *tl = nullptr;
  if (c.reject_mode == 1) {      // both models' logits of the step in flight
    dl = (float*)bump.take((size_t)c.max_batch * c.draft.vocab * 4);
    tl = (float*)bump.take((size_t)rows * c.target.vocab * 4);
  }
  SdBase sd;
  memset(&sd, 0, sizeof sd);
  RowDescW rd2{nullptr, nullptr, nullptr, nullptr, nullptr};
  if (c.sd_gamma > 0) {
    const size_t B = c.max_batch, G = c.sd_gamma;
    sd.len_dc = (int*)bump.take(B * 4);
    sd.win = (int*)bump.take(B * G * 4);
    sd.qrow = (int*)bump.take(B * G * 4);
    sd.kept = (unsigned char*)bump.take(B * G);
    sd.alt = (int*)bump.take(B * (G + 1) * 4);
    sd.d0_n = (int*)bump.take(4);
    sd.d0_b = (int*)bump.take(2 * B * 4);
    sd.d0_tok = (int*)bump.take(2 * B * 4);
    sd.d0_pos = (int*)bump.take(2 * B * 4);
    sd.d0_last = (int*)bump.take(2 * B * 4);
    sd.o_cnt = (int*)bump.take(B * 4);
    sd.dlw = (float*)bump.take((G + 1) * B * c.draft.vocab * 4);
    sd.tlw = (float*)bump.take((G + 1) * B * c.target.vocab * 4);
    rd2.n_rows = (int*)bump.take(4);
    rd2.b = (int*)bump.take(B * 4);
    rd2.tok = (int*)bump.take(B * 4);
    rd2.pos = (int*)bump.take(B * 4);
    rd2.slot = (int*)bump.take(B * 4);
  }
  float* tau = (float*)bump.take(4);
  int* draft_tok = (int*)bump.take((size_t)c.max_batch * 4);
  float* score = (float*)bump.take((size_t)c.max_batch * 4);
  unsigned char* accept = (unsigned char*)bump.take((size_t)c.max_batch);
  int* rej_idx = (int*)bump.take((size_t)c.max_batch * 4);
  int* n_rej = (int*)bump.take(4);
  int* committed = (int*)bump.take((size_t)c.max_batch * 4);
  unsigned long long* dev_counts = (unsigned long long*)bump.take(256);
  size_t total = (bump.off + 255) & ~(size_t)255;
  if (ctx) {
    ctx->ver_part = ver_part; ctx->ver_chunks = chunks; ctx->st = st; ctx->tau_dev = tau;
    ctx->draft_tok = draft_tok; ctx->score = score; ctx->accept = accept; ctx->rej_idx = rej_idx;
    ctx->n_rej = n_rej; ctx->committed = committed; ctx->rows_alloc = rows; ctx->dev_counts = dev_counts;
    ctx->ent_off = ent_off; ctx->t_last = t_last; ctx->coin_kept = coin_kept; ctx->dl = dl; ctx->tl = tl;
    sd.st = st; sd.coin_kept = coin_kept; sd.V = c.target.vocab;
    sd.seed_lo = (unsigned)(c.seed & 0xFFFFFFFFull); sd.seed_hi = (unsigned)(c.seed >> 32);
    sd.inv_temperature = c.temperature > 0.f ? 1.0f / c.temperature : 0.f;
    ctx->sd = sd; ctx->sd_rd2 = rd2;
  }
  (void)scratch_begin; (void)scratch_end;
  return total;
}

// One model forward over the rows described by rd (device-side count).
// shared_caches: several rows of rd may belong to one batch row (consecutive positions): every layer appends all
// new keys / values first and attends in a second launch.  long_runs: those entries come in long runs of
// consecutive positions (prefill), so the attending launch lets 8 queries share one pass over the row's cache.
void forward(sprinter_ctx* ctx, Model& m, const RowDesc& rd, int max_rows, bool want_head, unsigned stream_id,
             float* logits_out, bool shared_caches = false, bool long_runs = false) {
  const int dt = ctx->cfg.dtype;
  const ModelDims& md = m.md;
  hipStream_t s = ctx->stream;
  ModelScratch& sc = m.sc;
  const int rows = ctx->rows_alloc;
  // elements the activation buffers hold (their row tiles bound what a kernel may fetch)
  const size_t pl_d = act_elems(dt, rows, md.d), pl_a = act_elems(dt, rows, md.H * md.dh), pl_f = act_elems(dt, rows, md.ff);
  launch_embed(dt, md, m.tok_emb, m.pos_emb, rd, sc.h, sc.rope, max_rows, s);
  // bf16: O-proj and FFN-down split K over workgroups and leave partial products; the norm that follows folds
  // them (and the bias) into the residual stream before it normalises the row.
  const bool split = norm_takes_pending(dt, md.d);
  const size_t part_stride = (size_t)rows * md.d;
  NormPending pend{sc.part, part_stride, 0, nullptr};
  auto resid_gemm = [&](const void* W, const void* X, size_t plane, int K, const float* bias) {
    if (split) {
      pend.shares = launch_gemm_part(W, X, plane, rd.n_rows, md.d, K, sc.part, part_stride, PART_SHARES, max_rows, s);
      pend.bias = bias;
    } else {
      launch_gemm(dt, EPI_RESID, W, nullptr, X, plane, rd.n_rows, md.d, K, bias, sc.h, md.d, nullptr, 0, max_rows, s);
    }
  };
  auto norm = [&](const float* g, const float* b, void* out, float* f32_out) {
    launch_norm(dt, md.arch, sc.h, g, b, md.eps, md.d, rd.n_rows, out, f32_out, max_rows, s,
                pend.shares > 0 ? &pend : nullptr);
    pend.shares = 0;
  };
  for (int i = 0; i < md.n_layer; ++i) {
    const LayerW& L = m.layers[i];
    norm(L.n1g, L.n1b, sc.xn, nullptr);
    launch_gemm(dt, EPI_F32, L.wqkv, nullptr, sc.xn, pl_d, rd.n_rows, md.dqkv, md.d, L.bqkv, sc.y, md.dqkv, nullptr, 0,
                max_rows, s);
    if (shared_caches) {
      launch_attention(dt, md, sc.y, sc.rope, rd, m.kcache, m.vcache, m.layer_stride * i, ctx->max_prompt_len + (int)ctx->steps_done,
                       kv_slots(ctx->cfg), sc.ao, max_rows, s, 1);
      launch_attention(dt, md, sc.y, sc.rope, rd, m.kcache, m.vcache, m.layer_stride * i, ctx->max_prompt_len + (int)ctx->steps_done,
                       kv_slots(ctx->cfg), sc.ao, max_rows, s, long_runs ? 3 : 2);
    } else {
      launch_attention(dt, md, sc.y, sc.rope, rd, m.kcache, m.vcache, m.layer_stride * i, ctx->max_prompt_len + (int)ctx->steps_done,
                       kv_slots(ctx->cfg), sc.ao, max_rows, s);
    }
    if (!want_head && i + 1 == md.n_layer) break;   // a prefill position only has to fill the caches
    resid_gemm(L.wo, sc.ao, pl_a, md.H * md.dh, L.bo);
    norm(L.n2g, L.n2b, sc.xn, nullptr);
    if (md.arch == SPRINTER_ARCH_GPT)
      launch_gemm(dt, EPI_GELU, L.w1, nullptr, sc.xn, pl_d, rd.n_rows, md.ff, md.d, L.b1, nullptr, 0, sc.mid, md.ff,
                  max_rows, s);
    else
      launch_gemm(dt, EPI_SWIGLU, L.wg, L.wu, sc.xn, pl_d, rd.n_rows, md.ff, md.d, nullptr, nullptr, 0, sc.mid, md.ff,
                  max_rows, s);
    resid_gemm(L.w2, sc.mid, pl_f, md.ff, L.b2);
  }
  if (!want_head) return;
  norm((const float*)m.normf_g, (const float*)m.normf_b, sc.hfn, sc.hf);
  SamplerArgs sa;
  sa.seed_lo = (unsigned)(ctx->cfg.seed & 0xFFFFFFFFull);
  sa.seed_hi = (unsigned)(ctx->cfg.seed >> 32);
  sa.stream = stream_id;
  sa.inv_temperature = ctx->cfg.temperature > 0.f ? 1.0f / ctx->cfg.temperature : 0.f;
  launch_lmhead(dt, m.lm_head, sc.hfn, pl_d, rd, md.V, md.d, sa, sc.am_part, sc.n_lm_wg, ctx->rows_alloc, logits_out,
                max_rows, s);
}

int check_ready(sprinter_ctx* ctx) {
  if (!ctx->draft.loaded || !ctx->target.loaded || !ctx->v_loaded)
    return fail(ctx, SPRINTER_E_WEIGHTS, "weights not loaded (draft %d, target %d, verifier %d)", (int)ctx->draft.loaded,
                (int)ctx->target.loaded, (int)ctx->v_loaded);
  return SPRINTER_OK;
}

int check_room(sprinter_ctx* ctx, long long extra_steps) {
  if (!ctx->prefilled) return fail(ctx, SPRINTER_E_STATE, "no prefill has been done");
  long long last_slot = (long long)ctx->max_prompt_len - 1 + ctx->steps_done + extra_steps - 1;
  if (last_slot > ctx->cfg.max_seq - 1)
    return fail(ctx, SPRINTER_E_RANGE, "prompt length %d + %lld generated tokens exceeds max_seq %d",
                ctx->max_prompt_len, ctx->steps_done + extra_steps, ctx->cfg.max_seq);
  return SPRINTER_OK;
}

// Polls a pinned word a kernel stores (ticket << 32) | value into; after 2 s without the ticket it falls back to
// a stream synchronisation.
int wait_ticket(sprinter_ctx* ctx, volatile unsigned long long* word, unsigned ticket, int* value, const char* what) {
  if (ctx->static_dev >= 0) {
    // no pinned memory in this kind of context: the kernels store the words in the workspace; fetch them
    if (hipMemcpyAsync(ctx->static_words, ctx->dev_counts, sizeof ctx->static_words, hipMemcpyDeviceToHost, ctx->stream) != hipSuccess ||
        hipStreamSynchronize(ctx->stream) != hipSuccess)
      return fail(ctx, SPRINTER_E_HIP, "waiting for the device failed: %s", hipGetErrorString(hipGetLastError()));
    const unsigned long long v = *word;
    if ((unsigned)(v >> 32) != ticket) return fail(ctx, SPRINTER_E_HIP, "%s", what);
    *value = (int)(unsigned)(v & 0xFFFFFFFFull);
    return SPRINTER_OK;
  }
  const auto t0 = std::chrono::steady_clock::now();
  for (unsigned spin = 0;; ++spin) {
    const unsigned long long v = *word;
    if ((unsigned)(v >> 32) == ticket) { *value = (int)(unsigned)(v & 0xFFFFFFFFull); return SPRINTER_OK; }
    if ((spin & 0xFFF) == 0xFFF && std::chrono::steady_clock::now() - t0 > std::chrono::seconds(2)) {
      if (hipStreamSynchronize(ctx->stream) != hipSuccess)
        return fail(ctx, SPRINTER_E_HIP, "waiting for the device failed: %s", hipGetErrorString(hipGetLastError()));
      const unsigned long long v2 = *word;
      if ((unsigned)(v2 >> 32) != ticket) return fail(ctx, SPRINTER_E_HIP, "%s", what);
      *value = (int)(unsigned)(v2 & 0xFFFFFFFFull);
      return SPRINTER_OK;
    }
  }
}

int enqueue_step(sprinter_ctx* ctx, const sprinter_step_out* out, int n_tokens, int32_t* g_tok, uint8_t* g_accept,
                  float* g_score, int32_t* g_draft_tok) {
  hipStream_t s = ctx->stream;
  const int B = ctx->B;
  Model &dq = ctx->draft, &tp = ctx->target;
  const bool sd = ctx->cfg.reject_mode == 1;
  forward(ctx, dq, dq.rd(), B, true, 0u, sd ? ctx->dl : (out ? out->draft_logits : nullptr));
  if (sd && out && out->draft_logits) launch_copy_f32(ctx->dl, out->draft_logits, dq.rd_n, dq.md.V, B, s);
  if (out && out->draft_hidden) launch_copy_f32(dq.sc.hf, out->draft_hidden, dq.rd_n, dq.md.d, B, s);
  launch_verifier_part(dq.sc.hf, dq.md.d, ctx->cfg.ver_d_hidden, (const float*)ctx->v_w1, (const float*)ctx->v_b1,
                       (const float*)ctx->v_w2, dq.rd_n, ctx->ver_part, B, s);
  DecideArgs da;
  da.am_part = dq.sc.am_part; da.n_lm_wg = dq.sc.n_lm_wg; da.Mpad = ctx->rows_alloc;
  da.ver_part = ctx->ver_part; da.n_chunks = ctx->ver_chunks; da.b2 = (const float*)ctx->v_b2; da.tau_ptr = ctx->tau_dev;
  da.B = B; da.st = ctx->st;
  da.draft_tok = ctx->draft_tok; da.score = ctx->score; da.accept = ctx->accept; da.rej_idx = ctx->rej_idx;
  da.n_rej = ctx->n_rej; da.committed = ctx->committed;
  da.t_n_rows = tp.rd_n; da.t_b = tp.rd_b; da.t_tok = tp.rd_tok; da.t_pos = tp.rd_pos; da.t_slot = tp.rd_slot;
  da.o_draft_tok = out ? out->draft_tok : nullptr; da.o_score = out ? out->score : nullptr;
  da.o_accept = out ? out->accept : nullptr; da.o_rej_idx = out ? out->rej_idx : nullptr;
  da.o_n_rej = out ? out->n_rej : nullptr;
  const int mode = ctx->cfg.target_ctx_mode;
  da.ctx_mode = mode; da.ent_off = ctx->ent_off;
  da.host_word = ctx->kernel_word; da.ticket = ++ctx->ticket;
  if (da.ticket == 0) da.ticket = ++ctx->ticket;   // 0 is the word's initial value
  launch_draft_decide(da, s);
  // The host waits for the number of rejected rows R: the target's kernels are then launched for exactly R
  // rows (row-tile count and K split follow R, not the batch size), and not at all when every row accepted.
  // The decide kernel stores (ticket, R) into pinned memory and the host polls that word, which costs a few
  // microseconds; after 2 s without the ticket it falls back to a stream synchronisation.
  int R = -1;
  {
    int rc = wait_ticket(ctx, ctx->host_counts, da.ticket, &R, "the draft pass did not report its rejected rows");
    if (rc) return rc;
  }
  if (R < 0 || R > B) return fail(ctx, SPRINTER_E_HIP, "device reported %d rejected rows of %d", R, B);
  SdArgs sa;
  memset(&sa, 0, sizeof sa);
  if (sd) {
    sa.dl = ctx->dl; sa.tl = ctx->tl; sa.n_rows = tp.rd_n; sa.t_b = tp.rd_b; sa.t_pos = tp.rd_pos;
    sa.draft_tok = ctx->draft_tok; sa.V = tp.md.V; sa.inv_temperature = 1.0f / ctx->cfg.temperature;
    sa.seed_lo = (unsigned)(ctx->cfg.seed & 0xFFFFFFFFull); sa.seed_hi = (unsigned)(ctx->cfg.seed >> 32);
    sa.committed = ctx->committed; sa.coin_kept = ctx->coin_kept;
  }
  if (R > 0 && mode == 0) {
    forward(ctx, tp, tp.rd(), R, true, 1u, sd ? ctx->tl : (out ? out->target_logits : nullptr));
    if (sd) {
      launch_sd_correct(sa, R, s);
      if (out && out->target_logits) launch_copy_f32(ctx->tl, out->target_logits, tp.rd_n, tp.md.V, R, s);
    }
    if (out && out->target_hidden) launch_copy_f32(tp.sc.hf, out->target_hidden, tp.rd_n, tp.md.d, R, s);
  } else if (R > 0) {
    // full prefix: the work list (E entries, at least one per rejected row) goes through the target in chunks of
    // at most rows_alloc entries, in list order, so that a later entry of a row finds the earlier ones cached
    const long long E = (long long)((volatile unsigned long long*)ctx->host_counts)[1];
    if (E < R || E > (long long)B * ctx->cfg.max_seq) return fail(ctx, SPRINTER_E_HIP, "device reported %lld work-list entries for %d rows", E, R);
    CatchupArgs ca;
    ca.st = ctx->st; ca.rej_idx = ctx->rej_idx; ca.n_rej = ctx->n_rej; ca.ent_off = ctx->ent_off;
    ca.t_n_rows = tp.rd_n; ca.t_b = tp.rd_b; ca.t_tok = tp.rd_tok; ca.t_pos = tp.rd_pos; ca.t_slot = tp.rd_slot;
    ca.t_last = ctx->t_last;
    for (long long start = 0; start < E; start += ctx->rows_alloc) {
      const int n = (int)std::min<long long>(ctx->rows_alloc, E - start);
      ca.start = (int)start; ca.n = n;
      launch_catchup_chunk(ca, s);
      forward(ctx, tp, tp.rd(), n, true, 1u, sd ? ctx->tl : nullptr, true);
      if (sd) {
        sa.t_last = ctx->t_last;
        launch_sd_correct(sa, n, s);
      } else {
        launch_catchup_collect(tp.sc.am_part, tp.sc.n_lm_wg, ctx->rows_alloc, tp.rd_n, tp.rd_b, ctx->t_last,
                               ctx->committed, n, s);
      }
    }
  }
  FinishArgs fa;
  fa.am_part = tp.sc.am_part; fa.n_lm_wg = tp.sc.n_lm_wg; fa.Mpad = ctx->rows_alloc; fa.B = B; fa.st = ctx->st;
  fa.draft_tok = ctx->draft_tok; fa.score = ctx->score; fa.accept = ctx->accept; fa.rej_idx = ctx->rej_idx;
  fa.n_rej = ctx->n_rej; fa.committed = ctx->committed;
  fa.d_n_rows = dq.rd_n; fa.d_b = dq.rd_b; fa.d_tok = dq.rd_tok; fa.d_pos = dq.rd_pos; fa.d_slot = dq.rd_slot;
  fa.o_committed = out ? out->committed_tok : nullptr;
  fa.ctx_mode = mode; fa.pre_merged = (mode == 1 || sd) ? 1 : 0;
  fa.n_tokens = n_tokens; fa.g_tok = g_tok; fa.g_accept = g_accept; fa.g_score = g_score; fa.g_draft_tok = g_draft_tok;
  launch_step_finish(fa, s);
  return SPRINTER_OK;
}

int hip_status(sprinter_ctx* ctx, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, SPRINTER_E_HIP, "%s: %s", what, hipGetErrorString(e));
  return SPRINTER_OK;
}

// What sprinter_create and sprinter_create_static share: cfg is valid and the workspace large enough.
// static_dev >= 0: the workspace is the library's static array on that device and the context must not allocate
// anything, pinned host memory included.
int create_common(const sprinter_cfg* cfg, void* dev_workspace, void* hip_stream, int static_dev, sprinter_ctx** out_ctx) {
  sprinter_ctx* ctx = new sprinter_ctx();
  ctx->cfg = *cfg;
  ctx->stream = (hipStream_t)hip_stream;
  ctx->err[0] = 0;
  carve(*cfg, dev_workspace, ctx, nullptr, nullptr);
  // verifier tensors
  auto vwant = [&](const char* name, int64_t r, int64_t c, const void** slot) {
    ctx->v_expected.push_back(Expected{name, r, c, false, slot, nullptr, nullptr, nullptr, false});
  };
  if (cfg->ver_d_hidden > 0) {
    vwant("v.w1", cfg->ver_d_hidden, cfg->ver_d_in, &ctx->v_w1);
    vwant("v.b1", cfg->ver_d_hidden, 0, &ctx->v_b1);
    vwant("v.w2", cfg->ver_d_hidden, 0, &ctx->v_w2);
  } else {
    vwant("v.w2", cfg->ver_d_in, 0, &ctx->v_w2);
  }
  vwant("v.b2", 1, 0, &ctx->v_b2);
  for (size_t i = 0; i < ctx->v_expected.size(); ++i) ctx->v_index[ctx->v_expected[i].name] = (int)i;
  // activation scratch must start at zero (padding lanes of operand tiles are never written)
  for (Model* m : {&ctx->draft, &ctx->target}) {
    const int rows = ctx->rows_alloc;
    const size_t es = esize(cfg->dtype);
    launch_fill_zero(m->sc.xn, act_elems(cfg->dtype, rows, m->md.d) * es, ctx->stream);
    launch_fill_zero(m->sc.ao, act_elems(cfg->dtype, rows, m->md.H * m->md.dh) * es, ctx->stream);
    launch_fill_zero(m->sc.mid, act_elems(cfg->dtype, rows, m->md.ff) * es, ctx->stream);
    launch_fill_zero(m->sc.hfn, act_elems(cfg->dtype, rows, m->md.d) * es, ctx->stream);
  }
  launch_set_f32(ctx->tau_dev, cfg->tau, ctx->stream);
  launch_fill_zero(ctx->dev_counts, 256, ctx->stream);
  if (static_dev >= 0) {
    ctx->static_dev = static_dev;
    ctx->host_counts = ctx->static_words;
    ctx->kernel_word = ctx->dev_counts;
  } else {
    if (hipHostMalloc((void**)&ctx->host_counts, 256, hipHostMallocDefault) != hipSuccess) {
      delete ctx;
      return fail(nullptr, SPRINTER_E_HIP, "allocation of the pinned count buffer failed");
    }
    memset(ctx->host_counts, 0, 256);
    ctx->kernel_word = ctx->host_counts;
  }
  int rc = hip_status(ctx, "sprinter_create");
  if (rc) {
    if (static_dev >= 0) { ctx->static_dev = -1; ctx->host_counts = nullptr; }   // (the caller releases the static workspace)
    sprinter_destroy(ctx);
    return rc;
  }
  *out_ctx = ctx;
  return SPRINTER_OK;
}


}  // namespace

extern "C" {

int sprinter_workspace_bytes(const sprinter_cfg* cfg, size_t* out_bytes) {
  if (!cfg || !out_bytes) return fail(nullptr, SPRINTER_E_NULL, "sprinter_workspace_bytes: NULL argument");
  char buf[256];
  int rc = validate_cfg(cfg, buf, sizeof buf);
  if (rc) return fail(nullptr, rc, "%s", buf);
  *out_bytes = carve(*cfg, nullptr, nullptr, nullptr, nullptr);
  return SPRINTER_OK;
}

int sprinter_create(const sprinter_cfg* cfg, void* dev_workspace, size_t workspace_bytes, void* hip_stream,
                    sprinter_ctx** out_ctx) {
  if (!cfg || !dev_workspace || !out_ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_create: NULL argument");
  *out_ctx = nullptr;
  char buf[256];
  int rc = validate_cfg(cfg, buf, sizeof buf);
  if (rc) return fail(nullptr, rc, "%s", buf);
  if (((uintptr_t)dev_workspace) & 255) return fail(nullptr, SPRINTER_E_WORKSPACE, "workspace is not 256-byte aligned");
  size_t need = carve(*cfg, nullptr, nullptr, nullptr, nullptr);
  if (workspace_bytes < need)
    return fail(nullptr, SPRINTER_E_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
  return create_common(cfg, dev_workspace, hip_stream, -1, out_ctx);
}

int sprinter_create_static(const sprinter_cfg* cfg, void* hip_stream, sprinter_ctx** out_ctx) {
  if (!cfg || !out_ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_create_static: NULL argument");
  *out_ctx = nullptr;
  char buf[256];
  int rc = validate_cfg(cfg, buf, sizeof buf);
  if (rc) return fail(nullptr, rc, "%s", buf);
  const size_t need = carve(*cfg, nullptr, nullptr, nullptr, nullptr);
  if (need > STATIC_WORKSPACE_BYTES)
    return fail(nullptr, SPRINTER_E_WORKSPACE, "this configuration needs %zu bytes of workspace, the static workspace holds %zu",
                need, STATIC_WORKSPACE_BYTES);
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_STATIC_DEVICES)
    return fail(nullptr, SPRINTER_E_HIP, "no current device with an index below %d", MAX_STATIC_DEVICES);
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    StaticSlot& slot = g_static[dev];
    if (!slot.base) {   // once per device, with that device current: every GPU holds its own copy of the array
      void* p = nullptr;
      const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return fail(nullptr, SPRINTER_E_HIP, "address of the static workspace on device %d: %s", dev, hipGetErrorString(e));
      if (((uintptr_t)p) & 255) return fail(nullptr, SPRINTER_E_WORKSPACE, "static workspace is not 256-byte aligned");
      slot.base = p;
    }
    if (slot.in_use)
      return fail(nullptr, SPRINTER_E_STATE, "device %d already has a live context on the static workspace; destroy it first", dev);
    slot.in_use = true;
    base = slot.base;
  }
  rc = create_common(cfg, base, hip_stream, dev, out_ctx);
  if (rc) {
    std::lock_guard<std::mutex> lock(g_static_mu);
    g_static[dev].in_use = false;
  }
  return rc;
}

int sprinter_load_weights(sprinter_ctx* ctx, int which, const char* const* names, const void* const* dev_ptrs,
                          const int64_t* shapes, int n) {
  if (!ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_load_weights: NULL context");
  if (!names || !dev_ptrs || !shapes || n < 0) return fail(ctx, SPRINTER_E_NULL, "sprinter_load_weights: NULL argument");
  std::vector<Expected>* exp;
  std::unordered_map<std::string, int>* idx;
  const char* who;
  if (which == SPRINTER_DRAFT) { exp = &ctx->draft.expected; idx = &ctx->draft.index; who = "draft"; }
  else if (which == SPRINTER_TARGET) { exp = &ctx->target.expected; idx = &ctx->target.index; who = "target"; }
  else if (which == SPRINTER_VERIFIER) { exp = &ctx->v_expected; idx = &ctx->v_index; who = "verifier"; }
  else return fail(ctx, SPRINTER_E_WEIGHTS, "unknown model selector %d", which);
  // validate everything before touching the device
  std::vector<int> hit(n, -1);
  std::vector<char> seen(exp->size(), 0);
  for (int i = 0; i < n; ++i) {
    if (!names[i] || !dev_ptrs[i]) return fail(ctx, SPRINTER_E_NULL, "%s tensor %d: NULL name or pointer", who, i);
    auto it = idx->find(names[i]);
    if (it == idx->end()) return fail(ctx, SPRINTER_E_WEIGHTS, "%s: unknown tensor name '%s'", who, names[i]);
    const Expected& e = (*exp)[it->second];
    const int64_t* sh = shapes + 4 * i;
    if (sh[0] != e.rows || sh[1] != e.cols || sh[2] != 0 || sh[3] != 0)
      return fail(ctx, SPRINTER_E_WEIGHTS, "%s: tensor '%s' has shape [%lld,%lld,%lld,%lld], expected [%lld,%lld]", who,
                  names[i], (long long)sh[0], (long long)sh[1], (long long)sh[2], (long long)sh[3], (long long)e.rows,
                  (long long)e.cols);
    if (((uintptr_t)dev_ptrs[i]) & 15)   // the kernels read borrowed tensors with 16-byte loads
      return fail(ctx, SPRINTER_E_WEIGHTS, "%s: tensor '%s' is not 16-byte aligned", who, names[i]);
    if (seen[it->second]) return fail(ctx, SPRINTER_E_WEIGHTS, "%s: tensor '%s' given twice", who, names[i]);
    seen[it->second] = 1;
    hit[i] = it->second;
  }
  for (size_t j = 0; j < exp->size(); ++j)
    if (!seen[j]) return fail(ctx, SPRINTER_E_WEIGHTS, "%s: tensor '%s' is missing", who, (*exp)[j].name.c_str());
  for (int i = 0; i < n; ++i) {
    Expected& e = (*exp)[hit[i]];
    if (e.pack) {
      launch_pack_bf16(dev_ptrs[i], e.packed, (int)e.rows, (int)e.cols, ctx->stream);
      *e.slot = e.packed;
    } else {
      *e.slot = dev_ptrs[i];
    }
    if (e.slot2) {   // tied LM head
      if (e.packed2) {
        launch_pack_bf16(dev_ptrs[i], e.packed2, (int)e.rows, (int)e.cols, ctx->stream);
        *e.slot2 = e.packed2;
      } else {
        *e.slot2 = dev_ptrs[i];
      }
    }
    e.seen = true;
  }
  if (which == SPRINTER_DRAFT) ctx->draft.loaded = true;
  else if (which == SPRINTER_TARGET) ctx->target.loaded = true;
  else ctx->v_loaded = true;
  return hip_status(ctx, "sprinter_load_weights");
}

int sprinter_prefill(sprinter_ctx* ctx, const int32_t* dev_prompt, const int32_t* host_prompt_len, int B,
                     int max_prompt) {
  if (!ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_prefill: NULL context");
  if (!dev_prompt || !host_prompt_len) return fail(ctx, SPRINTER_E_NULL, "sprinter_prefill: NULL argument");
  int rc = check_ready(ctx);
  if (rc) return rc;
  if (B < 1 || B > ctx->cfg.max_batch) return fail(ctx, SPRINTER_E_RANGE, "batch %d outside [1, %d]", B, ctx->cfg.max_batch);
  if (max_prompt < 1 || max_prompt > ctx->cfg.max_seq)
    return fail(ctx, SPRINTER_E_RANGE, "max_prompt %d outside [1, max_seq %d]", max_prompt, ctx->cfg.max_seq);
  int pmax = 0;
  for (int b = 0; b < B; ++b) {
    int P = host_prompt_len[b];
    if (P < 1 || P > max_prompt) return fail(ctx, SPRINTER_E_RANGE, "prompt length %d of row %d outside [1, %d]", P, b, max_prompt);
    if (P > pmax) pmax = P;
  }
  hipStream_t s = ctx->stream;
  if (hipMemcpyAsync(ctx->st.prompt_len, host_prompt_len, (size_t)B * 4, hipMemcpyHostToDevice, s) != hipSuccess)
    return fail(ctx, SPRINTER_E_HIP, "copy of prompt lengths failed");
  ctx->B = B;
  ctx->max_prompt_len = pmax;
  ctx->steps_done = 0;
  ctx->run_kind = 0; ctx->sd_wait_ticket = 0;
  Model &dq = ctx->draft, &tp = ctx->target;
  {
    // Chunked prefill: all (row, position) pairs, row-major, go through both models rows_alloc at a time with the
    // kernels of the multi-entry target pass (every layer appends the chunk's keys / values, then attends), so the
    // weights are streamed once per rows_alloc prompt tokens instead of once per position of the batch
    // (bf16: 4096 tokens per pass through the matrix-core kernels; float32: 16 unless cfg.chunk_rows says otherwise).
    std::vector<int> off((size_t)B + 1, 0);
    for (int b = 0; b < B; ++b) off[b + 1] = off[b] + host_prompt_len[b] - 1;
    const long long E = off[B];
    if (hipMemcpyAsync(ctx->ent_off, off.data(), ((size_t)B + 1) * 4, hipMemcpyHostToDevice, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)                  // (off is a local: the copy must be over before it goes)
      return fail(ctx, SPRINTER_E_HIP, "copy of the prefill work list failed");
    launch_prefill_begin(dev_prompt, max_prompt, B, ctx->st, ctx->rej_idx, ctx->n_rej, s);
    CatchupArgs ca;
    ca.st = ctx->st; ca.rej_idx = ctx->rej_idx; ca.n_rej = ctx->n_rej; ca.ent_off = ctx->ent_off;
    ca.t_n_rows = tp.rd_n; ca.t_b = tp.rd_b; ca.t_tok = tp.rd_tok; ca.t_pos = tp.rd_pos; ca.t_slot = tp.rd_slot;
    ca.t_last = ctx->t_last;
    int chunk = 0;
    for (long long start = 0; start < E; start += ctx->rows_alloc, ++chunk) {
      const int n = (int)std::min<long long>(ctx->rows_alloc, E - start);
      ca.start = (int)start; ca.n = n;
      launch_catchup_chunk(ca, s);
      forward(ctx, dq, tp.rd(), n, false, 0u, nullptr, true, true);
      forward(ctx, tp, tp.rd(), n, false, 1u, nullptr, true, true);
      // bound the number of launches in flight (tools that keep per-dispatch state have died on long backlogs)
      if ((chunk & 3) == 3 && hipStreamSynchronize(s) != hipSuccess) return fail(ctx, SPRINTER_E_HIP, "stream synchronisation failed");
    }
  }
  launch_prefill_finish(dev_prompt, max_prompt, B, ctx->st, dq.rd_n, dq.rd_b, dq.rd_tok, dq.rd_pos, dq.rd_slot, s);
  launch_set_i32(ctx->coin_kept, 0, s);
  ctx->prefilled = true;
  return hip_status(ctx, "sprinter_prefill");
}

int sprinter_step(sprinter_ctx* ctx, const sprinter_step_out* out) {
  if (!ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_step: NULL context");
  int rc = check_ready(ctx);
  if (rc) return rc;
  rc = check_room(ctx, 1);
  if (rc) return rc;
  if (ctx->run_kind == 2) return fail(ctx, SPRINTER_E_STATE, "speculative-decoding rounds were run since the last prefill");
  ctx->run_kind = 1;
  if (ctx->cfg.target_ctx_mode == 1 && out && (out->target_logits || out->target_hidden))
    return fail(ctx, SPRINTER_E_CONFIG, "target_logits / target_hidden are not produced with the full-prefix target context");
  rc = enqueue_step(ctx, out, 0, nullptr, nullptr, nullptr, nullptr);
  if (rc) return rc;
  ctx->steps_done += 1;
  return hip_status(ctx, "sprinter_step");
}

int sprinter_generate(sprinter_ctx* ctx, int n_tokens, int32_t* dev_out_tok, uint8_t* dev_out_accept,
                      float* dev_out_score, int32_t* dev_out_draft_tok) {
  if (!ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_generate: NULL context");
  if (n_tokens < 0) return fail(ctx, SPRINTER_E_RANGE, "n_tokens %d < 0", n_tokens);
  int rc = check_ready(ctx);
  if (rc) return rc;
  rc = check_room(ctx, n_tokens);
  if (rc) return rc;
  if (ctx->run_kind == 2) return fail(ctx, SPRINTER_E_STATE, "speculative-decoding rounds were run since the last prefill");
  if (n_tokens > 0) ctx->run_kind = 1;
  launch_reset_gen_idx(ctx->st.counters, ctx->stream);
  for (int g = 0; g < n_tokens; ++g) {
    rc = enqueue_step(ctx, nullptr, n_tokens, dev_out_tok, dev_out_accept, dev_out_score, dev_out_draft_tok);
    if (rc) return rc;
    ctx->steps_done += 1;
  }
  return hip_status(ctx, "sprinter_generate");
}

int sprinter_sd_generate(sprinter_ctx* ctx, int gamma, int n_rounds, int32_t* dev_out_tok, int tok_stride,
                         int32_t* dev_out_n_tok, int32_t* dev_out_n_acc, int32_t* dev_out_draft) {
  if (!ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_sd_generate: NULL context");
  int rc = check_ready(ctx);
  if (rc) return rc;
  if (!ctx->prefilled) return fail(ctx, SPRINTER_E_STATE, "no prefill has been done");
  if (ctx->cfg.sd_gamma <= 0) return fail(ctx, SPRINTER_E_CONFIG, "the context was created with sd_gamma = 0");
  if (gamma < 1 || gamma > ctx->cfg.sd_gamma)
    return fail(ctx, SPRINTER_E_RANGE, "gamma %d outside [1, sd_gamma = %d]", gamma, ctx->cfg.sd_gamma);
  if (!(ctx->cfg.temperature > 0.f)) return fail(ctx, SPRINTER_E_CONFIG, "speculative decoding needs a temperature > 0");
  if (n_rounds < 0) return fail(ctx, SPRINTER_E_RANGE, "n_rounds %d < 0", n_rounds);
  if (dev_out_tok && tok_stride < n_rounds * (gamma + 1))
    return fail(ctx, SPRINTER_E_RANGE, "tok_stride %d < n_rounds * (gamma + 1) = %d", tok_stride, n_rounds * (gamma + 1));
  if (ctx->run_kind == 1) return fail(ctx, SPRINTER_E_STATE, "decode steps were run since the last prefill");
  if ((long long)ctx->max_prompt_len - 1 + ctx->steps_done + (long long)n_rounds * (gamma + 1) > ctx->cfg.max_seq)
    return fail(ctx, SPRINTER_E_RANGE, "prompt length %d + %lld tokens so far + %d rounds of up to %d exceeds max_seq %d",
                ctx->max_prompt_len, ctx->steps_done, n_rounds, gamma + 1, ctx->cfg.max_seq);
  hipStream_t s = ctx->stream;
  const int B = ctx->B, rows = ctx->rows_alloc;
  Model &dq = ctx->draft, &tp = ctx->target;
  const size_t Vd = dq.md.V, Vt = tp.md.V;
  SdBase sd = ctx->sd;
  sd.B = B; sd.gamma = gamma;
  volatile unsigned long long* word = ctx->host_counts + 2;
  const bool fresh = ctx->run_kind == 0;
  launch_sd_begin(sd, fresh ? 1 : 0, s);       // clears the per-call token counts; fresh: one draft entry per row
  if (fresh) { ctx->sd_next_entries = B; ctx->sd_wait_ticket = 0; }
  if (n_rounds > 0) ctx->run_kind = 2;
  const RowDescW D[2] = {RowDescW{dq.rd_n, dq.rd_b, dq.rd_tok, dq.rd_pos, dq.rd_slot}, ctx->sd_rd2};
  const RowDescW T{tp.rd_n, tp.rd_b, tp.rd_tok, tp.rd_pos, tp.rd_slot};
  auto ro = [](const RowDescW& w) { return RowDesc{w.n_rows, w.b, w.tok, w.pos, w.slot}; };
  for (int r = 0; r < n_rounds; ++r) {
    // entries of the first draft pass: the previous round's finish kernel reports them (B plus the rows whose
    // window was kept whole)
    if (ctx->sd_wait_ticket) {
      int e0 = -1;
      rc = wait_ticket(ctx, word, ctx->sd_wait_ticket, &e0, "the previous round did not report its draft entries");
      if (rc) return rc;
      ctx->sd_wait_ticket = 0;
      ctx->sd_next_entries = e0;
    }
    const int E0 = ctx->sd_next_entries;
    if (E0 < B || E0 > 2 * B) return fail(ctx, SPRINTER_E_HIP, "device reported %d draft entries for %d rows", E0, B);
    ctx->steps_done += gamma + 1;
    // 1. gamma draft passes; the first may carry two entries for some rows (in list order, so that the second
    //    finds the first one cached)
    for (int start = 0; start < E0; start += rows) {
      const int n = std::min(rows, E0 - start);
      launch_sd_take_chunk(sd, start, n, D[0], ctx->t_last, s);
      forward(ctx, dq, ro(D[0]), n, true, 0u, sd.dlw + (size_t)start * Vd, E0 > B);
      launch_sd_draft_next(sd, 0, dq.sc.am_part, dq.sc.n_lm_wg, rows, ro(D[0]), ctx->t_last, start, D[1], n, s);
    }
    for (int j = 1; j < gamma; ++j) {
      const RowDescW &in = D[j & 1], &out = D[(j + 1) & 1];
      const int base = 2 * B + (j - 1) * B;
      forward(ctx, dq, ro(in), B, true, 0u, sd.dlw + (size_t)base * Vd, false);
      launch_sd_draft_next(sd, j, dq.sc.am_part, dq.sc.n_lm_wg, rows, ro(in), nullptr, base, out, B, s);
    }
    // 2. the target over gamma + 1 positions of every row, 3. coin / residual / extra token per entry
    const int E = B * (gamma + 1);
    for (int start = 0; start < E; start += rows) {
      const int n = std::min(rows, E - start);
      launch_sd_target_list(sd, start, n, T, s);
      forward(ctx, tp, tp.rd(), n, true, 1u, sd.tlw + (size_t)start * Vt, true);
      launch_sd_window_check(sd, start, n, tp.sc.am_part, tp.sc.n_lm_wg, rows, s);
    }
    // 4. commit
    SdFinishArgs fa;
    fa.round = r; fa.n_rounds = n_rounds; fa.tok_stride = tok_stride;
    fa.o_tok = dev_out_tok; fa.o_n_tok = dev_out_n_tok; fa.o_n_acc = dev_out_n_acc; fa.o_draft = dev_out_draft;
    fa.host_word = ctx->kernel_word + 2;
    fa.ticket = ++ctx->ticket;
    if (fa.ticket == 0) fa.ticket = ++ctx->ticket;
    launch_sd_round_finish(sd, fa, s);
    ctx->sd_wait_ticket = fa.ticket;
  }
  return hip_status(ctx, "sprinter_sd_generate");
}

int sprinter_set_tau(sprinter_ctx* ctx, float tau) {
  if (!ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_set_tau: NULL context");
  if (!(tau == tau)) return fail(ctx, SPRINTER_E_CONFIG, "tau is NaN");
  ctx->cfg.tau = tau;
  launch_set_f32(ctx->tau_dev, tau, ctx->stream);
  return hip_status(ctx, "sprinter_set_tau");
}

int sprinter_get_stats(sprinter_ctx* ctx, sprinter_stats* host_out, int64_t* host_target_calls) {
  if (!ctx) return fail(nullptr, SPRINTER_E_NULL, "sprinter_get_stats: NULL context");
  if (!host_out) return fail(ctx, SPRINTER_E_NULL, "sprinter_get_stats: NULL argument");
  if (hipStreamSynchronize(ctx->stream) != hipSuccess) return fail(ctx, SPRINTER_E_HIP, "stream synchronisation failed");
  long long c[4] = {0, 0, 0, 0};
  if (ctx->prefilled) {
    if (hipMemcpy(c, ctx->st.counters, sizeof c, hipMemcpyDeviceToHost) != hipSuccess)
      return fail(ctx, SPRINTER_E_HIP, "copy of counters failed");
    if (host_target_calls &&
        hipMemcpy(host_target_calls, ctx->st.n_target_calls, (size_t)ctx->B * 8, hipMemcpyDeviceToHost) != hipSuccess)
      return fail(ctx, SPRINTER_E_HIP, "copy of per-row target calls failed");
  }
  host_out->steps = c[0];
  host_out->steps_with_target = c[1];
  host_out->sum_rejected = c[2];
  host_out->batch = ctx->B;
  host_out->coin_kept = 0;
  if (ctx->prefilled && hipMemcpy(&host_out->coin_kept, ctx->coin_kept, 4, hipMemcpyDeviceToHost) != hipSuccess)
    return fail(ctx, SPRINTER_E_HIP, "copy of the coin counter failed");
  return SPRINTER_OK;
}

void sprinter_destroy(sprinter_ctx* ctx) {
  if (!ctx) return;
  (void)hipStreamSynchronize(ctx->stream);     // a decide kernel still in flight writes into the pinned word
  if (ctx->static_dev >= 0) {
    std::lock_guard<std::mutex> lock(g_static_mu);
    g_static[ctx->static_dev].in_use = false;
  } else if (ctx->host_counts) {
    (void)hipHostFree(ctx->host_counts);
  }
  delete ctx;
}

const char* sprinter_last_error(const sprinter_ctx* ctx) { return ctx ? ctx->err : g_err; }

}  // extern "C"
