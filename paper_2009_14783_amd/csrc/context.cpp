// Host-side state of libhetseq_hip: configuration checks, the flat parameter layout, the
// optional per-launch timing, and the C++ batch former.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <numeric>

#include "common.h"

static thread_local std::string g_last_error;

hs_status hs_fail(hs_ctx* ctx, hs_status st, const std::string& msg) {
  if (ctx) ctx->err = msg;
  g_last_error = msg;
  return st;
}

bool hs_cfg_valid(const hs_model_cfg* c, std::string* why) {
  auto bad = [&](const char* m) { if (why) *why = m; return false; };
  if (!c) return bad("cfg is NULL");
  if (c->n_layers < 1) return bad("n_layers < 1");
  if (c->hidden < 64 || c->hidden % 64 != 0 || c->hidden > 1024) return bad("hidden must be a multiple of 64 in [64, 1024]");
  if (c->n_heads < 1 || c->hidden != c->n_heads * 64) return bad("hidden / n_heads must be 64");
  if (c->ffn < 64 || c->ffn % 64 != 0) return bad("ffn must be a multiple of 64");
  if (c->vocab < 8) return bad("vocab < 8");
  if (c->max_pos < 8) return bad("max_pos < 8");
  if (!(c->ln_eps >= 0.0f)) return bad("ln_eps < 0");
  if (c->compute != HS_FP32 && c->compute != HS_BF16) return bad("compute must be HS_FP32 or HS_BF16");
  return true;
}

namespace {
struct Shape { std::string name; int64_t rows, cols; };
std::vector<Shape> model_shapes(const hs_model_cfg& c) {
  const int64_t H = c.hidden, F = c.ffn, V = c.vocab;
  std::vector<Shape> s = {{"emb.word", V, H}, {"emb.pos", c.max_pos, H}, {"emb.ln.g", 1, H}, {"emb.ln.b", 1, H}};
  for (int i = 0; i < c.n_layers; ++i) {
    std::string p = "l" + std::to_string(i) + ".";
    s.push_back({p + "qkv.w", 3 * H, H}); s.push_back({p + "qkv.b", 1, 3 * H});
    s.push_back({p + "o.w", H, H});       s.push_back({p + "o.b", 1, H});
    s.push_back({p + "ln1.g", 1, H});     s.push_back({p + "ln1.b", 1, H});
    s.push_back({p + "ffn1.w", F, H});    s.push_back({p + "ffn1.b", 1, F});
    s.push_back({p + "ffn2.w", H, F});    s.push_back({p + "ffn2.b", 1, H});
    s.push_back({p + "ln2.g", 1, H});     s.push_back({p + "ln2.b", 1, H});
  }
  s.push_back({"head.t.w", H, H}); s.push_back({"head.t.b", 1, H});
  s.push_back({"head.ln.g", 1, H}); s.push_back({"head.ln.b", 1, H});
  s.push_back({"head.dec.b", 1, V});
  return s;
}
}  // namespace

void hs_model_offsets(const hs_model_cfg& c, ModelOff* o) {
  auto shapes = model_shapes(c);
  std::vector<int64_t> off(shapes.size() + 1, 0);
  for (size_t i = 0; i < shapes.size(); ++i) off[i + 1] = off[i] + shapes[i].rows * shapes[i].cols;
  size_t k = 0;
  o->emb_word = off[k++]; o->emb_pos = off[k++]; o->emb_ln_g = off[k++]; o->emb_ln_b = off[k++];
  o->layer.resize(c.n_layers);
  for (int i = 0; i < c.n_layers; ++i) {
    LayerOff& l = o->layer[i];
    l.qkv_w = off[k++]; l.qkv_b = off[k++]; l.o_w = off[k++]; l.o_b = off[k++]; l.ln1_g = off[k++]; l.ln1_b = off[k++];
    l.ffn1_w = off[k++]; l.ffn1_b = off[k++]; l.ffn2_w = off[k++]; l.ffn2_b = off[k++]; l.ln2_g = off[k++]; l.ln2_b = off[k++];
  }
  o->head_t_w = off[k++]; o->head_t_b = off[k++]; o->head_ln_g = off[k++]; o->head_ln_b = off[k++]; o->head_dec_b = off[k++];
  o->total = off.back();
}

// ---- per-launch timing ---------------------------------------------------------------------
struct Profiler {
  static const int kMaxSlots = 8192;
  std::vector<hipEvent_t> start, stop;
  std::vector<int> kclass;
  std::vector<double> flops, bytes;
  int used = 0;
  int64_t dropped = 0;
  bool ok = true;
  Profiler() {
    start.resize(kMaxSlots); stop.resize(kMaxSlots); kclass.resize(kMaxSlots); flops.resize(kMaxSlots); bytes.resize(kMaxSlots);
    for (int i = 0; i < kMaxSlots; ++i) {
      if (hipEventCreate(&start[i]) != hipSuccess || hipEventCreate(&stop[i]) != hipSuccess) { ok = false; break; }
    }
  }
  ~Profiler() {
    for (auto e : start) if (e) (void)hipEventDestroy(e);
    for (auto e : stop) if (e) (void)hipEventDestroy(e);
  }
};

KScope::KScope(Profiler* p, int kc, double fl, double by, hipStream_t s) : prof(p), slot(-1), stream(s) {
  if (!prof) return;
  if (prof->used >= Profiler::kMaxSlots) { prof->dropped++; return; }
  slot = prof->used++;
  prof->kclass[slot] = kc; prof->flops[slot] = fl; prof->bytes[slot] = by;
  (void)hipEventRecord(prof->start[slot], stream);
}
KScope::~KScope() {
  if (prof && slot >= 0) (void)hipEventRecord(prof->stop[slot], stream);
}

static const char* kclass_name(int k) {
  static const char* names[KC_COUNT] = {"gemm_fwd", "gemm_dx", "gemm_dw", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd",
                                        "embed", "colsum", "loss", "elemwise", "accum", "adam"};
  return (k >= 0 && k < KC_COUNT) ? names[k] : "?";
}

extern "C" {

hs_status hs_ctx_create(const hs_model_cfg* cfg, hs_ctx** out) {
  if (!out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  std::string why;
  if (!hs_cfg_valid(cfg, &why)) return hs_fail(nullptr, HS_ERR_SHAPE, "hs_ctx_create: " + why);
  hs_ctx* c = new hs_ctx();
  c->cfg = *cfg;
  hs_model_offsets(*cfg, &c->off);
  c->prof = nullptr;
  c->side = nullptr;
  c->drop = DropCfg{0u, 1.0f, 0u, 0u, 0u};
  c->armed.on = false;
  c->upd = nullptr;
  c->is_s2s = false;
  *out = c;
  return HS_OK;
}

hs_status hs_ctx_destroy(hs_ctx* ctx) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  delete ctx->prof;
  for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  if (ctx->upd) (void)hipStreamDestroy(ctx->upd);
  delete ctx;
  return HS_OK;
}

const char* hs_last_error(const hs_ctx* ctx) { return ctx ? ctx->err.c_str() : g_last_error.c_str(); }

size_t hs_param_count(const hs_model_cfg* cfg) {
  if (!hs_cfg_valid(cfg, nullptr)) return 0;
  ModelOff o;
  hs_model_offsets(*cfg, &o);
  return (size_t)o.total;
}

hs_status hs_param_layout(const hs_model_cfg* cfg, hs_param_entry* out, int32_t* n) {
  std::string why;
  if (!n) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "n is NULL");
  if (!hs_cfg_valid(cfg, &why)) return hs_fail(nullptr, HS_ERR_SHAPE, "hs_param_layout: " + why);
  auto shapes = model_shapes(*cfg);
  if (!out) { *n = (int32_t)shapes.size(); return HS_OK; }
  if (*n < (int32_t)shapes.size()) { *n = (int32_t)shapes.size(); return hs_fail(nullptr, HS_ERR_INVALID_ARG, "layout table too small"); }
  int64_t off = 0;
  for (size_t i = 0; i < shapes.size(); ++i) {
    memset(&out[i], 0, sizeof(out[i]));
    snprintf(out[i].name, sizeof(out[i].name), "%s", shapes[i].name.c_str());
    out[i].offset = off; out[i].rows = (int32_t)shapes[i].rows; out[i].cols = (int32_t)shapes[i].cols;
    off += shapes[i].rows * shapes[i].cols;
  }
  *n = (int32_t)shapes.size();
  return HS_OK;
}

hs_status hs_profile_enable(hs_ctx* ctx, int32_t on) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  if (on && !ctx->prof) {
    ctx->prof = new Profiler();
    if (!ctx->prof->ok) { delete ctx->prof; ctx->prof = nullptr; return hs_fail(ctx, HS_ERR_HIP, "could not create timing events"); }
  } else if (!on && ctx->prof) {
    delete ctx->prof; ctx->prof = nullptr;
  }
  return HS_OK;
}

hs_status hs_profile_read(hs_ctx* ctx, hs_profile_entry* out, int32_t* n) {
  if (!ctx || !out || !n) return HS_ERR_INVALID_ARG;
  if (!ctx->prof) return hs_fail(ctx, HS_ERR_STATE, "timing is not enabled");
  if (*n < KC_COUNT) return hs_fail(ctx, HS_ERR_INVALID_ARG, "need room for all kernel classes");
  Profiler* p = ctx->prof;
  for (int k = 0; k < KC_COUNT; ++k) {
    memset(&out[k], 0, sizeof(out[k]));
    snprintf(out[k].name, sizeof(out[k].name), "%s", kclass_name(k));
  }
  for (int i = 0; i < p->used; ++i) {
    HS_HIP_CHECK(ctx, hipEventSynchronize(p->stop[i]));
    float ms = 0.f;
    HS_HIP_CHECK(ctx, hipEventElapsedTime(&ms, p->start[i], p->stop[i]));
    hs_profile_entry& e = out[p->kclass[i]];
    e.launches++; e.ms += ms; e.flops += p->flops[i]; e.bytes += p->bytes[i];
  }
  p->used = 0; p->dropped = 0;
  *n = KC_COUNT;
  return HS_OK;
}

// ---- batch formation -------------------------------------------------------------------------
hs_status hs_make_batches(const int32_t* lengths, int64_t n, int32_t bucket_width, int64_t max_tokens, int32_t cap_mode,
                          int32_t* seq_index_out, int64_t* batch_offsets_out, int32_t* batch_pad_len_out,
                          int64_t* n_batches_out) {
  if (!n_batches_out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "n_batches_out is NULL");
  *n_batches_out = 0;
  if (n < 0 || bucket_width < 1 || max_tokens < 1 || (cap_mode != 0 && cap_mode != 1))
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_make_batches: bad n, bucket_width, max_tokens or cap_mode");
  if (n > 0 && (!lengths || !seq_index_out || !batch_offsets_out || !batch_pad_len_out))
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_make_batches: NULL array");
  if (n == 0) { if (batch_offsets_out) batch_offsets_out[0] = 0; return HS_OK; }
  auto padded = [&](int64_t len) { return (len + bucket_width - 1) / bucket_width * bucket_width; };
  for (int64_t i = 0; i < n; ++i) {
    if (lengths[i] < 1) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_make_batches: length < 1");
    int64_t cost = cap_mode == 0 ? (int64_t)lengths[i] : padded(lengths[i]);
    if (cost > max_tokens || padded(lengths[i]) > INT32_MAX)
      return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_make_batches: a sequence alone exceeds the cap");
  }
  // order by (length, index): the two packed into one 64-bit key, so a plain sort of scalars does it
  // (millions of lengths sort several times faster than through an indirect comparison)
  if (n > (int64_t)INT32_MAX) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_make_batches: more than 2^31 - 1 sequences");
  std::vector<uint64_t> order((size_t)n);
  for (int64_t i = 0; i < n; ++i) order[(size_t)i] = ((uint64_t)(uint32_t)lengths[i] << 32) | (uint64_t)i;
  std::sort(order.begin(), order.end());
  int64_t nb = 0, count = 0, tokens = 0, pad = 0;
  batch_offsets_out[0] = 0;
  for (int64_t k = 0; k < n; ++k) {
    const int64_t i = (int64_t)(order[(size_t)k] & 0xffffffffull), len = lengths[i], p = padded(len);
    if (count > 0) {
      const int64_t would = cap_mode == 0 ? tokens + len : (count + 1) * p;
      if (p != pad || would > max_tokens) {
        batch_pad_len_out[nb] = (int32_t)pad;
        batch_offsets_out[++nb] = k;
        count = 0; tokens = 0;
      }
    }
    seq_index_out[k] = (int32_t)i;
    ++count; tokens += len; pad = p;
  }
  batch_pad_len_out[nb] = (int32_t)pad;
  batch_offsets_out[++nb] = n;
  *n_batches_out = nb;
  return HS_OK;
}

}  // extern "C"

// ---- learning-rate schedule and checkpoints (host only) ---------------------------------------
#include <cmath>
#include <cstdio>
#include <limits>

extern "C" double hs_lr_linear(int64_t t, double max_lr, int64_t warmup, int64_t total) {
  if (t < 1 || warmup < 0 || total < 1 || total < warmup || !(max_lr >= 0.0) || !std::isfinite(max_lr)) {
    hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_lr_linear: need t >= 1, 0 <= warmup <= total, total >= 1 and a finite max_lr >= 0");
    return std::numeric_limits<double>::quiet_NaN();
  }
  if (t <= warmup) return max_lr * (double)t / (double)warmup;
  if (t >= total) return 0.0;
  return max_lr * (double)(total - t) / (double)(total - warmup);
}

namespace {
const char kCkptMagic[8] = {'H', 'S', 'C', 'K', 'P', 'T', '0', '1'};

struct Fnv {
  uint64_t h = 1469598103934665603ull;
  void add(const void* p, size_t n) {
    const unsigned char* b = (const unsigned char*)p;
    for (size_t i = 0; i < n; ++i) { h ^= b[i]; h *= 1099511628211ull; }
  }
};

struct File {
  FILE* f;
  explicit File(FILE* fp) : f(fp) {}
  ~File() { if (f) fclose(f); }
};

bool header_ok(const hs_ckpt_header& h, std::string* why) {
  if (!hs_cfg_valid(&h.cfg, why)) return false;
  if (h.n_params != (int64_t)hs_param_count(&h.cfg)) { *why = "n_params does not match the model"; return false; }
  if (h.epoch < 0 || h.step < 0) { *why = "negative epoch or step"; return false; }
  return true;
}
}  // namespace

extern "C" hs_status hs_checkpoint_write(const char* path, const hs_ckpt_header* header, const float* w, const float* m, const float* v) {
  if (!path || !header || !w || !m || !v) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_checkpoint_write: NULL argument");
  std::string why;
  if (!header_ok(*header, &why)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_checkpoint_write: " + why);
  const std::string tmp = std::string(path) + ".tmp";
  const size_t bytes = (size_t)header->n_params * sizeof(float);
  Fnv sum;
  bool ok = false;
  {
    File out(fopen(tmp.c_str(), "wb"));
    if (!out.f) return hs_fail(nullptr, HS_ERR_STATE, "hs_checkpoint_write: cannot create " + tmp);
    auto put = [&](const void* p, size_t n) { sum.add(p, n); return fwrite(p, 1, n, out.f) == n; };
    ok = put(kCkptMagic, sizeof(kCkptMagic)) && put(header, sizeof(*header)) && put(w, bytes) && put(m, bytes) && put(v, bytes);
    const uint64_t h = sum.h;
    ok = ok && fwrite(&h, 1, sizeof(h), out.f) == sizeof(h) && fflush(out.f) == 0;
  }
  if (!ok || rename(tmp.c_str(), path) != 0) {
    remove(tmp.c_str());
    return hs_fail(nullptr, HS_ERR_STATE, std::string("hs_checkpoint_write: could not write ") + path);
  }
  return HS_OK;
}

static hs_status read_header(FILE* f, const char* path, hs_ckpt_header* h, Fnv* sum) {
  char magic[8];
  if (fread(magic, 1, 8, f) != 8 || memcmp(magic, kCkptMagic, 8) != 0)
    return hs_fail(nullptr, HS_ERR_STATE, std::string("checkpoint: bad magic in ") + path);
  if (fread(h, 1, sizeof(*h), f) != sizeof(*h)) return hs_fail(nullptr, HS_ERR_STATE, std::string("checkpoint: truncated header in ") + path);
  std::string why;
  if (!header_ok(*h, &why)) return hs_fail(nullptr, HS_ERR_STATE, std::string("checkpoint: ") + why);
  if (sum) { sum->add(magic, 8); sum->add(h, sizeof(*h)); }
  return HS_OK;
}

extern "C" hs_status hs_checkpoint_read_header(const char* path, hs_ckpt_header* header_out) {
  if (!path || !header_out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_checkpoint_read_header: NULL argument");
  File in(fopen(path, "rb"));
  if (!in.f) return hs_fail(nullptr, HS_ERR_STATE, std::string("checkpoint: cannot open ") + path);
  return read_header(in.f, path, header_out, nullptr);
}

extern "C" hs_status hs_checkpoint_read(const char* path, hs_ckpt_header* header_out, float* w, float* m, float* v, size_t n) {
  if (!path || !header_out || !w || !m || !v) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_checkpoint_read: NULL argument");
  File in(fopen(path, "rb"));
  if (!in.f) return hs_fail(nullptr, HS_ERR_STATE, std::string("checkpoint: cannot open ") + path);
  Fnv sum;
  hs_status st = read_header(in.f, path, header_out, &sum);
  if (st != HS_OK) return st;
  if ((int64_t)n != header_out->n_params) return hs_fail(nullptr, HS_ERR_SHAPE, "hs_checkpoint_read: array size does not match the file");
  const size_t bytes = n * sizeof(float);
  float* dst[3] = {w, m, v};
  for (float* d : dst) {
    if (fread(d, 1, bytes, in.f) != bytes) return hs_fail(nullptr, HS_ERR_STATE, std::string("checkpoint: truncated file ") + path);
    sum.add(d, bytes);
  }
  uint64_t stored = 0;
  if (fread(&stored, 1, sizeof(stored), in.f) != sizeof(stored) || stored != sum.h)
    return hs_fail(nullptr, HS_ERR_STATE, std::string("checkpoint: checksum mismatch in ") + path);
  return HS_OK;
}

// ---- dropout state of a context ------------------------------------------------------------------
extern "C" hs_status hs_set_dropout(hs_ctx* ctx, double p, uint64_t seed, uint32_t stream) {
  if (!ctx) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_set_dropout: ctx is NULL");
  if (!(p >= 0.0) || !(p < 1.0)) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_set_dropout: p must be in [0, 1)");
  const double t = std::floor(p * 4294967296.0);
  ctx->drop.thr = (uint32_t)(t > 4294967295.0 ? 4294967295.0 : t);
  ctx->drop.scale = (float)(1.0 / (1.0 - p));
  ctx->drop.k0 = (uint32_t)(seed & 0xffffffffull);
  ctx->drop.k1 = (uint32_t)(seed >> 32);
  ctx->drop.stream = stream;
  ctx->drop.g0 = ctx->drop.g1 = 0;
  return HS_OK;
}
