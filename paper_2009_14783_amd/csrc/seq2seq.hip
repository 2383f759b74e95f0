// Training-step entry points of the translation workload (encoder-decoder Transformer): forward, label-smoothed
// loss with the output projection, backward.  Host orchestration only: every arithmetic step is a kernel in
// gemm.hip / attention*.hip / rowops.hip / seq2seq_ops.hip.  One stream; the optimizer entry points are shared with
// the encoder-only path.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>

#include "common.h"

namespace {

struct Carver {
  char* base; size_t off;
  explicit Carver(void* p) : base((char*)p), off(0) {}
  void* take(size_t bytes) { void* r = base ? base + off : nullptr; off += align_up(bytes, 256); return r; }
};

struct Shape { std::string name; int64_t rows, cols; };

void block_shapes(std::vector<Shape>& s, const std::string& p, int64_t H, int64_t F, bool cross) {
  s.push_back({p + "qkv.w", 3 * H, H}); s.push_back({p + "qkv.b", 1, 3 * H});
  s.push_back({p + "o.w", H, H});       s.push_back({p + "o.b", 1, H});
  s.push_back({p + "ln1.g", 1, H});     s.push_back({p + "ln1.b", 1, H});
  if (cross) {
    s.push_back({p + "cq.w", H, H});       s.push_back({p + "cq.b", 1, H});
    s.push_back({p + "ckv.w", 2 * H, H});  s.push_back({p + "ckv.b", 1, 2 * H});
    s.push_back({p + "co.w", H, H});       s.push_back({p + "co.b", 1, H});
    s.push_back({p + "lnc.g", 1, H});      s.push_back({p + "lnc.b", 1, H});
  }
  s.push_back({p + "ffn1.w", F, H});    s.push_back({p + "ffn1.b", 1, F});
  s.push_back({p + "ffn2.w", H, F});    s.push_back({p + "ffn2.b", 1, H});
  s.push_back({p + "ln2.g", 1, H});     s.push_back({p + "ln2.b", 1, H});
}

std::vector<Shape> s2s_shapes(const hs_s2s_cfg& c) {
  std::vector<Shape> s = {{"emb", c.vocab, c.hidden}};
  for (int i = 0; i < c.n_enc; ++i) block_shapes(s, "enc" + std::to_string(i) + ".", c.hidden, c.ffn, false);
  for (int i = 0; i < c.n_dec; ++i) block_shapes(s, "dec" + std::to_string(i) + ".", c.hidden, c.ffn, true);
  return s;
}

struct BlockOff {
  int64_t qkv_w, qkv_b, o_w, o_b, ln1_g, ln1_b, cq_w, cq_b, ckv_w, ckv_b, co_w, co_b, lnc_g, lnc_b, ffn1_w, ffn1_b, ffn2_w, ffn2_b, ln2_g,
      ln2_b;
};
struct S2SOff { int64_t emb; std::vector<BlockOff> enc, dec; int64_t total; };

S2SOff s2s_offsets(const hs_s2s_cfg& c) {
  const auto shapes = s2s_shapes(c);
  std::vector<int64_t> off(shapes.size() + 1, 0);
  for (size_t i = 0; i < shapes.size(); ++i) off[i + 1] = off[i] + shapes[i].rows * shapes[i].cols;
  size_t k = 0;
  S2SOff o;
  o.emb = off[k++];
  auto block = [&](bool cross) {
    BlockOff b{};
    b.qkv_w = off[k++]; b.qkv_b = off[k++]; b.o_w = off[k++]; b.o_b = off[k++]; b.ln1_g = off[k++]; b.ln1_b = off[k++];
    if (cross) {
      b.cq_w = off[k++]; b.cq_b = off[k++]; b.ckv_w = off[k++]; b.ckv_b = off[k++]; b.co_w = off[k++]; b.co_b = off[k++];
      b.lnc_g = off[k++]; b.lnc_b = off[k++];
    }
    b.ffn1_w = off[k++]; b.ffn1_b = off[k++]; b.ffn2_w = off[k++]; b.ffn2_b = off[k++]; b.ln2_g = off[k++]; b.ln2_b = off[k++];
    return b;
  };
  for (int i = 0; i < c.n_enc; ++i) o.enc.push_back(block(false));
  for (int i = 0; i < c.n_dec; ++i) o.dec.push_back(block(true));
  o.total = off.back();
  return o;
}

hs_model_cfg shared_sizes(const hs_s2s_cfg& c) {
  hs_model_cfg m;
  m.n_layers = c.n_enc; m.hidden = c.hidden; m.n_heads = c.n_heads; m.ffn = c.ffn; m.vocab = c.vocab; m.max_pos = c.max_pos;
  m.ln_eps = c.ln_eps; m.compute = c.compute;
  return m;
}

bool s2s_cfg_valid(const hs_s2s_cfg* c, std::string* why) {
  if (!c) { if (why) *why = "cfg is NULL"; return false; }
  if (c->n_dec < 1) { if (why) *why = "n_dec < 1"; return false; }
  const hs_model_cfg m = shared_sizes(*c);
  return hs_cfg_valid(&m, why);
}

// ---- saved activations ------------------------------------------------------------------------
struct EncActs { void *qkv, *ctx, *y1, *x1, *h, *y2, *x2; float *lse, *st1, *st2; };
struct DecActs { void *qkv, *ctx, *y1s, *y1, *cq, *ckv, *cctx, *ycs, *yc, *h, *y2s, *y2; float *lse, *clse, *st1, *stc, *st2; };
struct Acts { float* pe; void *x0, *t0; std::vector<EncActs> enc; std::vector<DecActs> dec; size_t total; };

Acts carve_acts(const hs_s2s_cfg& c, int B, int Ls, int Lt, void* base) {
  const size_t Ts = (size_t)B * Ls, Tt = (size_t)B * Lt, H = c.hidden, F = c.ffn, es = esize(c.compute), A = c.n_heads;
  Carver cv(base);
  Acts a;
  a.pe = (float*)cv.take((size_t)std::max(Ls, Lt) * H * sizeof(float));
  a.x0 = cv.take(Ts * H * es); a.t0 = cv.take(Tt * H * es);
  a.enc.resize(c.n_enc); a.dec.resize(c.n_dec);
  for (auto& l : a.enc) {
    l.qkv = cv.take(Ts * 3 * H * es); l.lse = (float*)cv.take((size_t)B * A * Ls * sizeof(float)); l.ctx = cv.take(Ts * H * es);
    l.y1 = cv.take(Ts * H * es); l.st1 = (float*)cv.take(2 * Ts * sizeof(float)); l.x1 = cv.take(Ts * H * es);
    l.h = cv.take(Ts * F * es);
    l.y2 = cv.take(Ts * H * es); l.st2 = (float*)cv.take(2 * Ts * sizeof(float)); l.x2 = cv.take(Ts * H * es);
  }
  for (size_t i = 0; i < a.dec.size(); ++i) {
    DecActs& l = a.dec[i];
    l.qkv = cv.take(Tt * 3 * H * es); l.lse = (float*)cv.take((size_t)B * A * Lt * sizeof(float)); l.ctx = cv.take(Tt * H * es);
    l.y1s = cv.take(Tt * H * es); l.st1 = (float*)cv.take(2 * Tt * sizeof(float)); l.y1 = cv.take(Tt * H * es);
    l.cq = cv.take(Tt * H * es); l.ckv = cv.take(Ts * 2 * H * es); l.clse = (float*)cv.take((size_t)B * A * Lt * sizeof(float));
    l.cctx = cv.take(Tt * H * es);
    l.ycs = cv.take(Tt * H * es); l.stc = (float*)cv.take(2 * Tt * sizeof(float)); l.yc = cv.take(Tt * H * es);
    l.h = cv.take(Tt * F * es);
    l.y2s = cv.take(Tt * H * es); l.st2 = (float*)cv.take(2 * Tt * sizeof(float));
    l.y2 = (i + 1 < a.dec.size()) ? cv.take(Tt * H * es) : nullptr;      // the last layer writes dec_out
  }
  a.total = cv.off;
  return a;
}

int padded_vocab(int V) { return (V + 63) / 64 * 64; }
size_t gemm_scratch_bytes(const hs_s2s_cfg& c) {
  return std::max<size_t>((size_t)32 << 20, (size_t)8 * c.hidden * std::max(c.ffn, 3 * c.hidden) * sizeof(float));
}

struct LossWs { float *logits, *row_loss, *row_nll; void *dlogits, *gemm_ws, *xc, *dxc; int32_t* rows; size_t gemm_ws_bytes, total; };
LossWs carve_loss(const hs_s2s_cfg& c, int B, int Lt, void* base) {
  const size_t Tt = (size_t)B * Lt, Vp = padded_vocab(c.vocab), es = esize(c.compute);
  Carver cv(base);
  LossWs w;
  w.logits = (float*)cv.take(Tt * Vp * sizeof(float));
  w.dlogits = cv.take(Tt * Vp * es);
  w.row_loss = (float*)cv.take(Tt * sizeof(float)); w.row_nll = (float*)cv.take(Tt * sizeof(float));
  // compaction of the real target rows: their positions, the gathered decoder outputs and their gradients
  w.rows = (int32_t*)cv.take(Tt * sizeof(int32_t)); w.xc = cv.take(Tt * c.hidden * es); w.dxc = cv.take(Tt * c.hidden * es);
  w.gemm_ws_bytes = gemm_scratch_bytes(c);
  w.gemm_ws = cv.take(w.gemm_ws_bytes);
  w.total = cv.off;
  return w;
}

// Backward workspace.  The buffers that the weight-gradient GEMMs and bias column sums read (they run on a second stream
// beside the chain of activation gradients) exist once per layer and sub-layer, so that the chain never has to wait
// before it overwrites anything; buffers that only the chain touches are shared by all layers.
struct LayerGrads { void *s2, *m2, *sc, *mc, *s1, *m1, *dh, *dcq, *dckv, *dqkv, *p2, *pc, *p1; };   // p*: LayerNorm column partials
struct BwdWs {
  void *da, *db, *dctx, *denc[2], *de_tgt, *de_src, *cs_part, *emb, *gemm_ws_side;
  std::vector<LayerGrads> enc, dec;
  float* dvec;
  size_t gemm_ws_bytes, total;
};
BwdWs carve_bwd(const hs_s2s_cfg& c, int B, int Ls, int Lt, void* base) {
  const size_t Tm = (size_t)B * std::max(Ls, Lt), Ts = (size_t)B * Ls, Tt = (size_t)B * Lt, H = c.hidden, F = c.ffn, es = esize(c.compute);
  Carver cv(base);
  BwdWs w;
  w.da = cv.take(Tm * H * es); w.db = cv.take(Tm * H * es); w.dctx = cv.take(Tm * H * es);
  w.denc[0] = cv.take(Ts * H * es); w.denc[1] = cv.take(Ts * H * es);
  w.de_tgt = cv.take(Tt * H * es); w.de_src = cv.take(Ts * H * es);      // scaled, masked embedding gradients (read on the second stream)
  w.enc.resize(c.n_enc); w.dec.resize(c.n_dec);
  for (auto& l : w.enc) {
    l = LayerGrads{};
    l.s2 = cv.take(Ts * H * es); l.m2 = cv.take(Ts * H * es); l.s1 = cv.take(Ts * H * es); l.m1 = cv.take(Ts * H * es);
    l.dh = cv.take(Ts * F * es); l.dqkv = cv.take(Ts * 3 * H * es);
    l.p2 = cv.take(layernorm_bwd_scratch((int)Ts, (int)H)); l.p1 = cv.take(layernorm_bwd_scratch((int)Ts, (int)H));
  }
  for (auto& l : w.dec) {
    l.s2 = cv.take(Tt * H * es); l.m2 = cv.take(Tt * H * es); l.sc = cv.take(Tt * H * es); l.mc = cv.take(Tt * H * es);
    l.s1 = cv.take(Tt * H * es); l.m1 = cv.take(Tt * H * es);
    l.dh = cv.take(Tt * F * es); l.dcq = cv.take(Tt * H * es); l.dckv = cv.take(Ts * 2 * H * es); l.dqkv = cv.take(Tt * 3 * H * es);
    l.p2 = cv.take(layernorm_bwd_scratch((int)Tt, (int)H)); l.pc = cv.take(layernorm_bwd_scratch((int)Tt, (int)H));
    l.p1 = cv.take(layernorm_bwd_scratch((int)Tt, (int)H));
  }
  w.dvec = (float*)cv.take((size_t)B * c.n_heads * std::max(Ls, Lt) * sizeof(float));
  w.cs_part = cv.take(colsum_scratch((int)Tm, (int)std::max(F, 3 * H)));
  w.emb = cv.take(embed_bwd_scratch((int)Tm, (int)H));
  w.gemm_ws_bytes = gemm_scratch_bytes(c);
  w.gemm_ws_side = cv.take(w.gemm_ws_bytes);      // split-K partial sums of the weight-gradient GEMMs (second stream)
  w.total = cv.off;
  return w;
}

// second stream + ordering events of a context, created on first use
hs_status ensure_side_stream(hs_ctx* ctx, size_t n_events) {
  if (!ctx->side) HS_HIP_CHECK(ctx, hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking));
  while (ctx->events.size() < n_events) {
    hipEvent_t e;
    HS_HIP_CHECK(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
    ctx->events.push_back(e);
  }
  return HS_OK;
}

bool shape_ok(const hs_s2s_cfg& c, int B, int Ls, int Lt, std::string* why) {
  if (B < 0 || Ls < 1 || Lt < 1) { *why = "B < 0 or a length < 1"; return false; }
  if ((Ls % 8) || (Lt % 8)) { *why = "Ls and Lt must be multiples of 8"; return false; }
  if (Ls > c.max_pos || Lt > c.max_pos) { *why = "a length exceeds max_pos"; return false; }
  if ((int64_t)B * std::max(Ls, Lt) > (int64_t)1 << 24) { *why = "B * L too large"; return false; }
  return true;
}

const void* W(int dt, const void* w, int64_t off) { return dt == HS_BF16 ? (const void*)((const bf16*)w + off) : (const void*)((const float*)w + off); }
const void* at(int dt, const void* p, int64_t elems) { return (const char*)p + elems * (int64_t)esize(dt); }
void* at(int dt, void* p, int64_t elems) { return (char*)p + elems * (int64_t)esize(dt); }

GemmArgs gemm_args(int dtype, int ak, int bk, int M, int N, int K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                   int64_t ldc) {
  GemmArgs g{};
  g.dtype = dtype; g.a_kmajor = ak; g.b_kmajor = bk; g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  return g;
}

#define HS_TRY(expr) do { hs_status st_ = (expr); if (st_ != HS_OK) return st_; } while (0)

uint32_t site_src() { return 0; }
uint32_t site_tgt() { return 1; }
uint32_t site_enc(int layer, int which) { return 2 + 2 * (uint32_t)layer + which; }
uint32_t site_dec(const hs_s2s_cfg& c, int layer, int which) { return 2 + 2 * (uint32_t)c.n_enc + 3 * (uint32_t)layer + which; }

// y = x W^T + b
hs_status linear(hs_ctx* ctx, int dt, int T, int N, int K, const void* x, const void* Wm, const void* b, void* y, hipStream_t s) {
  GemmArgs g = gemm_args(dt, 1, 1, T, N, K, x, K, Wm, K, y, N);
  g.bias = b;
  return launch_gemm(ctx, g, s);
}
// sum = res + drop(x W^T + b) ; out = LN(sum)
hs_status linear_res_ln(hs_ctx* ctx, int dt, int T, int H, int K, const void* x, const void* Wm, const void* b, const void* res, void* sum,
                        const void* gain, const void* beta, void* out, float* stats, int stat_ld, float eps, const DropCfg* drop,
                        uint32_t site, hipStream_t s) {
  GemmArgs g = gemm_args(dt, 1, 1, T, H, K, x, K, Wm, K, sum, H);
  g.bias = b; g.epi = 1; g.aux = res; g.ldaux = H; g.drop = drop; g.drop_site = site;
  HS_TRY(launch_gemm(ctx, g, s));
  return launch_layernorm_fwd(ctx, dt, sum, gain, beta, out, stats, T, H, eps, s, stat_ld);
}

}  // namespace

extern "C" {

hs_status hs_s2s_ctx_create(const hs_s2s_cfg* cfg, hs_ctx** out) {
  if (!out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  std::string why;
  if (!s2s_cfg_valid(cfg, &why)) return hs_fail(nullptr, HS_ERR_SHAPE, "hs_s2s_ctx_create: " + why);
  const hs_model_cfg m = shared_sizes(*cfg);
  hs_status st = hs_ctx_create(&m, out);
  if (st != HS_OK) return st;
  (*out)->is_s2s = true;
  (*out)->s2s = *cfg;
  return HS_OK;
}

size_t hs_s2s_param_count(const hs_s2s_cfg* cfg) { return s2s_cfg_valid(cfg, nullptr) ? (size_t)s2s_offsets(*cfg).total : 0; }

hs_status hs_s2s_param_layout(const hs_s2s_cfg* cfg, hs_param_entry* out, int32_t* n) {
  std::string why;
  if (!n) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "n is NULL");
  if (!s2s_cfg_valid(cfg, &why)) return hs_fail(nullptr, HS_ERR_SHAPE, "hs_s2s_param_layout: " + why);
  const auto shapes = s2s_shapes(*cfg);
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

size_t hs_s2s_acts_bytes(const hs_s2s_cfg* cfg, int32_t B, int32_t Ls, int32_t Lt) {
  if (!s2s_cfg_valid(cfg, nullptr) || B < 0 || Ls < 0 || Lt < 0) return 0;
  return std::max<size_t>(carve_acts(*cfg, B, Ls, Lt, nullptr).total, 256);
}

size_t hs_s2s_workspace_bytes(const hs_s2s_cfg* cfg, int32_t B, int32_t Ls, int32_t Lt) {
  if (!s2s_cfg_valid(cfg, nullptr) || B < 0 || Ls < 0 || Lt < 0) return 0;
  return std::max<size_t>(std::max(carve_loss(*cfg, B, Lt, nullptr).total, carve_bwd(*cfg, B, Ls, Lt, nullptr).total), 256);
}

hs_status hs_s2s_fwd(hs_ctx* ctx, const void* w, const int32_t* src, const int32_t* src_lens, const int32_t* tgt_in, const int32_t* tgt_lens,
                     int32_t B, int32_t Ls, int32_t Lt, void* acts, void* dec_out, void* stream) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  if (!ctx->is_s2s) return hs_fail(ctx, HS_ERR_STATE, "hs_s2s_fwd: the context was not made by hs_s2s_ctx_create");
  const hs_s2s_cfg& c = ctx->s2s;
  std::string why;
  if (!shape_ok(c, B, Ls, Lt, &why)) return hs_fail(ctx, HS_ERR_SHAPE, "hs_s2s_fwd: " + why);
  if (B == 0) return HS_OK;
  if (!w || !src || !src_lens || !tgt_in || !tgt_lens || !acts || !dec_out) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_s2s_fwd: NULL buffer");
  const S2SOff o = s2s_offsets(c);
  const int dt = c.compute, H = c.hidden, F = c.ffn, A = c.n_heads, Ts = B * Ls, Tt = B * Lt;
  hipStream_t s = (hipStream_t)stream;
  Acts a = carve_acts(c, B, Ls, Lt, acts);
  const DropCfg* drop = ctx->drop.thr ? &ctx->drop : nullptr;
  const float scale = sqrtf((float)H);
  const int64_t es = (int64_t)esize(dt);

  // Sentence pairs are independent in the forward pass.  A batch of some size runs as two halves on two streams (the
  // caller's and the context's second one) over row ranges of the same buffers: one half's launch ramp-ups and tails
  // fill with the other half's work, and the results are those of one pass (dropout numbers the elements of the whole
  // batch: each half gets the state with its offset).  Not with per-launch timing.
  const bool split = ctx->prof == nullptr && B >= 2 && std::min(Ts, Tt) >= 2048;
  HS_TRY(launch_position_table(ctx, a.pe, std::max(Ls, Lt), H, s));
  if (split) {
    HS_TRY(ensure_side_stream(ctx, 2));
    HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[0], s));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(ctx->side, ctx->events[0], 0));
  }
  struct Part { int b0, nb; hipStream_t st; };
  const Part part[2] = {{0, split ? B / 2 : B, s}, {B / 2, B - B / 2, split ? ctx->side : s}};
  const int nparts = split ? 2 : 1;
  DropCfg drop_src[2], drop_tgt[2];      // dropout state of a half for tensors of [Ts, H] and [Tt, H] elements
  for (int k = 0; k < 2; ++k) {
    drop_src[k] = drop_at(ctx->drop, (uint64_t)part[k].b0 * Ls * H);
    drop_tgt[k] = drop_at(ctx->drop, (uint64_t)part[k].b0 * Lt * H);
  }
  // rows of sequence b0 onwards in a buffer with L positions per sequence and `width` elements per position
  auto src_rows = [&](const void* p, const Part& pt, int64_t width) { return (const void*)((const char*)p + (int64_t)pt.b0 * Ls * width * es); };
  auto tgt_rows = [&](const void* p, const Part& pt, int64_t width) { return (const void*)((const char*)p + (int64_t)pt.b0 * Lt * width * es); };
  auto mut = [](const void* p) { return const_cast<void*>(p); };

  // ---- encoder ----
  for (int k = 0; k < nparts; ++k) {
    const Part& pt = part[k];
    HS_TRY(launch_embed_scale_pos(ctx, dt, W(dt, w, o.emb), src + (size_t)pt.b0 * Ls, a.pe, mut(src_rows(a.x0, pt, H)), pt.nb, Ls, H, c.vocab, scale,
                                  drop ? &drop_src[k] : nullptr, site_src(), pt.st));
  }
  const void* x = a.x0;
  for (int i = 0; i < c.n_enc; ++i) {
    const BlockOff& lo = o.enc[i];
    EncActs& la = a.enc[i];
    for (int k = 0; k < nparts; ++k) {
      const Part& pt = part[k];
      const int T = pt.nb * Ls;
      hipStream_t st = pt.st;
      auto R = [&](const void* p, int64_t width) { return src_rows(p, pt, width); };
      HS_TRY(linear(ctx, dt, T, 3 * H, H, R(x, H), W(dt, w, lo.qkv_w), W(dt, w, lo.qkv_b), mut(R(la.qkv, 3 * H)), st));
      HS_TRY(launch_attention_fwd(ctx, dt, R(la.qkv, 3 * H), src_lens + pt.b0, pt.nb, Ls, A, mut(R(la.ctx, H)), la.lse + (size_t)pt.b0 * A * Ls, st));
      HS_TRY(linear_res_ln(ctx, dt, T, H, H, R(la.ctx, H), W(dt, w, lo.o_w), W(dt, w, lo.o_b), R(x, H), mut(R(la.y1, H)), W(dt, w, lo.ln1_g),
                           W(dt, w, lo.ln1_b), mut(R(la.x1, H)), la.st1 + (size_t)pt.b0 * Ls, Ts, c.ln_eps, drop ? &drop_src[k] : nullptr, site_enc(i, 0), st));
      HS_TRY(linear(ctx, dt, T, F, H, R(la.x1, H), W(dt, w, lo.ffn1_w), W(dt, w, lo.ffn1_b), mut(R(la.h, F)), st));
      HS_TRY(launch_relu(ctx, dt, mut(R(la.h, F)), (size_t)T * F, st));
      HS_TRY(linear_res_ln(ctx, dt, T, H, F, R(la.h, F), W(dt, w, lo.ffn2_w), W(dt, w, lo.ffn2_b), R(la.x1, H), mut(R(la.y2, H)), W(dt, w, lo.ln2_g),
                           W(dt, w, lo.ln2_b), mut(R(la.x2, H)), la.st2 + (size_t)pt.b0 * Ls, Ts, c.ln_eps, drop ? &drop_src[k] : nullptr, site_enc(i, 1), st));
    }
    x = la.x2;
  }
  const void* enc_out = x;

  // ---- decoder ----
  for (int k = 0; k < nparts; ++k) {
    const Part& pt = part[k];
    HS_TRY(launch_embed_scale_pos(ctx, dt, W(dt, w, o.emb), tgt_in + (size_t)pt.b0 * Lt, a.pe, mut(tgt_rows(a.t0, pt, H)), pt.nb, Lt, H, c.vocab,
                                  scale, drop ? &drop_tgt[k] : nullptr, site_tgt(), pt.st));
  }
  const void* y = a.t0;
  for (int i = 0; i < c.n_dec; ++i) {
    const BlockOff& lo = o.dec[i];
    DecActs& la = a.dec[i];
    void* y2 = la.y2 ? la.y2 : dec_out;
    for (int k = 0; k < nparts; ++k) {
      const Part& pt = part[k];
      const int T = pt.nb * Lt, TS = pt.nb * Ls;
      hipStream_t st = pt.st;
      auto R = [&](const void* p, int64_t width) { return tgt_rows(p, pt, width); };
      const int32_t* tl = tgt_lens + pt.b0;
      const int32_t* sl = src_lens + pt.b0;
      HS_TRY(linear(ctx, dt, T, 3 * H, H, R(y, H), W(dt, w, lo.qkv_w), W(dt, w, lo.qkv_b), mut(R(la.qkv, 3 * H)), st));
      const void* qkv = R(la.qkv, 3 * H);
      AttnOperands self{qkv, at(dt, qkv, H), at(dt, qkv, 2 * H), 3 * (int64_t)H, 3 * (int64_t)H, tl, tl, Lt, Lt, A, 1};
      HS_TRY(launch_attention_general_fwd(ctx, dt, self, pt.nb, mut(R(la.ctx, H)), la.lse + (size_t)pt.b0 * A * Lt, st));
      HS_TRY(linear_res_ln(ctx, dt, T, H, H, R(la.ctx, H), W(dt, w, lo.o_w), W(dt, w, lo.o_b), R(y, H), mut(R(la.y1s, H)), W(dt, w, lo.ln1_g),
                           W(dt, w, lo.ln1_b), mut(R(la.y1, H)), la.st1 + (size_t)pt.b0 * Lt, Tt, c.ln_eps, drop ? &drop_tgt[k] : nullptr, site_dec(c, i, 0), st));
      HS_TRY(linear(ctx, dt, T, H, H, R(la.y1, H), W(dt, w, lo.cq_w), W(dt, w, lo.cq_b), mut(R(la.cq, H)), st));
      const void* ckv = src_rows(la.ckv, pt, 2 * H);
      HS_TRY(linear(ctx, dt, TS, 2 * H, H, src_rows(enc_out, pt, H), W(dt, w, lo.ckv_w), W(dt, w, lo.ckv_b), mut(ckv), st));
      AttnOperands cross{R(la.cq, H), ckv, at(dt, ckv, H), (int64_t)H, 2 * (int64_t)H, tl, sl, Lt, Ls, A, 0};
      HS_TRY(launch_attention_general_fwd(ctx, dt, cross, pt.nb, mut(R(la.cctx, H)), la.clse + (size_t)pt.b0 * A * Lt, st));
      HS_TRY(linear_res_ln(ctx, dt, T, H, H, R(la.cctx, H), W(dt, w, lo.co_w), W(dt, w, lo.co_b), R(la.y1, H), mut(R(la.ycs, H)),
                           W(dt, w, lo.lnc_g), W(dt, w, lo.lnc_b), mut(R(la.yc, H)), la.stc + (size_t)pt.b0 * Lt, Tt, c.ln_eps, drop ? &drop_tgt[k] : nullptr,
                           site_dec(c, i, 1), st));
      HS_TRY(linear(ctx, dt, T, F, H, R(la.yc, H), W(dt, w, lo.ffn1_w), W(dt, w, lo.ffn1_b), mut(R(la.h, F)), st));
      HS_TRY(launch_relu(ctx, dt, mut(R(la.h, F)), (size_t)T * F, st));
      HS_TRY(linear_res_ln(ctx, dt, T, H, F, R(la.h, F), W(dt, w, lo.ffn2_w), W(dt, w, lo.ffn2_b), R(la.yc, H), mut(R(la.y2s, H)),
                           W(dt, w, lo.ln2_g), W(dt, w, lo.ln2_b), mut(R(y2, H)), la.st2 + (size_t)pt.b0 * Lt, Tt, c.ln_eps, drop ? &drop_tgt[k] : nullptr,
                           site_dec(c, i, 2), st));
    }
    y = y2;
  }
  if (split) {     // the second half is ordered before whatever the caller enqueues next
    HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[1], ctx->side));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, ctx->events[1], 0));
  }
  return HS_OK;
}

hs_status hs_s2s_loss(hs_ctx* ctx, const void* w, const void* dec_out, const int32_t* tgt_out, const int32_t* tgt_lens,
                      const int32_t* tgt_lens_host, int32_t B, int32_t Lt, double eps, float* loss_sum, float* nll_sum, void* d_dec_out, float* g,
                      int32_t accumulate, void* workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  if (!ctx->is_s2s) return hs_fail(ctx, HS_ERR_STATE, "hs_s2s_loss: the context was not made by hs_s2s_ctx_create");
  const hs_s2s_cfg& c = ctx->s2s;
  std::string why;
  if (!shape_ok(c, B, 8, Lt, &why)) return hs_fail(ctx, HS_ERR_SHAPE, "hs_s2s_loss: " + why);
  if (!(eps >= 0.0 && eps < 1.0)) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_s2s_loss: eps must be in [0, 1)");
  if (!loss_sum) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_s2s_loss: NULL output");
  hipStream_t s = (hipStream_t)stream;
  if (B == 0) {
    HS_TRY(launch_fill_zero(ctx, loss_sum, sizeof(float), s));
    return nll_sum ? launch_fill_zero(ctx, nll_sum, sizeof(float), s) : HS_OK;
  }
  if (!w || !dec_out || !tgt_out || !tgt_lens || !d_dec_out || !g || !workspace) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_s2s_loss: NULL buffer");
  if (workspace_bytes < carve_loss(c, B, Lt, nullptr).total) return hs_fail(ctx, HS_ERR_WORKSPACE, "hs_s2s_loss: workspace too small");
  const S2SOff o = s2s_offsets(c);
  const int dt = c.compute, H = c.hidden, V = c.vocab, Vp = padded_vocab(V), Tt = B * Lt;
  LossWs h = carve_loss(c, B, Lt, workspace);
  // With the lengths known on the host the padding rows are left out of the vocabulary projection: the real rows are
  // gathered, projected and scored, and their gradient rows scattered back into a zeroed d dec_out.
  int M = Tt;
  if (tgt_lens_host) {
    int64_t n_real = 0;
    for (int b = 0; b < B; ++b) {
      if (tgt_lens_host[b] < 1 || tgt_lens_host[b] > Lt) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_s2s_loss: tgt_lens[b] outside [1, Lt]");
      n_real += tgt_lens_host[b];
    }
    M = (int)n_real;
  }
  const bool compact = M < Tt;
  const void* X = dec_out;
  void* dX = d_dec_out;
  const int32_t* rows = nullptr;
  if (compact) {
    HS_TRY(launch_real_rows(ctx, tgt_lens, B, Lt, h.rows, M, s));
    HS_TRY(launch_gather_rows(ctx, dt, dec_out, h.rows, M, H, h.xc, s));
    X = h.xc; dX = h.dxc; rows = h.rows;
  }
  // logits = x E^T, fp32, row stride Vp
  GemmArgs ga = gemm_args(dt, 1, 1, M, V, H, X, H, W(dt, w, o.emb), H, h.logits, Vp);
  ga.c_f32 = 1; ga.ws = h.gemm_ws; ga.ws_bytes = h.gemm_ws_bytes;
  HS_TRY(launch_gemm(ctx, ga, s));
  HS_TRY(launch_smoothed_ce(ctx, dt, h.logits, Vp, tgt_out, tgt_lens, M, Lt, V, (float)eps, h.dlogits, h.row_loss, h.row_nll, loss_sum, nll_sum,
                            rows, s));
  // dE [V,H] (+)= dlogits^T x ; dx = dlogits E
  ga = gemm_args(dt, 0, 0, V, H, M, h.dlogits, Vp, X, H, g + o.emb, H);
  ga.c_f32 = 1; ga.beta = accumulate ? 1.f : 0.f; ga.ws = h.gemm_ws; ga.ws_bytes = h.gemm_ws_bytes;
  HS_TRY(launch_gemm(ctx, ga, s));
  ga = gemm_args(dt, 1, 0, M, H, V, h.dlogits, Vp, W(dt, w, o.emb), H, dX, H);
  ga.ws = h.gemm_ws; ga.ws_bytes = h.gemm_ws_bytes;
  HS_TRY(launch_gemm(ctx, ga, s));
  if (compact) {
    HS_TRY(launch_fill_zero(ctx, d_dec_out, (size_t)Tt * H * esize(dt), s));
    HS_TRY(launch_scatter_rows(ctx, dt, h.dxc, h.rows, M, H, d_dec_out, s));
  }
  return HS_OK;
}

hs_status hs_s2s_bwd(hs_ctx* ctx, const void* w, const void* acts, const int32_t* src, const int32_t* src_lens, const int32_t* tgt_in,
                     const int32_t* tgt_lens, int32_t B, int32_t Ls, int32_t Lt, const void* d_dec_out, float* g, int32_t accumulate,
                     void* workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  const hs_ctx::Armed upd = ctx->armed;       // an update armed with hs_arm_update is consumed by this call, whatever its outcome
  ctx->armed.on = false;
  if (!ctx->is_s2s) return hs_fail(ctx, HS_ERR_STATE, "hs_s2s_bwd: the context was not made by hs_s2s_ctx_create");
  if (upd.on && upd.G != g) return hs_fail(ctx, HS_ERR_STATE, "hs_s2s_bwd: an update is armed for another gradient buffer");
  const hs_s2s_cfg& c = ctx->s2s;
  std::string why;
  if (!shape_ok(c, B, Ls, Lt, &why)) return hs_fail(ctx, HS_ERR_SHAPE, "hs_s2s_bwd: " + why);
  if (B == 0) {      // nothing to back-propagate: an armed update still takes place, on the caller's stream
    if (upd.on) return update_slice(ctx, upd, 0, s2s_offsets(c).total, (hipStream_t)stream);
    return HS_OK;
  }
  if (!w || !acts || !src || !src_lens || !tgt_in || !tgt_lens || !d_dec_out || !g || !workspace)
    return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_s2s_bwd: NULL buffer");
  if (workspace_bytes < carve_bwd(c, B, Ls, Lt, nullptr).total) return hs_fail(ctx, HS_ERR_WORKSPACE, "hs_s2s_bwd: workspace too small");
  const S2SOff o = s2s_offsets(c);
  const int dt = c.compute, H = c.hidden, F = c.ffn, A = c.n_heads, Ts = B * Ls, Tt = B * Lt;
  hipStream_t s = (hipStream_t)stream;
  Acts a = carve_acts(c, B, Ls, Lt, const_cast<void*>(acts));
  BwdWs ws = carve_bwd(c, B, Ls, Lt, workspace);
  const float beta = accumulate ? 1.f : 0.f;
  const DropCfg* drop = ctx->drop.thr ? &ctx->drop : nullptr;
  const float scale = sqrtf((float)H);

  // The weight gradients and bias column sums only consume what the chain of activation gradients produces: they run on
  // the context's second stream, each after the event that marks its operand ready, and the caller's stream waits for
  // them once, at the end.  With per-launch timing enabled everything stays on the caller's stream.
  const bool overlap = ctx->prof == nullptr;
  const size_t n_events = (size_t)6 * c.n_dec + 4 * c.n_enc + 2 + 1 + (upd.on ? (size_t)2 * (c.n_dec + c.n_enc) + 2 : 0);
  if (overlap) HS_TRY(ensure_side_stream(ctx, n_events));
  hipStream_t sd = overlap ? ctx->side : s;
  size_t next_event = 0;
  // An armed optimizer update runs on a third stream: the slice of a layer is normalised and updated as soon as both
  // streams have finished that layer (its gradient is final and its weights are no longer read), the shared embedding last.
  if (overlap && upd.on && !ctx->upd) HS_HIP_CHECK(ctx, hipStreamCreateWithFlags(&ctx->upd, hipStreamNonBlocking));
  hipStream_t su = (overlap && upd.on) ? ctx->upd : s;
  auto update_after_both = [&](int64_t begin, int64_t end) -> hs_status {
    if (!upd.on) return HS_OK;
    if (overlap) {
      hipEvent_t e1 = ctx->events[next_event++], e2 = ctx->events[next_event++];
      HS_HIP_CHECK(ctx, hipEventRecord(e1, sd));
      HS_HIP_CHECK(ctx, hipStreamWaitEvent(su, e1, 0));
      HS_HIP_CHECK(ctx, hipEventRecord(e2, s));
      HS_HIP_CHECK(ctx, hipStreamWaitEvent(su, e2, 0));
    }
    return update_slice(ctx, upd, begin, end, su);
  };
  auto hand_over = [&]() -> hs_status {       // what the caller's stream has produced so far may now be read on the second one
    if (!overlap) return HS_OK;
    hipEvent_t e = ctx->events[next_event++];
    HS_HIP_CHECK(ctx, hipEventRecord(e, s));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(sd, e, 0));
    return HS_OK;
  };
  auto wgrad = [&](int M, int N, int K, const void* dy, int64_t ldd, const void* xin, int64_t ldx, float* dst) {   // dst [M,N] (+)= dy^T x
    GemmArgs ga = gemm_args(dt, 0, 0, M, N, K, dy, ldd, xin, ldx, dst, N);
    // at most four k-splits: these run beside the chain on the second stream, where the round trip of more partial sums
    // through memory costs the chain more than a fuller grid gains (measured: 32 splits 6.78 ms per step, 8: 6.56, 4: 6.48)
    ga.c_f32 = 1; ga.beta = beta; ga.ws = ws.gemm_ws_side;
    ga.ws_bytes = std::min(ws.gemm_ws_bytes, (size_t)4 * M * N * sizeof(float));
    return launch_gemm(ctx, ga, sd);
  };
  auto bias_grad = [&](const void* dy, int T, int N, float* dst) { return launch_colsum(ctx, dt, dy, N, T, N, dst, beta, ws.cs_part, sd); };
  auto dgrad = [&](int T, int N, int K, const void* dy, const void* Wm, void* dx, const void* res) {   // dx [T,N] = dy [T,K] W [K,N] (+ res)
    GemmArgs ga = gemm_args(dt, 1, 0, T, N, K, dy, K, Wm, N, dx, N);
    if (res) { ga.epi = 1; ga.aux = res; ga.ldaux = N; }
    return launch_gemm(ctx, ga, s);      // no split-K scratch: at K = 512 .. 2048 the reduction pass costs more than the idle CUs
                                         // (7.13 -> 6.78 ms per step)
  };
  // LayerNorm backward of a sub-layer: dsum = d(residual sum); the branch takes dsum through the sub-layer's dropout
  // (dmask; dsum itself without dropout).  The rows go on the chain; the column sums of its partials (gain and bias
  // gradients, and the bias gradient of the sub-layer's last linear map = column sums of the branch gradient) on the
  // second stream, which from here on may read what the chain has produced.  Returns the branch gradient.
  auto ln_bwd = [&](int T, const void* dy, const void* sum, const float* stats, int64_t gain, int64_t lnb, int64_t last_bias, uint32_t site,
                    void* dsum, void* dmask, void* partials, const void** branch) -> hs_status {
    *branch = drop ? dmask : dsum;
    HS_TRY(launch_layernorm_bwd_rows(ctx, dt, dy, sum, stats, W(dt, w, gain), dsum, T, H, partials, s, drop, site, drop ? 2 : 0,
                                     drop ? dmask : nullptr));
    HS_TRY(hand_over());
    return launch_layernorm_bwd_cols(ctx, partials, g + gain, g + lnb, g + last_bias, beta, T, H, sd);
  };
  // feed-forward backward: from the branch gradient to d(input of the sub-layer) = dsum + dh W1, written to out
  auto ffn_bwd = [&](int T, const BlockOff& lo, const LayerGrads& lg, const void* branch, const void* xin, const void* h, void* out) -> hs_status {
    HS_TRY(wgrad(H, F, T, branch, H, h, F, g + lo.ffn2_w));
    HS_TRY(dgrad(T, F, H, branch, W(dt, w, lo.ffn2_w), lg.dh, nullptr));
    HS_TRY(launch_relu_bwd(ctx, dt, lg.dh, h, (size_t)T * F, s));
    HS_TRY(hand_over());
    HS_TRY(bias_grad(lg.dh, T, F, g + lo.ffn1_b));
    HS_TRY(wgrad(F, H, T, lg.dh, F, xin, H, g + lo.ffn1_w));
    return dgrad(T, H, F, lg.dh, W(dt, w, lo.ffn1_w), out, lg.s2);
  };

  // ---- decoder ----
  const void* enc_out = a.enc[c.n_enc - 1].x2;
  const void* dcur = d_dec_out;
  int pe = 0;                      // which of the two encoder-gradient buffers holds the running sum
  bool have_denc = false;
  for (int i = c.n_dec - 1; i >= 0; --i) {
    const BlockOff& lo = o.dec[i];
    DecActs& la = a.dec[i];
    const LayerGrads& lg = ws.dec[i];
    const void* y_in = (i == 0) ? a.t0 : a.dec[i - 1].y2;
    const void* br;
    // feed-forward sub-layer
    HS_TRY(ln_bwd(Tt, dcur, la.y2s, la.st2, lo.ln2_g, lo.ln2_b, lo.ffn2_b, site_dec(c, i, 2), lg.s2, lg.m2, lg.p2, &br));
    HS_TRY(ffn_bwd(Tt, lo, lg, br, la.yc, la.h, ws.da));
    // attention over the encoder output
    HS_TRY(ln_bwd(Tt, ws.da, la.ycs, la.stc, lo.lnc_g, lo.lnc_b, lo.co_b, site_dec(c, i, 1), lg.sc, lg.mc, lg.pc, &br));
    HS_TRY(wgrad(H, H, Tt, br, H, la.cctx, H, g + lo.co_w));
    HS_TRY(dgrad(Tt, H, H, br, W(dt, w, lo.co_w), ws.dctx, nullptr));
    AttnOperands cross{la.cq, la.ckv, at(dt, (const void*)la.ckv, H), (int64_t)H, 2 * (int64_t)H, tgt_lens, src_lens, Lt, Ls, A, 0};
    HS_TRY(launch_attention_general_bwd(ctx, dt, cross, B, la.cctx, la.clse, ws.dctx, lg.dcq, H, lg.dckv, at(dt, lg.dckv, H), 2 * (int64_t)H,
                                        ws.dvec, s));
    HS_TRY(hand_over());
    HS_TRY(bias_grad(lg.dckv, Ts, 2 * H, g + lo.ckv_b));
    HS_TRY(wgrad(2 * H, H, Ts, lg.dckv, 2 * H, enc_out, H, g + lo.ckv_w));
    HS_TRY(bias_grad(lg.dcq, Tt, H, g + lo.cq_b));
    HS_TRY(wgrad(H, H, Tt, lg.dcq, H, la.y1, H, g + lo.cq_w));
    HS_TRY(dgrad(Ts, H, 2 * H, lg.dckv, W(dt, w, lo.ckv_w), ws.denc[pe ^ 1], have_denc ? ws.denc[pe] : nullptr));
    pe ^= 1; have_denc = true;
    HS_TRY(dgrad(Tt, H, H, lg.dcq, W(dt, w, lo.cq_w), ws.db, lg.sc));
    // causal self-attention
    HS_TRY(ln_bwd(Tt, ws.db, la.y1s, la.st1, lo.ln1_g, lo.ln1_b, lo.o_b, site_dec(c, i, 0), lg.s1, lg.m1, lg.p1, &br));
    HS_TRY(wgrad(H, H, Tt, br, H, la.ctx, H, g + lo.o_w));
    HS_TRY(dgrad(Tt, H, H, br, W(dt, w, lo.o_w), ws.dctx, nullptr));
    AttnOperands self{la.qkv, at(dt, (const void*)la.qkv, H), at(dt, (const void*)la.qkv, 2 * H), 3 * (int64_t)H, 3 * (int64_t)H, tgt_lens, tgt_lens,
                      Lt, Lt, A, 1};
    HS_TRY(launch_attention_general_bwd(ctx, dt, self, B, la.ctx, la.lse, ws.dctx, lg.dqkv, 3 * (int64_t)H, at(dt, lg.dqkv, H),
                                        at(dt, lg.dqkv, 2 * H), 3 * (int64_t)H, ws.dvec, s));
    HS_TRY(hand_over());
    HS_TRY(bias_grad(lg.dqkv, Tt, 3 * H, g + lo.qkv_b));
    HS_TRY(wgrad(3 * H, H, Tt, lg.dqkv, 3 * H, y_in, H, g + lo.qkv_w));
    HS_TRY(dgrad(Tt, H, 3 * H, lg.dqkv, W(dt, w, lo.qkv_w), ws.da, lg.s1));
    dcur = ws.da;
    HS_TRY(update_after_both(lo.qkv_w, i + 1 < c.n_dec ? o.dec[i + 1].qkv_w : o.total));
  }
  // target embedding: d E[id] += sqrt(H) * (gradient through the embedding dropout).  The scatter (sort of the ids, segment
  // sums) runs on the second stream like the weight gradients; both embedding scatters add into the same slice, in this order.
  HS_TRY(launch_mask_scale(ctx, dt, dcur, ws.de_tgt, (size_t)Tt * H, scale, drop, site_tgt(), s));
  HS_TRY(hand_over());
  HS_TRY(launch_embed_bwd(ctx, dt, ws.de_tgt, tgt_in, B, Lt, H, c.vocab, 0, g + o.emb, nullptr, 0.f, ws.emb, sd));

  // ---- encoder ----
  dcur = ws.denc[pe];
  for (int i = c.n_enc - 1; i >= 0; --i) {
    const BlockOff& lo = o.enc[i];
    EncActs& la = a.enc[i];
    const LayerGrads& lg = ws.enc[i];
    const void* x_in = (i == 0) ? a.x0 : a.enc[i - 1].x2;
    const void* br;
    HS_TRY(ln_bwd(Ts, dcur, la.y2, la.st2, lo.ln2_g, lo.ln2_b, lo.ffn2_b, site_enc(i, 1), lg.s2, lg.m2, lg.p2, &br));
    HS_TRY(ffn_bwd(Ts, lo, lg, br, la.x1, la.h, ws.da));
    HS_TRY(ln_bwd(Ts, ws.da, la.y1, la.st1, lo.ln1_g, lo.ln1_b, lo.o_b, site_enc(i, 0), lg.s1, lg.m1, lg.p1, &br));
    HS_TRY(wgrad(H, H, Ts, br, H, la.ctx, H, g + lo.o_w));
    HS_TRY(dgrad(Ts, H, H, br, W(dt, w, lo.o_w), ws.dctx, nullptr));
    HS_TRY(launch_attention_bwd(ctx, dt, la.qkv, la.ctx, la.lse, ws.dctx, src_lens, B, Ls, A, lg.dqkv, ws.dvec, s));
    HS_TRY(hand_over());
    HS_TRY(bias_grad(lg.dqkv, Ts, 3 * H, g + lo.qkv_b));
    HS_TRY(wgrad(3 * H, H, Ts, lg.dqkv, 3 * H, x_in, H, g + lo.qkv_w));
    HS_TRY(dgrad(Ts, H, 3 * H, lg.dqkv, W(dt, w, lo.qkv_w), ws.db, lg.s1));
    dcur = ws.db;
    HS_TRY(update_after_both(lo.qkv_w, i + 1 < c.n_enc ? o.enc[i + 1].qkv_w : o.dec[0].qkv_w));
  }
  HS_TRY(launch_mask_scale(ctx, dt, dcur, ws.de_src, (size_t)Ts * H, scale, drop, site_src(), s));
  HS_TRY(hand_over());
  HS_TRY(launch_embed_bwd(ctx, dt, ws.de_src, src, B, Ls, H, c.vocab, 0, g + o.emb, nullptr, 0.f, ws.emb, sd));
  if (upd.on) {      // the shared embedding: its gradient is complete only now
    if (overlap) {
      hipEvent_t e = ctx->events[next_event++];
      HS_HIP_CHECK(ctx, hipEventRecord(e, sd));
      HS_HIP_CHECK(ctx, hipStreamWaitEvent(su, e, 0));
    }
    HS_TRY(update_slice(ctx, upd, o.emb, o.enc[0].qkv_w, su));
    if (overlap) {
      hipEvent_t e = ctx->events[next_event++];
      HS_HIP_CHECK(ctx, hipEventRecord(e, su));
      HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, e, 0));
    }
  }
  if (overlap) {     // everything the second stream did is ordered before whatever the caller enqueues next
    hipEvent_t e = ctx->events[n_events - 1];
    HS_HIP_CHECK(ctx, hipEventRecord(e, sd));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, e, 0));
  }
  return HS_OK;
}

hs_status hs_op_attention_general_fwd(int32_t dtype, const void* q, int64_t ldq, const void* k, const void* v, int64_t ldkv,
                                      const int32_t* qlens, const int32_t* klens, int32_t B, int32_t Lq, int32_t Lk, int32_t A, int32_t causal,
                                      void* ctx_out, float* lse, void* stream) {
  if (dtype != HS_FP32 && dtype != HS_BF16) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_general_fwd: bad dtype");
  if (B < 0) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_general_fwd: bad size");
  if (B > 0 && (!ctx_out || !lse)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_general_fwd: NULL buffer");
  AttnOperands x{q, k, v, ldq, ldkv, qlens, klens, Lq, Lk, A, causal ? 1 : 0};
  return launch_attention_general_fwd(nullptr, dtype, x, B, ctx_out, lse, (hipStream_t)stream);
}

hs_status hs_op_attention_general_bwd(int32_t dtype, const void* q, int64_t ldq, const void* k, const void* v, int64_t ldkv,
                                      const int32_t* qlens, const int32_t* klens, int32_t B, int32_t Lq, int32_t Lk, int32_t A, int32_t causal,
                                      const void* ctx_in, const float* lse, const void* d_ctx, void* dq, int64_t lddq, void* dk, void* dv,
                                      int64_t lddkv, float* dvec, void* stream) {
  if (dtype != HS_FP32 && dtype != HS_BF16) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_general_bwd: bad dtype");
  if (B < 0) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_general_bwd: bad size");
  AttnOperands x{q, k, v, ldq, ldkv, qlens, klens, Lq, Lk, A, causal ? 1 : 0};
  return launch_attention_general_bwd(nullptr, dtype, x, B, ctx_in, lse, d_ctx, dq, lddq, dk, dv, lddkv, dvec, (hipStream_t)stream);
}

}  // extern "C"
