// The training-step entry points: encoder forward, masked-LM loss (forward + backward of the
// head), encoder backward; plus the exported building blocks.  Host orchestration only: every
// arithmetic step is a kernel in gemm.hip / attention.hip / rowops.hip.
#include "common.h"
#include <mutex>

namespace {

struct Carver {
  char* base; size_t off;
  explicit Carver(void* p) : base((char*)p), off(0) {}
  void* take(size_t bytes) { void* r = base ? base + off : nullptr; off += align_up(bytes, 256); return r; }
};

struct LayerActs { void *qkv, *ctx, *y1, *x1, *hpre, *h, *y2, *x2; float *lse, *st1, *st2; };
struct Acts {
  void *e_pre, *x0; float* emb_stats;
  std::vector<LayerActs> layer;
  size_t total;
};

Acts carve_acts(const hs_model_cfg& c, int B, int L, void* base) {
  const size_t T = (size_t)B * L, H = c.hidden, F = c.ffn, es = esize(c.compute);
  Carver cv(base);
  Acts a;
  a.e_pre = cv.take(T * H * es); a.x0 = cv.take(T * H * es); a.emb_stats = (float*)cv.take(2 * T * sizeof(float));
  a.layer.resize(c.n_layers);
  for (int i = 0; i < c.n_layers; ++i) {
    LayerActs& l = a.layer[i];
    l.qkv = cv.take(T * 3 * H * es);
    l.lse = (float*)cv.take((size_t)B * c.n_heads * L * sizeof(float));
    l.ctx = cv.take(T * H * es);
    l.y1 = cv.take(T * H * es); l.st1 = (float*)cv.take(2 * T * sizeof(float)); l.x1 = cv.take(T * H * es);
    l.hpre = cv.take(T * F * es); l.h = cv.take(T * F * es);
    l.y2 = cv.take(T * H * es); l.st2 = (float*)cv.take(2 * T * sizeof(float));
    l.x2 = (i + 1 < c.n_layers) ? cv.take(T * H * es) : nullptr;   // the last layer writes hidden_out
  }
  a.total = cv.off;
  return a;
}

int padded_vocab(int V) { return (V + 63) / 64 * 64; }

// scratch for split-K partial sums: room for 8 partial copies of the largest weight-gradient matrix
size_t gemm_scratch_bytes(const hs_model_cfg& c) {
  return std::max<size_t>((size_t)32 << 20, (size_t)8 * c.hidden * std::max(c.ffn, 3 * c.hidden) * sizeof(float));
}

struct HeadWs {
  void *grow, *tpre, *tact, *t, *dlogits, *dt, *dtact, *dtpre, *dg, *ln_part, *cs_part, *cs_part_side, *gemm_ws;
  float *stats, *logits, *row_loss;
  size_t total, gemm_ws_bytes;
};
HeadWs carve_head(const hs_model_cfg& c, int M, void* base) {
  const size_t H = c.hidden, es = esize(c.compute), Vp = padded_vocab(c.vocab), m = (size_t)M;
  Carver cv(base);
  HeadWs w;
  w.grow = cv.take(m * H * es); w.tpre = cv.take(m * H * es); w.tact = cv.take(m * H * es); w.t = cv.take(m * H * es);
  w.stats = (float*)cv.take(2 * m * sizeof(float));
  w.logits = (float*)cv.take(m * Vp * sizeof(float));
  w.dlogits = cv.take(m * Vp * es);
  w.row_loss = (float*)cv.take(m * sizeof(float));
  w.dt = cv.take(m * H * es); w.dtact = cv.take(m * H * es); w.dtpre = cv.take(m * H * es); w.dg = cv.take(m * H * es);
  w.ln_part = cv.take(layernorm_bwd_scratch(M, (int)H));
  w.cs_part = cv.take(colsum_scratch(M, (int)Vp));
  w.cs_part_side = cv.take(colsum_scratch(M, (int)Vp));
  w.gemm_ws_bytes = gemm_scratch_bytes(c);
  w.gemm_ws = cv.take(w.gemm_ws_bytes);
  w.total = cv.off;
  return w;
}

struct BwdWs {
  // dy2, dy1, dh and dqkv exist twice (by layer parity): the weight-gradient GEMMs that read them run
  // on a second stream and may still be in flight while the next layer produces its own
  void *dxa, *dxb, *dy2[2], *dy1[2], *dy2m[2], *dy1m[2], *dh[2], *dqkv[2], *dctx, *ln_part, *ln_part2[2], *ln_part1[2], *cs_part, *emb, *gemm_ws, *gemm_ws_side, *ones;
  float* dvec;
  size_t total, gemm_ws_bytes;
};
BwdWs carve_bwd(const hs_model_cfg& c, int B, int L, void* base) {
  const size_t T = (size_t)B * L, H = c.hidden, F = c.ffn, es = esize(c.compute);
  Carver cv(base);
  BwdWs w;
  w.dxa = cv.take(T * H * es); w.dxb = cv.take(T * H * es); w.dctx = cv.take(T * H * es);
  for (int k = 0; k < 2; ++k) {
    w.dy2[k] = cv.take(T * H * es); w.dy1[k] = cv.take(T * H * es);
    w.dy2m[k] = cv.take(T * H * es); w.dy1m[k] = cv.take(T * H * es);     // masked copies (dropout only)
    w.dh[k] = cv.take(T * F * es); w.dqkv[k] = cv.take(T * 3 * H * es);
  }
  w.dvec = (float*)cv.take((size_t)B * c.n_heads * L * sizeof(float));
  w.ln_part = cv.take(layernorm_bwd_scratch((int)T, (int)H));
  for (int k = 0; k < 2; ++k) {
    w.ln_part2[k] = cv.take(layernorm_bwd_scratch((int)T, (int)H));
    w.ln_part1[k] = cv.take(layernorm_bwd_scratch((int)T, (int)H));
  }
  w.cs_part = cv.take(colsum_scratch((int)T, (int)std::max(F, 3 * H)));
  w.emb = cv.take(embed_bwd_scratch((int)T, (int)H));
  w.gemm_ws_bytes = gemm_scratch_bytes(c);
  w.gemm_ws = cv.take(w.gemm_ws_bytes);
  w.gemm_ws_side = cv.take(w.gemm_ws_bytes);
  w.ones = cv.take(T * 8 * es);          // [T, 8] of 1.0: bias gradients as products with a column of ones
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

bool shape_ok(hs_ctx* ctx, int B, int L, std::string* why) {
  if (B < 0 || L < 1) { *why = "B < 0 or L < 1"; return false; }
  if (L % 8) { *why = "L must be a multiple of 8"; return false; }
  if (L > ctx->cfg.max_pos) { *why = "L exceeds max_pos"; return false; }
  if ((int64_t)B * L > (int64_t)1 << 24) { *why = "B*L too large"; return false; }
  return true;
}

template <class T> const void* wptr(const void* w, int64_t off) { return (const T*)w + off; }
const void* W(const hs_ctx* ctx, const void* w, int64_t off) {
  return ctx->cfg.compute == HS_BF16 ? wptr<bf16>(w, off) : wptr<float>(w, off);
}

GemmArgs gemm_args(int dtype, int ak, int bk, int M, int N, int K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                   int64_t ldc) {
  GemmArgs g{};
  g.dtype = dtype; g.a_kmajor = ak; g.b_kmajor = bk; g.M = M; g.N = N; g.K = K;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.c_f32 = 0; g.beta = 0.f; g.bias = nullptr; g.epi = 0; g.aux = nullptr; g.ldaux = 0; g.C2 = nullptr;
  g.ws = nullptr; g.ws_bytes = 0;
  g.drop = nullptr; g.drop_site = 0;
  return g;
}

#define HS_TRY(expr) do { hs_status st_ = (expr); if (st_ != HS_OK) return st_; } while (0)

}  // namespace

extern "C" {

size_t hs_acts_bytes(const hs_model_cfg* cfg, int32_t B, int32_t L, int32_t M) {
  (void)M;
  if (!hs_cfg_valid(cfg, nullptr) || B < 0 || L < 0) return 0;
  return carve_acts(*cfg, B, L, nullptr).total;
}

size_t hs_workspace_bytes(const hs_model_cfg* cfg, int32_t B, int32_t L, int32_t M) {
  if (!hs_cfg_valid(cfg, nullptr) || B < 0 || L < 0 || M < 0) return 0;
  const size_t a = carve_head(*cfg, M, nullptr).total, b = carve_bwd(*cfg, B, L, nullptr).total;
  return std::max<size_t>(std::max(a, b), 256);
}

hs_status hs_encoder_fwd(hs_ctx* ctx, const void* w, const int32_t* ids, const int32_t* lens, const int32_t* lens_host, int32_t B,
                         int32_t L, void* acts, void* hidden_out, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace; (void)workspace_bytes;
  if (!ctx) return HS_ERR_INVALID_ARG;
  std::string why;
  if (!shape_ok(ctx, B, L, &why)) return hs_fail(ctx, HS_ERR_SHAPE, "hs_encoder_fwd: " + why);
  if (B == 0) return HS_OK;
  if (!w || !ids || !lens || !acts || !hidden_out) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_encoder_fwd: NULL buffer");
  if (lens_host)
    for (int b = 0; b < B; ++b)
      if (lens_host[b] < 1 || lens_host[b] > L) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_encoder_fwd: lens[b] outside [1, L]");
  const hs_model_cfg& c = ctx->cfg;
  const ModelOff& o = ctx->off;
  const int dt = c.compute, H = c.hidden, F = c.ffn, T = B * L;
  hipStream_t s = (hipStream_t)stream;
  Acts a = carve_acts(c, B, L, acts);

  const DropCfg* drop = ctx->drop.thr ? &ctx->drop : nullptr;
  const size_t es = esize(dt);
  // Sequences are independent in the forward pass.  A large batch is run as two halves on two streams (the
  // caller's and the context's second one): one half's launch ramp-ups, epilogues and tails fill with the
  // other half's work.  Every kernel sees a row range of the same buffers, so the results are those of one
  // pass (dropout numbers the elements of the whole batch: each half gets the state with its offset).  Not with
  // per-launch timing.
  // (Measured on 64 x 128 tokens, 12 layers: one part 2.76 ms, two 2.43 ms, three 2.49 ms, four 2.46 ms.)
  const bool split = ctx->prof == nullptr && B >= 2 && T >= 4096;
  const int nparts = split ? 2 : 1;
  if (split) HS_TRY(ensure_side_stream(ctx, 2));
  if (split) {
    HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[0], s));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(ctx->side, ctx->events[0], 0));
  }
  struct Part { int b0, nb; hipStream_t st; };
  Part part[2] = {{0, split ? B / 2 : B, s}, {B / 2, B - B / 2, split ? ctx->side : s}};
  auto rows = [&](const void* p, const Part& pt, size_t width) { return (const void*)((const char*)p + (size_t)pt.b0 * L * width * es); };
  auto rows_w = [&](void* p, const Part& pt, size_t width) { return (void*)((char*)p + (size_t)pt.b0 * L * width * es); };

  // dropout state of a half for tensors of [T, H] elements and for the attention probabilities [B, A, L, L]
  DropCfg drop_rows[2], drop_prob[2];
  for (int k = 0; k < 2; ++k) {
    drop_rows[k] = drop_at(ctx->drop, (uint64_t)part[k].b0 * L * H);
    drop_prob[k] = drop_at(ctx->drop, (uint64_t)part[k].b0 * c.n_heads * L * L);
  }
  for (int k = 0; k < nparts; ++k) {
    const Part& pt = part[k];
    HS_TRY(launch_embed_ln_fwd(ctx, dt, W(ctx, w, o.emb_word), W(ctx, w, o.emb_pos), W(ctx, w, o.emb_ln_g), W(ctx, w, o.emb_ln_b),
                               ids + (size_t)pt.b0 * L, rows_w(a.e_pre, pt, H), rows_w(a.x0, pt, H), a.emb_stats + (size_t)pt.b0 * L, pt.nb, L, H,
                               c.vocab, c.ln_eps, pt.st, &drop_rows[k], T));
  }
  const void* x = a.x0;
  for (int i = 0; i < c.n_layers; ++i) {
    const LayerOff& lo = o.layer[i];
    LayerActs& la = a.layer[i];
    void* x2 = la.x2 ? la.x2 : hidden_out;
    for (int k = 0; k < nparts; ++k) {
      const Part& pt = part[k];
      const int Tp = pt.nb * L;
      hipStream_t st = pt.st;
      // q | k | v = x Wqkv^T + b
      GemmArgs g = gemm_args(dt, 1, 1, Tp, 3 * H, H, rows(x, pt, H), H, W(ctx, w, lo.qkv_w), H, rows_w(la.qkv, pt, 3 * H), 3 * H);
      g.bias = W(ctx, w, lo.qkv_b);
      HS_TRY(launch_gemm(ctx, g, st));
      HS_TRY(launch_attention_fwd(ctx, dt, rows(la.qkv, pt, 3 * H), lens + pt.b0, pt.nb, L, c.n_heads, rows_w(la.ctx, pt, H),
                                  la.lse + (size_t)pt.b0 * c.n_heads * L, st, drop ? &drop_prob[k] : nullptr, site_attention_prob(i)));
      // y1 = x + ctx Wo^T + bo ; x1 = LN(y1)
      g = gemm_args(dt, 1, 1, Tp, H, H, rows(la.ctx, pt, H), H, W(ctx, w, lo.o_w), H, rows_w(la.y1, pt, H), H);
      g.bias = W(ctx, w, lo.o_b); g.epi = 1; g.aux = rows(x, pt, H); g.ldaux = H;
      g.drop = drop ? &drop_rows[k] : nullptr; g.drop_site = site_attention_out(i);
      HS_TRY(launch_gemm(ctx, g, st));
      HS_TRY(launch_layernorm_fwd(ctx, dt, rows(la.y1, pt, H), W(ctx, w, lo.ln1_g), W(ctx, w, lo.ln1_b), rows_w(la.x1, pt, H),
                                  la.st1 + (size_t)pt.b0 * L, Tp, H, c.ln_eps, st, T));
      // hpre = x1 W1^T + b1 ; h = GELU(hpre)
      g = gemm_args(dt, 1, 1, Tp, F, H, rows(la.x1, pt, H), H, W(ctx, w, lo.ffn1_w), H, rows_w(la.hpre, pt, F), F);
      g.bias = W(ctx, w, lo.ffn1_b); g.epi = 2; g.C2 = rows_w(la.h, pt, F);
      HS_TRY(launch_gemm(ctx, g, st));
      // y2 = x1 + h W2^T + b2 ; x2 = LN(y2)
      g = gemm_args(dt, 1, 1, Tp, H, F, rows(la.h, pt, F), F, W(ctx, w, lo.ffn2_w), F, rows_w(la.y2, pt, H), H);
      g.bias = W(ctx, w, lo.ffn2_b); g.epi = 1; g.aux = rows(la.x1, pt, H); g.ldaux = H;
      g.drop = drop ? &drop_rows[k] : nullptr; g.drop_site = site_ffn_out(i);
      HS_TRY(launch_gemm(ctx, g, st));
      HS_TRY(launch_layernorm_fwd(ctx, dt, rows(la.y2, pt, H), W(ctx, w, lo.ln2_g), W(ctx, w, lo.ln2_b), rows_w(x2, pt, H),
                                  la.st2 + (size_t)pt.b0 * L, Tp, H, c.ln_eps, st, T));
    }
    x = x2;
  }
  if (split) {     // the second half is ordered before whatever the caller enqueues next
    HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[1], ctx->side));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, ctx->events[1], 0));
  }
  return HS_OK;
}

hs_status hs_mlm_loss(hs_ctx* ctx, const void* w, const void* hidden, const int32_t* mlm_pos, const int32_t* mlm_label, int32_t M,
                      int32_t B, int32_t L, float* loss_sum, void* d_hidden, float* g, int32_t accumulate, void* workspace,
                      size_t workspace_bytes, void* stream) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  std::string why;
  if (!shape_ok(ctx, B, L, &why)) return hs_fail(ctx, HS_ERR_SHAPE, "hs_mlm_loss: " + why);
  if (M < 0 || (int64_t)M > (int64_t)B * L) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_mlm_loss: M outside [0, B*L]");
  if (!loss_sum || (B > 0 && !d_hidden)) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_mlm_loss: NULL output");
  const hs_model_cfg& c = ctx->cfg;
  const ModelOff& o = ctx->off;
  const int dt = c.compute, H = c.hidden, V = c.vocab, Vp = padded_vocab(V);
  const size_t es = esize(dt);
  hipStream_t s = (hipStream_t)stream;
  if (M > 0) {
    if (!w || !hidden || !mlm_pos || !mlm_label || !g || !workspace) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_mlm_loss: NULL buffer");
    if (workspace_bytes < carve_head(c, M, nullptr).total) return hs_fail(ctx, HS_ERR_WORKSPACE, "hs_mlm_loss: workspace too small");
  }
  HS_TRY(launch_fill_zero(ctx, d_hidden, (size_t)B * L * H * es, s));
  if (M == 0) {
    // defined: loss 0, zero d_hidden, g untouched
    return launch_fill_zero(ctx, loss_sum, sizeof(float), s);
  }
  HeadWs h = carve_head(c, M, workspace);
  const float beta = accumulate ? 1.f : 0.f;
  auto run_gemm = [&](GemmArgs& a) { a.ws = h.gemm_ws; a.ws_bytes = h.gemm_ws_bytes; return launch_gemm(ctx, a, s); };

  HS_TRY(launch_gather_rows(ctx, dt, hidden, mlm_pos, M, H, h.grow, s));
  GemmArgs ga = gemm_args(dt, 1, 1, M, H, H, h.grow, H, W(ctx, w, o.head_t_w), H, h.tpre, H);
  ga.bias = W(ctx, w, o.head_t_b); ga.epi = 2; ga.C2 = h.tact;
  HS_TRY(run_gemm(ga));
  HS_TRY(launch_layernorm_fwd(ctx, dt, h.tact, W(ctx, w, o.head_ln_g), W(ctx, w, o.head_ln_b), h.t, h.stats, M, H, c.ln_eps, s));
  // logits = t E^T + b_dec, fp32, row stride Vp
  ga = gemm_args(dt, 1, 1, M, V, H, h.t, H, W(ctx, w, o.emb_word), H, h.logits, Vp);
  ga.c_f32 = 1; ga.beta = 0.f; ga.bias = W(ctx, w, o.head_dec_b);
  HS_TRY(run_gemm(ga));
  HS_TRY(launch_ce_loss(ctx, dt, h.logits, Vp, mlm_label, M, V, h.dlogits, h.row_loss, loss_sum, s));
  // Decoder bias and the decoder's share of the tied word embedding only consume d logits: beside the chain
  // that goes on to d hidden, on the context's second stream (own partial-sum buffer, no split-K scratch),
  // joined before this call returns work to the caller's stream.
  const bool overlap = ctx->prof == nullptr;
  hipStream_t sd = s;
  if (overlap) {
    HS_TRY(ensure_side_stream(ctx, 2));
    sd = ctx->side;
    HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[0], s));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(sd, ctx->events[0], 0));
  }
  HS_TRY(launch_colsum(ctx, dt, h.dlogits, Vp, M, V, g + o.head_dec_b, beta, h.cs_part_side, sd));
  ga = gemm_args(dt, 0, 0, V, H, M, h.dlogits, Vp, h.t, H, g + o.emb_word, H);
  ga.c_f32 = 1; ga.beta = beta;
  if (overlap) HS_TRY(launch_gemm(ctx, ga, sd)); else HS_TRY(run_gemm(ga));
  if (overlap) HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[1], sd));
  // dt = dlogits E
  ga = gemm_args(dt, 1, 0, M, H, V, h.dlogits, Vp, W(ctx, w, o.emb_word), H, h.dt, H);
  HS_TRY(run_gemm(ga));
  HS_TRY(launch_layernorm_bwd(ctx, dt, h.dt, h.tact, h.stats, W(ctx, w, o.head_ln_g), h.dtact, g + o.head_ln_g, g + o.head_ln_b, nullptr,
                              beta, M, H, h.ln_part, s));
  HS_TRY(launch_gelu_bwd(ctx, dt, h.dtact, h.tpre, h.dtpre, (size_t)M * H, s));
  HS_TRY(launch_colsum(ctx, dt, h.dtpre, H, M, H, g + o.head_t_b, beta, h.cs_part, s));
  ga = gemm_args(dt, 0, 0, H, H, M, h.dtpre, H, h.grow, H, g + o.head_t_w, H);
  ga.c_f32 = 1; ga.beta = beta;
  HS_TRY(run_gemm(ga));
  ga = gemm_args(dt, 1, 0, M, H, H, h.dtpre, H, W(ctx, w, o.head_t_w), H, h.dg, H);
  HS_TRY(run_gemm(ga));
  HS_TRY(launch_scatter_rows(ctx, dt, h.dg, mlm_pos, M, H, d_hidden, s));
  if (overlap) HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, ctx->events[1], 0));
  return HS_OK;
}

hs_status hs_arm_update(hs_ctx* ctx, float* w, float* m, float* v, float* G, void* w_lowp_out, double denom, double lr, double beta1,
                        double beta2, double eps, double weight_decay, int64_t t) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  if (!w || !m || !v || !G) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_arm_update: NULL buffer");
  if (t < 1) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_arm_update: t must be >= 1");
  if (!(denom >= 0.0) || std::isinf(denom)) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_arm_update: denom must be finite and >= 0");
  if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0) || !(eps >= 0.0))
    return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_arm_update: betas must be in [0,1), eps >= 0");
  if (((uintptr_t)w % 16) || ((uintptr_t)m % 16) || ((uintptr_t)v % 16) || ((uintptr_t)G % 16) || ((uintptr_t)w_lowp_out % 8))
    return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_arm_update: buffers must be 16-byte aligned");
  ctx->armed = hs_ctx::Armed{true, w, m, v, G, w_lowp_out, denom, lr, beta1, beta2, eps, weight_decay, t};
  return HS_OK;
}

}  // extern "C"

// normalise + Adam on the parameters [begin, end) of an armed update
hs_status update_slice(hs_ctx* ctx, const hs_ctx::Armed& u, int64_t begin, int64_t end, hipStream_t s) {
  const size_t n = (size_t)(end - begin);
  if (n == 0) return HS_OK;
  hs_status st = hs_grad_accum_normalize(u.G + begin, nullptr, n, 0, u.denom, s);
  if (st != HS_OK) return hs_fail(ctx, st, hs_last_error(nullptr));
  void* wl = u.wl ? (void*)((bf16*)u.wl + begin) : nullptr;
  st = hs_adam_step(u.w + begin, u.m + begin, u.v + begin, u.G + begin, wl, n, u.lr, u.beta1, u.beta2, u.eps, u.wd, u.t, s);
  if (st != HS_OK) return hs_fail(ctx, st, hs_last_error(nullptr));
  return HS_OK;
}

extern "C" {

static hs_status encoder_bwd_impl(hs_ctx* ctx, const hs_ctx::Armed& upd, const void* w, const void* acts, const int32_t* ids,
                                  const int32_t* lens, int32_t B, int32_t L, const void* d_hidden, float* g, int32_t accumulate,
                                  void* workspace, size_t workspace_bytes, void* stream);

hs_status hs_encoder_bwd(hs_ctx* ctx, const void* w, const void* acts, const int32_t* ids, const int32_t* lens, int32_t B, int32_t L,
                         const void* d_hidden, float* g, int32_t accumulate, void* workspace, size_t workspace_bytes, void* stream) {
  if (!ctx) return HS_ERR_INVALID_ARG;
  const hs_ctx::Armed upd = ctx->armed;       // consumed by this call, whatever its outcome
  ctx->armed.on = false;
  if (upd.on && upd.G != g) return hs_fail(ctx, HS_ERR_STATE, "hs_encoder_bwd: an update is armed for another gradient buffer");
  return encoder_bwd_impl(ctx, upd, w, acts, ids, lens, B, L, d_hidden, g, accumulate, workspace, workspace_bytes, stream);
}

static hs_status encoder_bwd_impl(hs_ctx* ctx, const hs_ctx::Armed& upd, const void* w, const void* acts, const int32_t* ids,
                                  const int32_t* lens, int32_t B, int32_t L, const void* d_hidden, float* g, int32_t accumulate,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  std::string why;
  if (!shape_ok(ctx, B, L, &why)) return hs_fail(ctx, HS_ERR_SHAPE, "hs_encoder_bwd: " + why);
  if (B == 0) {      // nothing to back-propagate: an armed update still takes place, on the caller's stream
    if (upd.on) return update_slice(ctx, upd, 0, ctx->off.total, (hipStream_t)stream);
    return HS_OK;
  }
  if (!w || !acts || !ids || !lens || !d_hidden || !g || !workspace) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_encoder_bwd: NULL buffer");
  const hs_model_cfg& c = ctx->cfg;
  const ModelOff& o = ctx->off;
  if (workspace_bytes < carve_bwd(c, B, L, nullptr).total) return hs_fail(ctx, HS_ERR_WORKSPACE, "hs_encoder_bwd: workspace too small");
  const int dt = c.compute, H = c.hidden, F = c.ffn, T = B * L;
  hipStream_t s = (hipStream_t)stream;
  Acts a = carve_acts(c, B, L, const_cast<void*>(acts));
  BwdWs ws = carve_bwd(c, B, L, workspace);
  const float beta = accumulate ? 1.f : 0.f;
  const DropCfg* drop = ctx->drop.thr ? &ctx->drop : nullptr;
  auto run_gemm = [&](GemmArgs& a) { a.ws = ws.gemm_ws; a.ws_bytes = ws.gemm_ws_bytes; return launch_gemm(ctx, a, s); };

  // The weight-gradient GEMMs only consume; they run on a second stream so that their ramp-up and tail
  // overlap the activation-gradient chain.  Per layer: four "operand ready" events (main -> side),
  // one "layer done" event (side -> main, waited on before the operand buffers of that parity are
  // reused two layers later and at the end of the call).  With per-launch timing enabled everything
  // stays on the caller's stream so that the timings do not overlap.
  const bool overlap = ctx->prof == nullptr;
  const int NL = c.n_layers;
  if (overlap) HS_TRY(ensure_side_stream(ctx, (size_t)6 * NL + 5));
  hipStream_t sd = overlap ? ctx->side : s;
  // third stream for an armed optimizer update (events 6 NL .. 6 NL + 2: head ready, embeddings ready, done)
  if (overlap && upd.on && !ctx->upd) HS_HIP_CHECK(ctx, hipStreamCreateWithFlags(&ctx->upd, hipStreamNonBlocking));
  hipStream_t su = (overlap && upd.on) ? ctx->upd : s;
  // the update stream continues after the caller's stream has got here (the caller's stream may be the
  // null stream, so it cannot double as a flag) ...
  auto after_main = [&](hipEvent_t e) -> hs_status {
    if (!overlap) return HS_OK;
    HS_HIP_CHECK(ctx, hipEventRecord(e, s));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(su, e, 0));
    return HS_OK;
  };
  // ... or after an event that has already been recorded on the second stream
  auto after_event = [&](hipEvent_t e) -> hs_status {
    if (!overlap) return HS_OK;
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(su, e, 0));
    return HS_OK;
  };
  if (upd.on) {      // the head's gradients were completed by hs_mlm_loss, earlier on the caller's stream
    HS_TRY(after_main(ctx->events[(size_t)6 * NL]));
    HS_TRY(update_slice(ctx, upd, o.head_t_w, o.total, su));
  }
  auto ev = [&](int layer, int k) { return ctx->events[(size_t)layer * 6 + k]; };
  auto hand_over = [&](int layer, int k) -> hs_status {      // main has produced operand k of this layer
    if (!overlap) return HS_OK;
    HS_HIP_CHECK(ctx, hipEventRecord(ev(layer, k), s));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(sd, ev(layer, k), 0));
    return HS_OK;
  };
  auto side_gemm = [&](GemmArgs& a) { a.ws = ws.gemm_ws_side; a.ws_bytes = ws.gemm_ws_bytes; a.c_f32 = 1; a.beta = beta; return launch_gemm(ctx, a, sd); };

  // bf16: the weight gradients of a layer go out as one grouped launch once the layer's last operand (d qkv) exists
  const bool grouped = dt == HS_BF16;
  if (grouped) HS_TRY(launch_fill_value(ctx, dt, ws.ones, (size_t)T * 8, 1.0f, s));
  // The sort of the token ids that the embedding gradient needs depends on nothing computed here: on the second
  // stream, ahead of everything else (events 6 NL + 3: the caller's stream has got here, 6 NL + 4: sorted).
  if (overlap) {
    HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[(size_t)6 * NL + 3], s));
    HS_HIP_CHECK(ctx, hipStreamWaitEvent(sd, ctx->events[(size_t)6 * NL + 3], 0));
    HS_TRY(launch_embed_sort(ctx, ids, T, c.vocab, ws.emb, sd));
    HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[(size_t)6 * NL + 4], sd));
  }
  const void* dcur = d_hidden;
  for (int i = NL - 1; i >= 0; --i) {
    const LayerOff& lo = o.layer[i];
    LayerActs& la = a.layer[i];
    const void* x_in = (i == 0) ? a.x0 : a.layer[i - 1].x2;
    const int par = i & 1;
    void *dy2 = ws.dy2[par], *dy1 = ws.dy1[par], *dh = ws.dh[par], *dqkv = ws.dqkv[par];
    // With dropout the gradient that enters the two dropped branches is the masked one; the residual paths
    // keep the unmasked gradient.
    void* dy2b = drop ? ws.dy2m[par] : dy2;
    void* dy1b = drop ? ws.dy1m[par] : dy1;
    if (overlap && i + 2 < NL) HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, ev(i + 2, 4), 0));   // buffers of this parity are free again
    // LN2 backward: dy2 on the main chain; d gain/bias and colsum(dy2) = d b2 from its partials beside it
    HS_TRY(launch_layernorm_bwd_rows(ctx, dt, dcur, la.y2, la.st2, W(ctx, w, lo.ln2_g), dy2, T, H, ws.ln_part2[par], s, drop,
                                     site_ffn_out(i), drop ? 2 : 0, dy2b));
    if (!grouped) {
      HS_TRY(hand_over(i, 0));
      HS_TRY(launch_layernorm_bwd_cols(ctx, ws.ln_part2[par], g + lo.ln2_g, g + lo.ln2_b, g + lo.ffn2_b, beta, T, H, sd));
    }
    // dW2 [H,F] = dy2^T h
    GemmArgs gw2 = gemm_args(dt, 0, 0, H, F, T, dy2b, H, la.h, F, g + lo.ffn2_w, F);
    if (!grouped) HS_TRY(side_gemm(gw2));
    // dhpre [T,F] = (dy2 W2) * GELU'(hpre)
    GemmArgs ga = gemm_args(dt, 1, 0, T, F, H, dy2b, H, W(ctx, w, lo.ffn2_w), F, dh, F);
    ga.epi = 3; ga.aux = la.hpre; ga.ldaux = F;
    HS_TRY(run_gemm(ga));
    if (!grouped) {
      HS_TRY(hand_over(i, 1));
      HS_TRY(launch_colsum(ctx, dt, dh, F, T, F, g + lo.ffn1_b, beta, ws.cs_part, sd));
    }
    // dW1 [F,H] = dhpre^T x1
    GemmArgs gw1 = gemm_args(dt, 0, 0, F, H, T, dh, F, la.x1, H, g + lo.ffn1_w, H);
    if (!grouped) HS_TRY(side_gemm(gw1));
    // dx1 [T,H] = dhpre W1 + dy2
    ga = gemm_args(dt, 1, 0, T, H, F, dh, F, W(ctx, w, lo.ffn1_w), H, ws.dxa, H);
    ga.epi = 1; ga.aux = dy2; ga.ldaux = H;
    HS_TRY(run_gemm(ga));
    // LN1 backward: dy1, d gain/bias, colsum(dy1) = d bo
    HS_TRY(launch_layernorm_bwd_rows(ctx, dt, ws.dxa, la.y1, la.st1, W(ctx, w, lo.ln1_g), dy1, T, H, ws.ln_part1[par], s, drop,
                                     site_attention_out(i), drop ? 2 : 0, dy1b));
    if (!grouped) {
      HS_TRY(hand_over(i, 2));
      HS_TRY(launch_layernorm_bwd_cols(ctx, ws.ln_part1[par], g + lo.ln1_g, g + lo.ln1_b, g + lo.o_b, beta, T, H, sd));
    }
    // dWo [H,H] = dy1^T ctx ; dctx = dy1 Wo
    GemmArgs gwo = gemm_args(dt, 0, 0, H, H, T, dy1b, H, la.ctx, H, g + lo.o_w, H);
    if (!grouped) HS_TRY(side_gemm(gwo));
    ga = gemm_args(dt, 1, 0, T, H, H, dy1b, H, W(ctx, w, lo.o_w), H, ws.dctx, H);
    HS_TRY(run_gemm(ga));
    HS_TRY(launch_attention_bwd(ctx, dt, la.qkv, la.ctx, la.lse, ws.dctx, lens, B, L, c.n_heads, dqkv, ws.dvec, s, drop,
                                site_attention_prob(i)));
    HS_TRY(hand_over(i, 3));
    // dWqkv [3H,H] = dqkv^T x_in ; dx_in = dqkv Wqkv + dy1
    GemmArgs gwq = gemm_args(dt, 0, 0, 3 * H, H, T, dqkv, 3 * H, x_in, H, g + lo.qkv_w, H);
    if (!grouped) {
      HS_TRY(launch_colsum(ctx, dt, dqkv, 3 * H, T, 3 * H, g + lo.qkv_b, beta, ws.cs_part, sd));
      HS_TRY(side_gemm(gwq));
    } else {
      // Every weight gradient of the layer, and the two bias gradients that are not by-products of a LayerNorm
      // backward (as products with a column of ones), in ONE launch on the second stream: 237 tiles of 256 x 128 for
      // 256 CUs at BERT-base size, each over the whole contraction, so no partial sums travel through memory.
      HS_TRY(launch_layernorm_bwd_cols(ctx, ws.ln_part2[par], g + lo.ln2_g, g + lo.ln2_b, g + lo.ffn2_b, beta, T, H, sd));
      HS_TRY(launch_layernorm_bwd_cols(ctx, ws.ln_part1[par], g + lo.ln1_g, g + lo.ln1_b, g + lo.o_b, beta, T, H, sd));
      GemmArgs gb1 = gemm_args(dt, 0, 0, F, 1, T, dh, F, ws.ones, 8, g + lo.ffn1_b, 1);
      GemmArgs gbq = gemm_args(dt, 0, 0, 3 * H, 1, T, dqkv, 3 * H, ws.ones, 8, g + lo.qkv_b, 1);
      GemmArgs group[6] = {gw2, gw1, gwq, gwo, gb1, gbq};
      for (GemmArgs& a : group) { a.c_f32 = 1; a.beta = beta; }
      HS_TRY(launch_gemm_group(ctx, group, 6, sd));
    }
    if (overlap) HS_HIP_CHECK(ctx, hipEventRecord(ev(i, 4), sd));
    ga = gemm_args(dt, 1, 0, T, H, 3 * H, dqkv, 3 * H, W(ctx, w, lo.qkv_w), H, ws.dxb, H);
    ga.epi = 1; ga.aux = dy1; ga.ldaux = H;
    HS_TRY(run_gemm(ga));
    dcur = ws.dxb;
    if (upd.on) {
      // Every gradient of this layer is final once the second stream has got to its "layer done" event, and
      // its weights are no longer read once the main chain has finished the GEMM above.
      HS_TRY(after_event(ev(i, 4)));
      HS_TRY(after_main(ev(i, 5)));
      HS_TRY(update_slice(ctx, upd, lo.qkv_w, i + 1 < NL ? o.layer[i + 1].qkv_w : o.head_t_w, su));
    }
  }
  // embedding LayerNorm, then the two embedding tables
  HS_TRY(launch_layernorm_bwd(ctx, dt, dcur, a.e_pre, a.emb_stats, W(ctx, w, o.emb_ln_g), ws.dxa, g + o.emb_ln_g,
                              g + o.emb_ln_b, nullptr, beta, T, H, ws.ln_part, s, drop, site_embedding(), drop ? 1 : 0, nullptr));
  if (overlap) HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, ctx->events[(size_t)6 * NL + 4], 0));
  HS_TRY(launch_embed_bwd(ctx, dt, ws.dxa, ids, B, L, H, c.vocab, c.max_pos, g + o.emb_word, g + o.emb_pos, beta, ws.emb, s, overlap));
  if (upd.on) {      // the embedding tables and their LayerNorm last
    HS_TRY(after_main(ctx->events[(size_t)6 * NL + 1]));
    HS_TRY(update_slice(ctx, upd, 0, o.layer[0].qkv_w, su));
    if (overlap) {
      HS_HIP_CHECK(ctx, hipEventRecord(ctx->events[(size_t)6 * NL + 2], su));
      HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, ctx->events[(size_t)6 * NL + 2], 0));
    }
  }
  // everything the second stream did is ordered before whatever the caller enqueues next
  if (overlap) HS_HIP_CHECK(ctx, hipStreamWaitEvent(s, ev(0, 4), 0));
  return HS_OK;
}

// ---- building blocks ----------------------------------------------------------------------------
hs_status hs_tune_gemm_variant(int32_t variant) {
  if (variant < -1 || variant >= gemm_variant_count())
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_tune_gemm_variant: variant must be -1 (automatic) or a configuration number");
  gemm_set_variant(variant);
  return HS_OK;
}

hs_status hs_op_gemm(int32_t dtype, int32_t a_kmajor, int32_t b_kmajor, int32_t M, int32_t N, int32_t K, const void* A, int64_t lda,
                     const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_f32, float beta, const void* bias, int32_t epi,
                     const void* aux, int64_t ldaux, void* C2, void* scratch, size_t scratch_bytes, void* stream) {
  if (dtype != HS_FP32 && dtype != HS_BF16) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_gemm: bad dtype");
  if (M < 0 || N < 0 || K < 0) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_gemm: negative size");
  GemmArgs g = gemm_args(dtype, a_kmajor ? 1 : 0, b_kmajor ? 1 : 0, M, N, K, A, lda, B, ldb, C, ldc);
  g.c_f32 = c_f32 ? 1 : 0; g.beta = beta; g.bias = bias; g.epi = epi; g.aux = aux; g.ldaux = ldaux; g.C2 = C2;
  g.ws = scratch; g.ws_bytes = scratch ? scratch_bytes : 0;
  return launch_gemm(nullptr, g, (hipStream_t)stream);
}

static bool ln_shape_ok(int R, int H) { return R >= 0 && H >= 64 && H % 64 == 0 && H <= 1024; }

hs_status hs_op_layernorm_fwd(int32_t dtype, const void* x, const void* gain, const void* bias, void* y, float* stats, int32_t R,
                              int32_t H, float eps, void* stream) {
  if (!ln_shape_ok(R, H)) return hs_fail(nullptr, HS_ERR_SHAPE, "hs_op_layernorm_fwd: H must be a multiple of 64, <= 1024");
  if (R > 0 && (!x || !gain || !bias || !y || !stats)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_layernorm_fwd: NULL buffer");
  return launch_layernorm_fwd(nullptr, dtype, x, gain, bias, y, stats, R, H, eps, (hipStream_t)stream);
}

size_t hs_op_layernorm_bwd_scratch(int32_t R, int32_t H) { return ln_shape_ok(R, H) ? layernorm_bwd_scratch(R, H) : 0; }

hs_status hs_op_layernorm_bwd(int32_t dtype, const void* dy, const void* x, const float* stats, const void* gain, void* dx, float* d_gain,
                              float* d_bias, float* d_colsum, float beta, int32_t R, int32_t H, void* partials, void* stream) {
  if (!ln_shape_ok(R, H)) return hs_fail(nullptr, HS_ERR_SHAPE, "hs_op_layernorm_bwd: H must be a multiple of 64, <= 1024");
  if (R > 0 && (!dy || !x || !stats || !gain || !dx || !partials)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_layernorm_bwd: NULL buffer");
  return launch_layernorm_bwd(nullptr, dtype, dy, x, stats, gain, dx, d_gain, d_bias, d_colsum, beta, R, H, partials, (hipStream_t)stream);
}

// ---- LayerNorm backward for callers that cannot allocate ---------------------------------------------
// Same kernels as hs_op_layernorm_bwd; the per-block partial column sums live in this file-scope array
// instead of a caller buffer.  Each GPU holds its own copy at its own address, resolved once per device.
namespace {
constexpr int kNoAllocMaxRows = 1 << 24, kNoAllocMaxH = 1024;
constexpr size_t kNoAllocFloats = (size_t)768 * 3 * kNoAllocMaxH;      // blocks x 3 x H peaks at 768 blocks of H = 1024 (= 1024 blocks of H = 768)
static __device__ __align__(256) float scratch[kNoAllocFloats];        // 9 MiB per GPU, held until the process ends
constexpr int kMaxDevices = 64;
float* scratch_ptr[kMaxDevices] = {};                                    // device address of `scratch`, per device
std::mutex scratch_mu;
}  // namespace

hs_status hs_op_layernorm_bwd_noalloc(int32_t dtype, const void* dy, const void* x, const float* stats, const void* gain, void* dx,
                                      float* d_gain, float* d_bias, float* d_colsum, float beta, int32_t R, int32_t H, void* stream) {
  if (dtype != HS_FP32 && dtype != HS_BF16) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_layernorm_bwd_noalloc: bad dtype");
  if (!ln_shape_ok(R, H) || H > kNoAllocMaxH || R > kNoAllocMaxRows)
    return hs_fail(nullptr, HS_ERR_SHAPE, "hs_op_layernorm_bwd_noalloc: needs H a multiple of 64 and <= 1024, R <= 2^24 (the built-in scratch is sized for that)");
  if (layernorm_bwd_scratch(R, H) > sizeof(float) * kNoAllocFloats)
    return hs_fail(nullptr, HS_ERR_SHAPE, "hs_op_layernorm_bwd_noalloc: (R, H) needs more than the built-in scratch of 9437184 bytes");
  if (R > 0 && (!dy || !x || !stats || !gain || !dx)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_layernorm_bwd_noalloc: NULL buffer");
  if (R == 0) return HS_OK;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hs_fail(nullptr, HS_ERR_HIP, std::string("hs_op_layernorm_bwd_noalloc: hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return hs_fail(nullptr, HS_ERR_STATE, "hs_op_layernorm_bwd_noalloc: device index out of range");
  float* part = nullptr;
  {
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_ptr[dev]) {
      void* p = nullptr;
      e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return hs_fail(nullptr, HS_ERR_HIP, std::string("hs_op_layernorm_bwd_noalloc: hipGetSymbolAddress: ") + hipGetErrorString(e));
      scratch_ptr[dev] = (float*)p;
    }
    part = scratch_ptr[dev];
  }
  // The row kernel writes every partial that the column kernel reads, so nothing has to start at zero.
  return launch_layernorm_bwd(nullptr, dtype, dy, x, stats, gain, dx, d_gain, d_bias, d_colsum, beta, R, H, part, (hipStream_t)stream);
}

hs_status hs_op_attention_fwd(int32_t dtype, const void* qkv, const int32_t* lens, int32_t B, int32_t L, int32_t A, void* ctx_out,
                              float* lse, void* stream) {
  if (B < 0 || L < 0 || A < 1) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_fwd: bad size");
  if (B > 0 && L > 0 && (!qkv || !lens || !ctx_out || !lse)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_fwd: NULL buffer");
  return launch_attention_fwd(nullptr, dtype, qkv, lens, B, L, A, ctx_out, lse, (hipStream_t)stream);
}

hs_status hs_op_attention_bwd(int32_t dtype, const void* qkv, const void* ctx_in, const float* lse, const void* d_ctx, const int32_t* lens,
                              int32_t B, int32_t L, int32_t A, void* dqkv, float* dvec, void* stream) {
  if (B < 0 || L < 0 || A < 1) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_bwd: bad size");
  if (B > 0 && L > 0 && (!qkv || !ctx_in || !lse || !d_ctx || !lens || !dqkv || !dvec))
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_op_attention_bwd: NULL buffer");
  return launch_attention_bwd(nullptr, dtype, qkv, ctx_in, lse, d_ctx, lens, B, L, A, dqkv, dvec, (hipStream_t)stream);
}

}  // extern "C"
