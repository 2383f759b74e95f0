// Shared device/host helpers of libhetseq_hip (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "hetseq_hip.h"

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define HS_WAVE 64

template <class T> __device__ __forceinline__ float to_f(T x);
template <> __device__ __forceinline__ float to_f<float>(float x) { return x; }
template <> __device__ __forceinline__ float to_f<bf16>(bf16 x) { return (float)x; }
template <class T> __device__ __forceinline__ T from_f(float x);
template <> __device__ __forceinline__ float from_f<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float x) { return (bf16)x; }  // round to nearest even

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

// exact-erf GELU and its derivative
__device__ __forceinline__ float gelu_f(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_f(float x) {
  return 0.5f * (1.0f + erff(x * 0.70710678118654752440f)) + x * 0.39894228040143267794f * __expf(-0.5f * x * x);
}

// Cheaper forms for the bf16 GEMM epilogues: erf by the rational-exponential fit 7.1.26 of Abramowitz &
// Stegun (absolute error below 1.5e-7, far under bf16 resolution).  The Gaussian e^{-x^2/2} it needs is
// the same one GELU' needs, so both cost one exponential and one reciprocal.
__device__ __forceinline__ void normal_cdf_pdf(float x, float& cdf, float& pdf) {
  const float ax = fabsf(x) * 0.70710678118654752440f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  const float e = __expf(-ax * ax);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float erf_abs = fmaf(-poly, e, 1.0f);
  cdf = 0.5f * (1.0f + copysignf(erf_abs, x));
  pdf = 0.39894228040143267794f * e;
}
__device__ __forceinline__ float gelu_fast(float x) { float c, d; normal_cdf_pdf(x, c, d); return x * c; }
__device__ __forceinline__ float gelu_grad_fast(float x) { float c, d; normal_cdf_pdf(x, c, d); return fmaf(x, d, c); }

// ---- dropout with a counter-based generator ---------------------------------------------------
// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel random numbers: as easy as 1, 2, 3",
// SC'11), from its published definition.  Element e of dropout site `site` uses word e % 4 of the block
// with counter (e / 4 low, e / 4 high, site, stream) under the key (seed low, seed high) and is dropped
// when that word is below thr = floor(p * 2^32); survivors are scaled by 1 / (1 - p).  thr == 0: off.
struct DropCfg {
  uint32_t thr;
  float scale;
  uint32_t k0, k1;
  uint32_t stream;
  // Offset, in groups of four elements, added to every element index: a kernel that works on a row range of a
  // tensor (pointers already advanced) still numbers the elements of the whole tensor.
  uint32_t g0, g1;
};
// the same dropout state for a kernel whose pointers start `elems` elements (a multiple of 4) into the tensor
static inline DropCfg drop_at(const DropCfg& d, uint64_t elems) {
  DropCfg r = d;
  const uint64_t g = (((uint64_t)d.g1 << 32) | d.g0) + (elems >> 2);
  r.g0 = (uint32_t)g; r.g1 = (uint32_t)(g >> 32);
  return r;
}
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                              uint32_t (&out)[4]) {
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0; c1 = lo1; c2 = hi0 ^ c3 ^ k1; c3 = lo0;
    k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
// factors (0 or scale) of the four elements 4*group .. 4*group + 3 of a site
__device__ __forceinline__ void drop_factors4(const DropCfg& d, uint32_t site, uint64_t group, float (&f)[4]) {
  uint32_t w[4];
  group += ((uint64_t)d.g1 << 32) | d.g0;
  philox4x32_10((uint32_t)group, (uint32_t)(group >> 32), site, d.stream, d.k0, d.k1, w);
#pragma unroll
  for (int t = 0; t < 4; ++t) f[t] = (w[t] >= d.thr) ? d.scale : 0.0f;
}
// keep bits of the four elements 4*group .. 4*group + 3 of a site (bit t set: element 4*group + t survives)
__device__ __forceinline__ int drop_keep4(const DropCfg& d, uint32_t site, uint64_t group) {
  uint32_t w[4];
  group += ((uint64_t)d.g1 << 32) | d.g0;
  philox4x32_10((uint32_t)group, (uint32_t)(group >> 32), site, d.stream, d.k0, d.k1, w);
  return (w[0] >= d.thr ? 1 : 0) | (w[1] >= d.thr ? 2 : 0) | (w[2] >= d.thr ? 4 : 0) | (w[3] >= d.thr ? 8 : 0);
}
// factor of the single element e
__device__ __forceinline__ float drop_factor1(const DropCfg& d, uint32_t site, uint64_t e) {
  uint32_t w[4];
  const uint64_t group = (e >> 2) + (((uint64_t)d.g1 << 32) | d.g0);
  philox4x32_10((uint32_t)group, (uint32_t)(group >> 32), site, d.stream, d.k0, d.k1, w);
  const uint32_t x = (e & 3) == 0 ? w[0] : ((e & 3) == 1 ? w[1] : ((e & 3) == 2 ? w[2] : w[3]));
  return (x >= d.thr) ? d.scale : 0.0f;
}
// site numbers: the embedding output, then per layer the attention probabilities, the attention
// output and the feed-forward output (the last two before the residual is added)
__host__ __device__ static inline uint32_t site_embedding() { return 0; }
__host__ __device__ static inline uint32_t site_attention_prob(int layer) { return 1 + 3 * (uint32_t)layer; }
__host__ __device__ static inline uint32_t site_attention_out(int layer) { return 2 + 3 * (uint32_t)layer; }
__host__ __device__ static inline uint32_t site_ffn_out(int layer) { return 3 + 3 * (uint32_t)layer; }

// ---- kernel classes for the optional per-launch timing ---------------------------------
enum KClass {
  KC_GEMM_FWD = 0,   // A k-major, B k-major   (y = x W^T)
  KC_GEMM_DX,        // A k-major, B n-major   (dx = dy W)
  KC_GEMM_DW,        // A m-major, B n-major   (dW = dy^T x)
  KC_ATTN_FWD,
  KC_ATTN_BWD,
  KC_LN_FWD,
  KC_LN_BWD,
  KC_EMBED,
  KC_COLSUM,
  KC_LOSS,
  KC_ELEMWISE,
  KC_ACCUM,
  KC_ADAM,
  KC_COUNT
};

struct Profiler;  // host side, see context.cpp

// One timing scope around a launch; no-op when prof is null.
struct KScope {
  Profiler* prof;
  int slot;
  hipStream_t stream;
  KScope(Profiler* p, int kclass, double flops, double bytes, hipStream_t s);
  ~KScope();
};

// ---- host-side model tables --------------------------------------------------------------
struct LayerOff {
  int64_t qkv_w, qkv_b, o_w, o_b, ln1_g, ln1_b, ffn1_w, ffn1_b, ffn2_w, ffn2_b, ln2_g, ln2_b;
};
struct ModelOff {
  int64_t emb_word, emb_pos, emb_ln_g, emb_ln_b;
  std::vector<LayerOff> layer;
  int64_t head_t_w, head_t_b, head_ln_g, head_ln_b, head_dec_b;
  int64_t total;
};
bool hs_cfg_valid(const hs_model_cfg* cfg, std::string* why);
void hs_model_offsets(const hs_model_cfg& cfg, ModelOff* out);

struct hs_ctx {
  hs_model_cfg cfg;
  ModelOff off;
  std::string err;
  Profiler* prof;  // null unless enabled
  // a second stream on which the weight-gradient GEMMs of the backward pass run beside the
  // activation-gradient chain, with the events that order the two (created on first use)
  hipStream_t side;
  std::vector<hipEvent_t> events;
  DropCfg drop;    // dropout of the forward/backward calls on this context (thr == 0: off)
  // an optimizer update armed for the next backward call: each parameter group is normalised and updated
  // on a third stream as soon as its gradient is final
  struct Armed { bool on; float *w, *m, *v, *G; void* wl; double denom, lr, beta1, beta2, eps, wd; int64_t t; } armed;
  hipStream_t upd;
  // translation workload (contexts made by hs_s2s_ctx_create): cfg above holds the shared sizes (n_layers = encoder layers)
  bool is_s2s;
  hs_s2s_cfg s2s;
};

hs_status hs_fail(hs_ctx* ctx, hs_status st, const std::string& msg);  // records msg, returns st
// normalise + Adam on the parameters [begin, end) of an armed update (api.hip)
hs_status update_slice(hs_ctx* ctx, const hs_ctx::Armed& u, int64_t begin, int64_t end, hipStream_t s);
#define HS_HIP_CHECK(ctx, expr)                                                              \
  do {                                                                                       \
    hipError_t e_ = (expr);                                                                  \
    if (e_ != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline size_t esize(int dtype) { return dtype == HS_BF16 ? 2 : 4; }

// ---- internal launchers (each checks nothing; callers validate) ----------------------------
struct GemmArgs {
  int dtype;  // hs_dtype
  int a_kmajor, b_kmajor;
  int M, N, K;
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  void* C; int64_t ldc;
  int c_f32; float beta;
  const void* bias;
  int epi; const void* aux; int64_t ldaux; void* C2;
  void* ws; size_t ws_bytes;   // optional scratch for split-K partial sums
  const DropCfg* drop; uint32_t drop_site;   // optional (epi == 1): dropout of product + bias before the residual
};
hs_status launch_gemm(hs_ctx* ctx, const GemmArgs& g, hipStream_t s);
// up to 8 weight-gradient products (A m-major, B n-major, fp32 C = beta C + product) in one launch; other argument
// sets run one by one
// timing runs: every bf16 product with M, N, K >= 256 that configuration `variant` can serve uses it (-1: automatic choice); process-wide
int gemm_variant_count();
void gemm_set_variant(int variant);
hs_status launch_gemm_group(hs_ctx* ctx, const GemmArgs* gs, int n, hipStream_t s);

// stats: R means, then (stat_ld floats after the first mean; default R) R reciprocal standard deviations
hs_status launch_layernorm_fwd(hs_ctx* ctx, int dtype, const void* x, const void* gain, const void* bias, void* y,
                               float* stats, int R, int H, float eps, hipStream_t s, int stat_ld = 0);
size_t layernorm_bwd_scratch(int R, int H);
// drop_mode 0: no dropout.  1: dy is the gradient of this LayerNorm's dropped output (site) and is masked as
// it is read.  2: dx also feeds a dropped branch (site): dxm gets its masked copy and d_colsum sums that copy.
hs_status launch_layernorm_bwd(hs_ctx* ctx, int dtype, const void* dy, const void* x, const float* stats, const void* gain,
                               void* dx, float* d_gain, float* d_bias, float* d_colsum, float beta, int R, int H,
                               void* partials, hipStream_t s, const DropCfg* drop = nullptr, uint32_t site = 0, int drop_mode = 0,
                               void* dxm = nullptr);
hs_status launch_layernorm_bwd_rows(hs_ctx* ctx, int dtype, const void* dy, const void* x, const float* stats, const void* gain, void* dx,
                                    int R, int H, void* partials, hipStream_t s, const DropCfg* drop = nullptr, uint32_t site = 0,
                                    int drop_mode = 0, void* dxm = nullptr);
hs_status launch_layernorm_bwd_cols(hs_ctx* ctx, const void* partials, float* d_gain, float* d_bias, float* d_colsum, float beta, int R, int H,
                                    hipStream_t s);
hs_status launch_embed_ln_fwd(hs_ctx* ctx, int dtype, const void* word, const void* pos, const void* gain, const void* bias,
                              const int32_t* ids, void* e_pre, void* x0, float* stats, int B, int L, int H, int V, float eps,
                              hipStream_t s, const DropCfg* drop = nullptr, int stat_ld = 0);
size_t embed_bwd_scratch(int T, int H);
// sorted: launch_embed_sort has already run on the same scratch (ordered before this call)
hs_status launch_embed_sort(hs_ctx* ctx, const int32_t* ids, int T, int V, void* scratch, hipStream_t s);
hs_status launch_embed_bwd(hs_ctx* ctx, int dtype, const void* de, const int32_t* ids, int B, int L, int H, int V, int max_pos,
                           float* g_word, float* g_pos, float beta_pos, void* scratch, hipStream_t s, bool sorted = false);
// drop/site: dropout of the attention probabilities (element ((b*A + h)*L + query)*L + key of the site)
hs_status launch_attention_fwd(hs_ctx* ctx, int dtype, const void* qkv, const int32_t* lens, int B, int L, int A, void* out,
                               float* lse, hipStream_t s, const DropCfg* drop = nullptr, uint32_t site = 0);
hs_status launch_attention_bwd(hs_ctx* ctx, int dtype, const void* qkv, const void* out, const float* lse, const void* d_out,
                               const int32_t* lens, int B, int L, int A, void* dqkv, float* dvec, hipStream_t s,
                               const DropCfg* drop = nullptr, uint32_t site = 0);
size_t colsum_scratch(int R, int C);
hs_status launch_colsum(hs_ctx* ctx, int dtype, const void* x, int64_t ldx, int R, int C, float* out, float beta, void* partials,
                        hipStream_t s);
hs_status launch_gather_rows(hs_ctx* ctx, int dtype, const void* src, const int32_t* idx, int M, int H, void* dst, hipStream_t s);
hs_status launch_scatter_rows(hs_ctx* ctx, int dtype, const void* src, const int32_t* idx, int M, int H, void* dst, hipStream_t s);
hs_status launch_fill_zero(hs_ctx* ctx, void* p, size_t bytes, hipStream_t s);
hs_status launch_fill_value(hs_ctx* ctx, int dtype, void* p, size_t n, float value, hipStream_t s);   // n elements of the activation type
hs_status launch_gelu_fwd(hs_ctx* ctx, int dtype, const void* x, void* y, size_t n, hipStream_t s);
hs_status launch_gelu_bwd(hs_ctx* ctx, int dtype, const void* dy, const void* pre, void* dx, size_t n, hipStream_t s);
// Attention with separate query and key/value sequences (attention_general.hip).  Row b*Lq + i of q (stride ldq) is
// query i of sequence b, row b*Lk + j of k and v (stride ldkv) key j; key j takes part iff j < klens[b] and, when
// causal (Lq == Lk), j <= i; queries at or beyond qlens[b] get zero gradients.  out/d_out are [B*Lq, A*64], lse and
// dvec [B, A, Lq]; dq (stride lddq), dk and dv (stride lddkv) are written for every row.
struct AttnOperands {
  const void *q, *k, *v;
  int64_t ldq, ldkv;
  const int32_t *qlens, *klens;
  int Lq, Lk, A, causal;
};
hs_status launch_attention_general_fwd(hs_ctx* ctx, int dtype, const AttnOperands& x, int B, void* out, float* lse, hipStream_t s);
hs_status launch_attention_general_bwd(hs_ctx* ctx, int dtype, const AttnOperands& x, int B, const void* out, const float* lse,
                                       const void* d_out, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv, float* dvec,
                                       hipStream_t s);
// translation workload (seq2seq_ops.hip)
hs_status launch_position_table(hs_ctx* ctx, float* pe, int L, int H, hipStream_t s);     // pe [L, H] fp32
hs_status launch_embed_scale_pos(hs_ctx* ctx, int dtype, const void* emb, const int32_t* ids, const float* pe, void* x, int B, int L, int H, int V,
                                 float scale, const DropCfg* drop, uint32_t site, hipStream_t s);
hs_status launch_mask_scale(hs_ctx* ctx, int dtype, const void* x, void* y, size_t n, float alpha, const DropCfg* drop, uint32_t site,
                            hipStream_t s);
hs_status launch_relu(hs_ctx* ctx, int dtype, void* x, size_t n, hipStream_t s);
hs_status launch_relu_bwd(hs_ctx* ctx, int dtype, void* dx, const void* h, size_t n, hipStream_t s);
hs_status launch_real_rows(hs_ctx* ctx, const int32_t* lens, int B, int L, int32_t* rows, int capacity, hipStream_t s);
hs_status launch_smoothed_ce(hs_ctx* ctx, int dtype, const float* logits, int64_t ldl, const int32_t* labels, const int32_t* lens, int M, int L,
                             int V, float eps, void* dlogits, float* row_loss, float* row_nll, float* loss_sum, float* nll_sum,
                             const int32_t* rows, hipStream_t s);
hs_status launch_ce_loss(hs_ctx* ctx, int dtype, const float* logits, int64_t ldl, const int32_t* labels, int M, int V, void* dlogits,
                         float* row_loss, float* loss_sum, hipStream_t s);
