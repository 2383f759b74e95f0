// Row and element kernels of the translation workload that the encoder-only path does not have:
// scaled token embedding plus the fixed sinusoidal position table, ReLU and its gradient, a dropout
// mask with a scale applied to a gradient, and the label-smoothed cross-entropy over fp32 logits.
#include "common.h"

namespace {

#define S2S_LAUNCH_CHECK(ctx, what)                                                                    \
  do {                                                                                                 \
    hipError_t e_ = hipGetLastError();                                                                 \
    if (e_ != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e_)); \
  } while (0)

template <class T> struct V4;
template <> struct V4<float> {
  static __device__ __forceinline__ float4 ld(const float* p) { return *(const float4*)p; }
  static __device__ __forceinline__ void st(float* p, float4 v) { *(float4*)p = v; }
};
template <> struct V4<bf16> {
  static __device__ __forceinline__ float4 ld(const bf16* p) {
    const bf16x4 v = *(const bf16x4*)p;
    return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
  }
  static __device__ __forceinline__ void st(bf16* p, float4 v) {
    bf16x4 o;
    o[0] = (bf16)v.x; o[1] = (bf16)v.y; o[2] = (bf16)v.z; o[3] = (bf16)v.w;
    *(bf16x4*)p = o;
  }
};

// PE[l, 2i] = sin(l / 10000^(2i/H)), PE[l, 2i+1] = cos(same), evaluated in double
__global__ __launch_bounds__(256) void position_table_kernel(float* __restrict__ pe, int L, int H) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= L * H) return;
  const int l = i / H, c = i - l * H;
  const double angle = (double)l * exp(-(double)(2 * (c >> 1)) / (double)H * 9.210340371976184 /* ln 10000 */);
  pe[i] = (float)((c & 1) ? cos(angle) : sin(angle));
}

// x[b, l, c] = drop(scale * E[ids[b, l], c] + PE[l, c]); one block per token, four columns per thread
template <class T>
__global__ __launch_bounds__(128) void embed_scale_pos_kernel(const T* __restrict__ emb, const int32_t* __restrict__ ids,
                                                              const float* __restrict__ pe, T* __restrict__ x, int L, int H, int V, float scale,
                                                              DropCfg drop, uint32_t site) {
  const int64_t row = blockIdx.x;
  const int l = (int)(row % L);
  int id = ids[row];
  id = id < 0 ? 0 : (id >= V ? V - 1 : id);
  for (int c = 4 * threadIdx.x; c < H; c += 512) {
    const float4 e = V4<T>::ld(emb + (int64_t)id * H + c);
    const float4 p = *(const float4*)(pe + (int64_t)l * H + c);
    float4 v = make_float4(fmaf(scale, e.x, p.x), fmaf(scale, e.y, p.y), fmaf(scale, e.z, p.z), fmaf(scale, e.w, p.w));
    if (drop.thr) {
      float f[4];
      drop_factors4(drop, site, ((uint64_t)row * H + c) >> 2, f);
      v.x *= f[0]; v.y *= f[1]; v.z *= f[2]; v.w *= f[3];
    }
    V4<T>::st(x + row * H + c, v);
  }
}

// y = alpha * f * x with f the dropout factors of `site` (f = 1 when off); four elements per thread
template <class T>
__global__ __launch_bounds__(256) void mask_scale_kernel(const T* __restrict__ x, T* __restrict__ y, size_t n4, float alpha, DropCfg drop,
                                                         uint32_t site) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 v = V4<T>::ld(x + 4 * i);
  float f[4] = {1.f, 1.f, 1.f, 1.f};
  if (drop.thr) drop_factors4(drop, site, (uint64_t)i, f);
  v.x *= alpha * f[0]; v.y *= alpha * f[1]; v.z *= alpha * f[2]; v.w *= alpha * f[3];
  V4<T>::st(y + 4 * i, v);
}

template <class T>
__global__ __launch_bounds__(256) void relu_kernel(T* __restrict__ x, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 v = V4<T>::ld(x + 4 * i);
  v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f);
  V4<T>::st(x + 4 * i, v);
}

// dx *= (h > 0), h the ReLU's output
template <class T>
__global__ __launch_bounds__(256) void relu_bwd_kernel(T* __restrict__ dx, const T* __restrict__ h, size_t n4) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n4) return;
  float4 d = V4<T>::ld(dx + 4 * i);
  const float4 a = V4<T>::ld(h + 4 * i);
  d.x = a.x > 0.f ? d.x : 0.f; d.y = a.y > 0.f ? d.y : 0.f; d.z = a.z > 0.f ? d.z : 0.f; d.w = a.w > 0.f ? d.w : 0.f;
  V4<T>::st(dx + 4 * i, d);
}

__device__ __forceinline__ float block_reduce256(float v, bool is_max, float* sh) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  float r = sh[0];
  for (int w = 1; w < 4; ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
  return r;
}

// One block per target position (row b*L + l of the logits).  Real positions (l < lens[b]):
//   nll = lse - z[label];  loss = (1 - eps) nll + eps (lse - mean_v z_v);  d z_v = softmax_v - (1 - eps)[v == label] - eps / V.
// Padding positions: zero loss, zero gradient row.  Columns V .. ldl-1 of the gradient row are written as zeros.
template <class T>
__global__ __launch_bounds__(256) void smoothed_ce_kernel(const float* __restrict__ logits, int64_t ldl, const int32_t* __restrict__ labels,
                                                          const int32_t* __restrict__ lens, int L, int V, float eps,
                                                          T* __restrict__ dlogits, float* __restrict__ row_loss, float* __restrict__ row_nll,
                                                          const int32_t* __restrict__ rows) {
  __shared__ float sh[4];
  const int m = blockIdx.x;
  const int pos = rows ? rows[m] : m;          // position b*L + l of this row of logits
  const int b = pos / L, l = pos - b * L;
  T* d = dlogits + (int64_t)m * ldl;
  if (l >= lens[b]) {       // block-uniform
    for (int v = threadIdx.x; v < (int)ldl; v += 256) d[v] = from_f<T>(0.f);
    if (threadIdx.x == 0) { row_loss[m] = 0.f; row_nll[m] = 0.f; }
    return;
  }
  const float* z = logits + (int64_t)m * ldl;
  float mx = -3.0e38f, sz = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) { const float t = z[v]; mx = fmaxf(mx, t); sz += t; }
  mx = block_reduce256(mx, true, sh);
  sz = block_reduce256(sz, false, sh);
  float se = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) se += __expf(z[v] - mx);
  se = block_reduce256(se, false, sh);
  const float lse = mx + logf(se);
  int lab = labels[pos];
  lab = lab < 0 ? 0 : (lab >= V ? V - 1 : lab);
  if (threadIdx.x == 0) {
    const float nll = lse - z[lab];
    row_nll[m] = nll;
    row_loss[m] = (1.0f - eps) * nll + eps * (lse - sz / (float)V);
  }
  const float u = eps / (float)V, on = 1.0f - eps;
  for (int v = threadIdx.x; v < (int)ldl; v += 256) {
    float p = 0.f;
    if (v < V) p = __expf(z[v] - lse) - u - (v == lab ? on : 0.0f);
    d[v] = from_f<T>(p);
  }
}

// The same with the whole row held in registers (one read of the logits): 1024 threads, up to ten 4-element chunks per
// thread, so rows of up to 40960 padded columns; row stride a multiple of 4, 16-byte aligned rows.
constexpr int SCE_NT = 1024, SCE_MAXCH = 10;
__device__ __forceinline__ float block_reduce1024(float v, bool is_max, float* sh) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  float r = sh[0];
  for (int w = 1; w < SCE_NT / 64; ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
  return r;
}
template <class T>
__global__ __launch_bounds__(SCE_NT) void smoothed_ce_row_kernel(const float* __restrict__ logits, int64_t ldl, const int32_t* __restrict__ labels,
                                                                const int32_t* __restrict__ lens, int L, int V, float eps,
                                                                T* __restrict__ dlogits, float* __restrict__ row_loss, float* __restrict__ row_nll,
                                                                const int32_t* __restrict__ rows) {
  __shared__ float sh[SCE_NT / 64];
  const int m = blockIdx.x;
  const int pos = rows ? rows[m] : m;          // position b*L + l of this row of logits
  const int b = pos / L, l = pos - b * L;
  const int nch = (int)(ldl / 4);
  T* d = dlogits + (int64_t)m * ldl;
  if (l >= lens[b]) {       // block-uniform
    for (int ch = threadIdx.x; ch < nch; ch += SCE_NT) V4<T>::st(d + 4 * ch, make_float4(0.f, 0.f, 0.f, 0.f));
    if (threadIdx.x == 0) { row_loss[m] = 0.f; row_nll[m] = 0.f; }
    return;
  }
  const float* z = logits + (int64_t)m * ldl;
  float4 x[SCE_MAXCH];
  float mx = -3.0e38f, sz = 0.f;
#pragma unroll
  for (int c = 0; c < SCE_MAXCH; ++c) {
    const int ch = threadIdx.x + c * SCE_NT, v = ch * 4;
    x[c] = make_float4(-3.0e38f, -3.0e38f, -3.0e38f, -3.0e38f);
    if (ch < nch) {
      if (v + 3 < V) { x[c] = *(const float4*)(z + v); sz += (x[c].x + x[c].y) + (x[c].z + x[c].w); }
      else {
        if (v < V) { x[c].x = z[v]; sz += x[c].x; }
        if (v + 1 < V) { x[c].y = z[v + 1]; sz += x[c].y; }
        if (v + 2 < V) { x[c].z = z[v + 2]; sz += x[c].z; }
      }
    }
    mx = fmaxf(mx, fmaxf(fmaxf(x[c].x, x[c].y), fmaxf(x[c].z, x[c].w)));
  }
  mx = block_reduce1024(mx, true, sh);
  sz = block_reduce1024(sz, false, sh);
  float se = 0.f;
#pragma unroll
  for (int c = 0; c < SCE_MAXCH; ++c)     // excluded positions hold -3e38: their exponential is exactly 0
    se += (__expf(x[c].x - mx) + __expf(x[c].y - mx)) + (__expf(x[c].z - mx) + __expf(x[c].w - mx));
  se = block_reduce1024(se, false, sh);
  const float lse = mx + logf(se);
  int lab = labels[pos];
  lab = lab < 0 ? 0 : (lab >= V ? V - 1 : lab);
  if (threadIdx.x == 0) {
    const float nll = lse - z[lab];
    row_nll[m] = nll;
    row_loss[m] = (1.0f - eps) * nll + eps * (lse - sz / (float)V);
  }
  const float u = eps / (float)V, on = 1.0f - eps;
#pragma unroll
  for (int c = 0; c < SCE_MAXCH; ++c) {
    const int ch = threadIdx.x + c * SCE_NT, v = ch * 4;
    if (ch < nch) {
      float4 p;      // columns at or beyond V hold -3e38: exp gives exactly 0, and they get 0, not -u
      p.x = (v < V) ? __expf(x[c].x - lse) - u - (v == lab ? on : 0.0f) : 0.f;
      p.y = (v + 1 < V) ? __expf(x[c].y - lse) - u - (v + 1 == lab ? on : 0.0f) : 0.f;
      p.z = (v + 2 < V) ? __expf(x[c].z - lse) - u - (v + 2 == lab ? on : 0.0f) : 0.f;
      p.w = (v + 3 < V) ? __expf(x[c].w - lse) - u - (v + 3 == lab ? on : 0.0f) : 0.f;
      V4<T>::st(d + v, p);
    }
  }
}

// rows[k] = b*L + l for the real positions (l < lens[b]) in ascending order: one block walks the sequences in chunks
// of 1024 with a running offset (a block-wide exclusive scan of the clamped lengths per chunk)
__global__ __launch_bounds__(1024) void real_rows_kernel(const int32_t* __restrict__ lens, int B, int L, int32_t* __restrict__ rows, int capacity) {
  __shared__ int scan[1024];
  __shared__ int base_s;
  if (threadIdx.x == 0) base_s = 0;
  __syncthreads();
  for (int b0 = 0; b0 < B; b0 += 1024) {
    const int b = b0 + threadIdx.x;
    int n = 0;
    if (b < B) { n = lens[b]; n = n < 0 ? 0 : (n > L ? L : n); }
    scan[threadIdx.x] = n;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {          // inclusive scan
      const int v = threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    const int start = base_s + scan[threadIdx.x] - n;
    for (int l = 0; l < n; ++l) if (start + l < capacity) rows[start + l] = b * L + l;
    __syncthreads();
    if (threadIdx.x == 1023) base_s += scan[1023];
    __syncthreads();
  }
  // a caller whose count exceeds the real one still gets valid positions (position 0) in the tail
  for (int k = base_s + threadIdx.x; k < capacity; k += 1024) rows[k] = 0;
}

// fixed-order sums of two vectors of n floats by one block
__global__ __launch_bounds__(256) void sum_two_kernel(const float* __restrict__ a, const float* __restrict__ b, int n, float* __restrict__ out_a,
                                                      float* __restrict__ out_b) {
  __shared__ float sh[4];
  float sa = 0.f, sb = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) { sa += a[i]; sb += b[i]; }
  sa = block_reduce256(sa, false, sh);
  sb = block_reduce256(sb, false, sh);
  if (threadIdx.x == 0) { *out_a = sa; if (out_b) *out_b = sb; }
}

}  // namespace

hs_status launch_position_table(hs_ctx* ctx, float* pe, int L, int H, hipStream_t s) {
  if (L <= 0) return HS_OK;
  KScope scope(ctx ? ctx->prof : nullptr, KC_EMBED, 0.0, 4.0 * L * H, s);
  hipLaunchKernelGGL(position_table_kernel, dim3((L * H + 255) / 256), dim3(256), 0, s, pe, L, H);
  S2S_LAUNCH_CHECK(ctx, "position_table");
  return HS_OK;
}

hs_status launch_embed_scale_pos(hs_ctx* ctx, int dtype, const void* emb, const int32_t* ids, const float* pe, void* x, int B, int L, int H, int V,
                                 float scale, const DropCfg* drop_in, uint32_t site, hipStream_t s) {
  if (B <= 0 || L <= 0) return HS_OK;
  const DropCfg drop = (drop_in && drop_in->thr) ? *drop_in : DropCfg{0u, 1.0f, 0u, 0u, 0u};
  KScope scope(ctx ? ctx->prof : nullptr, KC_EMBED, 2.0 * B * L * H, 2.0 * B * L * H * esize(dtype), s);
  dim3 grid((unsigned)(B * L));
  if (dtype == HS_BF16) hipLaunchKernelGGL(embed_scale_pos_kernel<bf16>, grid, dim3(128), 0, s, (const bf16*)emb, ids, pe, (bf16*)x, L, H, V, scale, drop, site);
  else hipLaunchKernelGGL(embed_scale_pos_kernel<float>, grid, dim3(128), 0, s, (const float*)emb, ids, pe, (float*)x, L, H, V, scale, drop, site);
  S2S_LAUNCH_CHECK(ctx, "embed_scale_pos");
  return HS_OK;
}

hs_status launch_mask_scale(hs_ctx* ctx, int dtype, const void* x, void* y, size_t n, float alpha, const DropCfg* drop_in, uint32_t site,
                            hipStream_t s) {
  if (n == 0) return HS_OK;
  if (n & 3) return hs_fail(ctx, HS_ERR_SHAPE, "mask_scale: element count must be a multiple of 4");
  const DropCfg drop = (drop_in && drop_in->thr) ? *drop_in : DropCfg{0u, 1.0f, 0u, 0u, 0u};
  KScope scope(ctx ? ctx->prof : nullptr, KC_ELEMWISE, (double)n, 2.0 * n * esize(dtype), s);
  const size_t n4 = n / 4;
  dim3 grid((unsigned)((n4 + 255) / 256));
  if (dtype == HS_BF16) hipLaunchKernelGGL(mask_scale_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)x, (bf16*)y, n4, alpha, drop, site);
  else hipLaunchKernelGGL(mask_scale_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (float*)y, n4, alpha, drop, site);
  S2S_LAUNCH_CHECK(ctx, "mask_scale");
  return HS_OK;
}

hs_status launch_relu(hs_ctx* ctx, int dtype, void* x, size_t n, hipStream_t s) {
  if (n == 0) return HS_OK;
  if (n & 3) return hs_fail(ctx, HS_ERR_SHAPE, "relu: element count must be a multiple of 4");
  KScope scope(ctx ? ctx->prof : nullptr, KC_ELEMWISE, (double)n, 2.0 * n * esize(dtype), s);
  const size_t n4 = n / 4;
  dim3 grid((unsigned)((n4 + 255) / 256));
  if (dtype == HS_BF16) hipLaunchKernelGGL(relu_kernel<bf16>, grid, dim3(256), 0, s, (bf16*)x, n4);
  else hipLaunchKernelGGL(relu_kernel<float>, grid, dim3(256), 0, s, (float*)x, n4);
  S2S_LAUNCH_CHECK(ctx, "relu");
  return HS_OK;
}

hs_status launch_relu_bwd(hs_ctx* ctx, int dtype, void* dx, const void* h, size_t n, hipStream_t s) {
  if (n == 0) return HS_OK;
  if (n & 3) return hs_fail(ctx, HS_ERR_SHAPE, "relu_bwd: element count must be a multiple of 4");
  KScope scope(ctx ? ctx->prof : nullptr, KC_ELEMWISE, (double)n, 3.0 * n * esize(dtype), s);
  const size_t n4 = n / 4;
  dim3 grid((unsigned)((n4 + 255) / 256));
  if (dtype == HS_BF16) hipLaunchKernelGGL(relu_bwd_kernel<bf16>, grid, dim3(256), 0, s, (bf16*)dx, (const bf16*)h, n4);
  else hipLaunchKernelGGL(relu_bwd_kernel<float>, grid, dim3(256), 0, s, (float*)dx, (const float*)h, n4);
  S2S_LAUNCH_CHECK(ctx, "relu_bwd");
  return HS_OK;
}

hs_status launch_real_rows(hs_ctx* ctx, const int32_t* lens, int B, int L, int32_t* rows, int capacity, hipStream_t s) {
  if (B <= 0) return HS_OK;
  KScope scope(ctx ? ctx->prof : nullptr, KC_ELEMWISE, 0.0, 4.0 * capacity, s);
  hipLaunchKernelGGL(real_rows_kernel, dim3(1), dim3(1024), 0, s, lens, B, L, rows, capacity);
  S2S_LAUNCH_CHECK(ctx, "real_rows");
  return HS_OK;
}

// M rows of logits; rows == NULL: row m is position m of the [B, L] batch (padding rows give zero loss and gradient);
// otherwise row m is position rows[m], which must be real.
hs_status launch_smoothed_ce(hs_ctx* ctx, int dtype, const float* logits, int64_t ldl, const int32_t* labels, const int32_t* lens, int M, int L,
                             int V, float eps, void* dlogits, float* row_loss, float* row_nll, float* loss_sum, float* nll_sum,
                             const int32_t* rows, hipStream_t s) {
  if (M <= 0) return HS_OK;
  KScope scope(ctx ? ctx->prof : nullptr, KC_LOSS, 5.0 * M * V, (double)M * V * (4.0 + esize(dtype)), s);
  const bool in_regs = (ldl % 4) == 0 && ldl <= (int64_t)4 * SCE_NT * SCE_MAXCH && ((uintptr_t)logits % 16) == 0 && ((uintptr_t)dlogits % 16) == 0;
  if (in_regs) {
    if (dtype == HS_BF16) hipLaunchKernelGGL(smoothed_ce_row_kernel<bf16>, dim3(M), dim3(SCE_NT), 0, s, logits, ldl, labels, lens, L, V, eps, (bf16*)dlogits, row_loss, row_nll, rows);
    else hipLaunchKernelGGL(smoothed_ce_row_kernel<float>, dim3(M), dim3(SCE_NT), 0, s, logits, ldl, labels, lens, L, V, eps, (float*)dlogits, row_loss, row_nll, rows);
  } else if (dtype == HS_BF16) hipLaunchKernelGGL(smoothed_ce_kernel<bf16>, dim3(M), dim3(256), 0, s, logits, ldl, labels, lens, L, V, eps, (bf16*)dlogits, row_loss, row_nll, rows);
  else hipLaunchKernelGGL(smoothed_ce_kernel<float>, dim3(M), dim3(256), 0, s, logits, ldl, labels, lens, L, V, eps, (float*)dlogits, row_loss, row_nll, rows);
  S2S_LAUNCH_CHECK(ctx, "smoothed_ce");
  hipLaunchKernelGGL(sum_two_kernel, dim3(1), dim3(256), 0, s, (const float*)row_loss, (const float*)row_nll, M, loss_sum, nll_sum);
  S2S_LAUNCH_CHECK(ctx, "loss sums");
  return HS_OK;
}
