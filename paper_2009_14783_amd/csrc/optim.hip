// Flat-buffer kernels: gradient accumulation and normalisation by the global weight, fused Adam,
// fp32 -> low-precision parameter copy, key mask.  Single pass over HBM, 16-byte accesses.
#include <cmath>

#include "common.h"

namespace {

__global__ __launch_bounds__(256) void accum_normalize_kernel(float* __restrict__ G, const float* __restrict__ g, size_t n, int add,
                                                              int scale, float denom) {
  const size_t n4 = n / 4;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  float4* G4 = (float4*)G;
  const float4* g4 = (const float4*)g;
  for (size_t i = i0; i < n4; i += stride) {
    float4 a = G4[i];
    if (add) { const float4 b = g4[i]; a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w; }
    if (scale) { a.x /= denom; a.y /= denom; a.z /= denom; a.w /= denom; }
    G4[i] = a;
  }
  for (size_t i = n4 * 4 + i0; i < n; i += stride) {
    float a = G[i];
    if (add) a += g[i];
    if (scale) a /= denom;
    G[i] = a;
  }
}

struct AdamConst { float lr, b1, b2, omb1, omb2, eps, inv_c1, inv_c2, lr_wd; };

__device__ __forceinline__ float adam_one(float& w, float& m, float& v, float g, const AdamConst& k) {
  m = k.b1 * m + k.omb1 * g;
  v = k.b2 * v + k.omb2 * (g * g);
  const float mhat = m * k.inv_c1;
  const float vhat = v * k.inv_c2;
  if (k.lr_wd != 0.f) w -= k.lr_wd * w;
  w -= k.lr * mhat / (sqrtf(vhat) + k.eps);
  return w;
}

__global__ __launch_bounds__(256) void adam_kernel(float* __restrict__ w, float* __restrict__ m, float* __restrict__ v,
                                                   const float* __restrict__ G, bf16* __restrict__ wl, size_t n, AdamConst k) {
  const size_t n4 = n / 4;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (size_t i = i0; i < n4; i += stride) {
    float4 w4 = ((float4*)w)[i], m4 = ((float4*)m)[i], v4 = ((float4*)v)[i];
    const float4 g4 = ((const float4*)G)[i];
    adam_one(w4.x, m4.x, v4.x, g4.x, k);
    adam_one(w4.y, m4.y, v4.y, g4.y, k);
    adam_one(w4.z, m4.z, v4.z, g4.z, k);
    adam_one(w4.w, m4.w, v4.w, g4.w, k);
    ((float4*)w)[i] = w4; ((float4*)m)[i] = m4; ((float4*)v)[i] = v4;
    if (wl) {
      bf16x4 o;
      o[0] = (bf16)w4.x; o[1] = (bf16)w4.y; o[2] = (bf16)w4.z; o[3] = (bf16)w4.w;
      ((bf16x4*)wl)[i] = o;
    }
  }
  for (size_t i = n4 * 4 + i0; i < n; i += stride) {
    float ww = w[i], mm = m[i], vv = v[i];
    adam_one(ww, mm, vv, G[i], k);
    w[i] = ww; m[i] = mm; v[i] = vv;
    if (wl) wl[i] = (bf16)ww;
  }
}

template <class T>
__global__ __launch_bounds__(256) void cast_kernel(const float* __restrict__ src, T* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = from_f<T>(src[i]);
}

__global__ void key_mask_kernel(const int32_t* __restrict__ lens, int B, int L, uint8_t* __restrict__ mask) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)B * L) return;
  const int b = (int)(i / L), l = (int)(i % L);
  mask[i] = (l < lens[b]) ? 1 : 0;
}

__global__ void keep_mask_kernel(DropCfg d, uint32_t site, size_t n, uint8_t* __restrict__ mask) {
  const size_t g = (size_t)blockIdx.x * blockDim.x + threadIdx.x;     // one group of four elements per thread
  if (4 * g >= n) return;
  float f[4];
  drop_factors4(d, site, g, f);
  for (int t = 0; t < 4; ++t) if (4 * g + t < n) mask[4 * g + t] = f[t] != 0.0f ? 1 : 0;
}

unsigned flat_grid(size_t work_items) {
  size_t blocks = (work_items + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 256 * 16) blocks = 256 * 16;   // 16 blocks per compute unit, grid-stride beyond
  return (unsigned)blocks;
}

hs_status check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(nullptr, HS_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
  return HS_OK;
}

// the loss sums of the workers / passes added in index order by one wave, times 1 / (global weight)
__global__ __launch_bounds__(64) void weighted_loss_kernel(const float* __restrict__ x, int n, float inv_denom, float* __restrict__ out) {
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 64) s += x[i];
  s = wave_sum(s);
  if (threadIdx.x == 0) *out = s * inv_denom;
}

}  // namespace

extern "C" {

hs_status hs_grad_accum_normalize(float* G, const float* g, size_t n, int32_t ignore, double denom, void* stream) {
  if (!G && n > 0) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_grad_accum_normalize: G is NULL");
  if (!(denom >= 0.0) || std::isinf(denom)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_grad_accum_normalize: denom must be finite and >= 0");
  if (((uintptr_t)G % 16) || ((uintptr_t)g % 16)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_grad_accum_normalize: buffers must be 16-byte aligned");
  const int add = (!ignore && g != nullptr) ? 1 : 0;
  const int scale = denom > 0.0 ? 1 : 0;
  if (n == 0 || (!add && !scale)) return HS_OK;
  hipLaunchKernelGGL(accum_normalize_kernel, dim3(flat_grid(n / 4 + 1)), dim3(256), 0, (hipStream_t)stream, G, add ? g : nullptr, n, add,
                     scale, (float)denom);
  return check_launch("hs_grad_accum_normalize");
}

hs_status hs_adam_step(float* w, float* m, float* v, const float* G, void* w_lowp_out, size_t n, double lr, double beta1, double beta2,
                       double eps, double weight_decay, int64_t t, void* stream) {
  if (n == 0) return HS_OK;
  if (!w || !m || !v || !G) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_adam_step: NULL buffer");
  if (t < 1) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_adam_step: t must be >= 1");
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_adam_step: betas must be in [0,1), eps >= 0");
  if (((uintptr_t)w % 16) || ((uintptr_t)m % 16) || ((uintptr_t)v % 16) || ((uintptr_t)G % 16) || ((uintptr_t)w_lowp_out % 8))
    return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_adam_step: buffers must be 16-byte aligned");
  AdamConst k;
  k.lr = lr; k.b1 = beta1; k.b2 = beta2; k.omb1 = (float)(1.0 - (double)beta1); k.omb2 = (float)(1.0 - (double)beta2); k.eps = eps;
  k.inv_c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)t)));
  k.inv_c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)t)));
  k.lr_wd = lr * weight_decay;
  hipLaunchKernelGGL(adam_kernel, dim3(flat_grid(n / 4 + 1)), dim3(256), 0, (hipStream_t)stream, w, m, v, G, (bf16*)w_lowp_out, n, k);
  return check_launch("hs_adam_step");
}

hs_status hs_fill_zero(void* dst, size_t bytes, void* stream) {
  if (bytes == 0) return HS_OK;
  if (!dst) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_fill_zero: NULL buffer");
  return launch_fill_zero(nullptr, dst, bytes, (hipStream_t)stream);
}

hs_status hs_weighted_loss(const float* loss_sums, int32_t n, double denom, float* loss_out, void* stream) {
  if (n < 0 || !(denom > 0.0) || std::isinf(denom)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_weighted_loss: n < 0 or denom not positive and finite");
  if (!loss_out || (n > 0 && !loss_sums)) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_weighted_loss: NULL buffer");
  hipLaunchKernelGGL(weighted_loss_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, loss_sums, n, (float)(1.0 / denom), loss_out);
  return check_launch("hs_weighted_loss");
}

hs_status hs_cast_params(const float* src, void* dst, size_t n, int32_t dst_dtype, void* stream) {
  if (n == 0) return HS_OK;
  if (!src || !dst) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_cast_params: NULL buffer");
  if (dst_dtype == HS_BF16) hipLaunchKernelGGL(cast_kernel<bf16>, dim3(flat_grid(n)), dim3(256), 0, (hipStream_t)stream, src, (bf16*)dst, n);
  else if (dst_dtype == HS_FP32) hipLaunchKernelGGL(cast_kernel<float>, dim3(flat_grid(n)), dim3(256), 0, (hipStream_t)stream, src, (float*)dst, n);
  else return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_cast_params: bad dtype");
  return check_launch("hs_cast_params");
}

hs_status hs_dropout_keep_mask(hs_ctx* ctx, uint32_t site, size_t n, uint8_t* mask_out, void* stream) {
  if (!ctx) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_dropout_keep_mask: ctx is NULL");
  if (n == 0) return HS_OK;
  if (!mask_out) return hs_fail(ctx, HS_ERR_INVALID_ARG, "hs_dropout_keep_mask: NULL buffer");
  const size_t groups = (n + 3) / 4;
  hipLaunchKernelGGL(keep_mask_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, (hipStream_t)stream, ctx->drop, site, n, mask_out);
  return check_launch("hs_dropout_keep_mask");
}

hs_status hs_key_mask(const int32_t* lens, int32_t B, int32_t L, uint8_t* mask_out, void* stream) {
  if (B < 0 || L < 0) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_key_mask: negative size");
  if ((int64_t)B * L == 0) return HS_OK;
  if (!lens || !mask_out) return hs_fail(nullptr, HS_ERR_INVALID_ARG, "hs_key_mask: NULL buffer");
  const int64_t n = (int64_t)B * L;
  hipLaunchKernelGGL(key_mask_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, lens, B, L, mask_out);
  return check_launch("hs_key_mask");
}

}  // extern "C"
