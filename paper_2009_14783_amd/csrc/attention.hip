// Softmax attention over the real keys of each sequence, head dimension 64.
// qkv is [B*L, 3H]: per token the query, key and value vectors of all heads; head h occupies
// columns h*64 .. h*64+63 of each third.  Key l' of sequence b takes part iff l' < lens[b].
//
// This file: the fp32 kernels (one thread per query or key row, K/V or Q/dO blocks of 64 rows
// staged in LDS as fp32, online softmax) and the dispatch; the bf16 MFMA kernels are in
// attention_mfma.hip.
#include "common.h"

namespace {

constexpr int D = 64;

template <class T>
__device__ __forceinline__ void stage_block(float (*dst)[D], const T* __restrict__ src, int64_t row_stride, int row0, int nrows_valid,
                                            int lane) {
  // 64 rows x 64 columns, coalesced along columns; rows beyond nrows_valid are zero
  for (int e = lane; e < 64 * D; e += 64) {
    const int r = e >> 6, c = e & 63;
    dst[r][c] = (r < nrows_valid) ? to_f(src[(int64_t)(row0 + r) * row_stride + c]) : 0.f;
  }
}

template <class T>
__global__ __launch_bounds__(64) void attn_fwd_simt(const T* __restrict__ qkv, const int32_t* __restrict__ lens, int L, int A,
                                                    T* __restrict__ out, float* __restrict__ lse, DropCfg drop, uint32_t site) {
  __shared__ float Ks[64][D];
  __shared__ float Vs[64][D];
  const int lane = threadIdx.x;
  const int b = blockIdx.z, h = blockIdx.y, qi = blockIdx.x * 64 + lane;
  const int H = A * D;
  const int64_t ld = 3 * (int64_t)H;
  int len = lens[b];
  len = len < 1 ? 1 : (len > L ? L : len);
  const T* base = qkv + (int64_t)b * L * ld + h * D;
  const bool active = qi < L;
  float q[D], acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) { q[c] = active ? 0.125f * to_f(base[(int64_t)qi * ld + c]) : 0.f; acc[c] = 0.f; }
  float m = -1.0e30f, l = 0.f;
  for (int k0 = 0; k0 < len; k0 += 64) {
    const int nv = min(64, len - k0);
    __syncthreads();
    stage_block<T>(Ks, base + H, ld, k0, nv, lane);
    stage_block<T>(Vs, base + 2 * H, ld, k0, nv, lane);
    __syncthreads();
    for (int j = 0; j < nv; ++j) {
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) s = fmaf(q[c], Ks[j][c], s);
      const float mn = fmaxf(m, s);
      const float alpha = __expf(m - mn), p = __expf(s - mn);
      l = l * alpha + p;
      // dropout acts on the normalised probabilities: the row sum keeps every key, the value sum the survivors
      const float pd = drop.thr ? p * drop_factor1(drop, site, (((uint64_t)b * A + h) * L + qi) * L + k0 + j) : p;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = fmaf(pd, Vs[j][c], acc[c] * alpha);
      m = mn;
    }
  }
  if (active) {
    const float inv = 1.0f / l;
    T* o = out + ((int64_t)b * L + qi) * H + h * D;
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] = from_f<T>(acc[c] * inv);
    lse[((int64_t)b * A + h) * L + qi] = m + logf(l);
  }
}

// dq and the row dot products dvec[i] = sum_c dO[i,c] * O[i,c]
template <class T>
__global__ __launch_bounds__(64) void attn_bwd_dq_simt(const T* __restrict__ qkv, const T* __restrict__ out, const float* __restrict__ lse,
                                                       const T* __restrict__ d_out, const int32_t* __restrict__ lens, int L, int A,
                                                       T* __restrict__ dqkv, float* __restrict__ dvec, DropCfg drop, uint32_t site) {
  __shared__ float Ks[64][D];
  __shared__ float Vs[64][D];
  const int lane = threadIdx.x;
  const int b = blockIdx.z, h = blockIdx.y, qi = blockIdx.x * 64 + lane;
  const int H = A * D;
  const int64_t ld = 3 * (int64_t)H;
  int len = lens[b];
  len = len < 1 ? 1 : (len > L ? L : len);
  const T* base = qkv + (int64_t)b * L * ld + h * D;
  const bool active = qi < len;     // padded query rows get zero gradient
  float q[D], go[D], dq[D];
  float dv_ = 0.f;
#pragma unroll
  for (int c = 0; c < D; ++c) {
    q[c] = active ? 0.125f * to_f(base[(int64_t)qi * ld + c]) : 0.f;
    go[c] = active ? to_f(d_out[((int64_t)b * L + qi) * H + h * D + c]) : 0.f;
    const float o = active ? to_f(out[((int64_t)b * L + qi) * H + h * D + c]) : 0.f;
    dv_ = fmaf(go[c], o, dv_);
    dq[c] = 0.f;
  }
  const float row_lse = active ? lse[((int64_t)b * A + h) * L + qi] : 0.f;
  for (int k0 = 0; k0 < len; k0 += 64) {
    const int nv = min(64, len - k0);
    __syncthreads();
    stage_block<T>(Ks, base + H, ld, k0, nv, lane);
    stage_block<T>(Vs, base + 2 * H, ld, k0, nv, lane);
    __syncthreads();
    if (active) {
      for (int j = 0; j < nv; ++j) {
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) { s = fmaf(q[c], Ks[j][c], s); dp = fmaf(go[c], Vs[j][c], dp); }
        const float p = __expf(s - row_lse);
        if (drop.thr) dp *= drop_factor1(drop, site, (((uint64_t)b * A + h) * L + qi) * L + k0 + j);
        const float ds = p * (dp - dv_);
#pragma unroll
        for (int c = 0; c < D; ++c) dq[c] = fmaf(ds, Ks[j][c], dq[c]);
      }
    }
  }
  if (qi < L) {
    T* o = dqkv + ((int64_t)b * L + qi) * ld + h * D;
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] = from_f<T>(0.125f * dq[c]);
    dvec[((int64_t)b * A + h) * L + qi] = dv_;
  }
}

template <class T>
__global__ __launch_bounds__(64) void attn_bwd_dkv_simt(const T* __restrict__ qkv, const float* __restrict__ lse,
                                                        const T* __restrict__ d_out, const float* __restrict__ dvec,
                                                        const int32_t* __restrict__ lens, int L, int A, T* __restrict__ dqkv, DropCfg drop,
                                                        uint32_t site) {
  __shared__ float Qs[64][D];
  __shared__ float Gs[64][D];
  __shared__ float lse_s[64], dvec_s[64];
  const int lane = threadIdx.x;
  const int b = blockIdx.z, h = blockIdx.y, kj = blockIdx.x * 64 + lane;
  const int H = A * D;
  const int64_t ld = 3 * (int64_t)H;
  int len = lens[b];
  len = len < 1 ? 1 : (len > L ? L : len);
  const T* base = qkv + (int64_t)b * L * ld + h * D;
  const bool active = kj < len;     // padded keys take no part
  float k[D], v[D], dk[D], dv[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    k[c] = active ? to_f(base[(int64_t)kj * ld + H + c]) : 0.f;
    v[c] = active ? to_f(base[(int64_t)kj * ld + 2 * H + c]) : 0.f;
    dk[c] = 0.f; dv[c] = 0.f;
  }
  for (int q0 = 0; q0 < len; q0 += 64) {     // padded queries carry zero gradient: skipped
    const int nv = min(64, len - q0);
    __syncthreads();
    stage_block<T>(Qs, base, ld, q0, nv, lane);
    stage_block<T>(Gs, d_out + (int64_t)b * L * H + h * D, (int64_t)H, q0, nv, lane);
    if (lane < nv) {
      lse_s[lane] = lse[((int64_t)b * A + h) * L + q0 + lane];
      dvec_s[lane] = dvec[((int64_t)b * A + h) * L + q0 + lane];
    }
    __syncthreads();
    if (active) {
      for (int i = 0; i < nv; ++i) {
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) { s = fmaf(Qs[i][c], k[c], s); dp = fmaf(Gs[i][c], v[c], dp); }
        const float p = __expf(0.125f * s - lse_s[i]);
        const float f = drop.thr ? drop_factor1(drop, site, (((uint64_t)b * A + h) * L + q0 + i) * L + kj) : 1.0f;
        const float ds = p * (f * dp - dvec_s[i]);
        const float pd = p * f;
#pragma unroll
        for (int c = 0; c < D; ++c) { dv[c] = fmaf(pd, Gs[i][c], dv[c]); dk[c] = fmaf(ds, Qs[i][c], dk[c]); }
      }
    }
  }
  if (kj < L) {
    T* o = dqkv + ((int64_t)b * L + kj) * ld + h * D;
#pragma unroll
    for (int c = 0; c < D; ++c) { o[H + c] = from_f<T>(0.125f * dk[c]); o[2 * H + c] = from_f<T>(dv[c]); }
  }
}

}  // namespace

void launch_attention_fwd_mfma(const void* qkv, const int32_t* lens, int B, int L, int A, void* out, float* lse, hipStream_t s,
                               const DropCfg& drop, uint32_t site);
void launch_attention_bwd_mfma(const void* qkv, const void* out, const float* lse, const void* d_out, const int32_t* lens, int B, int L,
                               int A, void* dqkv, float* dvec, hipStream_t s, const DropCfg& drop, uint32_t site);

hs_status launch_attention_fwd(hs_ctx* ctx, int dtype, const void* qkv, const int32_t* lens, int B, int L, int A, void* out, float* lse,
                               hipStream_t s, const DropCfg* drop_in, uint32_t site) {
  if (B <= 0 || L <= 0) return HS_OK;
  const DropCfg drop = (drop_in && drop_in->thr) ? *drop_in : DropCfg{0u, 1.0f, 0u, 0u, 0u};
  if (drop.thr && (L & 3)) return hs_fail(ctx, HS_ERR_SHAPE, "attention with dropout: the padded length must be a multiple of 4");
  const double fl = 4.0 * B * A * (double)L * L * D;
  const double by = (double)B * L * A * D * 4.0 * esize(dtype);
  KScope scope(ctx ? ctx->prof : nullptr, KC_ATTN_FWD, fl, by, s);
  dim3 grid((L + 63) / 64, A, B);
  if (dtype == HS_BF16) launch_attention_fwd_mfma(qkv, lens, B, L, A, out, lse, s, drop, site);
  else hipLaunchKernelGGL(attn_fwd_simt<float>, grid, dim3(64), 0, s, (const float*)qkv, lens, L, A, (float*)out, lse, drop, site);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("attention_fwd: ") + hipGetErrorString(e));
  return HS_OK;
}

hs_status launch_attention_bwd(hs_ctx* ctx, int dtype, const void* qkv, const void* out, const float* lse, const void* d_out,
                               const int32_t* lens, int B, int L, int A, void* dqkv, float* dvec, hipStream_t s, const DropCfg* drop_in,
                               uint32_t site) {
  if (B <= 0 || L <= 0) return HS_OK;
  const DropCfg drop = (drop_in && drop_in->thr) ? *drop_in : DropCfg{0u, 1.0f, 0u, 0u, 0u};
  if (drop.thr && (L & 3)) return hs_fail(ctx, HS_ERR_SHAPE, "attention with dropout: the padded length must be a multiple of 4");
  const double fl = 8.0 * B * A * (double)L * L * D;   // dV, dP, dQ, dK (recomputing the scores is not counted)
  const double by = (double)B * L * A * D * 8.0 * esize(dtype);
  KScope scope(ctx ? ctx->prof : nullptr, KC_ATTN_BWD, fl, by, s);
  dim3 grid((L + 63) / 64, A, B);
  if (dtype == HS_BF16) {
    launch_attention_bwd_mfma(qkv, out, lse, d_out, lens, B, L, A, dqkv, dvec, s, drop, site);
  } else {
    hipLaunchKernelGGL(attn_bwd_dq_simt<float>, grid, dim3(64), 0, s, (const float*)qkv, (const float*)out, lse, (const float*)d_out, lens, L, A, (float*)dqkv, dvec, drop, site);
    hipLaunchKernelGGL(attn_bwd_dkv_simt<float>, grid, dim3(64), 0, s, (const float*)qkv, lse, (const float*)d_out, (const float*)dvec, lens, L, A, (float*)dqkv, drop, site);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("attention_bwd: ") + hipGetErrorString(e));
  return HS_OK;
}
