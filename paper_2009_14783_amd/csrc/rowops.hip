// Row-wise and element-wise kernels: LayerNorm forward/backward, embedding forward/backward,
// column sums, gather/scatter of rows, GELU, cross-entropy.  All are HBM-bound single-pass
// kernels; statistics and reductions are fp32 and every reduction has a fixed order.
#include "common.h"

namespace {

constexpr int MAXC = 16;   // columns per lane (scalar access): hidden <= 1024
constexpr int MAXCH = 4;   // 4-element chunks per lane (vector access): hidden <= 1024

// 4 consecutive elements as float4 (8-byte access for bfloat16, 16-byte for float)
template <class T> struct Vec4;
template <> struct Vec4<float> {
  static __device__ __forceinline__ float4 ld(const float* p) { return *(const float4*)p; }
  static __device__ __forceinline__ void st(float* p, float4 v) { *(float4*)p = v; }
  static __device__ __forceinline__ float4 round(float4 v) { return v; }
};
template <> struct Vec4<bf16> {
  static __device__ __forceinline__ float4 ld(const bf16* p) {
    const bf16x4 v = *(const bf16x4*)p;
    return make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
  }
  static __device__ __forceinline__ void st(bf16* p, float4 v) {
    bf16x4 o;
    o[0] = (bf16)v.x; o[1] = (bf16)v.y; o[2] = (bf16)v.z; o[3] = (bf16)v.w;
    *(bf16x4*)p = o;
  }
  static __device__ __forceinline__ float4 round(float4 v) {   // what a store followed by a load gives
    return make_float4((float)(bf16)v.x, (float)(bf16)v.y, (float)(bf16)v.z, (float)(bf16)v.w);
  }
};

// ------------------------------------------------------------------------------------------
// LayerNorm forward: one wave per row; lane owns the 4-element chunks lane, lane+64, ...
// ------------------------------------------------------------------------------------------
template <class T>
__device__ __forceinline__ void ln_row(float4 (&v)[MAXCH], int nch, int H, int lane, const T* __restrict__ gain,
                                       const T* __restrict__ bias, float eps, T* __restrict__ y, float* mean_out, float* rstd_out,
                                       const DropCfg* drop = nullptr, uint32_t site = 0, int64_t row = 0) {
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) if (c * 64 + lane < nch) s += (v[c].x + v[c].y) + (v[c].z + v[c].w);
  const float mu = wave_sum(s) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) if (c * 64 + lane < nch) {
    const float a = v[c].x - mu, b = v[c].y - mu, d = v[c].z - mu, e = v[c].w - mu;
    q += (a * a + b * b) + (d * d + e * e);
  }
  const float var = wave_sum(q) / (float)H;
  const float rstd = 1.0f / sqrtf(var + eps);
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) if (c * 64 + lane < nch) {
    const int col = 4 * (c * 64 + lane);
    const float4 g = Vec4<T>::ld(gain + col), b = Vec4<T>::ld(bias + col);
    float4 o;
    o.x = (v[c].x - mu) * rstd * g.x + b.x; o.y = (v[c].y - mu) * rstd * g.y + b.y;
    o.z = (v[c].z - mu) * rstd * g.z + b.z; o.w = (v[c].w - mu) * rstd * g.w + b.w;
    if (drop) {                                   // dropout of the output: one generator block per chunk
      float f[4];
      drop_factors4(*drop, site, (uint64_t)(row * H + col) >> 2, f);
      o.x *= f[0]; o.y *= f[1]; o.z *= f[2]; o.w *= f[3];
    }
    Vec4<T>::st(y + col, o);
  }
  if (lane == 0) { *mean_out = mu; *rstd_out = rstd; }
}

template <class T>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gain, const T* __restrict__ bias,
                                                     T* __restrict__ y, float* __restrict__ stats, int R, int H, float eps, int stat_ld) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= R) return;
  const int nch = H / 4;
  float4 v[MAXCH];
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) if (c * 64 + lane < nch) v[c] = Vec4<T>::ld(x + (int64_t)row * H + 4 * (c * 64 + lane));
  ln_row<T>(v, nch, H, lane, gain, bias, eps, y + (int64_t)row * H, stats + row, stats + stat_ld + row);
}

template <class T>
__global__ __launch_bounds__(256) void embed_ln_fwd_kernel(const T* __restrict__ word, const T* __restrict__ pos,
                                                           const T* __restrict__ gain, const T* __restrict__ bias,
                                                           const int32_t* __restrict__ ids, T* __restrict__ e_pre, T* __restrict__ x0,
                                                           float* __restrict__ stats, int R, int L, int H, int V, float eps, DropCfg drop,
                                                           int stat_ld) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= R) return;
  int id = ids[row];
  id = id < 0 ? 0 : (id >= V ? V - 1 : id);  // ids are validated by contract; clamp keeps reads in bounds
  const int l = row % L;
  const int nch = H / 4;
  float4 v[MAXCH];
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) if (c * 64 + lane < nch) {
    const int col = 4 * (c * 64 + lane);
    const float4 a = Vec4<T>::ld(word + (int64_t)id * H + col), b = Vec4<T>::ld(pos + (int64_t)l * H + col);
    // the sum is rounded to the activation type because that is what the backward pass re-reads
    const float4 e = Vec4<T>::round(make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w));
    Vec4<T>::st(e_pre + (int64_t)row * H + col, e);
    v[c] = e;
  }
  ln_row<T>(v, nch, H, lane, gain, bias, eps, x0 + (int64_t)row * H, stats + row, stats + stat_ld + row, drop.thr ? &drop : nullptr,
            site_embedding(), row);
}

// ------------------------------------------------------------------------------------------
// LayerNorm backward.  Each wave walks rows with a fixed stride and keeps per-column partial
// sums of dy*xhat, dy and dx; blocks write partials, a second kernel adds them in block order.
// ------------------------------------------------------------------------------------------
// NC: 256-column slots per row that the registers hold (hidden <= 256 NC); EXACT: hidden == 256 NC, no slot is partly used.
template <class T, int drop_mode, int NC, bool EXACT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NC <= 3 ? 4 : 2, 4))) void ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x, const float* __restrict__ stats,
                                                     const T* __restrict__ gain, T* __restrict__ dx, float* __restrict__ partials,
                                                     int R, int H, DropCfg drop, uint32_t site, T* __restrict__ dxm) {
  // drop_mode 1: dy is the gradient of a dropped OUTPUT of this LayerNorm and is masked as it is read.
  // drop_mode 2: dx feeds a dropped branch (site) besides a residual path: dxm gets the masked copy and the
  //              column sums of dx (the bias gradient of that branch) are taken over the masked values.
  __shared__ float4 red[4][NC * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nch = H / 4;
  const float inv_h = 1.0f / (float)H;
  float4 g[NC], ag[NC], ab[NC], as[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    ag[c] = ab[c] = as[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    g[c] = (EXACT || c * 64 + lane < nch) ? Vec4<T>::ld(gain + 4 * (c * 64 + lane)) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  // Rows of one wave are software-pipelined: the loads of the wave's next row are issued before the
  // reductions of the current one, so two rows are in flight per wave.
  const int stride = gridDim.x * 4;
  int row = blockIdx.x * 4 + wave;
  float4 nx[NC], ndy[NC];
  float nmu = 0.f, nrstd = 0.f;
  if (row < R) {
    nmu = stats[row]; nrstd = stats[R + row];
#pragma unroll
    for (int c = 0; c < NC; ++c) if (EXACT || c * 64 + lane < nch) {
      const int64_t o = (int64_t)row * H + 4 * (c * 64 + lane);
      nx[c] = Vec4<T>::ld(x + o);
      ndy[c] = Vec4<T>::ld(dy + o);
    }
  }
  for (; row < R; row += stride) {
    const float mu = nmu, rstd = nrstd;
    float4 xh[NC], dyv[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) { xh[c] = nx[c]; dyv[c] = ndy[c]; }
    if (drop_mode == 1) {
#pragma unroll
      for (int c = 0; c < NC; ++c) if (EXACT || c * 64 + lane < nch) {
        float f[4];
        drop_factors4(drop, site, (uint64_t)((int64_t)row * H + 4 * (c * 64 + lane)) >> 2, f);
        dyv[c].x *= f[0]; dyv[c].y *= f[1]; dyv[c].z *= f[2]; dyv[c].w *= f[3];
      }
    }
    const int next = row + stride;
    if (next < R) {
      nmu = stats[next]; nrstd = stats[R + next];
#pragma unroll
      for (int c = 0; c < NC; ++c) if (EXACT || c * 64 + lane < nch) {
        const int64_t o = (int64_t)next * H + 4 * (c * 64 + lane);
        nx[c] = Vec4<T>::ld(x + o);
        ndy[c] = Vec4<T>::ld(dy + o);
      }
    }
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NC; ++c) if (EXACT || c * 64 + lane < nch) {
      const float4 xv = xh[c];
      xh[c] = make_float4((xv.x - mu) * rstd, (xv.y - mu) * rstd, (xv.z - mu) * rstd, (xv.w - mu) * rstd);
      const float4 d = make_float4(dyv[c].x * g[c].x, dyv[c].y * g[c].y, dyv[c].z * g[c].z, dyv[c].w * g[c].w);
      s1 += (d.x + d.y) + (d.z + d.w);
      s2 += (d.x * xh[c].x + d.y * xh[c].y) + (d.z * xh[c].z + d.w * xh[c].w);
    }
    s1 = wave_sum(s1) * inv_h;
    s2 = wave_sum(s2) * inv_h;
#pragma unroll
    for (int c = 0; c < NC; ++c) if (EXACT || c * 64 + lane < nch) {
      float4 d;
      d.x = rstd * (dyv[c].x * g[c].x - s1 - xh[c].x * s2); d.y = rstd * (dyv[c].y * g[c].y - s1 - xh[c].y * s2);
      d.z = rstd * (dyv[c].z * g[c].z - s1 - xh[c].z * s2); d.w = rstd * (dyv[c].w * g[c].w - s1 - xh[c].w * s2);
      float4 dm = d;
      d = Vec4<T>::round(d);
      Vec4<T>::st(dx + (int64_t)row * H + 4 * (c * 64 + lane), d);
      if (drop_mode == 2) {
        float f[4];
        drop_factors4(drop, site, (uint64_t)((int64_t)row * H + 4 * (c * 64 + lane)) >> 2, f);
        dm = Vec4<T>::round(make_float4(dm.x * f[0], dm.y * f[1], dm.z * f[2], dm.w * f[3]));
        Vec4<T>::st(dxm + (int64_t)row * H + 4 * (c * 64 + lane), dm);
      } else {
        dm = d;
      }
      ag[c].x += dyv[c].x * xh[c].x; ag[c].y += dyv[c].y * xh[c].y; ag[c].z += dyv[c].z * xh[c].z; ag[c].w += dyv[c].w * xh[c].w;
      ab[c].x += dyv[c].x; ab[c].y += dyv[c].y; ab[c].z += dyv[c].z; ab[c].w += dyv[c].w;
      as[c].x += dm.x; as[c].y += dm.y; as[c].z += dm.z; as[c].w += dm.w;
    }
  }
  // combine the four waves of the block in wave order, one quantity at a time
  float* out = partials + (int64_t)blockIdx.x * 3 * H;
#pragma unroll
  for (int q = 0; q < 3; ++q) {
#pragma unroll
    for (int c = 0; c < NC; ++c) if (EXACT || c * 64 + lane < nch) red[wave][c * 64 + lane] = (q == 0) ? ag[c] : (q == 1 ? ab[c] : as[c]);
    __syncthreads();
    for (int ch = threadIdx.x; ch < nch; ch += 256) {
      const float4 a = red[0][ch], b = red[1][ch], c2 = red[2][ch], d = red[3][ch];
      float4 t;
      t.x = ((a.x + b.x) + c2.x) + d.x; t.y = ((a.y + b.y) + c2.y) + d.y;
      t.z = ((a.z + b.z) + c2.z) + d.z; t.w = ((a.w + b.w) + c2.w) + d.w;
      *(float4*)(out + q * H + 4 * ch) = t;
    }
    __syncthreads();
  }
}

// out_q[col] = beta*out_q[col] + sum_p partials[p*pstride + q*qstride + col] for up to three quantities q
// (blockIdx.y).  Fixed summation tree: wave w of the block's 16 waves adds p = w, w+16, w+32, ... in
// ascending order, then the wave sums are added in wave order.
constexpr int SP_WAVES = 16;
__global__ __launch_bounds__(64 * SP_WAVES) void sum_partials_kernel(const float* __restrict__ partials, int np, int64_t pstride,
                                                                    int64_t qstride, int C, float* __restrict__ out0,
                                                                    float* __restrict__ out1, float* __restrict__ out2, float beta) {
  __shared__ float red[SP_WAVES][64];
  const int q = blockIdx.y;
  float* out = q == 0 ? out0 : (q == 1 ? out1 : out2);
  if (!out) return;                                   // uniform over the block
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (col < C) {
    const float* src = partials + q * qstride + col;
    int p = wave;
    for (; p + 7 * SP_WAVES < np; p += 8 * SP_WAVES) {
      float a[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) a[u] = src[(int64_t)(p + SP_WAVES * u) * pstride];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += a[u];
    }
    for (; p < np; p += SP_WAVES) s += src[(int64_t)p * pstride];
  }
  red[wave][lane] = s;
  __syncthreads();
  if (wave == 0 && col < C) {
    float t = red[0][lane];
#pragma unroll
    for (int w = 1; w < SP_WAVES; ++w) t += red[w][lane];
    out[col] = (beta != 0.f) ? beta * out[col] + t : t;
  }
}

// ------------------------------------------------------------------------------------------
// column sums of a [R, C] matrix
// ------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void colsum_kernel(const T* __restrict__ x, int64_t ldx, int R, int C, int rows_per_chunk,
                                                     float* __restrict__ partials) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= C) return;
  const int r0 = blockIdx.y * rows_per_chunk;
  const int r1 = min(R, r0 + rows_per_chunk);
  float s = 0.f;
  int r = r0;
  for (; r + 8 <= r1; r += 8) {
    float a[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] = to_f(x[(int64_t)(r + u) * ldx + col]);
#pragma unroll
    for (int u = 0; u < 8; ++u) s += a[u];
  }
  for (; r < r1; ++r) s += to_f(x[(int64_t)r * ldx + col]);
  partials[(int64_t)blockIdx.y * C + col] = s;
}

// ------------------------------------------------------------------------------------------
// rows: gather, scatter, zero fill, GELU
// ------------------------------------------------------------------------------------------
template <class T>
__global__ void gather_rows_kernel(const T* __restrict__ src, const int32_t* __restrict__ idx, int M, int H, T* __restrict__ dst, int scatter) {
  const int m = blockIdx.x;
  const int64_t r = idx[m];
  for (int c = threadIdx.x; c < H; c += blockDim.x) {
    if (scatter) dst[r * H + c] = src[(int64_t)m * H + c];
    else dst[(int64_t)m * H + c] = src[r * H + c];
  }
}

template <class T>
__global__ __launch_bounds__(256) void fill_value_kernel(T* p, size_t n, float value) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = from_f<T>(value);
}
__global__ void fill_bytes_kernel(unsigned char* p, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

__global__ void fill_zero_kernel(uint4* p, size_t n16, unsigned char* tail, size_t ntail) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t k = i; k < n16; k += stride) p[k] = make_uint4(0, 0, 0, 0);
  if (i < ntail) tail[i] = 0;
}

template <class T>
__global__ void gelu_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ pre, T* __restrict__ dx, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dx[i] = from_f<T>(to_f(dy[i]) * gelu_grad_f(to_f(pre[i])));
}
template <class T>
__global__ void gelu_fwd_kernel(const T* __restrict__ x, T* __restrict__ y, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) y[i] = from_f<T>(gelu_f(to_f(x[i])));
}

// ------------------------------------------------------------------------------------------
// cross-entropy over fp32 logits: one block per target row
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ float block_reduce(float v, bool is_max, float* sh) {
  v = is_max ? wave_max(v) : wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  float r = sh[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = is_max ? fmaxf(r, sh[w]) : r + sh[w];
  return r;
}

template <class T>
__global__ __launch_bounds__(256) void ce_loss_kernel(const float* __restrict__ logits, int64_t ldl, const int32_t* __restrict__ labels,
                                                      int V, T* __restrict__ dlogits, float* __restrict__ row_loss) {
  __shared__ float sh[8];
  const int m = blockIdx.x;
  const float* z = logits + (int64_t)m * ldl;
  float mx = -3.0e38f;
  for (int v = threadIdx.x; v < V; v += 256) mx = fmaxf(mx, z[v]);
  mx = block_reduce(mx, true, sh);
  float se = 0.f;
  for (int v = threadIdx.x; v < V; v += 256) se += __expf(z[v] - mx);
  se = block_reduce(se, false, sh);
  const float lse = mx + logf(se);
  int lab = labels[m];
  lab = lab < 0 ? 0 : (lab >= V ? V - 1 : lab);
  if (threadIdx.x == 0) row_loss[m] = lse - z[lab];
  T* d = dlogits + (int64_t)m * ldl;
  for (int v = threadIdx.x; v < (int)ldl; v += 256) {
    float p = 0.f;
    if (v < V) p = __expf(z[v] - lse) - (v == lab ? 1.0f : 0.0f);
    d[v] = from_f<T>(p);
  }
}

// The same with the whole row held in registers (one read of the logits): 1024 threads, up to eight
// 4-element chunks per thread, so rows of up to 32768 padded columns; row stride a multiple of 4.
// The padding columns of the logits buffer are never read; those of dlogits are written as zeros.
constexpr int CE_NT = 1024, CE_MAXCH = 8;
template <class T>
__global__ __launch_bounds__(CE_NT) void ce_loss_row_kernel(const float* __restrict__ logits, int64_t ldl, const int32_t* __restrict__ labels,
                                                           int V, T* __restrict__ dlogits, float* __restrict__ row_loss) {
  __shared__ float sh[CE_NT / 64];
  const int m = blockIdx.x;
  const float* z = logits + (int64_t)m * ldl;
  const int nch = (int)(ldl / 4);
  float4 x[CE_MAXCH];
  float mx = -3.0e38f;
#pragma unroll
  for (int c = 0; c < CE_MAXCH; ++c) {
    const int ch = threadIdx.x + c * CE_NT, v = ch * 4;
    x[c] = make_float4(-3.0e38f, -3.0e38f, -3.0e38f, -3.0e38f);
    if (ch < nch) {
      if (v + 3 < V) x[c] = *(const float4*)(z + v);
      else {
        if (v < V) x[c].x = z[v];
        if (v + 1 < V) x[c].y = z[v + 1];
        if (v + 2 < V) x[c].z = z[v + 2];
      }
    }
    mx = fmaxf(mx, fmaxf(fmaxf(x[c].x, x[c].y), fmaxf(x[c].z, x[c].w)));
  }
  mx = block_reduce(mx, true, sh);
  float se = 0.f;
#pragma unroll
  for (int c = 0; c < CE_MAXCH; ++c)     // excluded positions hold -3e38: their exponential is exactly 0
    se += (__expf(x[c].x - mx) + __expf(x[c].y - mx)) + (__expf(x[c].z - mx) + __expf(x[c].w - mx));
  se = block_reduce(se, false, sh);
  const float lse = mx + logf(se);
  int lab = labels[m];
  lab = lab < 0 ? 0 : (lab >= V ? V - 1 : lab);
  if (threadIdx.x == 0) row_loss[m] = lse - z[lab];
  T* d = dlogits + (int64_t)m * ldl;
#pragma unroll
  for (int c = 0; c < CE_MAXCH; ++c) {
    const int ch = threadIdx.x + c * CE_NT, v = ch * 4;
    if (ch < nch) {
      float4 p;
      p.x = __expf(x[c].x - lse) - (v == lab ? 1.0f : 0.0f);
      p.y = __expf(x[c].y - lse) - (v + 1 == lab ? 1.0f : 0.0f);
      p.z = __expf(x[c].z - lse) - (v + 2 == lab ? 1.0f : 0.0f);
      p.w = __expf(x[c].w - lse) - (v + 3 == lab ? 1.0f : 0.0f);
      Vec4<T>::st(d + v, p);
    }
  }
}

// fixed-order sum of n floats by one block
__global__ __launch_bounds__(256) void sum_vector_kernel(const float* __restrict__ x, int n, float* __restrict__ out) {
  __shared__ float sh[8];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += x[i];
  s = block_reduce(s, false, sh);
  if (threadIdx.x == 0) *out = s;
}

// ------------------------------------------------------------------------------------------
// embedding backward
// ------------------------------------------------------------------------------------------
// position table: g_pos[l, :] = beta*g_pos[l, :] + sum_b de[b, l, :]; rows l >= L get beta*old
template <class T>
__global__ void pos_grad_kernel(const T* __restrict__ de, int B, int L, int H, int max_pos, float* __restrict__ g_pos, float beta) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)max_pos * H) return;
  const int l = (int)(i / H), c = (int)(i % H);
  float s = 0.f;
  if (l < L) for (int b = 0; b < B; ++b) s += to_f(de[((int64_t)b * L + l) * H + c]);
  g_pos[i] = (beta != 0.f) ? beta * g_pos[i] + s : s;
}

// Stable LSD radix sort of (id, position) by id, 4 bits per pass, one block of 512 threads.
// Thread t owns the contiguous slice [t*per, (t+1)*per) in every pass, which keeps equal keys in
// their input order.  Result in (key_out, val_out) after an even number of passes.
__global__ __launch_bounds__(512) void sort_ids_kernel(const int32_t* __restrict__ ids, int T, int V, int32_t* k0, int32_t* v0,
                                                        int32_t* k1, int32_t* v1, int npass) {
  constexpr int NT = 512;
  __shared__ int cnt[16 * NT];
  __shared__ int wsum[NT / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int per = (T + NT - 1) / NT;
  const int beg = min(T, tid * per), end = min(T, beg + per);
  for (int pass = 0; pass < npass; ++pass) {
    const int shift = 4 * pass;
    const int32_t* kin = (pass & 1) ? k1 : k0;
    const int32_t* vin = (pass & 1) ? v1 : v0;
    int32_t* kout = (pass & 1) ? k0 : k1;
    int32_t* vout = (pass & 1) ? v0 : v1;
    for (int d = 0; d < 16; ++d) cnt[d * NT + tid] = 0;
    for (int i = beg; i < end; ++i) {
      int key;
      if (pass == 0) { key = ids[i]; key = key < 0 ? 0 : (key >= V ? V - 1 : key); } else key = kin[i];
      cnt[((key >> shift) & 15) * NT + tid]++;
    }
    __syncthreads();
    // exclusive scan over the 16*NT counters (digit-major): thread owns 16 consecutive entries
    int loc[16], s = 0;
    for (int j = 0; j < 16; ++j) { loc[j] = s; s += cnt[tid * 16 + j]; }
    int incl = s;
    for (int o = 1; o < 64; o <<= 1) { int t = __shfl_up(incl, o); if (lane >= o) incl += t; }
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    int base = 0;
    for (int w = 0; w < wave; ++w) base += wsum[w];
    base += incl - s;
    __syncthreads();
    for (int j = 0; j < 16; ++j) cnt[tid * 16 + j] = base + loc[j];
    __syncthreads();
    for (int i = beg; i < end; ++i) {
      int key, val;
      if (pass == 0) { key = ids[i]; key = key < 0 ? 0 : (key >= V ? V - 1 : key); val = i; } else { key = kin[i]; val = vin[i]; }
      const int pos = cnt[((key >> shift) & 15) * NT + tid]++;
      kout[pos] = key; vout[pos] = val;
    }
    __threadfence_block();
    __syncthreads();
  }
}

// Segmented sum over the sorted token list in chunks of CH entries, one wave per chunk.
// Runs that lie wholly inside a chunk are added to g_word directly (no other wave touches that
// row).  A run that continues into a neighbouring chunk is written to carry[chunk][0] (run open
// to the left, or spanning the whole chunk) or carry[chunk][1] (run open to the right only).
// All CH gradient rows of a chunk are fetched before any is used, so the loads overlap.
constexpr int CH = 8;
template <class T>
__global__ __launch_bounds__(256) void word_grad_chunks_kernel(const T* __restrict__ de, const int32_t* __restrict__ skey,
                                                               const int32_t* __restrict__ sval, int Ttok, int H,
                                                               float* __restrict__ g_word, float* __restrict__ carry) {
  const int lane = threadIdx.x & 63;
  const int chunk = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int i0 = chunk * CH;
  if (i0 >= Ttok) return;
  const int n = min(CH, Ttok - i0);
  const int nch = H / 4;
  int key[CH];
  float4 rowv[CH][MAXCH];
#pragma unroll
  for (int e = 0; e < CH; ++e) {
    key[e] = (e < n) ? skey[i0 + e] : -1;
    const int64_t t = (e < n) ? sval[i0 + e] : 0;
#pragma unroll
    for (int c = 0; c < MAXCH; ++c)
      rowv[e][c] = (e < n && c * 64 + lane < nch) ? Vec4<T>::ld(de + t * H + 4 * (c * 64 + lane)) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const int key_left = (i0 > 0) ? skey[i0 - 1] : -1;
  const int key_right = (i0 + n < Ttok) ? skey[i0 + n] : -1;
  float4 acc[MAXCH];
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
  bool run_from_start = true;
#pragma unroll
  for (int e = 0; e < CH; ++e) {
    if (e < n) {
#pragma unroll
      for (int c = 0; c < MAXCH; ++c) { acc[c].x += rowv[e][c].x; acc[c].y += rowv[e][c].y; acc[c].z += rowv[e][c].z; acc[c].w += rowv[e][c].w; }
      const bool last = (e + 1 == n);
      const bool run_ends = last || key[(e + 1) % CH] != key[e];
      if (run_ends) {
        const bool open_left = run_from_start && key_left == key[e];
        const bool open_right = last && key_right == key[e];
        float* dst;
        bool add;
        if (open_left) { dst = carry + ((int64_t)chunk * 2 + 0) * H; add = false; }
        else if (open_right) { dst = carry + ((int64_t)chunk * 2 + 1) * H; add = false; }
        else { dst = g_word + (int64_t)key[e] * H; add = true; }
#pragma unroll
        for (int c = 0; c < MAXCH; ++c) if (c * 64 + lane < nch) {
          float4* d4 = (float4*)(dst + 4 * (c * 64 + lane));
          float4 o = acc[c];
          if (add) { const float4 old = *d4; o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w; }
          *d4 = o;
          acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        run_from_start = false;
      }
    }
  }
}

// Joins the runs that cross chunk borders: the wave of the chunk in which such a run STARTS adds
// its right-open piece and every following left-open piece, in chunk order, then updates g_word.
// The end of the run is found by bisection in the sorted keys, after which the pieces are fetched
// eight at a time.
__global__ __launch_bounds__(256) void word_grad_join_kernel(const int32_t* __restrict__ skey, int Ttok, int H,
                                                             float* __restrict__ g_word, const float* __restrict__ carry) {
  const int lane = threadIdx.x & 63;
  const int chunk = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int i0 = chunk * CH;
  if (i0 >= Ttok) return;
  const int i1 = min(Ttok, i0 + CH);
  if (i1 >= Ttok) return;                       // nothing to the right
  const int key = skey[i1 - 1];
  if (skey[i1] != key) return;                  // last run is not open to the right
  // a run that also reaches back into the previous chunk is a continuation: its starting chunk handles it
  if (skey[i0] == key && i0 > 0 && skey[i0 - 1] == key) return;
  // last index of the run: largest j with skey[j] == key (keys ascend)
  int lo = i1, hi = Ttok - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (skey[mid] == key) lo = mid; else hi = mid - 1;
  }
  const int last_chunk = lo / CH;               // every chunk in (chunk, last_chunk] starts with this key
  const int nch = H / 4;
  float4 acc[MAXCH];
#pragma unroll
  for (int c = 0; c < MAXCH; ++c)
    acc[c] = (c * 64 + lane < nch) ? *(const float4*)(carry + ((int64_t)chunk * 2 + 1) * H + 4 * (c * 64 + lane)) : make_float4(0.f, 0.f, 0.f, 0.f);
  for (int ch = chunk + 1; ch <= last_chunk; ch += 8) {
    float4 v[8][MAXCH];
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int c = 0; c < MAXCH; ++c)
        v[u][c] = (ch + u <= last_chunk && c * 64 + lane < nch)
                      ? *(const float4*)(carry + ((int64_t)(ch + u) * 2 + 0) * H + 4 * (c * 64 + lane)) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int c = 0; c < MAXCH; ++c) { acc[c].x += v[u][c].x; acc[c].y += v[u][c].y; acc[c].z += v[u][c].z; acc[c].w += v[u][c].w; }
  }
#pragma unroll
  for (int c = 0; c < MAXCH; ++c) if (c * 64 + lane < nch) {
    float4* d4 = (float4*)(g_word + (int64_t)key * H + 4 * (c * 64 + lane));
    float4 o = *d4;
    o.x += acc[c].x; o.y += acc[c].y; o.z += acc[c].z; o.w += acc[c].w;
    *d4 = o;
  }
}

}  // namespace

// ==========================================================================================
// launchers
// ==========================================================================================
#define LAUNCH_CHECK(ctx, what)                                                                        \
  do {                                                                                                 \
    hipError_t e_ = hipGetLastError();                                                                 \
    if (e_ != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e_)); \
  } while (0)

static inline Profiler* prof_of(hs_ctx* ctx) { return ctx ? ctx->prof : nullptr; }

hs_status launch_layernorm_fwd(hs_ctx* ctx, int dtype, const void* x, const void* gain, const void* bias, void* y, float* stats,
                               int R, int H, float eps, hipStream_t s, int stat_ld) {
  if (R <= 0) return HS_OK;
  if (stat_ld <= 0) stat_ld = R;      // the reciprocal standard deviations start stat_ld floats after the means
  KScope scope(prof_of(ctx), KC_LN_FWD, 8.0 * R * H, 2.0 * R * H * esize(dtype), s);
  dim3 grid((R + 3) / 4);
  if (dtype == HS_BF16) hipLaunchKernelGGL(ln_fwd_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)x, (const bf16*)gain, (const bf16*)bias, (bf16*)y, stats, R, H, eps, stat_ld);
  else hipLaunchKernelGGL(ln_fwd_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (const float*)gain, (const float*)bias, (float*)y, stats, R, H, eps, stat_ld);
  LAUNCH_CHECK(ctx, "layernorm_fwd");
  return HS_OK;
}

// Blocks of ln_bwd_kernel: eight rows per block (two per wave, both in flight at once) up to the number of blocks
// that are resident together, which the kernel's register use sets: four per CU up to 768 columns, three beyond.
static int ln_bwd_blocks(int R, int H) {
  const int cap = H <= 768 ? 1024 : 768;
  const int nb = (R + 7) / 8;
  return nb < 1 ? 1 : (nb > cap ? cap : nb);
}
size_t layernorm_bwd_scratch(int R, int H) { return align_up((size_t)ln_bwd_blocks(R, H) * 3 * H * sizeof(float), 256); }

// main kernel: dx and the per-block partial column sums
hs_status launch_layernorm_bwd_rows(hs_ctx* ctx, int dtype, const void* dy, const void* x, const float* stats, const void* gain, void* dx,
                                    int R, int H, void* partials, hipStream_t s, const DropCfg* drop, uint32_t site, int drop_mode,
                                    void* dxm) {
  if (R <= 0) return HS_OK;
  const int nb = ln_bwd_blocks(R, H);
  KScope scope(prof_of(ctx), KC_LN_BWD, 14.0 * R * H, 3.0 * R * H * esize(dtype), s);
  DropCfg d{0u, 1.0f, 0u, 0u, 0u};
  if (drop && drop->thr && drop_mode) d = *drop; else drop_mode = 0;
  if (drop_mode == 2 && !dxm) return hs_fail(ctx, HS_ERR_INVALID_ARG, "layernorm_bwd: masked output buffer missing");
  const int nc = H <= 512 ? 2 : (H + 255) / 256;      // the NC the kernel is built with
  const bool exact = H == 256 * nc;
#define HS_LN_BWD4(TT, MODE, NC, EX) hipLaunchKernelGGL((ln_bwd_kernel<TT, MODE, NC, EX>), dim3(nb), dim3(256), 0, s, (const TT*)dy, (const TT*)x, stats, \
                                                       (const TT*)gain, (TT*)dx, (float*)partials, R, H, d, site, (TT*)dxm)
#define HS_LN_BWD3(TT, MODE, NC) do { if (exact) HS_LN_BWD4(TT, MODE, NC, true); else HS_LN_BWD4(TT, MODE, NC, false); } while (0)
#define HS_LN_BWD(TT, MODE) do { if (nc == 2) HS_LN_BWD3(TT, MODE, 2); else if (nc == 3) HS_LN_BWD3(TT, MODE, 3); else HS_LN_BWD3(TT, MODE, 4); } while (0)
  if (dtype == HS_BF16) { if (drop_mode == 0) HS_LN_BWD(bf16, 0); else if (drop_mode == 1) HS_LN_BWD(bf16, 1); else HS_LN_BWD(bf16, 2); }
  else { if (drop_mode == 0) HS_LN_BWD(float, 0); else if (drop_mode == 1) HS_LN_BWD(float, 1); else HS_LN_BWD(float, 2); }
#undef HS_LN_BWD4
#undef HS_LN_BWD3
#undef HS_LN_BWD
  LAUNCH_CHECK(ctx, "layernorm_bwd");
  return HS_OK;
}
// fixed-order sum of the partials into the three gradient vectors (may run on another stream)
hs_status launch_layernorm_bwd_cols(hs_ctx* ctx, const void* partials, float* d_gain, float* d_bias, float* d_colsum, float beta, int R, int H,
                                    hipStream_t s) {
  if (R <= 0 || !(d_gain || d_bias || d_colsum)) return HS_OK;
  KScope scope(prof_of(ctx), KC_LN_BWD, 0.0, 0.0, s);
  hipLaunchKernelGGL(sum_partials_kernel, dim3((H + 63) / 64, 3), dim3(64 * SP_WAVES), 0, s, (const float*)partials, ln_bwd_blocks(R, H), (int64_t)3 * H,
                     (int64_t)H, H, d_gain, d_bias, d_colsum, beta);
  LAUNCH_CHECK(ctx, "layernorm_bwd finalize");
  return HS_OK;
}
hs_status launch_layernorm_bwd(hs_ctx* ctx, int dtype, const void* dy, const void* x, const float* stats, const void* gain, void* dx,
                               float* d_gain, float* d_bias, float* d_colsum, float beta, int R, int H, void* partials, hipStream_t s,
                               const DropCfg* drop, uint32_t site, int drop_mode, void* dxm) {
  hs_status st = launch_layernorm_bwd_rows(ctx, dtype, dy, x, stats, gain, dx, R, H, partials, s, drop, site, drop_mode, dxm);
  if (st != HS_OK) return st;
  return launch_layernorm_bwd_cols(ctx, partials, d_gain, d_bias, d_colsum, beta, R, H, s);
}

hs_status launch_embed_ln_fwd(hs_ctx* ctx, int dtype, const void* word, const void* pos, const void* gain, const void* bias,
                              const int32_t* ids, void* e_pre, void* x0, float* stats, int B, int L, int H, int V, float eps, hipStream_t s,
                              const DropCfg* drop, int stat_ld) {
  const DropCfg dcfg = (drop && drop->thr) ? *drop : DropCfg{0u, 1.0f, 0u, 0u, 0u};
  if (stat_ld <= 0) stat_ld = B * L;
  const int R = B * L;
  if (R <= 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_EMBED, 10.0 * R * H, 4.0 * R * H * esize(dtype), s);
  dim3 grid((R + 3) / 4);
  if (dtype == HS_BF16) hipLaunchKernelGGL(embed_ln_fwd_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)word, (const bf16*)pos, (const bf16*)gain, (const bf16*)bias, ids, (bf16*)e_pre, (bf16*)x0, stats, R, L, H, V, eps, dcfg, stat_ld);
  else hipLaunchKernelGGL(embed_ln_fwd_kernel<float>, grid, dim3(256), 0, s, (const float*)word, (const float*)pos, (const float*)gain, (const float*)bias, ids, (float*)e_pre, (float*)x0, stats, R, L, H, V, eps, dcfg, stat_ld);
  LAUNCH_CHECK(ctx, "embed_ln_fwd");
  return HS_OK;
}

// scratch for the word-embedding gradient: 4 int arrays [T] + carry [chunks][2][H] floats
size_t embed_bwd_scratch(int T, int H) {
  const size_t chunks = ((size_t)T + CH - 1) / CH;
  return align_up(4 * (size_t)T * sizeof(int32_t), 256) + align_up(chunks * 2 * H * sizeof(float), 256);
}

// stable sort of the token ids (keys) with their positions (values) into the first two arrays of `scratch`; needs only the
// ids, so it can run ahead of the gradient that launch_embed_bwd scatters
hs_status launch_embed_sort(hs_ctx* ctx, const int32_t* ids, int T, int V, void* scratch, hipStream_t s) {
  if (T <= 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_EMBED, 0.0, 16.0 * T, s);
  int32_t* k0 = (int32_t*)scratch;
  int32_t* v0 = k0 + T; int32_t* k1 = v0 + T; int32_t* v1 = k1 + T;
  int bits = 1;
  while ((1 << bits) < V) ++bits;
  int npass = (bits + 3) / 4;
  if (npass & 1) ++npass;  // an even number of passes leaves the result in (k0, v0)
  hipLaunchKernelGGL(sort_ids_kernel, dim3(1), dim3(512), 0, s, ids, T, V, k0, v0, k1, v1, npass);
  LAUNCH_CHECK(ctx, "sort_ids");
  return HS_OK;
}

hs_status launch_embed_bwd(hs_ctx* ctx, int dtype, const void* de, const int32_t* ids, int B, int L, int H, int V, int max_pos,
                           float* g_word, float* g_pos, float beta_pos, void* scratch, hipStream_t s, bool sorted) {
  const int T = B * L;
  if (T <= 0) return HS_OK;
  if (!sorted) { hs_status st = launch_embed_sort(ctx, ids, T, V, scratch, s); if (st != HS_OK) return st; }
  KScope scope(prof_of(ctx), KC_EMBED, 2.0 * T * H, (double)T * H * (2.0 * esize(dtype) + 8.0) + 8.0 * max_pos * H, s);
  if (g_pos) {     // a model with a fixed position table has no position gradient
    const int64_t n = (int64_t)max_pos * H;
    dim3 grid((unsigned)((n + 255) / 256));
    if (dtype == HS_BF16) hipLaunchKernelGGL(pos_grad_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)de, B, L, H, max_pos, g_pos, beta_pos);
    else hipLaunchKernelGGL(pos_grad_kernel<float>, grid, dim3(256), 0, s, (const float*)de, B, L, H, max_pos, g_pos, beta_pos);
    LAUNCH_CHECK(ctx, "pos_grad");
  }
  int32_t* k0 = (int32_t*)scratch;
  int32_t* v0 = k0 + T;
  float* carry = (float*)((char*)scratch + align_up(4 * (size_t)T * sizeof(int32_t), 256));
  const int chunks = (T + CH - 1) / CH;
  dim3 grid((chunks + 3) / 4);
  if (dtype == HS_BF16) hipLaunchKernelGGL(word_grad_chunks_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)de, k0, v0, T, H, g_word, carry);
  else hipLaunchKernelGGL(word_grad_chunks_kernel<float>, grid, dim3(256), 0, s, (const float*)de, k0, v0, T, H, g_word, carry);
  LAUNCH_CHECK(ctx, "word_grad_chunks");
  hipLaunchKernelGGL(word_grad_join_kernel, grid, dim3(256), 0, s, k0, T, H, g_word, carry);
  LAUNCH_CHECK(ctx, "word_grad_join");
  return HS_OK;
}

static int colsum_chunks(int R) { int n = (R + 31) / 32; return n < 1 ? 1 : (n > 256 ? 256 : n); }
size_t colsum_scratch(int R, int C) { return align_up((size_t)colsum_chunks(R) * C * sizeof(float), 256); }

hs_status launch_colsum(hs_ctx* ctx, int dtype, const void* x, int64_t ldx, int R, int C, float* out, float beta, void* partials, hipStream_t s) {
  if (C <= 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_COLSUM, (double)R * C, (double)R * C * esize(dtype), s);
  const int nch = colsum_chunks(R);
  const int rpc = (R + nch - 1) / nch;
  dim3 grid((C + 255) / 256, nch);
  if (dtype == HS_BF16) hipLaunchKernelGGL(colsum_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)x, ldx, R, C, rpc, (float*)partials);
  else hipLaunchKernelGGL(colsum_kernel<float>, grid, dim3(256), 0, s, (const float*)x, ldx, R, C, rpc, (float*)partials);
  LAUNCH_CHECK(ctx, "colsum");
  hipLaunchKernelGGL(sum_partials_kernel, dim3((C + 63) / 64, 1), dim3(64 * SP_WAVES), 0, s, (const float*)partials, nch, (int64_t)C, (int64_t)0, C, out,
                     (float*)nullptr, (float*)nullptr, beta);
  LAUNCH_CHECK(ctx, "colsum finalize");
  return HS_OK;
}

static hs_status rows_move(hs_ctx* ctx, int dtype, const void* src, const int32_t* idx, int M, int H, void* dst, int scatter, hipStream_t s) {
  if (M <= 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_ELEMWISE, 0.0, 2.0 * M * H * esize(dtype), s);
  if (dtype == HS_BF16) hipLaunchKernelGGL(gather_rows_kernel<bf16>, dim3(M), dim3(128), 0, s, (const bf16*)src, idx, M, H, (bf16*)dst, scatter);
  else hipLaunchKernelGGL(gather_rows_kernel<float>, dim3(M), dim3(128), 0, s, (const float*)src, idx, M, H, (float*)dst, scatter);
  LAUNCH_CHECK(ctx, "gather/scatter rows");
  return HS_OK;
}
hs_status launch_gather_rows(hs_ctx* ctx, int dtype, const void* src, const int32_t* idx, int M, int H, void* dst, hipStream_t s) {
  return rows_move(ctx, dtype, src, idx, M, H, dst, 0, s);
}
hs_status launch_scatter_rows(hs_ctx* ctx, int dtype, const void* src, const int32_t* idx, int M, int H, void* dst, hipStream_t s) {
  return rows_move(ctx, dtype, src, idx, M, H, dst, 1, s);
}

hs_status launch_fill_zero(hs_ctx* ctx, void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_ELEMWISE, 0.0, (double)bytes, s);
  if ((uintptr_t)p % 16) {
    if (bytes > 4096) return hs_fail(ctx, HS_ERR_INVALID_ARG, "fill_zero: large buffers must be 16-byte aligned");
    hipLaunchKernelGGL(fill_bytes_kernel, dim3((unsigned)((bytes + 255) / 256)), dim3(256), 0, s, (unsigned char*)p, bytes);
    LAUNCH_CHECK(ctx, "fill_bytes");
    return HS_OK;
  }
  const size_t n16 = bytes / 16, ntail = bytes % 16;
  size_t blocks = (n16 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)p, n16, (unsigned char*)p + n16 * 16, ntail);
  LAUNCH_CHECK(ctx, "fill_zero");
  return HS_OK;
}

hs_status launch_fill_value(hs_ctx* ctx, int dtype, void* p, size_t n, float value, hipStream_t s) {
  if (n == 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_ELEMWISE, 0.0, (double)n * esize(dtype), s);
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == HS_BF16) hipLaunchKernelGGL(fill_value_kernel<bf16>, grid, dim3(256), 0, s, (bf16*)p, n, value);
  else hipLaunchKernelGGL(fill_value_kernel<float>, grid, dim3(256), 0, s, (float*)p, n, value);
  LAUNCH_CHECK(ctx, "fill_value");
  return HS_OK;
}

hs_status launch_gelu_fwd(hs_ctx* ctx, int dtype, const void* x, void* y, size_t n, hipStream_t s) {
  if (n == 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_ELEMWISE, 10.0 * n, 2.0 * n * esize(dtype), s);
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == HS_BF16) hipLaunchKernelGGL(gelu_fwd_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)x, (bf16*)y, n);
  else hipLaunchKernelGGL(gelu_fwd_kernel<float>, grid, dim3(256), 0, s, (const float*)x, (float*)y, n);
  LAUNCH_CHECK(ctx, "gelu_fwd");
  return HS_OK;
}
hs_status launch_gelu_bwd(hs_ctx* ctx, int dtype, const void* dy, const void* pre, void* dx, size_t n, hipStream_t s) {
  if (n == 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_ELEMWISE, 12.0 * n, 3.0 * n * esize(dtype), s);
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == HS_BF16) hipLaunchKernelGGL(gelu_bwd_kernel<bf16>, grid, dim3(256), 0, s, (const bf16*)dy, (const bf16*)pre, (bf16*)dx, n);
  else hipLaunchKernelGGL(gelu_bwd_kernel<float>, grid, dim3(256), 0, s, (const float*)dy, (const float*)pre, (float*)dx, n);
  LAUNCH_CHECK(ctx, "gelu_bwd");
  return HS_OK;
}

hs_status launch_ce_loss(hs_ctx* ctx, int dtype, const float* logits, int64_t ldl, const int32_t* labels, int M, int V, void* dlogits,
                         float* row_loss, float* loss_sum, hipStream_t s) {
  if (M <= 0) return HS_OK;
  KScope scope(prof_of(ctx), KC_LOSS, 4.0 * M * V, (double)M * V * (4.0 + esize(dtype)), s);
  const bool in_regs = (ldl % 4) == 0 && ldl <= (int64_t)4 * CE_NT * CE_MAXCH && ((uintptr_t)logits % 16) == 0 &&
                       ((uintptr_t)dlogits % 16) == 0;
  if (in_regs) {
    if (dtype == HS_BF16) hipLaunchKernelGGL(ce_loss_row_kernel<bf16>, dim3(M), dim3(CE_NT), 0, s, logits, ldl, labels, V, (bf16*)dlogits, row_loss);
    else hipLaunchKernelGGL(ce_loss_row_kernel<float>, dim3(M), dim3(CE_NT), 0, s, logits, ldl, labels, V, (float*)dlogits, row_loss);
  } else if (dtype == HS_BF16) hipLaunchKernelGGL(ce_loss_kernel<bf16>, dim3(M), dim3(256), 0, s, logits, ldl, labels, V, (bf16*)dlogits, row_loss);
  else hipLaunchKernelGGL(ce_loss_kernel<float>, dim3(M), dim3(256), 0, s, logits, ldl, labels, V, (float*)dlogits, row_loss);
  LAUNCH_CHECK(ctx, "ce_loss");
  hipLaunchKernelGGL(sum_vector_kernel, dim3(1), dim3(256), 0, s, (const float*)row_loss, M, loss_sum);
  LAUNCH_CHECK(ctx, "loss sum");
  return HS_OK;
}
