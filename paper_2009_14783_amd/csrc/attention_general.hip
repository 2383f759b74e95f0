// Softmax attention with separate query and key/value sequences (head dimension 64), forward and backward:
// the decoder's causal self-attention and its attention over the encoder output.  Queries, keys and values
// are row ranges of token-major matrices with their own row strides (head h = columns h*64 .. h*64+63);
// key j of sequence b takes part iff j < klens[b] and, when causal, j <= query index; queries at or beyond
// qlens[b] get zero gradients.  No dropout of the probabilities (the translation model drops sub-layer
// outputs only).
//
// bf16: MFMA kernels of the same shape as the self-attention ones (a wave owns 32 rows in registers and
// streams the other side through LDS in blocks of 64 rows; see attention_mfma.hip).  fp32: one thread per
// owned row, blocks of 64 streamed rows staged in LDS as fp32.
#include "attention_tiles.h"

namespace {

using namespace attn_tiles;

struct View {
  const void *q, *k, *v;      // first row of sequence 0
  int64_t ldq, ldkv;          // row strides in elements
  const int32_t *qlens, *klens;
  int Lq, Lk, A;
};

__device__ __forceinline__ int clamp_len(int n, int L) { return n < 1 ? 1 : (n > L ? L : n); }

// ------------------------------------------------------------------------------------------
// bf16 MFMA
// ------------------------------------------------------------------------------------------
template <bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void gen_fwd_mfma(View a, bf16* __restrict__ out, float* __restrict__ lse) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Vs[64 * LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int H = a.A * DH;
  const int klen = clamp_len(a.klens[b], a.Lk);
  const bf16* qb_ = (const bf16*)a.q + (int64_t)b * a.Lq * a.ldq + h * DH;
  const bf16* kb_ = (const bf16*)a.k + (int64_t)b * a.Lk * a.ldkv + h * DH;
  const bf16* vb_ = (const bf16*)a.v + (int64_t)b * a.Lk * a.ldkv + h * DH;
  const int q = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const int wave_qmax = blockIdx.x * 128 + wave * 32 + 31;
  const int kend = CAUSAL ? min(klen, (int)blockIdx.x * 128 + 128) : klen;      // block-uniform

  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qf[ks] = frag_rows_global(qb_, a.ldq, q, a.Lq, ks, lane);
  f32x16 o[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m2 = -1.0e30f, lsum = 0.f;

  for (int k0 = 0; k0 < kend; k0 += 64) {
    __syncthreads();
    stage64(Ks, kb_, a.ldkv, k0, klen, tid);
    stage64(Vs, vb_, a.ldkv, k0, klen, tid);
    __syncthreads();
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int kb = 32 * sub;
      if (k0 + kb < kend && (!CAUSAL || k0 + kb <= wave_qmax)) {
        f32x16 st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Ks, kb, ks, lane), qf[ks], st, 0, 0, 0);
        float mloc = -1.0e30f;
        bool okr[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + kb + tile_row(r, lane);
          okr[r] = key < klen && (!CAUSAL || key <= q);
          st[r] = okr[r] ? st[r] * SCALE2 : -1.0e30f;
          mloc = fmaxf(mloc, st[r]);
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float mn = fmaxf(m2, mloc);
        const float alpha = fast_exp2(m2 - mn);
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float p = okr[r] ? fast_exp2(st[r] - mn) : 0.f;
          st[r] = p;
          ps += p;
        }
        lsum = lsum * alpha + ps;
        m2 = mn;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
        const bf16x8 p0 = pack8(st, 0), p1 = pack8(st, 1);
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Vs, kb, 0, 32 * db, lane), p0, o[db], 0, 0, 0);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Vs, kb, 1, 32 * db, lane), p1, o[db], 0, 0, 0);
        }
      }
    }
  }
  lsum += __shfl_xor(lsum, 32);
  if (q < a.Lq) {
    store_owned_rows(out + ((int64_t)b * a.Lq + q) * H + h * DH, o, 1.0f / lsum, lane);
    if (lane < 32) lse[((int64_t)b * a.A + h) * a.Lq + q] = (m2 + __log2f(lsum)) * LN2;
  }
}

// dq and dvec[q] = sum_d dO[q,d] O[q,d]
template <bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void gen_bwd_dq_mfma(View a, const bf16* __restrict__ out, const float* __restrict__ lse,
                                                       const bf16* __restrict__ d_out, bf16* __restrict__ dq, int64_t lddq,
                                                       float* __restrict__ dvec) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Vs[64 * LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int H = a.A * DH;
  const int klen = clamp_len(a.klens[b], a.Lk), qlen = clamp_len(a.qlens[b], a.Lq);
  const bf16* qb_ = (const bf16*)a.q + (int64_t)b * a.Lq * a.ldq + h * DH;
  const bf16* kb_ = (const bf16*)a.k + (int64_t)b * a.Lk * a.ldkv + h * DH;
  const bf16* vb_ = (const bf16*)a.v + (int64_t)b * a.Lk * a.ldkv + h * DH;
  const bf16* go = d_out + (int64_t)b * a.Lq * H + h * DH;
  const bf16* oo = out + (int64_t)b * a.Lq * H + h * DH;
  const int q = blockIdx.x * 128 + wave * 32 + (lane & 31);
  const int wave_qmax = blockIdx.x * 128 + wave * 32 + 31;
  const int kend = CAUSAL ? min(klen, (int)blockIdx.x * 128 + 128) : klen;

  // padded queries (q >= qlen) own all-zero fragments and therefore produce zero rows
  bf16x8 qf[4], gf[4];
  float dpart = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qf[ks] = frag_rows_global(qb_, a.ldq, q, qlen, ks, lane);
    gf[ks] = frag_rows_global(go, H, q, qlen, ks, lane);
    const bf16x8 of = frag_rows_global(oo, H, q, qlen, ks, lane);
#pragma unroll
    for (int e = 0; e < 8; ++e) dpart = fmaf((float)gf[ks][e], (float)of[e], dpart);
  }
  const float dq_row = dpart + __shfl_xor(dpart, 32);
  const float lse2 = (q < qlen) ? lse[((int64_t)b * a.A + h) * a.Lq + q] * LOG2E : 0.f;
  f32x16 acc[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  for (int k0 = 0; k0 < kend; k0 += 64) {
    __syncthreads();
    stage64(Ks, kb_, a.ldkv, k0, klen, tid);
    stage64(Vs, vb_, a.ldkv, k0, klen, tid);
    __syncthreads();
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int kb = 32 * sub;
      if (k0 + kb < kend && (!CAUSAL || k0 + kb <= wave_qmax)) {
        f32x16 st, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Ks, kb, ks, lane), qf[ks], st, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Vs, kb, ks, lane), gf[ks], dp, 0, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + kb + tile_row(r, lane);
          const bool ok = key < klen && q < qlen && (!CAUSAL || key <= q);
          const float p = ok ? fast_exp2(st[r] * SCALE2 - lse2) : 0.f;
          st[r] = p * (dp[r] - dq_row);
        }
        const bf16x8 s0 = pack8(st, 0), s1 = pack8(st, 1);
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Ks, kb, 0, 32 * db, lane), s0, acc[db], 0, 0, 0);
          acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Ks, kb, 1, 32 * db, lane), s1, acc[db], 0, 0, 0);
        }
      }
    }
  }
  if (q < a.Lq) {
    store_owned_rows(dq + ((int64_t)b * a.Lq + q) * lddq + h * DH, acc, 0.125f, lane);
    if (lane < 32) dvec[((int64_t)b * a.A + h) * a.Lq + q] = dq_row;
  }
}

// wave owns 32 keys, streams queries / output gradients -> dk, dv
template <bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gen_bwd_dkv_mfma(View a, const float* __restrict__ lse, const bf16* __restrict__ d_out,
                                                        const float* __restrict__ dvec, bf16* __restrict__ dk_out,
                                                        bf16* __restrict__ dv_out, int64_t lddkv) {
  __shared__ __attribute__((aligned(16))) bf16 Qs[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Gs[64 * LDT];
  __shared__ float lse2_s[64], dvec_s[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int H = a.A * DH;
  const int klen = clamp_len(a.klens[b], a.Lk), qlen = clamp_len(a.qlens[b], a.Lq);
  const bf16* qb_ = (const bf16*)a.q + (int64_t)b * a.Lq * a.ldq + h * DH;
  const bf16* kb_ = (const bf16*)a.k + (int64_t)b * a.Lk * a.ldkv + h * DH;
  const bf16* vb_ = (const bf16*)a.v + (int64_t)b * a.Lk * a.ldkv + h * DH;
  const bf16* go = d_out + (int64_t)b * a.Lq * H + h * DH;
  const int kj = blockIdx.x * 128 + wave * 32 + (lane & 31);    // the key this lane owns
  const int wave_kmin = blockIdx.x * 128 + wave * 32;
  const bool wave_active = wave_kmin < klen;                    // wave-uniform

  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    kf[ks] = frag_rows_global(kb_, a.ldkv, kj, klen, ks, lane);
    vf[ks] = frag_rows_global(vb_, a.ldkv, kj, klen, ks, lane);
  }
  f32x16 dk[2], dv[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[db][r] = 0.f; dv[db][r] = 0.f; }

  // queries before the block's first key never see it when causal (block-uniform start, a multiple of 64)
  for (int q0 = CAUSAL ? (int)blockIdx.x * 128 : 0; q0 < qlen; q0 += 64) {
    __syncthreads();
    stage64(Qs, qb_, a.ldq, q0, qlen, tid);
    stage64(Gs, go, H, q0, qlen, tid);
    if (tid < 64) {
      const bool ok = q0 + tid < qlen;
      lse2_s[tid] = ok ? lse[((int64_t)b * a.A + h) * a.Lq + q0 + tid] * LOG2E : 0.f;
      dvec_s[tid] = ok ? dvec[((int64_t)b * a.A + h) * a.Lq + q0 + tid] : 0.f;
    }
    __syncthreads();
    if (wave_active) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int qb = 32 * sub;
        if (q0 + qb < qlen && (!CAUSAL || q0 + qb + 31 >= wave_kmin)) {
          f32x16 st, dp;
#pragma unroll
          for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Qs, qb, ks, lane), kf[ks], st, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Gs, qb, ks, lane), vf[ks], dp, 0, 0, 0);
          }
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qi = qb + tile_row(r, lane);
            const bool ok = (q0 + qi < qlen) && (kj < klen) && (!CAUSAL || kj <= q0 + qi);
            const float p = ok ? fast_exp2(st[r] * SCALE2 - lse2_s[qi]) : 0.f;
            st[r] = p;
            dp[r] = p * (dp[r] - dvec_s[qi]);
          }
          const bf16x8 p0 = pack8(st, 0), p1 = pack8(st, 1), s0 = pack8(dp, 0), s1 = pack8(dp, 1);
#pragma unroll
          for (int db = 0; db < 2; ++db) {
            dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Gs, qb, 0, 32 * db, lane), p0, dv[db], 0, 0, 0);
            dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Gs, qb, 1, 32 * db, lane), p1, dv[db], 0, 0, 0);
            dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Qs, qb, 0, 32 * db, lane), s0, dk[db], 0, 0, 0);
            dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(Qs, qb, 1, 32 * db, lane), s1, dk[db], 0, 0, 0);
          }
        }
      }
    }
  }
  if (kj < a.Lk) {
    store_owned_rows(dk_out + ((int64_t)b * a.Lk + kj) * lddkv + h * DH, dk, 0.125f, lane);
    store_owned_rows(dv_out + ((int64_t)b * a.Lk + kj) * lddkv + h * DH, dv, 1.0f, lane);
  }
}

// ------------------------------------------------------------------------------------------
// fp32: one thread per owned row
// ------------------------------------------------------------------------------------------
constexpr int D = 64;

__device__ __forceinline__ void stage_f32(float (*dst)[D], const float* __restrict__ src, int64_t row_stride, int row0, int nrows_valid,
                                          int lane) {
  for (int e = lane; e < 64 * D; e += 64) {
    const int r = e >> 6, c = e & 63;
    dst[r][c] = (r < nrows_valid) ? src[(int64_t)(row0 + r) * row_stride + c] : 0.f;
  }
}

template <bool CAUSAL>
__global__ __launch_bounds__(64) void gen_fwd_simt(View a, float* __restrict__ out, float* __restrict__ lse) {
  __shared__ float Ks[64][D];
  __shared__ float Vs[64][D];
  const int lane = threadIdx.x;
  const int b = blockIdx.z, h = blockIdx.y, qi = blockIdx.x * 64 + lane;
  const int H = a.A * D;
  const int klen = clamp_len(a.klens[b], a.Lk);
  const float* qb_ = (const float*)a.q + (int64_t)b * a.Lq * a.ldq + h * D;
  const float* kb_ = (const float*)a.k + (int64_t)b * a.Lk * a.ldkv + h * D;
  const float* vb_ = (const float*)a.v + (int64_t)b * a.Lk * a.ldkv + h * D;
  const bool active = qi < a.Lq;
  const int kend = CAUSAL ? min(klen, (int)blockIdx.x * 64 + 64) : klen;
  float q[D], acc[D];
#pragma unroll
  for (int c = 0; c < D; ++c) { q[c] = active ? 0.125f * qb_[(int64_t)qi * a.ldq + c] : 0.f; acc[c] = 0.f; }
  float m = -1.0e30f, l = 0.f;
  for (int k0 = 0; k0 < kend; k0 += 64) {
    const int nv = min(64, kend - k0);
    __syncthreads();
    stage_f32(Ks, kb_, a.ldkv, k0, nv, lane);
    stage_f32(Vs, vb_, a.ldkv, k0, nv, lane);
    __syncthreads();
    for (int j = 0; j < nv; ++j) {
      if (CAUSAL && k0 + j > qi) break;      // keys are visited in ascending order
      float s = 0.f;
#pragma unroll
      for (int c = 0; c < D; ++c) s = fmaf(q[c], Ks[j][c], s);
      const float mn = fmaxf(m, s);
      const float alpha = __expf(m - mn), p = __expf(s - mn);
      l = l * alpha + p;
#pragma unroll
      for (int c = 0; c < D; ++c) acc[c] = fmaf(p, Vs[j][c], acc[c] * alpha);
      m = mn;
    }
  }
  if (active) {
    const float inv = 1.0f / l;
    float* o = out + ((int64_t)b * a.Lq + qi) * H + h * D;
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] = acc[c] * inv;
    lse[((int64_t)b * a.A + h) * a.Lq + qi] = m + logf(l);
  }
}

template <bool CAUSAL>
__global__ __launch_bounds__(64) void gen_bwd_dq_simt(View a, const float* __restrict__ out, const float* __restrict__ lse,
                                                      const float* __restrict__ d_out, float* __restrict__ dq_out, int64_t lddq,
                                                      float* __restrict__ dvec) {
  __shared__ float Ks[64][D];
  __shared__ float Vs[64][D];
  const int lane = threadIdx.x;
  const int b = blockIdx.z, h = blockIdx.y, qi = blockIdx.x * 64 + lane;
  const int H = a.A * D;
  const int klen = clamp_len(a.klens[b], a.Lk), qlen = clamp_len(a.qlens[b], a.Lq);
  const float* qb_ = (const float*)a.q + (int64_t)b * a.Lq * a.ldq + h * D;
  const float* kb_ = (const float*)a.k + (int64_t)b * a.Lk * a.ldkv + h * D;
  const float* vb_ = (const float*)a.v + (int64_t)b * a.Lk * a.ldkv + h * D;
  const bool active = qi < qlen;     // padded query rows get zero gradient
  const int kend = CAUSAL ? min(klen, (int)blockIdx.x * 64 + 64) : klen;
  float q[D], go[D], dq[D];
  float dv_ = 0.f;
#pragma unroll
  for (int c = 0; c < D; ++c) {
    q[c] = active ? 0.125f * qb_[(int64_t)qi * a.ldq + c] : 0.f;
    go[c] = active ? d_out[((int64_t)b * a.Lq + qi) * H + h * D + c] : 0.f;
    const float o = active ? out[((int64_t)b * a.Lq + qi) * H + h * D + c] : 0.f;
    dv_ = fmaf(go[c], o, dv_);
    dq[c] = 0.f;
  }
  const float row_lse = active ? lse[((int64_t)b * a.A + h) * a.Lq + qi] : 0.f;
  for (int k0 = 0; k0 < kend; k0 += 64) {
    const int nv = min(64, kend - k0);
    __syncthreads();
    stage_f32(Ks, kb_, a.ldkv, k0, nv, lane);
    stage_f32(Vs, vb_, a.ldkv, k0, nv, lane);
    __syncthreads();
    if (active) {
      for (int j = 0; j < nv; ++j) {
        if (CAUSAL && k0 + j > qi) break;
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) { s = fmaf(q[c], Ks[j][c], s); dp = fmaf(go[c], Vs[j][c], dp); }
        const float ds = __expf(s - row_lse) * (dp - dv_);
#pragma unroll
        for (int c = 0; c < D; ++c) dq[c] = fmaf(ds, Ks[j][c], dq[c]);
      }
    }
  }
  if (qi < a.Lq) {
    float* o = dq_out + ((int64_t)b * a.Lq + qi) * lddq + h * D;
#pragma unroll
    for (int c = 0; c < D; ++c) o[c] = 0.125f * dq[c];
    dvec[((int64_t)b * a.A + h) * a.Lq + qi] = dv_;
  }
}

template <bool CAUSAL>
__global__ __launch_bounds__(64) void gen_bwd_dkv_simt(View a, const float* __restrict__ lse, const float* __restrict__ d_out,
                                                       const float* __restrict__ dvec, float* __restrict__ dk_out, float* __restrict__ dv_out,
                                                       int64_t lddkv) {
  __shared__ float Qs[64][D];
  __shared__ float Gs[64][D];
  __shared__ float lse_s[64], dvec_s[64];
  const int lane = threadIdx.x;
  const int b = blockIdx.z, h = blockIdx.y, kj = blockIdx.x * 64 + lane;
  const int H = a.A * D;
  const int klen = clamp_len(a.klens[b], a.Lk), qlen = clamp_len(a.qlens[b], a.Lq);
  const float* qb_ = (const float*)a.q + (int64_t)b * a.Lq * a.ldq + h * D;
  const float* kb_ = (const float*)a.k + (int64_t)b * a.Lk * a.ldkv + h * D;
  const float* vb_ = (const float*)a.v + (int64_t)b * a.Lk * a.ldkv + h * D;
  const bool active = kj < klen;     // padded keys take no part
  float k[D], v[D], dk[D], dv[D];
#pragma unroll
  for (int c = 0; c < D; ++c) {
    k[c] = active ? kb_[(int64_t)kj * a.ldkv + c] : 0.f;
    v[c] = active ? vb_[(int64_t)kj * a.ldkv + c] : 0.f;
    dk[c] = 0.f; dv[c] = 0.f;
  }
  for (int q0 = CAUSAL ? (int)blockIdx.x * 64 : 0; q0 < qlen; q0 += 64) {     // padded queries carry zero gradient: skipped
    const int nv = min(64, qlen - q0);
    __syncthreads();
    stage_f32(Qs, qb_, a.ldq, q0, nv, lane);
    stage_f32(Gs, d_out + (int64_t)b * a.Lq * H + h * D, (int64_t)H, q0, nv, lane);
    if (lane < nv) {
      lse_s[lane] = lse[((int64_t)b * a.A + h) * a.Lq + q0 + lane];
      dvec_s[lane] = dvec[((int64_t)b * a.A + h) * a.Lq + q0 + lane];
    }
    __syncthreads();
    if (active) {
      for (int i = 0; i < nv; ++i) {
        if (CAUSAL && q0 + i < kj) continue;
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int c = 0; c < D; ++c) { s = fmaf(Qs[i][c], k[c], s); dp = fmaf(Gs[i][c], v[c], dp); }
        const float p = __expf(0.125f * s - lse_s[i]);
        const float ds = p * (dp - dvec_s[i]);
#pragma unroll
        for (int c = 0; c < D; ++c) { dv[c] = fmaf(p, Gs[i][c], dv[c]); dk[c] = fmaf(ds, Qs[i][c], dk[c]); }
      }
    }
  }
  if (kj < a.Lk) {
    float* ok_ = dk_out + ((int64_t)b * a.Lk + kj) * lddkv + h * D;
    float* ov_ = dv_out + ((int64_t)b * a.Lk + kj) * lddkv + h * D;
#pragma unroll
    for (int c = 0; c < D; ++c) { ok_[c] = 0.125f * dk[c]; ov_[c] = dv[c]; }
  }
}

View make_view(const AttnOperands& x) {
  View v;
  v.q = x.q; v.k = x.k; v.v = x.v; v.ldq = x.ldq; v.ldkv = x.ldkv; v.qlens = x.qlens; v.klens = x.klens;
  v.Lq = x.Lq; v.Lk = x.Lk; v.A = x.A;
  return v;
}

hs_status check_operands(hs_ctx* ctx, int dtype, const AttnOperands& x, const char* who) {
  if (x.A < 1 || x.Lq < 1 || x.Lk < 1) return hs_fail(ctx, HS_ERR_INVALID_ARG, std::string(who) + ": bad size");
  if (x.causal && x.Lq != x.Lk) return hs_fail(ctx, HS_ERR_SHAPE, std::string(who) + ": causal attention needs Lq == Lk");
  if (!x.q || !x.k || !x.v || !x.qlens || !x.klens) return hs_fail(ctx, HS_ERR_INVALID_ARG, std::string(who) + ": NULL operand");
  const int64_t H = (int64_t)x.A * 64;
  if (x.ldq < H || x.ldkv < H) return hs_fail(ctx, HS_ERR_SHAPE, std::string(who) + ": row stride smaller than A*64");
  if (dtype == HS_BF16) {       // 16-byte fragment loads
    if ((x.ldq & 7) || (x.ldkv & 7) || ((uintptr_t)x.q & 15) || ((uintptr_t)x.k & 15) || ((uintptr_t)x.v & 15))
      return hs_fail(ctx, HS_ERR_SHAPE, std::string(who) + ": bf16 operands must be 16-byte aligned with strides that are multiples of 8");
  }
  return HS_OK;
}

}  // namespace

hs_status launch_attention_general_fwd(hs_ctx* ctx, int dtype, const AttnOperands& x, int B, void* out, float* lse, hipStream_t s) {
  if (B <= 0) return HS_OK;
  hs_status st = check_operands(ctx, dtype, x, "attention_general_fwd");
  if (st != HS_OK) return st;
  const double pairs = (double)B * x.A * x.Lq * x.Lk * (x.causal ? 0.5 : 1.0);
  KScope scope(ctx ? ctx->prof : nullptr, KC_ATTN_FWD, 4.0 * pairs * 64, (double)B * x.A * 64 * (2.0 * x.Lq + 2.0 * x.Lk) * esize(dtype), s);
  const View v = make_view(x);
  if (dtype == HS_BF16) {
    dim3 grid((x.Lq + 127) / 128, x.A, B);
    if (x.causal) hipLaunchKernelGGL(gen_fwd_mfma<true>, grid, dim3(256), 0, s, v, (bf16*)out, lse);
    else hipLaunchKernelGGL(gen_fwd_mfma<false>, grid, dim3(256), 0, s, v, (bf16*)out, lse);
  } else {
    dim3 grid((x.Lq + 63) / 64, x.A, B);
    if (x.causal) hipLaunchKernelGGL(gen_fwd_simt<true>, grid, dim3(64), 0, s, v, (float*)out, lse);
    else hipLaunchKernelGGL(gen_fwd_simt<false>, grid, dim3(64), 0, s, v, (float*)out, lse);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("attention_general_fwd: ") + hipGetErrorString(e));
  return HS_OK;
}

hs_status launch_attention_general_bwd(hs_ctx* ctx, int dtype, const AttnOperands& x, int B, const void* out, const float* lse,
                                       const void* d_out, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv, float* dvec,
                                       hipStream_t s) {
  if (B <= 0) return HS_OK;
  hs_status st = check_operands(ctx, dtype, x, "attention_general_bwd");
  if (st != HS_OK) return st;
  if (!out || !lse || !d_out || !dq || !dk || !dv || !dvec) return hs_fail(ctx, HS_ERR_INVALID_ARG, "attention_general_bwd: NULL buffer");
  if (dtype == HS_BF16 && ((lddq & 3) || (lddkv & 3) || ((uintptr_t)dq & 7) || ((uintptr_t)dk & 7) || ((uintptr_t)dv & 7)))
    return hs_fail(ctx, HS_ERR_SHAPE, "attention_general_bwd: bf16 gradients must be 8-byte aligned with strides that are multiples of 4");
  const double pairs = (double)B * x.A * x.Lq * x.Lk * (x.causal ? 0.5 : 1.0);
  KScope scope(ctx ? ctx->prof : nullptr, KC_ATTN_BWD, 8.0 * pairs * 64, (double)B * x.A * 64 * (4.0 * x.Lq + 4.0 * x.Lk) * esize(dtype), s);
  const View v = make_view(x);
  if (dtype == HS_BF16) {
    dim3 gq((x.Lq + 127) / 128, x.A, B), gk((x.Lk + 127) / 128, x.A, B);
    if (x.causal) {
      hipLaunchKernelGGL(gen_bwd_dq_mfma<true>, gq, dim3(256), 0, s, v, (const bf16*)out, lse, (const bf16*)d_out, (bf16*)dq, lddq, dvec);
      hipLaunchKernelGGL(gen_bwd_dkv_mfma<true>, gk, dim3(256), 0, s, v, lse, (const bf16*)d_out, (const float*)dvec, (bf16*)dk, (bf16*)dv, lddkv);
    } else {
      hipLaunchKernelGGL(gen_bwd_dq_mfma<false>, gq, dim3(256), 0, s, v, (const bf16*)out, lse, (const bf16*)d_out, (bf16*)dq, lddq, dvec);
      hipLaunchKernelGGL(gen_bwd_dkv_mfma<false>, gk, dim3(256), 0, s, v, lse, (const bf16*)d_out, (const float*)dvec, (bf16*)dk, (bf16*)dv, lddkv);
    }
  } else {
    dim3 gq((x.Lq + 63) / 64, x.A, B), gk((x.Lk + 63) / 64, x.A, B);
    if (x.causal) {
      hipLaunchKernelGGL(gen_bwd_dq_simt<true>, gq, dim3(64), 0, s, v, (const float*)out, lse, (const float*)d_out, (float*)dq, lddq, dvec);
      hipLaunchKernelGGL(gen_bwd_dkv_simt<true>, gk, dim3(64), 0, s, v, lse, (const float*)d_out, (const float*)dvec, (float*)dk, (float*)dv, lddkv);
    } else {
      hipLaunchKernelGGL(gen_bwd_dq_simt<false>, gq, dim3(64), 0, s, v, (const float*)out, lse, (const float*)d_out, (float*)dq, lddq, dvec);
      hipLaunchKernelGGL(gen_bwd_dkv_simt<false>, gk, dim3(64), 0, s, v, lse, (const float*)d_out, (const float*)dvec, (float*)dk, (float*)dv, lddkv);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("attention_general_bwd: ") + hipGetErrorString(e));
  return HS_OK;
}
