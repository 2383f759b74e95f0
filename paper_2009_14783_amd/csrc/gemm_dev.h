// Shared by the GEMM translation units: the kernel arguments and the fused epilogues.
#pragma once
#include "common.h"

// arguments of every GEMM kernel (plain data, passed by value)
struct GemmDev {
  const void* A; const void* B; void* C; void* C2; const void* bias; const void* aux;
  int64_t lda, ldb, ldc, ldaux;
  int M, N, K;
  int c_f32, epi;
  float beta;
  float* partial;      // split-K partial sums [splits][M][N], or null
  int k_per_split;     // multiple of the k-tile
  const float2* gelu_tab;   // wide kernels, GELU epilogues: table for gelu_tab_eval (the cdf for epi 2, GELU' for epi 3)
  DropCfg drop;        // dropout of (product + bias) before the residual is added (epi == 1 only; thr == 0: off)
  uint32_t drop_site;  // element index of the site = row * N + col
};

// several products for one launch of the grouped kernel (gemm_wide.h)
struct GemmGroupDev {
  int n;                   // problems in use
  int first_tile[9];       // first_tile[i] .. first_tile[i + 1] - 1: the tiles of problem i
  GemmDev prob[8];
};
constexpr int kGroupBM = 256, kGroupBN = 128;   // tile of the grouped kernel

// Piecewise-linear tables of the normal cdf Phi (GELU(x) = x Phi(x)) and of GELU'(x) = Phi(x) + x pdf(x) on
// [-6, 6]: entry i holds the value at -6 + i h and the increment to the next node, h = 12 / 1024.  Error of the
// interpolation below 5e-6 (Phi) and 1.4e-5 (GELU'), three orders under bf16 resolution; outside the interval
// both functions equal their end values to 1e-7.
constexpr int kGeluTabN = 1024;
constexpr float kGeluTabR = 6.0f;

namespace {
// dropout factors of n (4 or 8) consecutive output columns of one row, starting at a column that is a
// multiple of 4: one generator block per four columns when the row length allows it
template <int NV>
__device__ __forceinline__ void drop_row_factors(const GemmDev& p, int row, int col, float (&f)[NV]) {
  const uint64_t e = (uint64_t)row * (uint64_t)p.N + (uint64_t)col;
  if ((p.N & 3) == 0) {
#pragma unroll
    for (int q = 0; q < NV / 4; ++q) {
      float t[4];
      drop_factors4(p.drop, p.drop_site, (e >> 2) + q, t);
      f[4 * q] = t[0]; f[4 * q + 1] = t[1]; f[4 * q + 2] = t[2]; f[4 * q + 3] = t[3];
    }
  } else {
#pragma unroll
    for (int t = 0; t < NV; ++t) f[t] = drop_factor1(p.drop, p.drop_site, e + t);
  }
}
__device__ __forceinline__ float drop_elem(const GemmDev& p, int row, int col) {
  return drop_factor1(p.drop, p.drop_site, (uint64_t)row * (uint64_t)p.N + (uint64_t)col);
}

template <class T>
__device__ __forceinline__ void epilogue_store(const GemmDev& p, int row, int col, float v) {
  if (row >= p.M || col >= p.N) return;
  if (p.bias) v += to_f(((const T*)p.bias)[col]);
  if (p.epi == 1 && p.drop.thr) v *= drop_elem(p, row, col);
  if (p.epi == 1) v += to_f(((const T*)p.aux)[(int64_t)row * p.ldaux + col]);
  else if (p.epi == 3) v *= gelu_grad_f(to_f(((const T*)p.aux)[(int64_t)row * p.ldaux + col]));
  const int64_t o = (int64_t)row * p.ldc + col;
  if (p.c_f32) {
    float* C = (float*)p.C;
    C[o] = (p.beta != 0.0f) ? p.beta * C[o] + v : v;
  } else {
    ((T*)p.C)[o] = from_f<T>(v);
    if (p.epi == 2) ((T*)p.C2)[o] = from_f<T>(gelu_f(v));
  }
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------
enum { EPI_PARTIAL = 0, EPI_F32, EPI_ACT, EPI_ACT_RES, EPI_ACT_GELU, EPI_ACT_DGELU };

// One group of four consecutive output columns of one row: bias, epilogue, store.  `vec` says that
// all four columns exist and every pointer involved is aligned for a 4-element access.
template <int MODE>
__device__ __forceinline__ void store_quad(const GemmDev& p, int row, int col, float4 v, bool vec, int split) {
  const bf16* bias = (const bf16*)p.bias;
  const bf16* aux = (const bf16*)p.aux;
  if (vec) {
    if (MODE != EPI_PARTIAL && bias) {
      const bf16x4 b = *(const bf16x4*)(bias + col);
      v.x += (float)b[0]; v.y += (float)b[1]; v.z += (float)b[2]; v.w += (float)b[3];
    }
    if (MODE == EPI_PARTIAL) {
      *(float4*)(p.partial + ((int64_t)split * p.M + row) * p.N + col) = v;
    } else if (MODE == EPI_F32) {
      float4* C = (float4*)((float*)p.C + (int64_t)row * p.ldc + col);
      if (p.beta != 0.0f) { const float4 o = *C; v.x += p.beta * o.x; v.y += p.beta * o.y; v.z += p.beta * o.z; v.w += p.beta * o.w; }
      *C = v;
    } else {
      const int64_t o = (int64_t)row * p.ldc + col;
      if (MODE == EPI_ACT_RES && p.drop.thr) {
        float f[4];
        drop_row_factors<4>(p, row, col, f);
        v.x *= f[0]; v.y *= f[1]; v.z *= f[2]; v.w *= f[3];
      }
      if (MODE == EPI_ACT_RES || MODE == EPI_ACT_DGELU) {
        const bf16x4 a = *(const bf16x4*)(aux + (int64_t)row * p.ldaux + col);
        if (MODE == EPI_ACT_RES) { v.x += (float)a[0]; v.y += (float)a[1]; v.z += (float)a[2]; v.w += (float)a[3]; }
        else { v.x *= gelu_grad_fast((float)a[0]); v.y *= gelu_grad_fast((float)a[1]); v.z *= gelu_grad_fast((float)a[2]); v.w *= gelu_grad_fast((float)a[3]); }
      }
      bf16x4 c;
      c[0] = (bf16)v.x; c[1] = (bf16)v.y; c[2] = (bf16)v.z; c[3] = (bf16)v.w;
      *(bf16x4*)((bf16*)p.C + o) = c;
      if (MODE == EPI_ACT_GELU) {
        bf16x4 g;
        g[0] = (bf16)gelu_fast(v.x); g[1] = (bf16)gelu_fast(v.y); g[2] = (bf16)gelu_fast(v.z); g[3] = (bf16)gelu_fast(v.w);
        *(bf16x4*)((bf16*)p.C2 + o) = g;
      }
    }
  } else {
    const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (col + t >= p.N) break;
      float x = e[t];
      if (MODE == EPI_PARTIAL) { p.partial[((int64_t)split * p.M + row) * p.N + col + t] = x; continue; }
      if (bias) x += (float)bias[col + t];
      if (MODE == EPI_F32) {
        float* C = (float*)p.C + (int64_t)row * p.ldc + col + t;
        *C = (p.beta != 0.0f) ? p.beta * *C + x : x;
      } else {
        const int64_t o = (int64_t)row * p.ldc + col + t;
        if (MODE == EPI_ACT_RES && p.drop.thr) x *= drop_elem(p, row, col + t);
        if (MODE == EPI_ACT_RES) x += (float)aux[(int64_t)row * p.ldaux + col + t];
        if (MODE == EPI_ACT_DGELU) x *= gelu_grad_fast((float)aux[(int64_t)row * p.ldaux + col + t]);
        ((bf16*)p.C)[o] = (bf16)x;
        if (MODE == EPI_ACT_GELU) ((bf16*)p.C2)[o] = (bf16)gelu_fast(x);
      }
    }
  }
}

// whether 4-element accesses are aligned for everything this mode touches
template <int MODE>
__device__ __forceinline__ bool quad_aligned(const GemmDev& p) {
  if (MODE == EPI_PARTIAL) return (p.N & 3) == 0;
  bool ok = (p.ldc & 3) == 0 && ((uintptr_t)p.C & 15) == 0;
  if (p.bias) ok = ok && ((uintptr_t)p.bias & 7) == 0;
  if (MODE == EPI_ACT_RES || MODE == EPI_ACT_DGELU) ok = ok && (p.ldaux & 3) == 0 && ((uintptr_t)p.aux & 7) == 0;
  if (MODE == EPI_ACT_GELU) ok = ok && ((uintptr_t)p.C2 & 7) == 0;
  return ok;
}

// Writes the TI x TJ grid of 32x32 result tiles of one wave.  Register r of lane l of a tile is
// row 8*(r/4) + 4*(l/32) + r%4, column l%32: one store instruction covers 64 contiguous bytes of two
// rows (measured faster than 8-byte pieces of 32 rows from transposed tiles).
template <int MODE, int TI, int TJ>
__device__ __forceinline__ void tile_epilogue(const GemmDev& p, const f32x16 (&acc)[TI][TJ], int rbase, int cbase, int lane, int split) {
  const bf16* bias = (const bf16*)p.bias;
  float bv[TJ];
  bool col_ok[TJ];
#pragma unroll
  for (int j = 0; j < TJ; ++j) {
    const int col = cbase + j * 32 + (lane & 31);
    col_ok[j] = col < p.N;
    bv[j] = (MODE != EPI_PARTIAL && bias && col_ok[j]) ? (float)bias[col] : 0.f;
  }
  const int col0 = cbase + (lane & 31);
#pragma unroll
  for (int i = 0; i < TI; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = rbase + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (row < p.M) {
        // row offsets are computed once per row and used for the TJ columns of this lane
        const int64_t oc = (MODE == EPI_PARTIAL) ? ((int64_t)split * p.M + row) * p.N + col0 : (int64_t)row * p.ldc + col0;
        const int64_t oa = (int64_t)row * p.ldaux + col0;
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
          if (!col_ok[j]) continue;
          float v = acc[i][j][r] + bv[j];
          if (MODE == EPI_PARTIAL) {
            p.partial[oc + j * 32] = v;
          } else if (MODE == EPI_F32) {
            float* C = (float*)p.C + oc + j * 32;
            *C = (p.beta != 0.0f) ? p.beta * *C + v : v;
          } else {
            if (MODE == EPI_ACT_RES && p.drop.thr) v *= drop_elem(p, row, col0 + j * 32);
            if (MODE == EPI_ACT_RES) v += (float)((const bf16*)p.aux)[oa + j * 32];
            if (MODE == EPI_ACT_DGELU) v *= gelu_grad_fast((float)((const bf16*)p.aux)[oa + j * 32]);
            ((bf16*)p.C)[oc + j * 32] = (bf16)v;
            if (MODE == EPI_ACT_GELU) ((bf16*)p.C2)[oc + j * 32] = (bf16)gelu_fast(v);
          }
        }
      }
    }
    // keep the scheduler from overlapping the loads and address arithmetic of different tile rows:
    // that would cost more registers than the main loop needs and lower the occupancy
    __builtin_amdgcn_sched_barrier(0);
  }
}

// Eight consecutive output columns of one row (as two float4): bias, epilogue, store.  `vec` says
// that all eight columns exist and every pointer involved is aligned for 16-byte accesses.
template <int MODE>
__device__ __forceinline__ void store_octet(const GemmDev& p, int row, int col, float4 lo, float4 hi, bool vec, int split) {
  const bf16* bias = (const bf16*)p.bias;
  const bf16* aux = (const bf16*)p.aux;
  float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  if (vec) {
    if (MODE == EPI_PARTIAL) {
      float* dst = p.partial + ((int64_t)split * p.M + row) * p.N + col;
      *(float4*)dst = lo; *(float4*)(dst + 4) = hi;
      return;
    }
    if (bias) {
      const bf16x8 b = *(const bf16x8*)(bias + col);
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] += (float)b[t];
    }
    if (MODE == EPI_F32) {
      float* C = (float*)p.C + (int64_t)row * p.ldc + col;
      if (p.beta != 0.0f) {
        const float4 o0 = *(const float4*)C, o1 = *(const float4*)(C + 4);
        v[0] += p.beta * o0.x; v[1] += p.beta * o0.y; v[2] += p.beta * o0.z; v[3] += p.beta * o0.w;
        v[4] += p.beta * o1.x; v[5] += p.beta * o1.y; v[6] += p.beta * o1.z; v[7] += p.beta * o1.w;
      }
      *(float4*)C = make_float4(v[0], v[1], v[2], v[3]);
      *(float4*)(C + 4) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
      const int64_t o = (int64_t)row * p.ldc + col;
      if (MODE == EPI_ACT_RES && p.drop.thr) {
        float f[8];
        drop_row_factors<8>(p, row, col, f);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] *= f[t];
      }
      if (MODE == EPI_ACT_RES || MODE == EPI_ACT_DGELU) {
        const bf16x8 a = *(const bf16x8*)(aux + (int64_t)row * p.ldaux + col);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = (MODE == EPI_ACT_RES) ? v[t] + (float)a[t] : v[t] * gelu_grad_fast((float)a[t]);
      }
      bf16x8 c;
#pragma unroll
      for (int t = 0; t < 8; ++t) c[t] = (bf16)v[t];
      *(bf16x8*)((bf16*)p.C + o) = c;
      if (MODE == EPI_ACT_GELU) {
        bf16x8 g;
#pragma unroll
        for (int t = 0; t < 8; ++t) g[t] = (bf16)gelu_fast(v[t]);
        *(bf16x8*)((bf16*)p.C2 + o) = g;
      }
    }
  } else {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      if (col + t >= p.N) break;
      float x = v[t];
      if (MODE == EPI_PARTIAL) { p.partial[((int64_t)split * p.M + row) * p.N + col + t] = x; continue; }
      if (bias) x += (float)bias[col + t];
      if (MODE == EPI_F32) {
        float* C = (float*)p.C + (int64_t)row * p.ldc + col + t;
        *C = (p.beta != 0.0f) ? p.beta * *C + x : x;
      } else {
        const int64_t o = (int64_t)row * p.ldc + col + t;
        if (MODE == EPI_ACT_RES && p.drop.thr) x *= drop_elem(p, row, col + t);
        if (MODE == EPI_ACT_RES) x += (float)aux[(int64_t)row * p.ldaux + col + t];
        if (MODE == EPI_ACT_DGELU) x *= gelu_grad_fast((float)aux[(int64_t)row * p.ldaux + col + t]);
        ((bf16*)p.C)[o] = (bf16)x;
        if (MODE == EPI_ACT_GELU) ((bf16*)p.C2)[o] = (bf16)gelu_fast(x);
      }
    }
  }
}

template <int MODE>
__device__ __forceinline__ bool octet_aligned(const GemmDev& p) {
  if (MODE == EPI_PARTIAL) return (p.N & 3) == 0;
  if (MODE == EPI_F32) return (p.ldc & 3) == 0 && ((uintptr_t)p.C & 15) == 0 && (!p.bias || ((uintptr_t)p.bias & 15) == 0);
  bool ok = (p.ldc & 7) == 0 && ((uintptr_t)p.C & 15) == 0 && (!p.bias || ((uintptr_t)p.bias & 15) == 0);
  if (MODE == EPI_ACT_RES || MODE == EPI_ACT_DGELU) ok = ok && (p.ldaux & 7) == 0 && ((uintptr_t)p.aux & 15) == 0;
  if (MODE == EPI_ACT_GELU) ok = ok && ((uintptr_t)p.C2 & 15) == 0;
  return ok;
}

// Epilogue through LDS: each wave writes one 32-row slab of its result tile to its own LDS region in
// row-major order and reads it back so that a lane holds 8 consecutive columns of one row; global
// accesses are then 16 bytes per lane and whole 128-byte lines per row.  LDS operations of one wave
// execute in order, so no barrier is needed inside a wave's region.
template <int MODE, int TI, int TJ>
__device__ __forceinline__ void tile_epilogue_lds(const GemmDev& p, const f32x16 (&acc)[TI][TJ], int rbase, int cbase, int lane, int split,
                                                  float* stage) {
  constexpr int WN = 32 * TJ, LDW = WN + 4;
  constexpr int LPR = WN / 8;           // 8-column pieces per row
  const bool vec = octet_aligned<MODE>(p);
#pragma unroll
  for (int i = 0; i < TI; ++i) {
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * LDW + j * 32 + (lane & 31)] = acc[i][j][r];
#pragma unroll
    for (int it = 0; it < 32 * LPR / 64; ++it) {
      const int piece = it * 64 + lane;
      const int lr = piece / LPR, lc = (piece % LPR) * 8;
      const float4 lo = *(const float4*)(stage + lr * LDW + lc), hi = *(const float4*)(stage + lr * LDW + lc + 4);
      const int row = rbase + i * 32 + lr, col = cbase + lc;
      if (row < p.M && col < p.N) store_octet<MODE>(p, row, col, lo, hi, vec && col + 7 < p.N, split);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

// table lookup for the epilogues of the wide kernels: tab (in LDS) as described at kGeluTabN
__device__ __forceinline__ float gelu_tab_eval(const float2* tab, float x) {
  const float xc = __builtin_amdgcn_fmed3f(x, -kGeluTabR, kGeluTabR * 0.9999999f);
  const float t = fmaf(xc, (float)kGeluTabN / (2.0f * kGeluTabR), 0.5f * (float)kGeluTabN);
  const float2 e = tab[(int)t];
  return fmaf(e.y, __builtin_amdgcn_fractf(t), e.x);
}

constexpr int MPAD = 32;   // m-major LDS rows: R + 32 elements  (row stride = 64 B mod 256 B)

}  // namespace
