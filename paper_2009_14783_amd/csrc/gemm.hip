// GEMM kernels: C[M,N] = sum_k A(m,k) B(n,k) with fused epilogues.
//   bf16: MFMA 32x32x16 tiles, fp32 accumulation, LDS double buffering.  Operands whose
//         contraction index is NOT the contiguous one are staged in their natural layout and read
//         with the LDS transpose read of gfx950, so every global and LDS access is 16/8 bytes wide.
//   fp32: plain tiled SIMT kernel (small reference-precision configurations only).
#include "common.h"

namespace {

struct GemmDev {
  const void* A; const void* B; void* C; void* C2; const void* bias; const void* aux;
  int64_t lda, ldb, ldc, ldaux;
  int M, N, K;
  int c_f32, epi;
  float beta;
  float* partial;      // split-K partial sums [splits][M][N], or null
  int k_per_split;     // multiple of the k-tile
  DropCfg drop;        // dropout of (product + bias) before the residual is added (epi == 1 only; thr == 0: off)
  uint32_t drop_site;  // element index of the site = row * N + col
};

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

constexpr int MPAD = 32;   // m-major LDS rows: R + 32 elements  (row stride = 64 B mod 256 B)

template <bool KMAJ, int R, int BK, int NT>
struct OperandTile {
  // k-major rows are stored without padding and with their 16-byte chunks permuted: chunk j of row r sits
  // at position j ^ ((r / 4) % 4).  Sixteen rows read at one k-offset then fall into sixteen different
  // 16-byte bank groups, and so do the four 64-byte rows that sixteen lanes write at once.
  static_assert(!KMAJ || BK == 32, "the chunk permutation is written for four chunks per row");
  static constexpr int LD = KMAJ ? BK : (R + MPAD);
  static __device__ __forceinline__ int swz(int row, int chunk) { return (chunk ^ ((row >> 2) & 3)) * 8; }
  static constexpr int ELEMS = KMAJ ? R * LD : BK * LD;
  static constexpr int CPR = KMAJ ? BK / 8 : R / 8;       // 8-element chunks per stored row
  static constexpr int NCH = R * BK / 8 / NT;             // chunks per thread
  static_assert(R * BK / 8 % NT == 0, "tile must split evenly over the threads");

  // Per-thread state of the global side: one 32-bit byte offset per chunk from the start of the matrix
  // (advanced every k-tile; the matrix start is uniform, so a load needs one address register) and whether
  // the chunk's position along the non-contraction index is inside the matrix.
  struct Cursor {
    const char* base;     // start of the matrix: always readable, also the address of masked-out chunks
    unsigned off[NCH];
    unsigned step;        // bytes from one k-tile to the next
    int koff[NCH];        // contraction offset of the chunk inside a k-tile
    bool ok[NCH];
  };
  static __device__ __forceinline__ void init(Cursor& cu, const bf16* __restrict__ base, int64_t ld, int row0, int rext, int kbeg, int tid) {
    cu.base = (const char*)base;
    cu.step = (unsigned)(KMAJ ? (int64_t)BK * 2 : (int64_t)BK * ld * 2);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * NT;
      const int a = c / CPR, b = (c % CPR) * 8;
      if (KMAJ) { cu.ok[i] = row0 + a < rext; cu.koff[i] = b; cu.off[i] = (unsigned)(((int64_t)(row0 + a) * ld + kbeg + b) * 2); }
      else      { cu.ok[i] = row0 + b < rext; cu.koff[i] = a; cu.off[i] = (unsigned)(((int64_t)(kbeg + a) * ld + row0 + b) * 2); }
    }
  }
  // global -> registers for the k-tile that starts at k0, then advance.  The loads are unconditional
  // (no branch, so the hardware load counter can be waited on exactly): a chunk outside the matrix or
  // beyond kend reads the start of the matrix instead and is zeroed when it is written to LDS.
  static __device__ __forceinline__ void load(uint4 (&reg)[NCH], Cursor& cu, int k0, int kend) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const bool ok = cu.ok[i] && k0 + cu.koff[i] < kend;
      reg[i] = *(const uint4*)(cu.base + (ok ? cu.off[i] : 0u));
      cu.off[i] += cu.step;
    }
  }
  // registers -> LDS for the k-tile that started at k0 (chunks that were masked out become zeros)
  static __device__ __forceinline__ void store(const uint4 (&reg)[NCH], bf16* s, int tid, const Cursor& cu, int k0, int kend) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * NT;
      const int a = c / CPR, b = (c % CPR) * 8;
      // branch-free select: an all-ones or all-zeros word per chunk
      const unsigned keep = (cu.ok[i] && k0 + cu.koff[i] < kend) ? 0xffffffffu : 0u;
      uint4 v = reg[i];
      v.x &= keep; v.y &= keep; v.z &= keep; v.w &= keep;
      *(uint4*)(s + a * LD + (KMAJ ? swz(a, b >> 3) : b)) = v;
    }
  }
  // LDS -> MFMA operand: lane gets elements (row = rbase + lane%32, k = ks*16 + 8*(lane/32) + 0..7)
  static __device__ __forceinline__ bf16x8 frag(const bf16* s, int rbase, int ks, int lane) {
    if (KMAJ) {
      const int row = rbase + (lane & 31);
      return *(const bf16x8*)(s + row * LD + swz(row, ks * 2 + (lane >> 5)));
    } else {
      // Transpose read: within each group of 16 lanes, lane i receives, as element e, the (i%4)-th
      // 16-bit value of the 8 bytes addressed by lane 4*e + i/4 of the group.  With lane s of a
      // group pointing at row (kb + s/4), columns nb + 4*(s%4)..+3, lane i ends up with rows
      // kb..kb+3 of column nb + i.
      const int kb = ks * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
      const int nb = rbase + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      typedef s16x4 __attribute__((address_space(3))) * lds_v4;
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + kb * LD + nb));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + (kb + 4) * LD + nb));
      union { struct { s16x4 lo, hi; } p; bf16x8 v; } u;
      u.p.lo = lo; u.p.hi = hi;
      return u.v;
    }
  }
};

// Block tile BM x BN x BK, WGM x WGN waves, each wave (BM/WGM) x (BN/WGN) as 32x32x16 MFMA tiles.
// A block's split index selects a contiguous range of k-tiles (split-K); with more than one split the raw fp32
// sums go to p.partial[z][M][N] and splitk_reduce_kernel applies the epilogue.
// waves per SIMD the register allocator should leave room for: accumulators take
// (BM/WGM)*(BN/WGN)/64 registers per lane out of 512
constexpr int gemm_occupancy(int bm, int bn, int wgm, int wgn) {
  const int acc = (bm / wgm) * (bn / wgn) / 64;
  return acc <= 64 ? 3 : (acc <= 128 ? 2 : 1);
}

// dynamic LDS of a block: the two pipeline stages of both operands, and at least the staging area of
// the epilogue (one 32-row slab of fp32 results per wave) when that is not much larger
template <bool AK, bool BKM, int BM, int BN, int BK, int WGM, int WGN>
constexpr size_t gemm_lds_bytes() {
  constexpr int NT = 64 * WGM * WGN;
  const size_t pipe = 2 * sizeof(bf16) * (size_t)(OperandTile<AK, BM, BK, NT>::ELEMS + OperandTile<BKM, BN, BK, NT>::ELEMS);
  const size_t stage = (size_t)WGM * WGN * 32 * (BN / WGN + 4) * sizeof(float);
  return (stage > pipe && stage <= pipe + pipe / 4) ? stage : pipe;
}

template <bool AK, bool BKM, int BM, int BN, int BK, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(gemm_occupancy(BM, BN, WGM, WGN), 8)))
void gemm_bf16_mfma(GemmDev p) {
  constexpr int NT = 64 * WGM * WGN;
  typedef OperandTile<AK, BM, BK, NT> TA;
  typedef OperandTile<BKM, BN, BK, NT> TB;
  constexpr int WM = BM / WGM, WN = BN / WGN, TI = WM / 32, TJ = WN / 32;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16* const sA0 = (bf16*)lds_raw;                       // two A buffers, then two B buffers
  bf16* const sB0 = (bf16*)lds_raw + 2 * TA::ELEMS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  // Tile order.  Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own
  // L2: give every XCD a contiguous range of tiles, and walk the tiles in groups of 8 tile rows so that
  // the tiles in flight on one XCD share operand panels.
  // The same holds across the k-splits (blockIdx.z): an XCD then works on one or two splits
  // instead of all of them, and fetches only their share of the operands.  Blocks beyond the last
  // multiple of 8 keep their place.
  const int nbx = gridDim.x, nby = gridDim.y, nb = nbx * nby;
  int v = (blockIdx.z * nby + blockIdx.y) * nbx + blockIdx.x;
  const int per_xcd = (nb * (int)gridDim.z) >> 3;
  if (v < 8 * per_xcd) v = (v & 7) * per_xcd + (v >> 3);
  const int split = v / nb;
  const int b = v - split * nb;
  constexpr int GM = 8;
  const int group = b / (GM * nbx), first_m = group * GM;
  const int gm = min(GM, nby - first_m);
  const int in_group = b - group * GM * nbx;
  const int m0 = (first_m + in_group % gm) * BM, n0 = (in_group / gm) * BN;
  const int kbeg = split * p.k_per_split;
  const int kend = min(p.K, kbeg + p.k_per_split);

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  typename TA::Cursor ca;
  typename TB::Cursor cb;
  TA::init(ca, (const bf16*)p.A, p.lda, m0, p.M, kbeg, tid);
  TB::init(cb, (const bf16*)p.B, p.ldb, n0, p.N, kbeg, tid);
  // Software pipeline with a prefetch distance of two k-tiles: tile t is fetched from global memory
  // into register set t%2 during iteration t-2, moved to LDS buffer t%2 during iteration t-1 and
  // consumed during iteration t, so a global load has two iterations of MFMA work to hide behind.
  // The tile count is rounded up to even; a tile beyond the range loads nothing real and is all zeros.
  uint4 ra0[TA::NCH], rb0[TB::NCH], ra1[TA::NCH], rb1[TB::NCH];
  const int nk = ((kend - kbeg + BK - 1) / BK + 1) & ~1;
  TA::load(ra0, ca, kbeg, kend);
  TB::load(rb0, cb, kbeg, kend);
  TA::load(ra1, ca, kbeg + BK, kend);
  TB::load(rb1, cb, kbeg + BK, kend);
  TA::store(ra0, sA0, tid, ca, kbeg, kend);
  TB::store(rb0, sB0, tid, cb, kbeg, kend);
  __syncthreads();

  // One k-tile of work, in the order the hardware queues like it: all fragment reads of the tile, the
  // MFMAs of its first half, then the LDS writes of the next tile (they need the global loads issued one
  // iteration ago and complete behind the second half's MFMAs), then the second half.
  static_assert(BK == 32, "the main loop is written for two 16-deep MFMA steps per k-tile");
  bf16x8 fa[2][TI], fb[2][TJ];
  auto frags = [&](int cur) {
    const bf16* sAc = sA0 + cur * TA::ELEMS;
    const bf16* sBc = sB0 + cur * TB::ELEMS;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
      for (int i = 0; i < TI; ++i) fa[ks][i] = TA::frag(sAc, wm * WM + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < TJ; ++j) fb[ks][j] = TB::frag(sBc, wn * WN + j * 32, ks, lane);
    }
  };
  auto mfmas = [&](int ks) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
  };

  for (int kt = 0; kt < nk; kt += 2) {
    const int k0 = kbeg + kt * BK;
    // even tile kt: in LDS buffer 0; register set 0 is free, set 1 holds tile kt+1
    TA::load(ra0, ca, k0 + 2 * BK, kend);
    TB::load(rb0, cb, k0 + 2 * BK, kend);
    frags(0);
    mfmas(0);
    TA::store(ra1, sA0 + TA::ELEMS, tid, ca, k0 + BK, kend);
    TB::store(rb1, sB0 + TB::ELEMS, tid, cb, k0 + BK, kend);
    mfmas(1);
    __syncthreads();
    // odd tile kt+1: in LDS buffer 1; register set 1 is free, set 0 holds tile kt+2
    TA::load(ra1, ca, k0 + 3 * BK, kend);
    TB::load(rb1, cb, k0 + 3 * BK, kend);
    frags(1);
    mfmas(0);
    if (kt + 2 < nk) {
      TA::store(ra0, sA0, tid, ca, k0 + 2 * BK, kend);
      TB::store(rb0, sB0, tid, cb, k0 + 2 * BK, kend);
    }
    mfmas(1);
    __syncthreads();
  }

  // The epilogue is selected once per block.  When the staging area fits into the LDS the main loop
  // used, results go out through LDS in whole lines; otherwise straight from the registers.
  const int rbase = m0 + wm * WM, cbase = n0 + wn * WN;
  constexpr int STAGE_FLOATS = 32 * (WN + 4);
  constexpr bool kStage = (size_t)WGM * WGN * STAGE_FLOATS * sizeof(float) <= gemm_lds_bytes<AK, BKM, BM, BN, BK, WGM, WGN>();
  if constexpr (kStage) {
    float* stage = (float*)lds_raw + wave * STAGE_FLOATS;     // the last loop iteration ended with a barrier
    if (p.partial) tile_epilogue_lds<EPI_PARTIAL, TI, TJ>(p, acc, rbase, cbase, lane, split, stage);
    else if (p.c_f32) tile_epilogue_lds<EPI_F32, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage);
    else if (p.epi == 0) tile_epilogue_lds<EPI_ACT, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage);
    else if (p.epi == 1) tile_epilogue_lds<EPI_ACT_RES, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage);
    else if (p.epi == 2) tile_epilogue_lds<EPI_ACT_GELU, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage);
    else tile_epilogue_lds<EPI_ACT_DGELU, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage);
  } else {
    if (p.partial) tile_epilogue<EPI_PARTIAL, TI, TJ>(p, acc, rbase, cbase, lane, split);
    else if (p.c_f32) tile_epilogue<EPI_F32, TI, TJ>(p, acc, rbase, cbase, lane, 0);
    else if (p.epi == 0) tile_epilogue<EPI_ACT, TI, TJ>(p, acc, rbase, cbase, lane, 0);
    else if (p.epi == 1) tile_epilogue<EPI_ACT_RES, TI, TJ>(p, acc, rbase, cbase, lane, 0);
    else if (p.epi == 2) tile_epilogue<EPI_ACT_GELU, TI, TJ>(p, acc, rbase, cbase, lane, 0);
    else tile_epilogue<EPI_ACT_DGELU, TI, TJ>(p, acc, rbase, cbase, lane, 0);
  }
}

// sums the split-K partials in split order and applies the epilogue (four columns per thread)
__global__ __launch_bounds__(256) void splitk_reduce_kernel(GemmDev p, int splits) {
  const int64_t mn = (int64_t)p.M * p.N;
  if ((p.N & 3) == 0) {
    const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (idx >= mn) return;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int z = 0; z < splits; ++z) {
      const float4 t = *(const float4*)(p.partial + z * mn + idx);
      s.x += t.x; s.y += t.y; s.z += t.z; s.w += t.w;
    }
    const int row = (int)(idx / p.N), col = (int)(idx % p.N);
    GemmDev q = p;
    q.partial = nullptr;
    if (p.c_f32) store_quad<EPI_F32>(q, row, col, s, quad_aligned<EPI_F32>(q), 0);
    else if (p.epi == 0) store_quad<EPI_ACT>(q, row, col, s, quad_aligned<EPI_ACT>(q), 0);
    else if (p.epi == 1) store_quad<EPI_ACT_RES>(q, row, col, s, quad_aligned<EPI_ACT_RES>(q), 0);
    else if (p.epi == 2) store_quad<EPI_ACT_GELU>(q, row, col, s, quad_aligned<EPI_ACT_GELU>(q), 0);
    else store_quad<EPI_ACT_DGELU>(q, row, col, s, quad_aligned<EPI_ACT_DGELU>(q), 0);
  } else {
    for (int t = 0; t < 4; ++t) {
      const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4 + t;
      if (idx >= mn) return;
      float s = 0.f;
      for (int z = 0; z < splits; ++z) s += p.partial[z * mn + idx];
      epilogue_store<bf16>(p, (int)(idx / p.N), (int)(idx % p.N), s);
    }
  }
}

// ------------------------------------------------------------------------------------------
// plain SIMT kernel (any element type, exact bounds checks, fp32 accumulation)
// ------------------------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(256) void gemm_simt(GemmDev p, int a_kmajor, int b_kmajor) {
  constexpr int TS = 64, KS = 16;
  __shared__ float sA[KS][TS + 1];
  __shared__ float sB[KS][TS + 1];
  const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
  const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  const T* A = (const T*)p.A;
  const T* B = (const T*)p.B;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;
  for (int k0 = 0; k0 < p.K; k0 += KS) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      int r, k;
      if (a_kmajor) { r = e / KS; k = e % KS; } else { k = e / TS; r = e % TS; }
      float v = 0.0f;
      if (m0 + r < p.M && k0 + k < p.K)
        v = to_f(a_kmajor ? A[(int64_t)(m0 + r) * p.lda + k0 + k] : A[(int64_t)(k0 + k) * p.lda + m0 + r]);
      sA[k][r] = v;
      if (b_kmajor) { r = e / KS; k = e % KS; } else { k = e / TS; r = e % TS; }
      v = 0.0f;
      if (n0 + r < p.N && k0 + k < p.K)
        v = to_f(b_kmajor ? B[(int64_t)(n0 + r) * p.ldb + k0 + k] : B[(int64_t)(k0 + k) * p.ldb + n0 + r]);
      sB[k][r] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < KS; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; b[i] = sB[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) epilogue_store<T>(p, m0 + ty * 4 + i, n0 + tx * 4 + j, acc[i][j]);
}

}  // namespace

namespace {

template <bool AK, bool BKM, int BM, int BN, int BK, int WGM, int WGN>
hipError_t launch_one(const GemmDev& p, dim3 grid, hipStream_t s) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr size_t lds = gemm_lds_bytes<AK, BKM, BM, BN, BK, WGM, WGN>();
  auto kern = gemm_bf16_mfma<AK, BKM, BM, BN, BK, WGM, WGN>;
  static bool configured = false;          // per instantiation; the attribute is per process and device-wide
  if (!configured && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  configured = true;
  hipLaunchKernelGGL(kern, grid, dim3(NT), lds, s, p);
  return hipSuccess;
}

template <int BM, int BN, int BK, int WGM, int WGN>
hipError_t launch_cfg(const GemmArgs& g, const GemmDev& p, int splits, hipStream_t s) {
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM, splits);
  if (g.a_kmajor && g.b_kmajor) return launch_one<true, true, BM, BN, BK, WGM, WGN>(p, grid, s);
  if (g.a_kmajor) return launch_one<true, false, BM, BN, BK, WGM, WGN>(p, grid, s);
  return launch_one<false, false, BM, BN, BK, WGM, WGN>(p, grid, s);
}

// The one tile shape in use: 128 x 128 x 32 with 2 x 2 waves, three blocks per CU.  Measured alternatives
// were equal or slower over the shapes of the training step and are not built: 256 x 128 and 256 x 256
// block tiles, 8-wave blocks, 64-deep k-tiles, asynchronous global->LDS rings with 4 stages, and a
// three-stage LDS pipeline with two fragment sets and a prescribed MFMA/LDS/global issue order (faster
// only with a single block per CU: 128 x 192 tiles gained 5-15 % on the N = 768 shapes and lost on the
// weight-gradient shapes).
constexpr int kBM = 128, kBN = 128, kBK = 32;

}  // namespace

hs_status launch_gemm(hs_ctx* ctx, const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return HS_OK;  // nothing to write
  if (g.K < 0) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: K < 0");
  if (!g.A || !g.B || !g.C) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: NULL operand");
  if ((g.epi == 1 || g.epi == 3) && !g.aux) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: epilogue needs aux");
  if (g.epi == 2 && (!g.C2 || g.c_f32)) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: GELU epilogue needs C2 and an activation-type C");
  if (g.epi < 0 || g.epi > 3) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: bad epilogue");
  GemmDev p;
  p.A = g.A; p.B = g.B; p.C = g.C; p.C2 = g.C2; p.bias = g.bias; p.aux = g.aux;
  p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldaux = g.ldaux;
  p.M = g.M; p.N = g.N; p.K = g.K; p.c_f32 = g.c_f32; p.epi = g.epi; p.beta = g.beta;
  p.partial = nullptr; p.k_per_split = g.K;
  p.drop = (g.drop && g.drop->thr && g.epi == 1) ? *g.drop : DropCfg{0u, 1.0f, 0u, 0u, 0u};
  p.drop_site = g.drop_site;
  const double flops = 2.0 * g.M * g.N * (double)g.K;
  const double bytes = ((double)g.M * g.K + (double)g.N * g.K) * esize(g.dtype) + (double)g.M * g.N * (g.c_f32 ? 4 : esize(g.dtype));
  const int kc = (g.a_kmajor && g.b_kmajor) ? KC_GEMM_FWD : (g.a_kmajor ? KC_GEMM_DX : KC_GEMM_DW);
  KScope scope(ctx ? ctx->prof : nullptr, kc, flops, bytes, s);
  if (g.dtype == HS_FP32) {
    dim3 grid((g.N + 63) / 64, (g.M + 63) / 64);
    hipLaunchKernelGGL(gemm_simt<float>, grid, dim3(256), 0, s, p, g.a_kmajor, g.b_kmajor);
  } else {
    if ((g.lda % 8) || (g.ldb % 8) || ((uintptr_t)g.A % 16) || ((uintptr_t)g.B % 16))
      return hs_fail(ctx, HS_ERR_SHAPE, "gemm(bf16): operand rows must be 16-byte aligned");
    if (g.a_kmajor && g.b_kmajor && (g.K % 8))
      return hs_fail(ctx, HS_ERR_SHAPE, "gemm(bf16): K must be a multiple of 8 when both operands are k-major");
    if (!g.a_kmajor && g.b_kmajor) return hs_fail(ctx, HS_ERR_UNIMPLEMENTED, "gemm(bf16): A m-major with B k-major is not built");
    // the kernel addresses each operand with 32-bit byte offsets from its start (one k-tile of slack)
    const int64_t a_rows = g.a_kmajor ? g.M : g.K, b_rows = g.b_kmajor ? g.N : g.K;
    const int64_t lim = ((int64_t)1 << 32) - 1;
    if ((a_rows + 2 * kBK) * g.lda * 2 + 4 * kBK > lim || (b_rows + 2 * kBK) * g.ldb * 2 + 4 * kBK > lim)
      return hs_fail(ctx, HS_ERR_SHAPE, "gemm(bf16): an operand exceeds 4 GiB");
    // split-K when the output has too few tiles to fill the chip and a scratch buffer was given
    const int64_t tiles = (int64_t)((g.M + kBM - 1) / kBM) * ((g.N + kBN - 1) / kBN);
    int splits = 1;
    if (g.ws && tiles < 256) {
      int64_t want = (512 + tiles - 1) / tiles;
      const int64_t by_k = g.K / (4 * kBK), by_ws = (int64_t)(g.ws_bytes / ((size_t)g.M * g.N * sizeof(float)));
      if (want > by_k) want = by_k;
      if (want > by_ws) want = by_ws;
      if (want > 32) want = 32;
      if (want > 1) splits = (int)want;
    }
    if (splits > 1) {
      p.partial = (float*)g.ws;
      p.k_per_split = (int)(((g.K + splits - 1) / splits + kBK - 1) / kBK * kBK);
      splits = (g.K + p.k_per_split - 1) / p.k_per_split;
    }
    hipError_t e = launch_cfg<kBM, kBN, kBK, 2, 2>(g, p, splits, s);
    if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("gemm launch: ") + hipGetErrorString(e));
    if (splits > 1) {
      const int64_t mn = (int64_t)g.M * g.N;
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((mn + 1023) / 1024)), dim3(256), 0, s, p, splits);
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("gemm launch: ") + hipGetErrorString(e));
  return HS_OK;
}
