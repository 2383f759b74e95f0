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
};

template <class T>
__device__ __forceinline__ void epilogue_store(const GemmDev& p, int row, int col, float v) {
  if (row >= p.M || col >= p.N) return;
  if (p.bias) v += to_f(((const T*)p.bias)[col]);
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
constexpr int KPAD = 8;    // k-major LDS rows: BK + 8 elements  (conflict-free 16-byte reads)
constexpr int MPAD = 32;   // m-major LDS rows: R + 32 elements  (row stride = 64 B mod 256 B)

template <bool KMAJ, int R, int BK>
struct OperandTile {
  static constexpr int LD = KMAJ ? (BK + KPAD) : (R + MPAD);
  static constexpr int ELEMS = KMAJ ? R * LD : BK * LD;
  static constexpr int CPR = KMAJ ? BK / 8 : R / 8;       // 8-element chunks per stored row
  static constexpr int NCH = R * BK / 8 / 256;            // chunks per thread
  static_assert(R * BK / 8 % 256 == 0, "tile must split evenly over 256 threads");

  // global -> registers (zero where out of range)
  static __device__ __forceinline__ void load(uint4 (&reg)[NCH], const bf16* __restrict__ base, int64_t ld, int row0, int rext,
                                              int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * 256;
      const int a = c / CPR, b = (c % CPR) * 8;
      int64_t off; bool ok;
      if (KMAJ) { ok = (row0 + a < rext) && (k0 + b < K); off = (int64_t)(row0 + a) * ld + k0 + b; }
      else      { ok = (k0 + a < K) && (row0 + b < rext); off = (int64_t)(k0 + a) * ld + row0 + b; }
      uint4 v = make_uint4(0, 0, 0, 0);
      if (ok) v = *(const uint4*)(base + off);
      reg[i] = v;
    }
  }
  // registers -> LDS
  static __device__ __forceinline__ void store(const uint4 (&reg)[NCH], bf16* s, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * 256;
      const int a = c / CPR, b = (c % CPR) * 8;
      *(uint4*)(s + a * LD + b) = reg[i];
    }
  }
  // LDS -> MFMA operand: lane gets elements (row = rbase + lane%32, k = ks*16 + 8*(lane/32) + 0..7)
  static __device__ __forceinline__ bf16x8 frag(const bf16* s, int rbase, int ks, int lane) {
    if (KMAJ) {
      return *(const bf16x8*)(s + (rbase + (lane & 31)) * LD + ks * 16 + (lane >> 5) * 8);
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

template <bool AK, bool BKM, int BM, int BN, int BK>
__global__ __launch_bounds__(256) void gemm_bf16_mfma(GemmDev p) {
  typedef OperandTile<AK, BM, BK> TA;
  typedef OperandTile<BKM, BN, BK> TB;
  constexpr int WM = BM / 2, WN = BN / 2, TI = WM / 32, TJ = WN / 32;
  __shared__ __attribute__((aligned(16))) bf16 sA[2][TA::ELEMS];
  __shared__ __attribute__((aligned(16))) bf16 sB[2][TB::ELEMS];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const bf16* A = (const bf16*)p.A;
  const bf16* B = (const bf16*)p.B;

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  uint4 ra[TA::NCH], rb[TB::NCH];
  const int nk = (p.K + BK - 1) / BK;
  TA::load(ra, A, p.lda, m0, p.M, 0, p.K, tid);
  TB::load(rb, B, p.ldb, n0, p.N, 0, p.K, tid);
  TA::store(ra, sA[0], tid);
  TB::store(rb, sB[0], tid);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) {
      TA::load(ra, A, p.lda, m0, p.M, (kt + 1) * BK, p.K, tid);
      TB::load(rb, B, p.ldb, n0, p.N, (kt + 1) * BK, p.K, tid);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[TI], fb[TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i) fa[i] = TA::frag(sA[cur], wm * WM + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < TJ; ++j) fb[j] = TB::frag(sB[cur], wn * WN + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      TA::store(ra, sA[cur ^ 1], tid);
      TB::store(rb, sB[cur ^ 1], tid);
    }
    __syncthreads();
  }

  // result layout of the 32x32 tile: register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        const int col = n0 + wn * WN + j * 32 + (lane & 31);
        epilogue_store<bf16>(p, row, col, acc[i][j][r]);
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
    constexpr int BM = 128, BN = 128, BK = 32;
    dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM);
    if (g.a_kmajor && g.b_kmajor) hipLaunchKernelGGL((gemm_bf16_mfma<true, true, BM, BN, BK>), grid, dim3(256), 0, s, p);
    else if (g.a_kmajor) hipLaunchKernelGGL((gemm_bf16_mfma<true, false, BM, BN, BK>), grid, dim3(256), 0, s, p);
    else hipLaunchKernelGGL((gemm_bf16_mfma<false, false, BM, BN, BK>), grid, dim3(256), 0, s, p);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("gemm launch: ") + hipGetErrorString(e));
  return HS_OK;
}
