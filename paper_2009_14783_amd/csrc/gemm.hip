// GEMM kernels: C[M,N] = sum_k A(m,k) B(n,k) with fused epilogues.
//   bf16: MFMA 32x32x16 tiles, fp32 accumulation, LDS double buffering.  Operands whose
//         contraction index is NOT the contiguous one are staged in their natural layout and read
//         with the LDS transpose read of gfx950, so every global and LDS access is 16/8 bytes wide.
//   fp32: plain tiled SIMT kernel (small reference-precision configurations only).
#include "gemm_dev.h"

hipError_t gemm_wide_launch_kk(int cfg, const GemmDev& p, int splits, hipStream_t s);
hipError_t gemm_wide_launch_kn(int cfg, const GemmDev& p, int splits, hipStream_t s);
hipError_t gemm_wide_launch_nn(int cfg, const GemmDev& p, int splits, hipStream_t s);
hipError_t gemm_wide_group_launch_nn(const GemmGroupDev& g, hipStream_t s);

namespace {

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

// the two tables of gelu_tab_eval, filled once per process by a kernel on the stream of the first product that needs them
static __device__ float2 gelu_tables[2][kGeluTabN];
__global__ __launch_bounds__(256) void gelu_table_kernel(float2* tab) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= 2 * kGeluTabN) return;
  const int which = i / kGeluTabN, k = i % kGeluTabN;
  const double h = 2.0 * (double)kGeluTabR / kGeluTabN;
  auto f = [&](double x) {
    const double cdf = 0.5 * (1.0 + erf(x * 0.70710678118654752440));
    return which == 0 ? cdf : cdf + x * 0.39894228040143267794 * exp(-0.5 * x * x);
  };
  const double a = f(-(double)kGeluTabR + k * h), b = f(-(double)kGeluTabR + (k + 1) * h);
  tab[i] = make_float2((float)a, (float)(b - a));
}
static hipError_t gelu_table(int which, hipStream_t s, const float2** out) {
  static float2* dev_tab = nullptr;
  if (!dev_tab) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(gelu_tables));
    if (e != hipSuccess) return e;
    // every later use is ordered behind this launch only on `s`; other streams wait for it once, here
    hipLaunchKernelGGL(gelu_table_kernel, dim3(2 * kGeluTabN / 256), dim3(256), 0, s, (float2*)p);
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return e;
    dev_tab = (float2*)p;
  }
  *out = dev_tab + which * kGeluTabN;
  return hipSuccess;
}

// Tile configurations.  0 is gemm_bf16_mfma (128 x 128 x 32, three blocks per CU); 1..6 are gemm_bf16_wide (global ->
// registers -> LDS), 7..11 gemm_bf16_dma (global -> LDS directly).  In use: 0, 5 and 9 (see launch_gemm) and, for the
// grouped weight-gradient launch, the tile of 6.  The others are kept as measured alternatives, selectable for
// timing runs through gemm_set_variant: on the shapes of the training step they were equal or slower.
struct TileCfg { int bm, bn, bk; };
constexpr TileCfg kTileCfg[] = {{128, 128, 32}, {256, 256, 64}, {256, 192, 64}, {128, 192, 64}, {256, 128, 32}, {128, 128, 64}, {256, 128, 64},
                                {128, 128, 32}, {128, 128, 32}, {128, 128, 64}, {256, 128, 64}, {256, 128, 64}};
constexpr int kNumTileCfg = sizeof(kTileCfg) / sizeof(kTileCfg[0]);
int gemm_cfg_override = -1;    // >= 0: use this configuration for every bf16 product of some size that it can serve (timing runs)

constexpr int kMaxBK = 64;

}  // namespace

static hs_status check_gemm_args(hs_ctx* ctx, const GemmArgs& g) {
  if (g.K < 0) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: K < 0");
  if (!g.A || !g.B || !g.C) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: NULL operand");
  if ((g.epi == 1 || g.epi == 3) && !g.aux) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: epilogue needs aux");
  if (g.epi == 2 && (!g.C2 || g.c_f32)) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: GELU epilogue needs C2 and an activation-type C");
  if (g.epi < 0 || g.epi > 3) return hs_fail(ctx, HS_ERR_INVALID_ARG, "gemm: bad epilogue");
  if (g.dtype == HS_BF16) {
    if ((g.lda % 8) || (g.ldb % 8) || ((uintptr_t)g.A % 16) || ((uintptr_t)g.B % 16))
      return hs_fail(ctx, HS_ERR_SHAPE, "gemm(bf16): operand rows must be 16-byte aligned");
    if (g.a_kmajor && g.b_kmajor && (g.K % 8))
      return hs_fail(ctx, HS_ERR_SHAPE, "gemm(bf16): K must be a multiple of 8 when both operands are k-major");
    if (!g.a_kmajor && g.b_kmajor) return hs_fail(ctx, HS_ERR_UNIMPLEMENTED, "gemm(bf16): A m-major with B k-major is not built");
    // the kernels address each operand with 32-bit byte offsets from its start (a few k-tiles of slack)
    const int64_t a_rows = g.a_kmajor ? g.M : g.K, b_rows = g.b_kmajor ? g.N : g.K;
    const int64_t lim = ((int64_t)1 << 32) - 1;
    if ((a_rows + 3 * kMaxBK) * g.lda * 2 + 4 * kMaxBK > lim || (b_rows + 3 * kMaxBK) * g.ldb * 2 + 4 * kMaxBK > lim)
      return hs_fail(ctx, HS_ERR_SHAPE, "gemm(bf16): an operand exceeds 4 GiB");
  }
  return HS_OK;
}

static GemmDev gemm_dev_args(const GemmArgs& g) {
  GemmDev p;
  p.A = g.A; p.B = g.B; p.C = g.C; p.C2 = g.C2; p.bias = g.bias; p.aux = g.aux;
  p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldaux = g.ldaux;
  p.M = g.M; p.N = g.N; p.K = g.K; p.c_f32 = g.c_f32; p.epi = g.epi; p.beta = g.beta;
  p.partial = nullptr; p.k_per_split = g.K; p.gelu_tab = nullptr;
  p.drop = (g.drop && g.drop->thr && g.epi == 1) ? *g.drop : DropCfg{0u, 1.0f, 0u, 0u, 0u};
  p.drop_site = g.drop_site;
  return p;
}

int gemm_variant_count() { return kNumTileCfg; }
void gemm_set_variant(int variant) { gemm_cfg_override = variant; }

// Several weight-gradient products (A m-major, B n-major, fp32 C = beta C + A^T-style product, no epilogue) in ONE
// launch of the grouped kernel: no split-K, no partial sums in memory.  Anything else, or more than 8 products,
// runs as separate launches.
hs_status launch_gemm_group(hs_ctx* ctx, const GemmArgs* gs, int n, hipStream_t s) {
  bool groupable = n >= 1 && n <= 8;
  for (int i = 0; i < n && groupable; ++i) {
    const GemmArgs& g = gs[i];
    groupable = g.dtype == HS_BF16 && !g.a_kmajor && !g.b_kmajor && g.c_f32 && g.epi == 0 && !g.bias && g.M > 0 && g.N > 0 && g.K > 0;
  }
  if (!groupable) {
    for (int i = 0; i < n; ++i) { hs_status st = launch_gemm(ctx, gs[i], s); if (st != HS_OK) return st; }
    return HS_OK;
  }
  GemmGroupDev gd;
  gd.n = n;
  int tiles = 0;
  double flops = 0, bytes = 0;
  for (int i = 0; i < n; ++i) {
    hs_status st = check_gemm_args(ctx, gs[i]);
    if (st != HS_OK) return st;
    gd.prob[i] = gemm_dev_args(gs[i]);
    gd.first_tile[i] = tiles;
    tiles += ((gs[i].M + kGroupBM - 1) / kGroupBM) * ((gs[i].N + kGroupBN - 1) / kGroupBN);
    flops += 2.0 * gs[i].M * gs[i].N * (double)gs[i].K;
    bytes += ((double)gs[i].M * gs[i].K + (double)gs[i].N * gs[i].K) * 2 + (double)gs[i].M * gs[i].N * 4;
  }
  for (int i = n; i <= 8; ++i) gd.first_tile[i] = tiles;
  KScope scope(ctx ? ctx->prof : nullptr, KC_GEMM_DW, flops, bytes, s);
  hipError_t e = gemm_wide_group_launch_nn(gd, s);
  if (e == hipSuccess) e = hipGetLastError();
  if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("grouped gemm launch: ") + hipGetErrorString(e));
  return HS_OK;
}

// whether gemm_bf16_wide is built with the epilogue this product needs (see wide_epilogues in gemm_wide.h)
static bool wide_supports(const GemmArgs& g) {
  if (g.a_kmajor && g.b_kmajor) return g.c_f32 ? true : (g.epi == 0 || g.epi == 1 || g.epi == 2);
  if (g.a_kmajor) return !g.c_f32 && (g.epi == 0 || g.epi == 1 || g.epi == 3);
  return g.c_f32 != 0;
}

hs_status launch_gemm(hs_ctx* ctx, const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return HS_OK;  // nothing to write
  {
    hs_status st = check_gemm_args(ctx, g);
    if (st != HS_OK) return st;
  }
  GemmDev p = gemm_dev_args(g);
  const double flops = 2.0 * g.M * g.N * (double)g.K;
  const double bytes = ((double)g.M * g.K + (double)g.N * g.K) * esize(g.dtype) + (double)g.M * g.N * (g.c_f32 ? 4 : esize(g.dtype));
  const int kc = (g.a_kmajor && g.b_kmajor) ? KC_GEMM_FWD : (g.a_kmajor ? KC_GEMM_DX : KC_GEMM_DW);
  KScope scope(ctx ? ctx->prof : nullptr, kc, flops, bytes, s);
  if (g.dtype == HS_FP32) {
    dim3 grid((g.N + 63) / 64, (g.M + 63) / 64);
    hipLaunchKernelGGL(gemm_simt<float>, grid, dim3(256), 0, s, p, g.a_kmajor, g.b_kmajor);
  } else {
    // Configuration for products of some size whose epilogue the wide kernels are built with: 128 x 128 x 64 tiles, two
    // blocks per CU - the direct-to-LDS kernel for the activation-gradient products (A k-major, B n-major; it gained 6-12 %
    // on their shapes, whole output matrices of 8192 rows, and lost on the forward pass's half batches), the
    // register-staged kernel otherwise.  Small or ragged products and the remaining epilogues: the three-blocks-per-CU kernel.
    int cfg = !(g.M >= 256 && g.N >= 256 && g.K >= 256) ? 0
              : (gemm_cfg_override >= 0 && gemm_cfg_override < kNumTileCfg) ? gemm_cfg_override
              : ((g.a_kmajor && !g.b_kmajor) ? 9 : 5);
    if (cfg != 0 && !wide_supports(g)) cfg = 0;
    if (cfg >= 7 && g.K % kTileCfg[cfg].bk) cfg = 5;      // the direct-to-LDS kernel takes whole k-tiles only
    const int kBM = kTileCfg[cfg].bm, kBN = kTileCfg[cfg].bn, kBK = kTileCfg[cfg].bk;
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
    hipError_t e;
    if (cfg != 0 && (g.epi == 2 || g.epi == 3)) {
      e = gelu_table(g.epi == 2 ? 0 : 1, s, &p.gelu_tab);
      if (e != hipSuccess) return hs_fail(ctx, HS_ERR_HIP, std::string("gemm: GELU table: ") + hipGetErrorString(e));
    }
    if (cfg == 0) e = launch_cfg<128, 128, 32, 2, 2>(g, p, splits, s);
    else if (g.a_kmajor && g.b_kmajor) e = gemm_wide_launch_kk(cfg, p, splits, s);
    else if (g.a_kmajor) e = gemm_wide_launch_kn(cfg, p, splits, s);
    else e = gemm_wide_launch_nn(cfg, p, splits, s);
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
