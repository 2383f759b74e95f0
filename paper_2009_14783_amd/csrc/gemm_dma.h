// bf16 MFMA GEMM kernel whose operand tiles go from global memory straight into LDS (template); instantiated per
// operand layout in gemm_wide_*.hip beside the wide kernels, with which it shares fragments' layout and epilogues.
#pragma once
#include "gemm_wide.h"

namespace {

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel with direct global -> LDS operand loads
// ------------------------------------------------------------------------------------------
// Block tile (64 WGM) x 128 x BK, WGM x 2 waves of 64 x 64 (WGM = 2 or 4).  A k-tile is fetched by buffer loads that write LDS
// themselves (16 bytes per lane, one instruction fills 1 KiB of LDS in lane order), so that an operand byte never
// passes through a register and no LDS store instruction is issued.  S stages of LDS form a ring: the tile for
// k-step t + S - 1 is requested when step t starts, one barrier per k-tile.  What orders the loads against their
// readers is the wave's own load counter (the hardware retires these loads in order) followed by the barrier;
// both are written out by hand here, because a fence would make every wave wait for all of its loads.
//
// One instruction's 64 lanes land in consecutive 16-byte slots, so the bank-conflict-free LDS layouts are made on
// the global side: the lane that fills slot p of a row fetches the chunk whose number is p XOR a function of the row.
//   k-major operand ([rows, K], a row of the tile is BK contiguous elements): the layout of WideTile, rows
//     unpadded, chunk ^ ((row >> 1) & 7) for BK = 64 and chunk ^ ((row >> 2) & 3) for BK = 32.
//   m-major operand ([K, rows], a row of the tile is 128 or 256 contiguous elements of one contraction index k):
//     chunk ^ ((k & 3) << 2), which spreads the four k-rows that 16 lanes of a transposing read touch over four
//     64-byte bank groups.
// The contraction range of a block must be a multiple of BK (the launcher checks); rows beyond the matrix edge are
// clamped to the last row (their products are never stored).
typedef __attribute__((address_space(3))) void* lds_void_ptr;

// R: rows of the tile (128 or 256); NW: waves of the block, which share the tile's load instructions evenly
template <bool KMAJ, int BK, int R, int NW>
struct DmaTile {
  static_assert(BK == 32 || BK == 64, "k-tile of 32 or 64");
  static_assert(R == 128 || R == 256, "128 or 256 rows");
  static constexpr int BYTES = R * BK * 2;
  static constexpr int NI = BYTES / 1024 / NW;         // load instructions per wave and k-tile
  static_assert(NI >= 1 && NI * NW * 1024 == BYTES, "the tile must split evenly over the waves");
  static constexpr int CPR = BK / 8;                   // k-major: chunks per row
  static constexpr int RPI = 64 / CPR;                 // k-major: rows per instruction
  static constexpr int KPI = 64 / (R / 8);             // m-major: k-rows per instruction
  struct Cursor {
    __amdgpu_buffer_rsrc_t rsrc;
    unsigned off[NI];
    unsigned soff, step;
  };
  static __device__ __forceinline__ void init(Cursor& cu, const bf16* __restrict__ mat, int64_t ld, int row0, int rext, int kbeg, int K, int lane,
                                              int wave) {
    const int64_t rows = KMAJ ? rext : K, cols = KMAJ ? K : rext;
    const int64_t bytes = ((rows - 1) * ld + ((cols + 7) & ~(int64_t)7)) * 2;
    cu.rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)mat, 0, (int)(unsigned)bytes, 0x00020000);
    cu.step = (unsigned)(KMAJ ? (int64_t)BK * 2 : (int64_t)BK * ld * 2);
    cu.soff = (unsigned)(KMAJ ? (int64_t)kbeg * 2 : (int64_t)kbeg * ld * 2);
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int j = wave * NI + i;
      if (KMAJ) {
        const int row = j * RPI + lane / CPR, slot = lane % CPR;
        const int chunk = slot ^ (BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3));
        const int r = min(row0 + row, rext - 1);
        cu.off[i] = (unsigned)(((int64_t)r * ld + chunk * 8) * 2);
      } else {
        const int k = j * KPI + lane / (R / 8), slot = lane % (R / 8);
        const int chunk = slot ^ ((k & 3) << 2);
        const int n = min(row0 + chunk * 8, ((rext - 1) >> 3) << 3);
        cu.off[i] = (unsigned)(((int64_t)k * ld + n) * 2);
      }
    }
  }
  // request the cursor's k-tile into the tile at dst (wave-uniform) and advance
  static __device__ __forceinline__ void issue(Cursor& cu, unsigned char* __restrict__ dst, int wave) {
#pragma unroll
    for (int i = 0; i < NI; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(cu.rsrc, (lds_void_ptr)(dst + (wave * NI + i) * 1024), 16, (int)cu.off[i], (int)cu.soff, 0, 0);
    cu.soff += cu.step;
  }
  // LDS -> MFMA operand: lane gets elements (row = rbase + lane%32, k = ks*16 + 8*(lane/32) + 0..7)
  static __device__ __forceinline__ bf16x8 frag(const bf16* __restrict__ s, int rbase, int ks, int lane) {
    if (KMAJ) {
      return WideTile<true, R, BK, 64 * NW>::frag(s, rbase, ks, lane);
    } else {
      const int kb = ks * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
      const int nb = rbase + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
      const int pos = kb * R + ((((nb >> 3) ^ ((kb & 3) << 2))) << 3) + (nb & 7);     // kb + 4 has the same k & 3
      typedef s16x4 __attribute__((address_space(3))) * lds_v4;
      union { struct { s16x4 lo, hi; } p; bf16x8 v; } u;
      u.p.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + pos));
      u.p.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(s + pos + 4 * R));
      return u.v;
    }
  }
};

template <int BK, int S, int WGM>
constexpr size_t dma_lds_bytes() {
  const size_t pipe = (size_t)S * (64 * WGM + 128) * BK * 2;
  const size_t stage = (size_t)2 * WGM * 32 * (32 * 2 + 4) * sizeof(float) + kGeluTabN * sizeof(float2);
  return stage > pipe ? stage : pipe;
}

// s_waitcnt: the wave's vector-memory loads except the newest VM have completed, and so have all its LDS reads
template <int VM>
__device__ __forceinline__ void wait_loads() {
  static_assert(VM >= 0 && VM < 64, "6-bit counter");
  __builtin_amdgcn_s_waitcnt((VM & 15) | ((VM >> 4) << 14) | 0x70);
}

// One k-step: tile `cur` is read (after the wave's share of it has landed and every wave has arrived), the tile
// S - 1 steps ahead is requested into `nxt`, whose last readers passed the same barrier.
template <class TA, class TB, int KS, int AHEAD>
__device__ __forceinline__ void dma_step(typename TA::Cursor& ca, typename TB::Cursor& cb, unsigned char* __restrict__ nxt,
                                         const unsigned char* __restrict__ cur, f32x16 (&acc)[2][2], bool full_ring, bool request, int wm,
                                         int wn, int lane, int wave) {
  asm volatile("" ::: "memory");      // no LDS access of the step before moves below the barrier, none of this step above it
  if (full_ring) wait_loads<AHEAD*(TA::NI + TB::NI)>(); else wait_loads<0>();
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  if (request) {
    TA::issue(ca, nxt, wave);
    TB::issue(cb, nxt + TA::BYTES, wave);
  }
  const bf16* sA = (const bf16*)cur;
  const bf16* sB = (const bf16*)(cur + TA::BYTES);
  bf16x8 fa[KS][2], fb[KS][2];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
    for (int i = 0; i < 2; ++i) fa[ks][i] = TA::frag(sA, (wm * 2 + i) * 32, ks, lane);
#pragma unroll
    for (int j = 0; j < 2; ++j) fb[ks][j] = TB::frag(sB, (wn * 2 + j) * 32, ks, lane);
  }
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][i], fb[ks][j], acc[i][j], 0, 0, 0);
}

template <bool AK, bool BKM, int BK, int S, int WGM, int EPIS>
__device__ __forceinline__ void dma_tile(const GemmDev& p, int m0, int n0, int split, unsigned char* lds_raw) {
  constexpr int TI = 2, TJ = 2, KS = BK / 16, NW = 2 * WGM;
  static_assert(S >= 2 && S <= 4, "two to four stages");
  typedef DmaTile<AK, BK, 64 * WGM, NW> TA;
  typedef DmaTile<BKM, BK, 128, NW> TB;
  constexpr int STAGE = TA::BYTES + TB::BYTES;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int kbeg = split * p.k_per_split;
  const int kend = min(p.K, kbeg + p.k_per_split);
  const int nk = (kend - kbeg) / BK;

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  typename TA::Cursor ca;
  typename TB::Cursor cb;
  TA::init(ca, (const bf16*)p.A, p.lda, m0, p.M, kbeg, p.K, lane, wave);
  TB::init(cb, (const bf16*)p.B, p.ldb, n0, p.N, kbeg, p.K, lane, wave);

  // tiles 0 .. S-2 into stages 0 .. S-2
#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < nk) {
      TA::issue(ca, lds_raw + s * STAGE, wave);
      TB::issue(cb, lds_raw + s * STAGE + TA::BYTES, wave);
    }
  // Step t reads stage t % S and requests tile t + S - 1 into stage (t - 1) % S.  At its start the wave has
  // requested tiles up to min(t + S - 2, nk - 1): with all S - 2 tiles behind tile t in flight the counter is
  // waited down to their number of loads, otherwise (the last steps) to zero.
  for (int t0 = 0; t0 < nk; t0 += S) {
#pragma unroll
    for (int u = 0; u < S; ++u) {
      const int t = t0 + u;
      if (t < nk)
        dma_step<TA, TB, KS, S - 2>(ca, cb, lds_raw + ((u + S - 1) % S) * STAGE, lds_raw + u * STAGE, acc, t + S - 2 < nk, t + S - 1 < nk, wm, wn,
                                    lane, wave);
    }
  }
  asm volatile("" ::: "memory");
  wait_loads<0>();
  __builtin_amdgcn_s_barrier();   // every wave is done with the operand stages: they become the staging area of the epilogue
  asm volatile("" ::: "memory");

  const int rbase = m0 + wm * TI * 32, cbase = n0 + wn * TJ * 32;
  constexpr int STAGE_FLOATS = 32 * (32 * TJ + 4);
  float* stage = (float*)lds_raw + wave * STAGE_FLOATS;
  float2* const tab = (float2*)((float*)lds_raw + NW * STAGE_FLOATS);
  if (p.gelu_tab && (((EPIS >> EPI_ACT_GELU) | (EPIS >> EPI_ACT_DGELU)) & 1)) {
    for (int i = tid; i < kGeluTabN / 2; i += 64 * NW) ((float4*)tab)[i] = ((const float4*)p.gelu_tab)[i];
    __syncthreads();
  }
  constexpr auto has = [](int mode) { return (EPIS >> mode) & 1; };
  if (p.partial) { if constexpr (has(EPI_PARTIAL)) tile_epilogue_pipe<EPI_PARTIAL, TI, TJ>(p, acc, rbase, cbase, lane, split, stage, tab); }
  else if (p.c_f32) { if constexpr (has(EPI_F32)) tile_epilogue_pipe<EPI_F32, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage, tab); }
  else if (p.epi == 0) { if constexpr (has(EPI_ACT)) tile_epilogue_pipe<EPI_ACT, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage, tab); }
  else if (p.epi == 1) { if constexpr (has(EPI_ACT_RES)) tile_epilogue_pipe<EPI_ACT_RES, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage, tab); }
  else if (p.epi == 2) { if constexpr (has(EPI_ACT_GELU)) tile_epilogue_pipe<EPI_ACT_GELU, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage, tab); }
  else { if constexpr (has(EPI_ACT_DGELU)) tile_epilogue_pipe<EPI_ACT_DGELU, TI, TJ>(p, acc, rbase, cbase, lane, 0, stage, tab); }
}

// OCC: blocks per CU the register allocator leaves room for.
template <bool AK, bool BKM, int BK, int S, int WGM, int OCC>
__global__ __launch_bounds__(128 * WGM) __attribute__((amdgpu_waves_per_eu(OCC * WGM / 2, OCC * WGM / 2)))
void gemm_bf16_dma(GemmDev p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  // tile order as in gemm_bf16_wide
  const int nbx = gridDim.x, nby = gridDim.y, nb = nbx * nby;
  int v = (blockIdx.z * nby + blockIdx.y) * nbx + blockIdx.x;
  const int per_xcd = (nb * (int)gridDim.z) >> 3;
  if (v < 8 * per_xcd) v = (v & 7) * per_xcd + (v >> 3);
  const int split = v / nb;
  int tm, tn;
  tile_of_block<(WGM >= 4) ? 4 : 8>(v - split * nb, nbx, nby, tm, tn);
  dma_tile<AK, BKM, BK, S, WGM, wide_epilogues<AK, BKM>()>(p, tm * 64 * WGM, tn * 128, split, lds_raw);
}

template <bool AK, bool BKM, int BK, int S, int WGM, int OCC>
hipError_t launch_dma_one(const GemmDev& p, int splits, hipStream_t s) {
  constexpr size_t lds = dma_lds_bytes<BK, S, WGM>();
  static_assert(lds * OCC <= 160 * 1024, "stages do not fit the LDS of a CU");
  auto kern = gemm_bf16_dma<AK, BKM, BK, S, WGM, OCC>;
  static bool configured = false;
  if (!configured && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  configured = true;
  hipLaunchKernelGGL(kern, dim3((p.N + 127) / 128, (p.M + 64 * WGM - 1) / (64 * WGM), splits), dim3(128 * WGM), lds, s, p);
  return hipSuccess;
}

// the configurations of gemm_bf16_dma that are built: numbers continue those of launch_wide_layout
constexpr int kFirstDmaCfg = 7;
template <bool AK, bool BKM>
hipError_t launch_dma_layout(int cfg, const GemmDev& p, int splits, hipStream_t s) {
  switch (cfg) {
    case 7: return launch_dma_one<AK, BKM, 32, 4, 2, 2>(p, splits, s);
    case 8: return launch_dma_one<AK, BKM, 32, 3, 2, 3>(p, splits, s);
    case 9: return launch_dma_one<AK, BKM, 64, 2, 2, 2>(p, splits, s);
    case 10: return launch_dma_one<AK, BKM, 64, 3, 4, 1>(p, splits, s);
    case 11: return launch_dma_one<AK, BKM, 64, 2, 4, 1>(p, splits, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace
