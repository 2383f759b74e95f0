// The bf16 MFMA GEMM kernel with wide block tiles (template); instantiated per operand layout in gemm_wide_*.hip.
#pragma once
#include <type_traits>

#include "gemm_dev.h"

namespace {

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel with wide block tiles
// ------------------------------------------------------------------------------------------
// The same contraction with a block tile of (32 TI WGM) x (32 TJ WGN) x BK and one or two blocks per CU.
// What changes against the kernel above: each wave owns TI x TJ MFMA tiles (up to 128 x 128), so one operand
// fragment read from LDS feeds up to four MFMAs and a byte fetched from L2 up to twice as many flops; the
// main loop is one basic block without masks or selects (ragged edges are handled by clamping the global
// row of a chunk once, before the loop; only the last k-tiles, which may be partial or absent, go through a
// guarded copy of the loop body); one barrier per k-tile, placed before the last 16-deep step so that the
// matrix pipes have queued work while the waves meet; instruction order prescribed per MFMA.
template <bool KMAJ, int R, int BK, int NT>
struct WideTile {
  static_assert(BK == 32 || BK == 64, "k-tile of 32 or 64");
  static constexpr int CPK = BK / 8;                      // 16-byte chunks of a k-major row
  static constexpr int LD = KMAJ ? BK : (R + MPAD);
  static constexpr int ELEMS = KMAJ ? R * BK : BK * LD;
  static constexpr int CPR = KMAJ ? CPK : R / 8;          // chunks per stored row
  static constexpr int NCH = R * BK / 8 / NT;             // chunks per thread
  static_assert(R * BK / 8 % NT == 0, "tile must split evenly over the threads");
  // k-major rows sit in LDS unpadded with their chunks permuted so that 16 consecutive rows read at one
  // k-offset, and the two 128-byte (four 64-byte) rows that 16 lanes write at once, fall into 16 different
  // 16-byte bank groups.
  static __device__ __forceinline__ int swz(int row, int chunk) {
    return (BK == 64 ? (chunk ^ ((row >> 1) & 7)) : (chunk ^ ((row >> 2) & 3))) * 8;
  }
  // Global side: buffer loads with one 32-bit byte offset per chunk (row clamped into the matrix once) plus a
  // uniform offset that advances by one k-tile per load; reads beyond the operand's last readable chunk return
  // zero instead of faulting.
  struct Cursor {
    __amdgpu_buffer_rsrc_t rsrc;
    unsigned off[NCH];
    unsigned soff, step;
  };
  // rows x cols elements with leading dimension ld: KMAJ [rext, K], else [K, rext]
  static __device__ __forceinline__ void init(Cursor& cu, const bf16* __restrict__ mat, int64_t ld, int row0, int rext, int kbeg, int K, int tid) {
    const int64_t rows = KMAJ ? rext : K, cols = KMAJ ? K : rext;
    const int64_t bytes = ((rows - 1) * ld + ((cols + 7) & ~(int64_t)7)) * 2;
    cu.rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)mat, 0, (int)(unsigned)bytes, 0x00020000);
    cu.step = (unsigned)(KMAJ ? (int64_t)BK * 2 : (int64_t)BK * ld * 2);
    cu.soff = (unsigned)(KMAJ ? (int64_t)kbeg * 2 : (int64_t)kbeg * ld * 2);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * NT;
      const int a = c / CPR, b = (c % CPR) * 8;
      if (KMAJ) { const int r = min(row0 + a, rext - 1); cu.off[i] = (unsigned)(((int64_t)r * ld + b) * 2); }
      else      { const int r = min(row0 + b, ((rext - 1) >> 3) << 3); cu.off[i] = (unsigned)(((int64_t)a * ld + r) * 2); }
    }
  }
  // contraction offset of chunk i inside a k-tile
  static __device__ __forceinline__ int koff(int i, int tid) { const int c = tid + i * NT; return KMAJ ? (c % CPR) * 8 : c / CPR; }
  // global -> registers for the current k-tile, then advance.  GUARD: chunks at or beyond `kleft` contraction steps
  // from the tile start read the start of the tile row instead and are zeroed on their way to LDS.
  template <bool GUARD>
  static __device__ __forceinline__ void load_chunk(uint4& reg, const Cursor& cu, int i, int kleft, int tid) {
    typedef int v4i __attribute__((ext_vector_type(4)));
    const unsigned vo = (!GUARD || koff(i, tid) < kleft) ? cu.off[i] : 0u;
    const v4i v = __builtin_amdgcn_raw_buffer_load_b128(cu.rsrc, (int)vo, (int)((!GUARD || kleft > 0) ? cu.soff : 0u), 0);
    reg = make_uint4((unsigned)v.x, (unsigned)v.y, (unsigned)v.z, (unsigned)v.w);
  }
  template <bool GUARD>
  static __device__ __forceinline__ void load(uint4 (&reg)[NCH], Cursor& cu, int kleft, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) load_chunk<GUARD>(reg[i], cu, i, kleft, tid);
    cu.soff += cu.step;
  }
  template <bool GUARD>
  static __device__ __forceinline__ void store_chunk(const uint4& reg, bf16* s, int i, int kleft, int tid) {
    const int c = tid + i * NT;
    const int a = c / CPR, b = (c % CPR) * 8;
    uint4 v = reg;
    if (GUARD) {
      const unsigned keep = (koff(i, tid) < kleft) ? 0xffffffffu : 0u;
      v.x &= keep; v.y &= keep; v.z &= keep; v.w &= keep;
    }
    *(uint4*)(s + a * LD + (KMAJ ? swz(a, b >> 3) : b)) = v;
  }
  template <bool GUARD>
  static __device__ __forceinline__ void store(const uint4 (&reg)[NCH], bf16* s, int kleft, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) store_chunk<GUARD>(reg[i], s, i, kleft, tid);
  }
  // LDS -> MFMA operand: lane gets elements (row = rbase + lane%32, k = ks*16 + 8*(lane/32) + 0..7)
  static __device__ __forceinline__ bf16x8 frag(const bf16* s, int rbase, int ks, int lane) {
    if (KMAJ) {
      const int row = rbase + (lane & 31);
      return *(const bf16x8*)(s + row * LD + swz(row, ks * 2 + (lane >> 5)));
    } else {
      // transpose read, see OperandTile::frag
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

template <bool AK, bool BKM, int TI, int TJ, int WGM, int WGN, int BK>
constexpr size_t wide_lds_bytes() {
  constexpr int NT = 64 * WGM * WGN;
  const size_t pipe = 2 * sizeof(bf16) * (size_t)(WideTile<AK, 32 * TI * WGM, BK, NT>::ELEMS + WideTile<BKM, 32 * TJ * WGN, BK, NT>::ELEMS);
  const size_t stage = (size_t)WGM * WGN * 32 * (32 * TJ + 4) * sizeof(float) + kGeluTabN * sizeof(float2);   // + the GELU table
  return stage > pipe ? stage : pipe;
}

// Epilogue of a wave's TI x TJ result tiles for the wide kernels, which run one or two blocks per CU: with so few
// waves the memory latency of an epilogue has to be covered inside each wave.  Same staging through LDS as
// tile_epilogue_lds; the residual / pre-activation values (aux) of the next 32-row slab are requested before the
// current slab is worked on, and nothing keeps the compiler from overlapping slabs.  Regions that touch the matrix
// edge, unaligned operands and dropout take the general routine.
template <int MODE, int TI, int TJ>
__device__ __forceinline__ void tile_epilogue_pipe(const GemmDev& p, const f32x16 (&acc)[TI][TJ], int rbase, int cbase, int lane, int split,
                                                   float* stage, const float2* tab) {
  constexpr int WN = 32 * TJ, LDW = WN + 4;
  constexpr int LPR = WN / 8, NIT = 32 * LPR / 64;
  constexpr bool HAS_AUX = MODE == EPI_ACT_RES || MODE == EPI_ACT_DGELU;
  const bool inside = octet_aligned<MODE>(p) && rbase + 32 * TI <= p.M && cbase + WN <= p.N && !(MODE == EPI_ACT_RES && p.drop.thr);
  if (!inside) { tile_epilogue_lds<MODE, TI, TJ>(p, acc, rbase, cbase, lane, split, stage); return; }
  const bf16* bias = (const bf16*)p.bias;
  const bf16* aux = (const bf16*)p.aux;
  bf16x8 anext[NIT];
  auto load_aux = [&](int i) __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int piece = it * 64 + lane;
      const int row = rbase + i * 32 + piece / LPR, col = cbase + (piece % LPR) * 8;
      anext[it] = *(const bf16x8*)(aux + (int64_t)row * p.ldaux + col);
    }
  };
  if (HAS_AUX) load_aux(0);
#pragma unroll
  for (int i = 0; i < TI; ++i) {
    bf16x8 acur[NIT];
    if (HAS_AUX) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) acur[it] = anext[it];
      if (i + 1 < TI) load_aux(i + 1);
    }
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * LDW + j * 32 + (lane & 31)] = acc[i][j][r];
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int piece = it * 64 + lane;
      const int lr = piece / LPR, lc = (piece % LPR) * 8;
      const float4 lo = *(const float4*)(stage + lr * LDW + lc), hi = *(const float4*)(stage + lr * LDW + lc + 4);
      const int row = rbase + i * 32 + lr, col = cbase + lc;
      float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      if (MODE == EPI_PARTIAL) {
        float* dst = p.partial + ((int64_t)split * p.M + row) * p.N + col;
        *(float4*)dst = lo; *(float4*)(dst + 4) = hi;
        continue;
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
        if (HAS_AUX) {
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] = (MODE == EPI_ACT_RES) ? v[t] + (float)acur[it][t] : v[t] * gelu_tab_eval(tab, (float)acur[it][t]);
        }
        bf16x8 c;
#pragma unroll
        for (int t = 0; t < 8; ++t) c[t] = (bf16)v[t];
        *(bf16x8*)((bf16*)p.C + o) = c;
        if (MODE == EPI_ACT_GELU) {
          bf16x8 g;
#pragma unroll
          for (int t = 0; t < 8; ++t) g[t] = (bf16)(v[t] * gelu_tab_eval(tab, v[t]));
          *(bf16x8*)((bf16*)p.C2 + o) = g;
        }
      }
    }
  }
}

// One block tile of C for the k-range of `split`: main loop and epilogue.
// NSETS register sets hold the k-tiles in flight from global memory: a tile is requested NSETS iterations
// before it is written to LDS.  EPIS: bit mask (1 << mode) of the epilogues that are compiled in.
template <bool AK, bool BKM, int TI, int TJ, int WGM, int WGN, int BK, int NSETS, int EPIS>
__device__ __forceinline__ void wide_tile(const GemmDev& p, int m0, int n0, int split, unsigned char* lds_raw) {
  constexpr int NT = 64 * WGM * WGN, BM = 32 * TI * WGM, BN = 32 * TJ * WGN, KS = BK / 16;
  static_assert(NSETS == 1 || NSETS == 2, "one or two register sets");
  typedef WideTile<AK, BM, BK, NT> TA;
  typedef WideTile<BKM, BN, BK, NT> TB;
  bf16* const sA0 = (bf16*)lds_raw;                       // two A buffers, then two B buffers
  bf16* const sB0 = (bf16*)lds_raw + 2 * TA::ELEMS;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int kbeg = split * p.k_per_split;
  const int kend = min(p.K, kbeg + p.k_per_split);
  const int klen = kend - kbeg;
  const int nk = (klen + BK - 1) / BK;          // k-tiles, the last one possibly partial
  const int nfull = klen / BK;

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  typename TA::Cursor ca;
  typename TB::Cursor cb;
  TA::init(ca, (const bf16*)p.A, p.lda, m0, p.M, kbeg, p.K, tid);
  TB::init(cb, (const bf16*)p.B, p.ldb, n0, p.N, kbeg, p.K, tid);

  uint4 ra[NSETS][TA::NCH], rb[NSETS][TB::NCH];
  bf16x8 fa[2][TI], fb[2][TJ];
  auto frags = [&](int buf, int cur, int ks) __attribute__((always_inline)) {
    const bf16* sAc = sA0 + cur * TA::ELEMS;
    const bf16* sBc = sB0 + cur * TB::ELEMS;
#pragma unroll
    for (int i = 0; i < TI; ++i) fa[buf][i] = TA::frag(sAc, (wm * TI + i) * 32, ks, lane);
#pragma unroll
    for (int j = 0; j < TJ; ++j) fb[buf][j] = TB::frag(sBc, (wn * TJ + j) * 32, ks, lane);
  };
  // contraction steps left from the start of k-tile t (<= 0: the tile does not exist)
  auto kleft = [&](int t) __attribute__((always_inline)) { return klen - t * BK; };

  // prologue: tiles 0 .. NSETS requested, tile 0 in LDS buffer 0, its first fragments in registers
  TA::template load<true>(ra[0], ca, kleft(0), tid);
  TB::template load<true>(rb[0], cb, kleft(0), tid);
  if (NSETS == 2) {
    TA::template load<true>(ra[NSETS - 1], ca, kleft(1), tid);
    TB::template load<true>(rb[NSETS - 1], cb, kleft(1), tid);
  }
  TA::template store<true>(ra[0], sA0, kleft(0), tid);
  TB::template store<true>(rb[0], sB0, kleft(0), tid);
  TA::template load<true>(ra[0], ca, kleft(NSETS), tid);
  TB::template load<true>(rb[0], cb, kleft(NSETS), tid);
  __syncthreads();
  frags(0, 0, 0);
  static_assert((TA::NCH + TB::NCH + TI * TJ - 1) / (TI * TJ) <= 2, "at most two chunks per MFMA of step 0");
  static_assert(TI + TJ <= TI * TJ, "one fragment read per MFMA must cover a step");

  // One k-tile of work.  On entry LDS buffer `cur` holds tile t and fragment set 0 its first step; register set
  // `set` holds tile t+1.  Step 0 moves tile t+1 to the other LDS buffer and requests tile t+1+NSETS into the
  // freed registers; every step reads the fragments of the next one while its MFMAs run; the barrier sits
  // before the last step, whose MFMAs cover the wait and the first fragment reads of tile t+1.
  // FAST: the contraction range is a whole number of k-tiles: no guards, the body is one basic block, and it also runs
  // for the last iterations, whose requests go to tiles that do not exist: those are sent beyond the end of the
  // operand (see `past`), where a buffer load returns zeros without touching memory, and what they bring is written
  // to the LDS buffer nobody reads any more.
  const unsigned past = 0x80000000u;            // beyond any operand this kernel accepts less one k-tile row range
  auto body = [&](auto fast_tag, auto cur_tag, int t) __attribute__((always_inline)) {
    constexpr bool FAST = decltype(fast_tag)::value;
    constexpr int cur = decltype(cur_tag)::value, nxt = cur ^ 1, set = (NSETS == 2) ? nxt : 0;
    constexpr int NM = TI * TJ;
    constexpr int NF = TI + TJ;                                         // fragments per step
    constexpr int NWR = TA::NCH + TB::NCH;                              // LDS writes (= global loads) per k-tile
    constexpr int WR = (NWR + NM - 1) / NM;                             // ... per MFMA of step 0
    const bf16* const sAc = sA0 + cur * TA::ELEMS;
    const bf16* const sBc = sB0 + cur * TB::ELEMS;
    bf16* const sAn = sA0 + nxt * TA::ELEMS;
    bf16* const sBn = sB0 + nxt * TB::ELEMS;
    const int kl_store = kleft(t + 1), kl_load = kleft(t + 1 + NSETS);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int fc = s & 1, fn = fc ^ 1;                                // fragment sets: in use, being filled
      const bool last = (s == KS - 1);
      if (last) __syncthreads();
      // The source order is the issue order wanted: one MFMA, then one fragment read for the next step, then (step 0)
      // one chunk of tile t+1 written to LDS and the global load that refills its registers.
#pragma unroll
      for (int q = 0; q < NM; ++q) {
        const int i = q / TJ, j = q % TJ;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[fc][i], fb[fc][j], acc[i][j], 0, 0, 0);
        if (q < NF) {
          const bf16* sa = last ? (const bf16*)sAn : sAc;
          const bf16* sb = last ? (const bf16*)sBn : sBc;
          const int ks = last ? 0 : s + 1;
          if (q < TI) fa[fn][q] = TA::frag(sa, (wm * TI + q) * 32, ks, lane);
          else fb[fn][q - TI] = TB::frag(sb, (wn * TJ + (q - TI)) * 32, ks, lane);
        }
        if (s == 0) {
#pragma unroll
          for (int c = q * WR; c < (q + 1) * WR && c < NWR; ++c) {
            if (c < TA::NCH) {
              TA::template store_chunk<!FAST>(ra[set][c], sAn, c, kl_store, tid);
              TA::template load_chunk<!FAST>(ra[set][c], ca, c, kl_load, tid);
            } else {
              TB::template store_chunk<!FAST>(rb[set][c - TA::NCH], sBn, c - TA::NCH, kl_store, tid);
              TB::template load_chunk<!FAST>(rb[set][c - TA::NCH], cb, c - TA::NCH, kl_load, tid);
            }
          }
        }
        if (FAST) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                   // MFMA
          if (q < TI) __builtin_amdgcn_sched_group_barrier(0x100, AK ? 1 : 2, 0);            // its fragment read
          else if (q < NF) __builtin_amdgcn_sched_group_barrier(0x100, BKM ? 1 : 2, 0);
          if (s == 0 && q * WR < NWR) {
            __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                                 // LDS write
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                 // global load
            if (WR > 1 && q * WR + 1 < NWR) {
              __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
              __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            }
          }
        }
      }
      if (s == 0) {
        // the next request: one k-tile on, or nowhere once the range is used up (FAST only: the guarded loads look at kleft)
        const bool more = !FAST || t + 2 + NSETS < nk;
        ca.soff = more ? ca.soff + ca.step : past;
        cb.soff = more ? cb.soff + cb.step : past;
      }
    }
  };
  {
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    if (nfull == nk && nk > NSETS) {
      for (int t = 0; t < nk; t += 2) {
        body(std::true_type{}, I0{}, t);
        if (t + 1 < nk) body(std::true_type{}, I1{}, t + 1);
      }
    } else {
      // a partial last k-tile, or fewer tiles than the pipeline is deep: every iteration guarded
      for (int t = 0; t < nk; t += 2) {
        body(std::false_type{}, I0{}, t);
        if (t + 1 < nk) body(std::false_type{}, I1{}, t + 1);
      }
    }
  }
  __syncthreads();   // every wave is done with the operand buffers: they become the staging area of the epilogue

  const int rbase = m0 + wm * TI * 32, cbase = n0 + wn * TJ * 32;
  constexpr int STAGE_FLOATS = 32 * (32 * TJ + 4);
  float* stage = (float*)lds_raw + wave * STAGE_FLOATS;
  // GELU epilogues: the table moves into LDS behind the staging areas
  float2* const tab = (float2*)((float*)lds_raw + WGM * WGN * STAGE_FLOATS);
  if (p.gelu_tab && (((EPIS >> EPI_ACT_GELU) | (EPIS >> EPI_ACT_DGELU)) & 1)) {
    for (int i = tid; i < kGeluTabN / 2; i += NT) ((float4*)tab)[i] = ((const float4*)p.gelu_tab)[i];
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

// the epilogues each operand layout is built with (the training step needs no others; launch_gemm falls back
// to gemm_bf16_mfma for the rest)
template <bool AK, bool BKM>
constexpr int wide_epilogues() {
  return (AK && BKM) ? (1 << EPI_PARTIAL | 1 << EPI_F32 | 1 << EPI_ACT | 1 << EPI_ACT_RES | 1 << EPI_ACT_GELU)
         : AK        ? (1 << EPI_PARTIAL | 1 << EPI_ACT | 1 << EPI_ACT_RES | 1 << EPI_ACT_DGELU)
                     : (1 << EPI_PARTIAL | 1 << EPI_F32);
}

// position of linear block v in a grid of nbx x nby tiles: tile rows in groups of GM, rows fastest inside a group,
// so that the tiles in flight on one XCD share operand panels
template <int GM>
__device__ __forceinline__ void tile_of_block(int b, int nbx, int nby, int& tm, int& tn) {
  const int group = b / (GM * nbx), first_m = group * GM;
  const int gm = min(GM, nby - first_m);
  const int in_group = b - group * GM * nbx;
  tm = first_m + in_group % gm;
  tn = in_group / gm;
}

// OCC: blocks per CU the register allocator leaves room for.
template <bool AK, bool BKM, int TI, int TJ, int WGM, int WGN, int BK, int NSETS, int OCC>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(OCC * WGM * WGN / 4, OCC * WGM * WGN / 4)))
void gemm_bf16_wide(GemmDev p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  // tile order: as in gemm_bf16_mfma (a contiguous range of (split, tile) pairs per XCD, groups of tile rows)
  const int nbx = gridDim.x, nby = gridDim.y, nb = nbx * nby;
  int v = (blockIdx.z * nby + blockIdx.y) * nbx + blockIdx.x;
  const int per_xcd = (nb * (int)gridDim.z) >> 3;
  if (v < 8 * per_xcd) v = (v & 7) * per_xcd + (v >> 3);
  const int split = v / nb;
  int tm, tn;
  tile_of_block<(TI * WGM >= 8) ? 4 : 8>(v - split * nb, nbx, nby, tm, tn);
  wide_tile<AK, BKM, TI, TJ, WGM, WGN, BK, NSETS, wide_epilogues<AK, BKM>()>(p, tm * 32 * TI * WGM, tn * 32 * TJ * WGN, split, lds_raw);
}

// Several products in one launch: block v works on tile v - first_tile[i] of problem i (the problems' tiles are
// numbered one problem after the other; an XCD gets a contiguous range of them).  No split-K: every tile runs
// over the whole contraction.
template <bool AK, bool BKM, int TI, int TJ, int WGM, int WGN, int BK, int NSETS, int OCC>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(OCC * WGM * WGN / 4, OCC * WGM * WGN / 4)))
void gemm_bf16_wide_group(GemmGroupDev g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  constexpr int BM = 32 * TI * WGM, BN = 32 * TJ * WGN;
  int v = blockIdx.x;
  const int per_xcd = (int)gridDim.x >> 3;
  if (v < 8 * per_xcd) v = (v & 7) * per_xcd + (v >> 3);
  int i = 0;
  while (i + 1 < g.n && v >= g.first_tile[i + 1]) ++i;
  const GemmDev& p = g.prob[i];
  const int nbx = (p.N + BN - 1) / BN, nby = (p.M + BM - 1) / BM;
  int tm, tn;
  tile_of_block<(TI * WGM >= 8) ? 4 : 8>(v - g.first_tile[i], nbx, nby, tm, tn);
  wide_tile<AK, BKM, TI, TJ, WGM, WGN, BK, NSETS, wide_epilogues<AK, BKM>()>(p, tm * BM, tn * BN, 0, lds_raw);
}

template <bool AK, bool BKM, int TI, int TJ, int WGM, int WGN, int BK, int NSETS, int OCC>
hipError_t launch_wide_one(const GemmDev& p, dim3 grid, hipStream_t s) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr size_t lds = wide_lds_bytes<AK, BKM, TI, TJ, WGM, WGN, BK>();
  static_assert(lds <= 160 * 1024, "tile does not fit the LDS of a CU");
  auto kern = gemm_bf16_wide<AK, BKM, TI, TJ, WGM, WGN, BK, NSETS, OCC>;
  static bool configured = false;          // per instantiation; the attribute is per process and device-wide
  if (!configured && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  configured = true;
  hipLaunchKernelGGL(kern, grid, dim3(NT), lds, s, p);
  return hipSuccess;
}

template <bool AK, bool BKM, int TI, int TJ, int WGM, int WGN, int BK, int NSETS, int OCC>
hipError_t launch_wide_group_one(const GemmGroupDev& g, hipStream_t s) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr size_t lds = wide_lds_bytes<AK, BKM, TI, TJ, WGM, WGN, BK>();
  static_assert(lds <= 160 * 1024, "tile does not fit the LDS of a CU");
  auto kern = gemm_bf16_wide_group<AK, BKM, TI, TJ, WGM, WGN, BK, NSETS, OCC>;
  static bool configured = false;
  if (!configured && lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  configured = true;
  hipLaunchKernelGGL(kern, dim3(g.first_tile[g.n]), dim3(NT), lds, s, g);
  return hipSuccess;
}

// the configurations of gemm_bf16_wide that are built (index = configuration number - 1), one layout per translation unit
template <bool AK, bool BKM>
hipError_t launch_wide_layout(int cfg, const GemmDev& p, int splits, hipStream_t s) {
#define HS_WIDE(TI, TJ, WGM, WGN, BK, NSETS, OCC)                                                        \
  return launch_wide_one<AK, BKM, TI, TJ, WGM, WGN, BK, NSETS, OCC>(                                     \
      p, dim3((p.N + 32 * TJ * WGN - 1) / (32 * TJ * WGN), (p.M + 32 * TI * WGM - 1) / (32 * TI * WGM), splits), s)
  switch (cfg) {
    case 1: HS_WIDE(4, 4, 2, 2, 64, 1, 1);
    case 2: HS_WIDE(4, 3, 2, 2, 64, 2, 1);
    case 3: HS_WIDE(2, 3, 2, 2, 64, 2, 2);
    case 4: HS_WIDE(4, 2, 2, 2, 32, 2, 2);
    case 5: HS_WIDE(2, 2, 2, 2, 64, 2, 2);
    case 6: HS_WIDE(4, 2, 2, 2, 64, 2, 1);
    default: return hipErrorInvalidValue;
  }
#undef HS_WIDE
}

}  // namespace
