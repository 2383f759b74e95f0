// bf16 MFMA attention (head dimension 64), forward and backward, fp32 softmax statistics.
//
// Every kernel has the same shape.  A wave OWNS 32 rows (queries, or keys in the dK/dV kernel)
// whose vectors stay in registers as MFMA B operands, and STREAMS the other side through LDS in
// blocks of 64 rows kept in their natural [row][64] layout.  Score tiles are computed transposed,
// tile[streamed row][owned row], so that each lane holds ONE owned row (lane % 32) and 16 streamed
// rows: reductions over the streamed index are then in-lane plus one exchange between the two
// half-waves.  The second product needs the score tile as a B operand and the streamed block
// transposed as the A operand; the transposed fragment comes from the LDS transpose read, with
// the 16 contraction slots ordered exactly as the result registers of the score tile are
// (register r of lane l is streamed row 8*(r/4) + 4*(l/32) + r%4), so no data moves between lanes.
#include "attention_tiles.h"

namespace {

using namespace attn_tiles;

// ------------------------------------------------------------------------------------------
// forward: wave owns 32 queries, streams keys/values
// ------------------------------------------------------------------------------------------
template <bool DROP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4))) void attn_fwd_mfma(const bf16* __restrict__ qkv, const int32_t* __restrict__ lens, int L, int A,
                                                     bf16* __restrict__ out, float* __restrict__ lse, DropCfg drop, uint32_t site) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Vs[64 * LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int H = A * DH;
  const int64_t ld = 3 * (int64_t)H;
  int len = lens[b];
  len = len < 1 ? 1 : (len > L ? L : len);
  const bf16* base = qkv + (int64_t)b * L * ld + h * DH;
  const int q = blockIdx.x * 128 + wave * 32 + (lane & 31);     // the query this lane owns

  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qf[ks] = frag_rows_global(base, ld, q, L, ks, lane);
  f32x16 o[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m2 = -1.0e30f, lsum = 0.f;

  for (int k0 = 0; k0 < len; k0 += 64) {
    __syncthreads();
    stage64(Ks, base + H, ld, k0, len, tid);
    stage64(Vs, base + 2 * H, ld, k0, len, tid);
    __syncthreads();
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int kb = 32 * sub;
      if (k0 + kb < len) {
        f32x16 st;
#pragma unroll
        for (int r = 0; r < 16; ++r) st[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Ks, kb, ks, lane), qf[ks], st, 0, 0, 0);
        float mloc = -1.0e30f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool ok = k0 + kb + tile_row(r, lane) < len;
          st[r] = ok ? st[r] * SCALE2 : -1.0e30f;
          mloc = fmaxf(mloc, st[r]);
        }
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
        const float mn = fmaxf(m2, mloc);
        const float alpha = fast_exp2(m2 - mn);
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool ok = k0 + kb + tile_row(r, lane) < len;
          const float p = ok ? fast_exp2(st[r] - mn) : 0.f;
          st[r] = p;
          ps += p;
        }
        lsum = lsum * alpha + ps;
        m2 = mn;
        if (DROP) {      // the row sum keeps every key, the value sum only the survivors (scaled)
          f32x16 f;
          drop_tile_keys(drop, site, (((uint64_t)b * A + h) * L + q) * (uint64_t)L, k0 + kb, lane, f);
#pragma unroll
          for (int r = 0; r < 16; ++r) st[r] *= f[r];
        }
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
  if (q < L && lane < 32) lse[((int64_t)b * A + h) * L + q] = (m2 + __log2f(lsum)) * LN2;
  __syncthreads();      // every wave is done with the key/value tiles: each wave takes 32 rows of them as its staging area
  store_owned_rows_lds(out + (int64_t)b * L * H + h * DH, H, blockIdx.x * 128 + wave * 32, L, o, 1.0f / lsum, lane,
                       (wave < 2 ? Ks : Vs) + (wave & 1) * 32 * LDT);
}

// ------------------------------------------------------------------------------------------
// backward 1: wave owns 32 queries, streams keys/values -> dq and dvec[q] = sum_d dO[q,d] O[q,d]
// ------------------------------------------------------------------------------------------
template <bool DROP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3))) void attn_bwd_dq_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ out,
                                                        const float* __restrict__ lse, const bf16* __restrict__ d_out,
                                                        const int32_t* __restrict__ lens, int L, int A, bf16* __restrict__ dqkv,
                                                        float* __restrict__ dvec, DropCfg drop, uint32_t site) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Vs[64 * LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int H = A * DH;
  const int64_t ld = 3 * (int64_t)H;
  int len = lens[b];
  len = len < 1 ? 1 : (len > L ? L : len);
  const bf16* base = qkv + (int64_t)b * L * ld + h * DH;
  const bf16* go = d_out + (int64_t)b * L * H + h * DH;
  const bf16* oo = out + (int64_t)b * L * H + h * DH;
  const int q = blockIdx.x * 128 + wave * 32 + (lane & 31);

  // padded queries (q >= len) own all-zero fragments and therefore produce zero rows
  bf16x8 qf[4], gf[4];
  float dpart = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qf[ks] = frag_rows_global(base, ld, q, len, ks, lane);
    gf[ks] = frag_rows_global(go, H, q, len, ks, lane);
    const bf16x8 of = frag_rows_global(oo, H, q, len, ks, lane);
#pragma unroll
    for (int e = 0; e < 8; ++e) dpart = fmaf((float)gf[ks][e], (float)of[e], dpart);
  }
  const float dq_row = dpart + __shfl_xor(dpart, 32);
  const float lse2 = (q < len) ? lse[((int64_t)b * A + h) * L + q] * LOG2E : 0.f;
  f32x16 acc[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;

  for (int k0 = 0; k0 < len; k0 += 64) {
    __syncthreads();
    stage64(Ks, base + H, ld, k0, len, tid);
    stage64(Vs, base + 2 * H, ld, k0, len, tid);
    __syncthreads();
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      const int kb = 32 * sub;
      if (k0 + kb < len) {
        f32x16 st, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Ks, kb, ks, lane), qf[ks], st, 0, 0, 0);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Vs, kb, ks, lane), gf[ks], dp, 0, 0, 0);
        }
        if (DROP) {
          f32x16 f;
          drop_tile_keys(drop, site, (((uint64_t)b * A + h) * L + q) * (uint64_t)L, k0 + kb, lane, f);
#pragma unroll
          for (int r = 0; r < 16; ++r) dp[r] *= f[r];
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const bool ok = (k0 + kb + tile_row(r, lane) < len) && (q < len);
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
  if (q < L) {
    store_owned_rows(dqkv + ((int64_t)b * L + q) * ld + h * DH, acc, 0.125f, lane);
    if (lane < 32) dvec[((int64_t)b * A + h) * L + q] = dq_row;
  }
}

// ------------------------------------------------------------------------------------------
// backward 2: wave owns 32 keys, streams queries / output gradients -> dk, dv
// ------------------------------------------------------------------------------------------
template <bool DROP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dkv_mfma(const bf16* __restrict__ qkv, const float* __restrict__ lse,
                                                         const bf16* __restrict__ d_out, const float* __restrict__ dvec,
                                                         const int32_t* __restrict__ lens, int L, int A, bf16* __restrict__ dqkv, DropCfg drop,
                                                         uint32_t site) {
  __shared__ __attribute__((aligned(16))) bf16 Qs[64 * LDT];
  __shared__ __attribute__((aligned(16))) bf16 Gs[64 * LDT];
  __shared__ float lse2_s[64], dvec_s[64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z, h = blockIdx.y;
  const int H = A * DH;
  const int64_t ld = 3 * (int64_t)H;
  int len = lens[b];
  len = len < 1 ? 1 : (len > L ? L : len);
  const bf16* base = qkv + (int64_t)b * L * ld + h * DH;
  const bf16* go = d_out + (int64_t)b * L * H + h * DH;
  const int kj = blockIdx.x * 128 + wave * 32 + (lane & 31);    // the key this lane owns
  const bool wave_active = blockIdx.x * 128 + wave * 32 < len;  // wave-uniform

  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    kf[ks] = frag_rows_global(base + H, ld, kj, len, ks, lane);
    vf[ks] = frag_rows_global(base + 2 * H, ld, kj, len, ks, lane);
  }
  f32x16 dk[2], dv[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[db][r] = 0.f; dv[db][r] = 0.f; }

  for (int q0 = 0; q0 < len; q0 += 64) {        // padded queries carry no gradient
    __syncthreads();
    stage64(Qs, base, ld, q0, len, tid);
    stage64(Gs, go, H, q0, len, tid);
    if (tid < 64) {
      const bool ok = q0 + tid < len;
      lse2_s[tid] = ok ? lse[((int64_t)b * A + h) * L + q0 + tid] * LOG2E : 0.f;
      dvec_s[tid] = ok ? dvec[((int64_t)b * A + h) * L + q0 + tid] : 0.f;
    }
    __syncthreads();
    if (wave_active) {
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int qb = 32 * sub;
        if (q0 + qb < len) {
          f32x16 st, dp;
#pragma unroll
          for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) {
            st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Qs, qb, ks, lane), kf[ks], st, 0, 0, 0);
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(Gs, qb, ks, lane), vf[ks], dp, 0, 0, 0);
          }
          f32x16 f;
          if (DROP) drop_tile_queries(drop, site, ((uint64_t)b * A + h) * L, L, q0 + qb, kj, lane, f);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qi = qb + tile_row(r, lane);
            const bool ok = (q0 + qi < len) && (kj < len);
            const float p = ok ? fast_exp2(st[r] * SCALE2 - lse2_s[qi]) : 0.f;
            const float fr = DROP ? f[r] : 1.0f;
            st[r] = p * fr;
            dp[r] = p * (fr * dp[r] - dvec_s[qi]);
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
  if (kj < L) {
    bf16* row = dqkv + ((int64_t)b * L + kj) * ld + h * DH;
    store_owned_rows(row + H, dk, 0.125f, lane);
    store_owned_rows(row + 2 * H, dv, 1.0f, lane);
  }
}

// ------------------------------------------------------------------------------------------
// backward for sequences of at most 128 positions: one block per (sequence, head), no second launch.  Every
// wave first owns 32 queries (dq) with K and V streamed from two LDS tiles, then 32 keys (dk, dv) with Q and dO
// streamed from the SAME two tiles: owned rows never need LDS (their fragments come straight from global memory,
// or out of the tiles just before they are overwritten), so a block takes 37 KiB of LDS and three of them share a CU -
// one round for the 768 blocks of 64 sequences x 12 heads, and the second staging phase of one block runs under
// the arithmetic of the others.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void stage128(bf16* tile, const bf16* __restrict__ src, int64_t ld, int row_limit, int tid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int c = tid + i * 256;
    const int r = c >> 3, col = (c & 7) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < row_limit) v = *(const uint4*)(src + (int64_t)r * ld + col);
    *(uint4*)(tile + r * LDT + col) = v;
  }
}

template <bool DROP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void attn_bwd_fused128_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ out, const float* __restrict__ lse,
                            const bf16* __restrict__ d_out, const int32_t* __restrict__ lens, int L, int A, bf16* __restrict__ dqkv,
                            DropCfg drop, uint32_t site) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16* T0 = (bf16*)lds_raw;               // K, then Q
  bf16* T1 = T0 + 128 * LDT;               // V, then dO
  float* lse2_s = (float*)(T1 + 128 * LDT);
  float* dvec_s = lse2_s + 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.y, h = blockIdx.x;
  const int H = A * DH;
  const int64_t ld = 3 * (int64_t)H;
  int len = lens[b];
  len = len < 1 ? 1 : (len > L ? L : len);
  const bf16* base = qkv + (int64_t)b * L * ld + h * DH;
  const bf16* go = d_out + (int64_t)b * L * H + h * DH;
  const bf16* oo = out + (int64_t)b * L * H + h * DH;
  const int own = wave * 32 + (lane & 31);       // the query, then the key, this lane owns
  const bool wave_active = wave * 32 < len;      // wave-uniform

  stage128(T0, base + H, ld, len, tid);
  stage128(T1, base + 2 * H, ld, len, tid);
  // the owned queries' fragments of Q and dO, and the row dot product sum_d dO*O (lanes l and l + 32 hold the two halves of a row)
  bf16x8 qf[4], gf[4];
  float drow = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qf[ks] = frag_rows_global(base, ld, own, len, ks, lane);
    gf[ks] = frag_rows_global(go, H, own, len, ks, lane);
    const bf16x8 of = frag_rows_global(oo, H, own, len, ks, lane);
#pragma unroll
    for (int e = 0; e < 8; ++e) drow = fmaf((float)gf[ks][e], (float)of[e], drow);
  }
  drow += __shfl_xor(drow, 32);
  const float lse2 = (own < len) ? lse[((int64_t)b * A + h) * L + own] * LOG2E : 0.f;
  if (lane < 32) { dvec_s[own] = drow; lse2_s[own] = lse2; }
  __syncthreads();

  f32x16 acc[2], acc2[2];
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[db][r] = 0.f;
  // ---- queries owned: dq ----
  if (wave_active) {
    for (int kb = 0; kb < len; kb += 32) {
      f32x16 st, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(T0, kb, ks, lane), qf[ks], st, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(T1, kb, ks, lane), gf[ks], dp, 0, 0, 0);
      }
      if (DROP) {
        f32x16 f;
        drop_tile_keys(drop, site, (((uint64_t)b * A + h) * L + own) * (uint64_t)L, kb, lane, f);
#pragma unroll
        for (int r = 0; r < 16; ++r) dp[r] *= f[r];
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const bool ok = (kb + tile_row(r, lane) < len) && (own < len);
        const float pr = ok ? fast_exp2(st[r] * SCALE2 - lse2) : 0.f;
        st[r] = pr * (dp[r] - drow);
      }
      const bf16x8 s0 = pack8(st, 0), s1 = pack8(st, 1);
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(T0, kb, 0, 32 * db, lane), s0, acc[db], 0, 0, 0);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(T0, kb, 1, 32 * db, lane), s1, acc[db], 0, 0, 0);
      }
    }
  }
  // ---- keys owned: dk, dv ----
  // The owned key/value fragments are the last thing read from K and V.  After the barrier a wave's own 32 rows of
  // tile 0 stage the whole-row stores of dq; after the next one the tiles are refilled with Q and dO.
  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) { kf[ks] = frag_rows(T0, wave * 32, ks, lane); vf[ks] = frag_rows(T1, wave * 32, ks, lane); }
  __syncthreads();
  bf16* const dst = dqkv + (int64_t)b * L * ld + h * DH;
  store_owned_rows_lds(dst, ld, wave * 32, L, acc, 0.125f, lane, T0 + wave * 32 * LDT);
  __syncthreads();
  stage128(T0, base, ld, len, tid);
  stage128(T1, go, H, len, tid);
  __syncthreads();
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[db][r] = 0.f; acc2[db][r] = 0.f; }
  if (wave_active) {
    for (int qb = 0; qb < len; qb += 32) {
      f32x16 st, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { st[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(T0, qb, ks, lane), kf[ks], st, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_rows(T1, qb, ks, lane), vf[ks], dp, 0, 0, 0);
      }
      f32x16 f;
      if (DROP) drop_tile_queries(drop, site, ((uint64_t)b * A + h) * L, L, qb, own, lane, f);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int qi = qb + tile_row(r, lane);
        const bool ok = (qi < len) && (own < len);
        const float pr = ok ? fast_exp2(st[r] * SCALE2 - lse2_s[qi]) : 0.f;
        const float fr = DROP ? f[r] : 1.0f;
        st[r] = pr * fr;
        dp[r] = pr * (fr * dp[r] - dvec_s[qi]);
      }
      const bf16x8 p0 = pack8(st, 0), p1 = pack8(st, 1), s0 = pack8(dp, 0), s1 = pack8(dp, 1);
#pragma unroll
      for (int db = 0; db < 2; ++db) {
        acc2[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(T1, qb, 0, 32 * db, lane), p0, acc2[db], 0, 0, 0);
        acc2[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(T1, qb, 1, 32 * db, lane), p1, acc2[db], 0, 0, 0);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(T0, qb, 0, 32 * db, lane), s0, acc[db], 0, 0, 0);
        acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_cols_t(T0, qb, 1, 32 * db, lane), s1, acc[db], 0, 0, 0);
      }
    }
  }
  __syncthreads();     // every wave is done with Q and dO: own rows of the tiles stage the stores of dk and dv
  store_owned_rows_lds(dst + H, ld, wave * 32, L, acc, 0.125f, lane, T0 + wave * 32 * LDT);
  store_owned_rows_lds(dst + 2 * H, ld, wave * 32, L, acc2, 1.0f, lane, T1 + wave * 32 * LDT);
}

}  // namespace

void launch_attention_fwd_mfma(const void* qkv, const int32_t* lens, int B, int L, int A, void* out, float* lse, hipStream_t s,
                               const DropCfg& drop, uint32_t site) {
  dim3 grid((L + 127) / 128, A, B);
  if (drop.thr) hipLaunchKernelGGL(attn_fwd_mfma<true>, grid, dim3(256), 0, s, (const bf16*)qkv, lens, L, A, (bf16*)out, lse, drop, site);
  else hipLaunchKernelGGL(attn_fwd_mfma<false>, grid, dim3(256), 0, s, (const bf16*)qkv, lens, L, A, (bf16*)out, lse, drop, site);
}

void launch_attention_bwd_mfma(const void* qkv, const void* out, const float* lse, const void* d_out, const int32_t* lens, int B, int L,
                               int A, void* dqkv, float* dvec, hipStream_t s, const DropCfg& drop, uint32_t site) {
  if (L <= 128) {
    constexpr size_t lds = 2 * 128 * LDT * sizeof(bf16) + 2 * 128 * sizeof(float);
    static bool configured = false;
    if (!configured) {
      (void)hipFuncSetAttribute((const void*)attn_bwd_fused128_mfma<false>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      (void)hipFuncSetAttribute((const void*)attn_bwd_fused128_mfma<true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      configured = true;
    }
    if (drop.thr) hipLaunchKernelGGL(attn_bwd_fused128_mfma<true>, dim3(A, B), dim3(256), lds, s, (const bf16*)qkv, (const bf16*)out, lse,
                                     (const bf16*)d_out, lens, L, A, (bf16*)dqkv, drop, site);
    else hipLaunchKernelGGL(attn_bwd_fused128_mfma<false>, dim3(A, B), dim3(256), lds, s, (const bf16*)qkv, (const bf16*)out, lse,
                            (const bf16*)d_out, lens, L, A, (bf16*)dqkv, drop, site);
    return;
  }
  dim3 grid((L + 127) / 128, A, B);
  if (drop.thr) {
    hipLaunchKernelGGL(attn_bwd_dq_mfma<true>, grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)out, lse, (const bf16*)d_out, lens, L, A,
                       (bf16*)dqkv, dvec, drop, site);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma<true>, grid, dim3(256), 0, s, (const bf16*)qkv, lse, (const bf16*)d_out, (const float*)dvec, lens, L, A,
                       (bf16*)dqkv, drop, site);
  } else {
    hipLaunchKernelGGL(attn_bwd_dq_mfma<false>, grid, dim3(256), 0, s, (const bf16*)qkv, (const bf16*)out, lse, (const bf16*)d_out, lens, L, A,
                       (bf16*)dqkv, dvec, drop, site);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma<false>, grid, dim3(256), 0, s, (const bf16*)qkv, lse, (const bf16*)d_out, (const float*)dvec, lens, L, A,
                       (bf16*)dqkv, drop, site);
  }
}
