// Tile helpers of the bf16 MFMA attention kernels (head dimension 64): staging of 64-row blocks into LDS,
// row and transposed fragments, the result-register -> streamed-row map, dropout factors per tile,
// packing and the store of owned rows.  Included by the kernels' translation units only.
#pragma once
#include "common.h"

namespace attn_tiles {

constexpr int DH = 64;
constexpr int LDT = 72;                 // LDS row stride in elements (144 B: conflict-free 16-byte row reads)
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float SCALE2 = 0.125f * LOG2E;   // 1/sqrt(64) folded with the change to base 2

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// rows r0..r0+63 of a [*, ld] bf16 matrix (64 columns starting at the given pointer) -> LDS tile;
// rows at or beyond row_limit are zero.  256 threads, two 16-byte chunks each.
__device__ __forceinline__ void stage64(bf16* tile, const bf16* __restrict__ src, int64_t ld, int r0, int row_limit, int tid) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int c = tid + i * 256;
    const int r = c >> 3, col = (c & 7) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r0 + r < row_limit) v = *(const uint4*)(src + (int64_t)(r0 + r) * ld + col);
    *(uint4*)(tile + r * LDT + col) = v;
  }
}

// A/B fragment of tile rows: lane gets row rbase + lane%32, columns 16*ks + 8*(lane/32) .. +7
__device__ __forceinline__ bf16x8 frag_rows(const bf16* tile, int rbase, int ks, int lane) {
  return *(const bf16x8*)(tile + (rbase + (lane & 31)) * LDT + ks * 16 + (lane >> 5) * 8);
}
// the same fragment straight from global memory for the owned rows (zero beyond row_limit)
__device__ __forceinline__ bf16x8 frag_rows_global(const bf16* __restrict__ src, int64_t ld, int row, int row_limit, int ks, int lane) {
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = (bf16)0.0f;
  if (row < row_limit) z = *(const bf16x8*)(src + (int64_t)row * ld + ks * 16 + (lane >> 5) * 8);
  return z;
}
// Transposed A fragment: MFMA row i = tile column c0 + lane%32; contraction slot (g = lane/32, e)
// = tile row rb + 16*step + 4*g + (e & 3) + 8*(e >> 2).
__device__ __forceinline__ bf16x8 frag_cols_t(const bf16* tile, int rb, int step, int c0, int lane) {
  const int row = rb + 16 * step + 4 * (lane >> 5) + ((lane & 15) >> 2);
  const int col = c0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  typedef s16x4 __attribute__((address_space(3))) * lds_v4;
  union { struct { s16x4 lo, hi; } p; bf16x8 v; } u;
  u.p.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + row * LDT + col));
  u.p.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(tile + (row + 8) * LDT + col));
  return u.v;
}
// streamed-row index (within a 32-row tile) of result register r
__device__ __forceinline__ int tile_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }

// Dropout factors of a score tile whose STREAMED index is the key: registers 4a .. 4a+3 of a lane are four
// consecutive keys of one query, i.e. one generator block.  row_base = ((b*A + h)*L + query) * L.
__device__ __forceinline__ void drop_tile_keys(const DropCfg& d, uint32_t site, uint64_t row_base, int key0, int lane, f32x16& f) {
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    float t[4];
    drop_factors4(d, site, (row_base + (uint64_t)(key0 + 8 * a + 4 * (lane >> 5))) >> 2, t);
    f[4 * a] = t[0]; f[4 * a + 1] = t[1]; f[4 * a + 2] = t[2]; f[4 * a + 3] = t[3];
  }
}
// ... and of a tile whose STREAMED index is the query (the lane owns one key).  head_base = (b*A + h) * L; element =
// (head_base + query) * L + key.  The four lanes of a quad own the four keys of one aligned group (key % 4 == lane % 4),
// i.e. the four words of ONE generator block per query: for each group of four result registers (four consecutive
// queries) lane i of the quad evaluates the block of query i and the quad exchanges the keep bits, so a lane runs
// the generator 4 times per tile instead of 16.
template <int I>
__device__ __forceinline__ int quad_broadcast(int x) { return __builtin_amdgcn_mov_dpp(x, I * 0x55, 0xF, 0xF, true); }
__device__ __forceinline__ void drop_tile_queries(const DropCfg& d, uint32_t site, uint64_t head_base, int L, int query0, int key, int lane,
                                                  f32x16& f) {
  const int word = lane & 3;
#pragma unroll
  for (int a = 0; a < 4; ++a) {
    const int query = query0 + 8 * a + 4 * (lane >> 5) + word;        // = query0 + tile_row(4a + word, lane)
    const uint64_t e = (head_base + (uint64_t)query) * (uint64_t)L + (uint64_t)(key & ~3);
    const int mine = drop_keep4(d, site, e >> 2);
    const int k0 = quad_broadcast<0>(mine), k1 = quad_broadcast<1>(mine), k2 = quad_broadcast<2>(mine), k3 = quad_broadcast<3>(mine);
    f[4 * a + 0] = ((k0 >> word) & 1) ? d.scale : 0.0f;
    f[4 * a + 1] = ((k1 >> word) & 1) ? d.scale : 0.0f;
    f[4 * a + 2] = ((k2 >> word) & 1) ? d.scale : 0.0f;
    f[4 * a + 3] = ((k3 >> word) & 1) ? d.scale : 0.0f;
  }
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int step) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (bf16)v[8 * step + e];
  return o;
}

// writes a transposed [64 x 32] fp32 accumulator pair (two 32-row column blocks) as 32 rows of
// 64 bf16: lane owns row (lane%32) and, per register quad, 4 consecutive columns
__device__ __forceinline__ void store_owned_rows(bf16* __restrict__ dst_row, const f32x16 (&acc)[2], float scale, int lane) {
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)(acc[db][4 * qd + e] * scale);
      *(bf16x4*)(dst_row + 32 * db + 8 * qd + 4 * (lane >> 5)) = o;
    }
}

// The same rows through a wave-private LDS area of 32 x LDT elements, so that global memory sees whole 128-byte
// rows (8 lanes x 16 bytes) instead of 8-byte pieces: lane l first puts its pieces of row l % 32 into the area,
// then the wave writes the 32 rows out, 8 rows per store instruction.  LDS operations of one wave execute in
// order, so no barrier is needed.  Rows row0 + r >= row_limit are not written.
__device__ __forceinline__ void store_owned_rows_lds(bf16* __restrict__ dst, int64_t ld, int row0, int row_limit, const f32x16 (&acc)[2],
                                                     float scale, int lane, bf16* stage) {
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int qd = 0; qd < 4; ++qd) {
      bf16x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (bf16)(acc[db][4 * qd + e] * scale);
      *(bf16x4*)(stage + (lane & 31) * LDT + 32 * db + 8 * qd + 4 * (lane >> 5)) = o;
    }
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int c = it * 64 + lane;
    const int r = c >> 3, col = (c & 7) * 8;
    const uint4 v = *(const uint4*)(stage + r * LDT + col);
    if (row0 + r < row_limit) *(uint4*)(dst + (int64_t)(row0 + r) * ld + col) = v;
  }
}

}  // namespace attn_tiles
