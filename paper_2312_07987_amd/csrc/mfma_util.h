// Device helpers shared by the matrix-core (MFMA) kernels of libswitchhead: operand fragments of
// v_mfma_f32_32x32x16_bf16 from LDS, gate scaling of packed bf16 pieces, the XCD-aware work-group
// placement and the tile lookup among expert groups.  gfx950 only.
//
// Fragment layouts of v_mfma_f32_32x32x16_bf16 (lane = 32*g + r, g in {0,1}):
//   A operand: A[row r][k = 8g .. 8g+7]      B operand: B[k = 8g .. 8g+7][col r]
//   D: register q (0..15) holds D[8*(q/4) + 4g + q%4][col r]
#pragma once
#include "common.h"

namespace sh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// 8 consecutive bf16 of one LDS row -> operand fragment
__device__ __forceinline__ bf16x8 frag_rowmajor(const unsigned short* p) { return *(const bf16x8*)p; }

// Operand fragment from a tile stored [k][n] (n contiguous): the lane needs k = kb..kb+7 of
// column n.  Two transposing reads; inside each group of 16 lanes, lane s addresses row
// kb + s/4, columns 4*(s%4).. and receives rows kb..kb+3 of column s.
__device__ __forceinline__ bf16x8 frag_transposed(const unsigned short* tile, int ld, int kb, int nb, int lane) {
  const int s = lane & 15;
  const unsigned short* p = tile + (kb + (s >> 2)) * ld + nb + ((lane >> 4) & 1) * 16 + (s & 3) * 4;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, p + 4 * ld));
  union {
    struct {
      s16x4 a, b;
    } s2;
    bf16x8 v;
  } u;
  u.s2.a = lo;
  u.s2.b = hi;
  return u.v;
}

template <int VEC>
struct Chunk;
template <>
struct Chunk<8> {
  typedef uint4 type;
};
template <>
struct Chunk<4> {
  typedef uint2 type;
};

__device__ __forceinline__ float chunk_sumsq(uint4 v) {
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
  float s = 0.f;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const float lo = __uint_as_float(w[u] << 16), hi = __uint_as_float(w[u] & 0xffff0000u);
    s = fmaf(lo, lo, s);
    s = fmaf(hi, hi, s);
  }
  return s;
}
__device__ __forceinline__ float chunk_sumsq(uint2 v) { return chunk_sumsq(make_uint4(v.x, v.y, 0, 0)); }

template <int VEC>
__device__ __forceinline__ typename Chunk<VEC>::type zero_chunk() {
  typename Chunk<VEC>::type z;
  if constexpr (VEC == 8)
    z = make_uint4(0, 0, 0, 0);
  else
    z = make_uint2(0, 0);
  return z;
}

__device__ __forceinline__ unsigned scale_pair(unsigned w, float g) {
  float lo = __uint_as_float(w << 16) * g, hi = __uint_as_float(w & 0xffff0000u) * g;
  return pack_bf16x2(lo, hi);
}
__device__ __forceinline__ uint4 scale_chunk(uint4 c, float g) {
  return make_uint4(scale_pair(c.x, g), scale_pair(c.y, g), scale_pair(c.z, g), scale_pair(c.w, g));
}
__device__ __forceinline__ uint2 scale_chunk(uint2 c, float g) { return make_uint2(scale_pair(c.x, g), scale_pair(c.y, g)); }

// ----------------------------------------------------------------------------------------
// Work-group placement.  Consecutive work-group ids are dealt round-robin to the 8 XCDs,
// each with its own L2.  decode_block turns a linear id into (window, slot) such that all
// `per_window` slots of window w run on XCD w % 8 back to back: work-groups that read the
// same rows (the column tiles of a row tile; the same token window of every expert) then
// meet in one L2 instead of fetching the rows from HBM once per XCD.
// ----------------------------------------------------------------------------------------
// Row ids are divided by a small constant (the k slots of a token share a row): multiply-high by
// ceil(2^32 / d) is exact for ids below 2^32 / d; inv == 0 stands for d == 1.
__device__ __forceinline__ unsigned div_magic(int d) { return d > 1 ? 0xFFFFFFFFu / (unsigned)d + 1u : 0u; }
__device__ __forceinline__ int div_by(int id, unsigned inv) { return inv ? (int)__umulhi((unsigned)id, inv) : id; }

// The tile-th row tile of a head whose groups (experts or expert sets, at most 128) start at off[0..E]:
// every lane takes the groups `lane` and `lane + 64`, a wave prefix sum of their tile counts finds the
// group in one round of loads (a serial scan pays one dependent scalar load per group).  Returns false
// past the last tile.  All lanes get the same answer.
__device__ __forceinline__ bool find_tile_wave(const int* off, int E, int bm, int tile, int lane, int& e, int& row0, int& rows) {
  const int b0 = off[min(lane, E)], e0 = off[min(lane + 1, E)];
  const int b1 = off[min(lane + 64, E)], e1 = off[min(lane + 65, E)];
  const int c0 = (e0 - b0 + bm - 1) / bm, c1 = (e1 - b1 + bm - 1) / bm;   // 0 for lanes past the last group
  int p0 = c0, p1 = c1;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int u0 = __shfl_up(p0, d, 64), u1 = __shfl_up(p1, d, 64);
    if (lane >= d) {
      p0 += u0;
      p1 += u1;
    }
  }
  const int total0 = __shfl(p0, 63, 64);
  p1 += total0;
  const unsigned long long m0 = __ballot(tile < p0), m1 = __ballot(tile < p1);
  if (!(m0 | m1)) return false;
  const bool low = m0 != 0;
  const int src = low ? __builtin_ctzll(m0) : __builtin_ctzll(m1);
  e = low ? src : src + 64;
  const int first = __shfl(low ? p0 - c0 : p1 - c1, src, 64);   // tiles before this group
  const int beg = __shfl(low ? b0 : b1, src, 64), end = __shfl(low ? e0 : e1, src, 64);
  row0 = beg + (tile - first) * bm;
  rows = end - row0 < bm ? end - row0 : bm;
  return true;
}

__device__ __forceinline__ void decode_block(int L, int per_window, int& w, int& slot) {
  const int S = 8 * per_window;
  const int w8 = L / S, rr = L % S;
  w = w8 * 8 + (rr & 7);
  slot = rr >> 3;
}
static inline unsigned grid_windows(int nwin, int per_window) { return (unsigned)(((nwin + 7) / 8) * 8) * per_window; }

}  // namespace sh
