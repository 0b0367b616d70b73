// Fused attention on bf16 matrix cores for the SwitchHead layer (arXiv 2312.07987):
// A^h = softmax(Q^h K^h^T / sqrt(d_head)) and the read-out A^h V^h of Sec. 2.1, one
// attention matrix per head, computed tile by tile with a running maximum so that the
// T x T matrix of probabilities never exists in memory; plus the matching backward kernels
// (which, at head widths 64..128 and up to 1 GiB, do keep one T x T quantity between them: the
// score gradient dS in bf16, the visible half under a causal mask; see attn_ds_dims).
//
// Everything is computed transposed, S^T[key][query] = K Q^T, so that one query lives in
// one lane column of the MFMA result: the softmax statistics of a query are lane-local
// (plus one exchange between the two lane halves), and exp(S^T) is directly the B operand
// of the second product O^T[d][query] = V^T[d][key] P^T[key][query].  V tiles stay
// [key][d] in LDS and are read with transposing loads.
//
// v_mfma_f32_32x32x16_bf16, lane = 32*g + r:  A[row r][k = 8g..8g+7], B[k = 8g..8g+7][col r],
// D register q holds D[8*(q/4) + 4g + q%4][col r].
#include "common.h"

namespace sh {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

__device__ __forceinline__ bf16x8 rowfrag(const unsigned short* p) { return *(const bf16x8*)p; }

// Fragment for a tile stored [row][col] (col contiguous) when the MFMA reduction index is the
// tile row: the lane receives rows kb0..kb0+3 and kb1..kb1+3 of column nb + (lane%32).
__device__ __forceinline__ bf16x8 trfrag(const unsigned short* tile, int ld, int kb0, int kb1, int nb, int lane) {
  const int s = lane & 15;
  const int col = nb + ((lane >> 4) & 1) * 16 + (s & 3) * 4;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + (kb0 + (s >> 2)) * ld + col));
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, tile + (kb1 + (s >> 2)) * ld + col));
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

__device__ __forceinline__ bf16x8 pack8(const float* v) {
  bf16x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (__bf16)v[i];
  return o;
}

// row stride (elements) of a tile read with transposing loads: 16 banks (mod 64) apart
__host__ __device__ constexpr int ld_tr(int dh) { return dh <= 32 ? 32 : (dh <= 160 ? 160 : 288); }

// 8 consecutive elements of a global row as an operand fragment, zero beyond dh / invalid row
template <int VEC>
__device__ __forceinline__ bf16x8 global_frag(const unsigned short* row, int d, int dh, bool valid) {
  union {
    uint4 q;
    uint2 h[2];
    bf16x8 v;
  } u;
  u.q = make_uint4(0, 0, 0, 0);
  if (valid) {
    if constexpr (VEC == 8) {
      if (d < dh) u.q = *(const uint4*)(row + d);
    } else {
      if (d < dh) u.h[0] = *(const uint2*)(row + d);
      if (d + 4 < dh) u.h[1] = *(const uint2*)(row + d + 4);
    }
  }
  return u.v;
}

// NROWS rows of `dh` bf16 on their way from global memory to LDS: load() issues the global loads into registers,
// store() writes them to one or two LDS tiles (the second with another row stride, for the transposing reads).
// Keeping the two apart lets the next tile travel while the current one is used.
// The loads carry no tests (a test per load costs a branch and a dozen instructions, a fifth of the forward kernel's
// time at T = 4096): a row past `valid_rows` reads the last valid row instead, and a column past `dh` reads column 0
// and is replaced by zero in store().  The kernels mask every product that involves a row past the end (the
// probability of such a key or query is exactly zero), so what the repeated row holds does not matter as long as it
// is finite; the padding columns enter the sums over d and must be zero.
template <int DH, int VEC, int NROWS, int NT = 256>
struct RowTile {
  static constexpr int CPR = DH / VEC, TOTAL = NROWS * CPR, NCH = (TOTAL + NT - 1) / NT;
  uint4 r[NCH];   // VEC == 4 uses .x/.y only
  __device__ __forceinline__ void load(const unsigned short* src, long row_stride, int valid_rows, int dh, int tid) {
    if (valid_rows <= 0) {   // uniform: the tile lies past the end, nothing may be read
#pragma unroll
      for (int i = 0; i < NCH; ++i) r[i] = make_uint4(0, 0, 0, 0);
      return;
    }
    const int last = (valid_rows < NROWS ? valid_rows : NROWS) - 1;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * NT;
      const int row = c / CPR, d = (c % CPR) * VEC;
      const int rc = row < last ? row : last;
      const char* p = (const char*)src + ((unsigned)rc * (unsigned)row_stride + (unsigned)(d < dh ? d : 0)) * 2u;
      if constexpr (VEC == 8) {
        r[i] = *(const uint4*)p;
      } else {
        const uint2 v = *(const uint2*)p;
        r[i] = make_uint4(v.x, v.y, 0, 0);
      }
    }
  }
  __device__ __forceinline__ void store(unsigned short* t0, int ld0, unsigned short* t1, int ld1, int tid, int dh) const {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * NT;
      if (c >= TOTAL) continue;
      const int row = c / CPR, d = (c % CPR) * VEC;
      const uint4 v = d < dh ? r[i] : make_uint4(0, 0, 0, 0);
      if constexpr (VEC == 8) {
        *(uint4*)(t0 + row * ld0 + d) = v;
        if (t1 != t0) *(uint4*)(t1 + row * ld1 + d) = v;
      } else {
        *(uint2*)(t0 + row * ld0 + d) = make_uint2(v.x, v.y);
        if (t1 != t0) *(uint2*)(t1 + row * ld1 + d) = make_uint2(v.x, v.y);
      }
    }
  }
};

// Work-group -> (sequence, head, tile).  Under a causal mask the tiles differ in weight and the
// order decides the balance.  Where all work-groups of a launch are resident at once (`resident`
// per CU on 256 CUs) the first half of the grid holds the heavy tiles in descending order, the
// second half the light tiles in ascending order, and the CU that got the r-th heaviest tile also
// gets the r-th lightest.  A larger grid is handed out as CUs become free, so the tiles simply come
// heaviest first (longest-processing-time order): whichever CU frees up first takes the largest
// piece left.
// Consecutive ids go to different XCDs; id % 8 = (b*H + h) % 8 keeps all tiles of one
// (sequence, head) on one XCD, whose L2 then serves the K/V re-reads.
__device__ __forceinline__ void attn_block_map(int L, int ntile, int P, int H, bool causal, bool heavy_is_high, int resident,
                                               int& b, int& h, int& tile) {
  const int rank = L / P, pair = L % P;
  b = pair / H;
  h = pair % H;
  int t = rank;   // index counted from the heavy end
  if (causal && (long)ntile * P <= 256L * resident) {
    const int nheavy = (ntile + 1) / 2;
    t = rank < nheavy ? rank : ntile - 1 - (rank - nheavy);
  }
  tile = heavy_is_high ? ntile - 1 - t : t;
  if (!causal) tile = rank;
}

// ----------------------------------------------------------------------------------------
// forward: block = NG groups of 4 waves x 32 queries, key tiles of KT keys.  With NG = 2 the two wave groups work on the same
// 128 queries and take alternate key tiles (the serial chain of a long row of tiles halves and every SIMD holds two waves of
// the work-group throughout); their partial (o, m, l) are merged through LDS at the end.
// ----------------------------------------------------------------------------------------
template <int DH, int VEC, int NG = 1>
__global__ __launch_bounds__(256 * NG, (DH <= 128 && NG == 1) ? 2 : 1) void mfma_attn_fwd_kernel(AttnArgs a) {
  // two K/V buffers per group (one barrier per trip) for the long sequences that run two groups; short ones do better
  // with one buffer and two barriers (c2: 27 against 31 us)
  constexpr int NBUF = NG == 2 ? 2 : 1;
  constexpr int KT = DH > 128 ? 32 : 64;
  constexpr int LDK = DH + 8, LDV = ld_tr(DH);
  constexpr int NKD = DH / 16;   // k steps of Q K^T
  constexpr int NDB = DH / 32;   // 32-wide d blocks of the output
  constexpr int TILE = KT * (LDK + LDV);   // one K tile and one V tile
  __shared__ __attribute__((aligned(16))) unsigned short kv_[NG * NBUF * TILE];   // per group: NBUF buffers in turn

  int b, h, qt;
  const int T = a.T, dh = a.dh, Tq = a.Tq > 0 ? a.Tq : a.T;
  const int off = T - Tq;   // position of query 0 among the keys
  attn_block_map(blockIdx.x, (Tq + 127) / 128, a.B * a.H, a.H, a.causal, true, (DH <= 128 && NG == 1) ? 2 : 1, b, h, qt);
  const int q0 = qt * 128;
  const int grp = NG > 1 ? threadIdx.x >> 8 : 0;     // wave group: key tiles grp, grp + NG, ...
  const int tid = threadIdx.x & 255, lane = tid & 63, wave = tid >> 6;
  unsigned short* const kv = kv_ + grp * NBUF * TILE;
  const int r = lane & 31, g = lane >> 5;
  const long rs = (long)a.H * dh;
  const long base = ((long)b * T) * rs + (long)h * dh;
  const long qbase = ((long)b * Tq) * rs + (long)h * dh;
  const unsigned short* Q = (const unsigned short*)a.Q + qbase;
  const unsigned short* K = (const unsigned short*)a.K + base;
  const unsigned short* V = (const unsigned short*)a.V + base;

  const int q = q0 + wave * 32 + r;             // this lane's query
  const int qpos = q + off;                     // its position among the keys
  const int wq_last = q0 + wave * 32 + 31 + off;
  bf16x8 qf[NKD];
#pragma unroll
  for (int kk = 0; kk < NKD; ++kk) qf[kk] = global_frag<VEC>(Q + (long)q * rs, kk * 16 + 8 * g, dh, q < Tq);

  f32x16 o[NDB];
#pragma unroll
  for (int d = 0; d < NDB; ++d)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[d][i] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float sc = a.scale * 1.44269504088896340736f;   // logits in log2 units

  const int kend = a.causal ? min(T, q0 + 128 + off) : T;
  RowTile<DH, VEC, KT> tk, tv;
  // (rows past the end of the sequence load as zeros: a group whose first tile lies past `kend` stages zeros once)
  tk.load(K + (long)(grp * KT) * rs, rs, T - grp * KT, dh, tid);
  tv.load(V + (long)(grp * KT) * rs, rs, T - grp * KT, dh, tid);
  if constexpr (NBUF == 2) {
    tk.store(kv, LDK, kv, LDK, tid, dh);
    tv.store(kv + KT * LDK, LDV, kv + KT * LDK, LDV, tid, dh);
    if ((grp + NG) * KT < kend) {
      tk.load(K + (long)((grp + NG) * KT) * rs, rs, T - (grp + NG) * KT, dh, tid);
      tv.load(V + (long)((grp + NG) * KT) * rs, rs, T - (grp + NG) * KT, dh, tid);
    }
    __syncthreads();
  }
  // NBUF = 2, one barrier per trip: while a tile is multiplied out of one buffer the next one (loaded a trip ago) is
  // written into the other and the one after that starts to travel.  NBUF = 1: the tile in the registers is written
  // between two barriers and the next one starts to travel.  Every group makes the same number of trips (the barriers
  // are the work-group's); a trip past `kend` only waits.
  int cur = 0;
  for (int kb0 = 0; kb0 < kend; kb0 += NG * KT, cur ^= NBUF - 1) {
    const int k0 = kb0 + grp * KT;
    const unsigned short* Ks = kv + cur * TILE;
    const unsigned short* Vs = Ks + KT * LDK;
    if constexpr (NBUF == 2) {
      if (k0 + NG * KT < kend) {
        unsigned short* nk = kv + (cur ^ 1) * TILE;   // last read a trip ago, before the barrier that ended it
        tk.store(nk, LDK, nk, LDK, tid, dh);
        tv.store(nk + KT * LDK, LDV, nk + KT * LDK, LDV, tid, dh);
        if (k0 + 2 * NG * KT < kend) {
          tk.load(K + (long)(k0 + 2 * NG * KT) * rs, rs, T - k0 - 2 * NG * KT, dh, tid);
          tv.load(V + (long)(k0 + 2 * NG * KT) * rs, rs, T - k0 - 2 * NG * KT, dh, tid);
        }
      }
    } else {
      __syncthreads();
      tk.store(kv, LDK, kv, LDK, tid, dh);
      tv.store(kv + KT * LDK, LDV, kv + KT * LDK, LDV, tid, dh);
      __syncthreads();
      if (k0 + NG * KT < kend) {
        tk.load(K + (long)(k0 + NG * KT) * rs, rs, T - k0 - NG * KT, dh, tid);
        tv.load(V + (long)(k0 + NG * KT) * rs, rs, T - k0 - NG * KT, dh, tid);
      }
    }
    // wave-uniform: a trip past the end, or a tile with nothing visible to this wave
    if (k0 < kend && !(a.causal && k0 > wq_last)) {
      float s[KT / 32][16];
#pragma unroll
      for (int kb = 0; kb < KT / 32; ++kb) {
        f32x16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < NKD; ++kk)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowfrag(&Ks[(kb * 32 + r) * LDK + kk * 16 + 8 * g]), qf[kk], acc, 0,
                                                        0, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) s[kb][i] = acc[i];
      }
      const bool need_mask = (a.causal && k0 + KT - 1 > q0 + wave * 32 + off) || (k0 + KT > T);
      if (need_mask) {
#pragma unroll
        for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = k0 + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
            if (key >= T || (a.causal && key > qpos)) s[kb][i] = -INFINITY;
          }
      }
      float mt = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) mt = fmaxf(mt, s[kb][i]);
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64)) * sc;  // sc > 0: the maximum of the scaled logits
      const float mn = fmaxf(m, mt);
      const bool moved = mn > m;                    // wave-uniform test below: most tiles move no maximum
      const float alpha = moved ? __builtin_amdgcn_exp2f(m - mn) : 1.f;   // m = -inf on the first tile -> 0
      m = mn;
      // A query that has seen no key yet and sees none in this tile (the second wave group starts at tile 1, and with
      // fewer queries than keys a wave's tile can hold a row's first key in a later tile) has mn = -inf: take 0 as the
      // base there, -inf - (-inf) would be a NaN
      const float mb = mn == -INFINITY ? 0.f : mn;
      float ps = 0.f;
#pragma unroll
      for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          s[kb][i] = __builtin_amdgcn_exp2f(fmaf(s[kb][i], sc, -mb));   // masked: -inf -> 0
          ps += s[kb][i];
        }
      l = l * alpha + ps;
      if (__ballot(moved)) {
#pragma unroll
        for (int d = 0; d < NDB; ++d)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[d][i] *= alpha;
      }

#pragma unroll
      for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
          const bf16x8 pb = pack8(&s[kb][8 * st]);
          const int kr = kb * 32 + 16 * st + 4 * g;
#pragma unroll
          for (int d = 0; d < NDB; ++d)
            o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trfrag(Vs, LDV, kr, kr + 8, d * 32, lane), pb, o[d], 0, 0, 0);
        }
    }
    if constexpr (NBUF == 2) __syncthreads();
  }

  l += __shfl_xor(l, 32, 64);
  if constexpr (NG > 1) {
    // merge the groups' partial results: group 1 parks (o, m, l) in LDS (the key / value tiles are dead), group 0 of the
    // same wave index and lane holds the same query and the same output elements
    static_assert(NG == 2, "two groups");
    static_assert(4 * (NDB * 16 + 2) * 64 * 4 <= NG * NBUF * TILE * 2, "the parked accumulators fit in the tiles");
    float* park = (float*)kv_ + (long)wave * (NDB * 16 + 2) * 64;
    if (grp == 1) {
#pragma unroll
      for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int i = 0; i < 16; ++i) park[(d * 16 + i) * 64 + lane] = o[d][i];
      park[(NDB * 16) * 64 + lane] = m;
      park[(NDB * 16 + 1) * 64 + lane] = l;
    }
    __syncthreads();
    if (grp == 1) return;
    const float m1 = park[(NDB * 16) * 64 + lane], l1 = park[(NDB * 16 + 1) * 64 + lane];
    const float mn = fmaxf(m, m1);
    // a group that saw no key has m = -inf, l = 0, o = 0: its factor is exp2(-inf) = 0 (both empty cannot happen: key 0 is visible)
    const float f0 = __builtin_amdgcn_exp2f(m - mn), f1 = __builtin_amdgcn_exp2f(m1 - mn);
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[d][i] = o[d][i] * f0 + park[(d * 16 + i) * 64 + lane] * f1;
    l = l * f0 + l1 * f1;
    m = mn;
  }
  if (q < Tq) {
    const float inv = 1.f / l;
    unsigned short* O = (unsigned short*)a.O + qbase + (long)q * rs;
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int dd = d * 32 + 8 * i4 + 4 * g;
        if (dd < dh) {
          uint2 w;
          w.x = pack_bf16x2(o[d][4 * i4] * inv, o[d][4 * i4 + 1] * inv);
          w.y = pack_bf16x2(o[d][4 * i4 + 2] * inv, o[d][4 * i4 + 3] * inv);
          *(uint2*)(O + dd) = w;
        }
      }
    if (g == 0) a.lse[((long)b * a.H + h) * Tq + q] = (m + log2f(l)) * 0.69314718055994530942f;
  }
}

template <int NDB>
__device__ __forceinline__ void store_rows_T(unsigned short* dst, const f32x16* acc, float mul, int g, int dh) {
  // acc[d] holds X^T[32*d + 8*(i/4) + 4g + i%4][this lane's row]; dst points at that row
#pragma unroll
  for (int d = 0; d < NDB; ++d)
#pragma unroll
    for (int i4 = 0; i4 < 4; ++i4) {
      const int dd = d * 32 + 8 * i4 + 4 * g;
      if (dd < dh) {
        uint2 w;
        w.x = pack_bf16x2(acc[d][4 * i4] * mul, acc[d][4 * i4 + 1] * mul);
        w.y = pack_bf16x2(acc[d][4 * i4 + 2] * mul, acc[d][4 * i4 + 3] * mul);
        *(uint2*)(dst + dd) = w;
      }
    }
}

// ----------------------------------------------------------------------------------------
// backward, dK and dV: block = 4 waves x 32 keys (K, V rows of a wave live in registers as
// B operands); query tiles of 32 rows of Q and dO are staged in LDS.
//   S[q][key] = Q K^T,  P = exp(S - lse),  dP[q][key] = dO V^T,  dS = P (dP - delta)
//   dV^T[d][key] += dO^T[d][q] P[q][key],   dK^T[d][key] += Q^T[d][q] dS[q][key]
// ----------------------------------------------------------------------------------------
// Score-gradient scratch: first query column kept for the block of 128 keys number t (a multiple of 256 at or below the
// first query that sees one of the block's keys; `off` = position of query 0 among the keys), and where that block starts
// within its (sequence, head) part (elements).
__host__ __device__ inline int ds_block_start(int t, int off, int causal) {
  const int u = 128 * t - off;
  return causal && u > 0 ? (u >> 8) << 8 : 0;
}
__host__ __device__ inline long ds_block_offset(int t, int ld, int off, int causal) {
  long o = 0;
  for (int j = 0; j < t; ++j) o += 128L * (ld - ds_block_start(j, off, causal));
  return o;
}

// queries per staged tile of the dK / dV kernel; 64 (half the barriers, two independent blocks per trip) measured 6 %
// slower at T = 4096.  The dQ-from-dS kernel derives from it which part of a dS^T row was written.
constexpr int DKV_QT = 32;

template <int DH, int VEC, int NW, int QT>
__global__ __launch_bounds__(64 * NW, DH <= 64 ? 2 : 1) void mfma_attn_dkv_kernel(AttnBwdArgs a) {
  constexpr int KB = 32 * NW;    // keys per work-group
  constexpr int NQ = QT / 32;   // 32-query blocks per staged tile: independent chains the scheduler can interleave
  constexpr bool SEP = DH <= 128;                       // separate tiles for the two read patterns
  constexpr int LDR = SEP ? DH + 8 : ld_tr(DH), LDT = ld_tr(DH);
  constexpr int NKD = DH / 16, NDB = DH / 32;
  __shared__ __attribute__((aligned(16))) unsigned short Qr[QT * LDR];
  __shared__ __attribute__((aligned(16))) unsigned short Gr[QT * LDR];
  __shared__ __attribute__((aligned(16))) unsigned short Qt_[SEP ? QT * LDT : 8];
  __shared__ __attribute__((aligned(16))) unsigned short Gt_[SEP ? QT * LDT : 8];
  __shared__ __attribute__((aligned(16))) float lse_s[QT];
  __shared__ __attribute__((aligned(16))) float del_s[QT];
  unsigned short* Qt = SEP ? Qt_ : Qr;
  unsigned short* Gt = SEP ? Gt_ : Gr;

  int b, h, ktile;
  attn_block_map(blockIdx.x, (a.T + KB - 1) / KB, a.B * a.H, a.H, a.causal, false, DH <= 64 ? 2 : 1, b, h, ktile);
  const int k0 = ktile * KB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int T = a.T, dh = a.dh, Tq = a.Tq > 0 ? a.Tq : a.T;
  const int off = T - Tq;   // position of query 0 among the keys
  const long rs = (long)a.H * dh;
  const long base = ((long)b * T) * rs + (long)h * dh;
  const long qbase = ((long)b * Tq) * rs + (long)h * dh;
  const unsigned short* Q = (const unsigned short*)a.Q + qbase;
  const unsigned short* K = (const unsigned short*)a.K + base;
  const unsigned short* V = (const unsigned short*)a.V + base;
  const unsigned short* dO = (const unsigned short*)a.dO + qbase;
  const float* lse = a.lse + ((long)b * a.H + h) * Tq;
  const float* delta = a.delta + (long)b * Tq * a.H + h;

  const int key = k0 + wave * 32 + r;
  // this lane's row of dS^T (keys past T lie inside the padded row count and receive zeros)
  unsigned short* dsrow = nullptr;
  if (a.dSt) {
    static_assert(KB == 128, "the score-gradient scratch is laid out in blocks of 128 keys");
    const int s0 = ds_block_start(ktile, off, a.causal);
    dsrow = (unsigned short*)a.dSt + ((long)b * a.H + h) * a.ds_per + ds_block_offset(ktile, a.ds_ld, off, a.causal) +
            (long)(wave * 32 + r) * (a.ds_ld - s0) - s0 + 4 * g;
  }
  const int wk_first = k0 + wave * 32;
  bf16x8 kf[NKD], vf[NKD];
#pragma unroll
  for (int kk = 0; kk < NKD; ++kk) {
    kf[kk] = global_frag<VEC>(K + (long)key * rs, kk * 16 + 8 * g, dh, key < T);
    vf[kk] = global_frag<VEC>(V + (long)key * rs, kk * 16 + 8 * g, dh, key < T);
  }
  f32x16 accK[NDB], accV[NDB];
#pragma unroll
  for (int d = 0; d < NDB; ++d)
#pragma unroll
    for (int i = 0; i < 16; ++i) accK[d][i] = accV[d][i] = 0.f;
  const float sc = a.scale * 1.44269504088896340736f;

  const int qbeg = a.causal ? (max(k0 - off, 0) / QT) * QT : 0;   // first query tile that sees a key of this tile
  RowTile<DH, VEC, QT, 64 * NW> tq, tg;
  float nlse = 0.f, ndel = 0.f;
  auto prefetch = [&](int q0) {
    tq.load(Q + (long)q0 * rs, rs, Tq - q0, dh, tid);
    tg.load(dO + (long)q0 * rs, rs, Tq - q0, dh, tid);
    // the softmax statistics of the tile's queries: loaded by every thread from a clamped index and
    // left untouched until they are stored, so that neither a branch nor arithmetic on the loaded
    // value makes the wave wait for this prefetch before it multiplies the current tile (rows past
    // the end repeat the last query: their probabilities are masked to zero below)
    const int qi = min(q0 + (tid & (QT - 1)), Tq - 1);
    nlse = lse[qi];
    ndel = delta[(long)qi * a.H];
  };
  if (qbeg < Tq) prefetch(qbeg);
  // Every load issued so far (the K / V rows held in registers, the first tile) completes here.  Without
  // this the compiler, which cannot tell the first trip of the loop from the others, waits for ALL
  // outstanding loads, the prefetch of the next tile included, before the first product of every trip.
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0), other counters untouched
  for (int q0 = qbeg; q0 < Tq; q0 += QT) {
    __syncthreads();
    tq.store(Qr, LDR, Qt, LDT, tid, dh);
    tg.store(Gr, LDR, Gt, LDT, tid, dh);
    if (tid < QT) {
      lse_s[tid] = nlse * 1.44269504088896340736f;
      del_s[tid] = ndel;
    }
    __syncthreads();
    if (q0 + QT < Tq) prefetch(q0 + QT);
    // (a wave whose keys all follow the tile's queries multiplies zeros here: a branch around the
    //  body costs more registers than the diagonal tiles cost time)

    f32x16 S[NQ], dP[NQ];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) S[qb][i] = dP[qb][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < NKD; ++kk)
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        S[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowfrag(&Qr[(qb * 32 + r) * LDR + kk * 16 + 8 * g]), kf[kk], S[qb], 0, 0, 0);
        dP[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowfrag(&Gr[(qb * 32 + r) * LDR + kk * 16 + 8 * g]), vf[kk], dP[qb], 0, 0, 0);
      }
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
      const int qs = q0 + qb * 32;   // first query of this block
      float p[16], ds[16];
      // wave-uniform: most blocks lie wholly inside the visible region and need no per-element test
      const bool need_mask = qs + 32 > Tq || wk_first + 32 > T || (a.causal && wk_first + 31 > qs + off);
      if (need_mask) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const float4 L = *(const float4*)&lse_s[qb * 32 + 8 * i4 + 4 * g];
          const float4 D = *(const float4*)&del_s[qb * 32 + 8 * i4 + 4 * g];
          const float Lv[4] = {L.x, L.y, L.z, L.w}, Dv[4] = {D.x, D.y, D.z, D.w};
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int i = 4 * i4 + t;
            const int qq = qs + 8 * i4 + 4 * g + t;
            const bool vis = qq < Tq && key < T && (!a.causal || key <= qq + off);
            // the mask caps the argument (exp2(-inf) = 0): nothing is left that a branch could skip
            const float pv = __builtin_amdgcn_exp2f(fminf(fmaf(S[qb][i], sc, -Lv[t]), vis ? INFINITY : -INFINITY));
            p[i] = pv;
            ds[i] = pv * (dP[qb][i] - Dv[t]);
          }
        }
      } else {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const float4 L = *(const float4*)&lse_s[qb * 32 + 8 * i4 + 4 * g];
          const float4 D = *(const float4*)&del_s[qb * 32 + 8 * i4 + 4 * g];
          const float Lv[4] = {L.x, L.y, L.z, L.w}, Dv[4] = {D.x, D.y, D.z, D.w};
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int i = 4 * i4 + t;
            const float pv = __builtin_amdgcn_exp2f(fmaf(S[qb][i], sc, -Lv[t]));
            p[i] = pv;
            ds[i] = pv * (dP[qb][i] - Dv[t]);
          }
        }
      }
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        const bf16x8 pb = pack8(&p[8 * st]), db = pack8(&ds[8 * st]);
        const int kb0 = qb * 32 + 16 * st + 4 * g;
        if (dsrow) {   // uniform.  Elements 0..3 / 4..7 of db: queries qs + 16 st + 4 g + {0..3} / + 8 + {0..3} of this lane's key
          union {
            bf16x8 v;
            uint2 h[2];
          } u;
          u.v = db;
          *(uint2*)(dsrow + qs + 16 * st) = u.h[0];
          *(uint2*)(dsrow + qs + 16 * st + 8) = u.h[1];
        }
#pragma unroll
        for (int d = 0; d < NDB; ++d) {
          accV[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trfrag(Gt, LDT, kb0, kb0 + 8, d * 32, lane), pb, accV[d], 0, 0, 0);
          accK[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trfrag(Qt, LDT, kb0, kb0 + 8, d * 32, lane), db, accK[d], 0, 0, 0);
        }
      }
    }
  }
  if (key < T) {
    store_rows_T<NDB>((unsigned short*)a.dK + base + (long)key * rs, accK, a.scale, g, dh);
    store_rows_T<NDB>((unsigned short*)a.dV + base + (long)key * rs, accV, 1.f, g, dh);
  }
}

// ----------------------------------------------------------------------------------------
// backward, dK and dV with two kinds of waves (head widths 64 .. 128).  The kernel above runs one wave per SIMD (its
// accumulators and key / value fragments need more than 256 registers), and whatever such a wave does besides multiplying
// (the softmax arithmetic, LDS traffic, the staging of the next tile) is time the matrix cores stand idle.  Here a
// work-group has eight waves, two per SIMD, that split the work of a 32-key block between them:
//   a score wave   holds the block's K and V fragments, computes S = Q K^T and dP = dO V^T of one query tile, turns them
//                  into P and dS = P (dP - delta), and leaves both as bf16 operand fragments in LDS (and dS^T in memory
//                  for the dQ product);
//   a gradient wave holds the block's dK and dV accumulators and adds dO^T P and Q^T dS of the PREVIOUS query tile, taken
//                  from those fragments.
// Each needs well under 256 registers, both issue 16 MFMAs per tile, and on every SIMD one of each kind is resident: the
// gradient wave's products fill the time the score wave spends on exponentials and conversions.  Query tiles go through
// three LDS stages (written one trip ahead, read by the score waves in the next trip and by the gradient waves in the
// one after), the fragments through two buffers; one work-group barrier per trip.
// ----------------------------------------------------------------------------------------
template <int DH, int VEC>
__global__ __launch_bounds__(512, 1) void mfma_attn_dkv_ws_kernel(AttnBwdArgs a) {
  constexpr int QT = DKV_QT, KB = 128, NST = 3;
  static_assert(QT == 32, "one 32-query block per tile");
  // One tile per matrix serves both read patterns: rows 2 DH + 32 bytes apart put the 8 rows a 16-byte fragment read
  // touches per clock 8 banks apart, and the 4 rows x 32 bytes of a transposing read's 16 lanes in 4 different bank groups.
  constexpr int LD = DH + 16;
  constexpr int NKD = DH / 16, NDB = DH / 32;
  constexpr int STAGE = 2 * QT * LD;   // Q tile, dO tile
  __shared__ __attribute__((aligned(16))) unsigned short tiles[NST * STAGE];
  __shared__ __attribute__((aligned(16))) uint4 hand[2][4][4][64];   // [buffer][key block][P st 0, P st 1, dS st 0, dS st 1][lane]
  __shared__ __attribute__((aligned(16))) float lse_s[NST][QT];
  __shared__ __attribute__((aligned(16))) float del_s[NST][QT];

  int b, h, ktile;
  attn_block_map(blockIdx.x, (a.T + KB - 1) / KB, a.B * a.H, a.H, a.causal, false, 1, b, h, ktile);
  const int k0 = ktile * KB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int blk = wave & 3;          // 32-key block of the wave
  const bool score = wave < 4;       // waves 0..3 score, 4..7 gradient: one of each per SIMD
  const int r = lane & 31, g = lane >> 5;
  const int T = a.T, dh = a.dh, Tq = a.Tq > 0 ? a.Tq : a.T;
  const int off = T - Tq;   // position of query 0 among the keys
  const long rs = (long)a.H * dh;
  const long base = ((long)b * T) * rs + (long)h * dh;
  const long qbase = ((long)b * Tq) * rs + (long)h * dh;
  const unsigned short* Q = (const unsigned short*)a.Q + qbase;
  const unsigned short* dO = (const unsigned short*)a.dO + qbase;
  const float* lse = a.lse + ((long)b * a.H + h) * Tq;
  const float* delta = a.delta + (long)b * Tq * a.H + h;
  const int key = k0 + blk * 32 + r;
  const int wk_first = k0 + blk * 32;

  const int qbeg = a.causal ? (max(k0 - off, 0) / QT) * QT : 0;   // first query tile that sees a key of this tile
  const int n = qbeg < Tq ? (Tq - qbeg + QT - 1) / QT : 0;        // query tiles
  // The gradient waves (threads 256..511) also move the query tiles: they have the time, the score waves' chain of
  // products, exponentials and conversions is what a trip waits for.  (A second register set, so that a tile has two
  // trips to arrive, cost more registers than the kernel has: 334 against 238 us at T = 4096.)
  const int gt = tid - 256;
  RowTile<DH, VEC, QT, 256> tq, tg;
  float nlse = 0.f, ndel = 0.f;
  auto prefetch = [&](int q0) {
    tq.load(Q + (long)q0 * rs, rs, Tq - q0, dh, gt);
    tg.load(dO + (long)q0 * rs, rs, Tq - q0, dh, gt);
    const int qi = min(q0 + (gt & (QT - 1)), Tq - 1);   // rows past the end repeat the last query: masked below
    nlse = lse[qi];
    ndel = delta[(long)qi * a.H];
  };
  auto stage = [&](int st) {
    unsigned short* t = tiles + st * STAGE;
    tq.store(t, LD, t, LD, gt, dh);
    tg.store(t + QT * LD, LD, t + QT * LD, LD, gt, dh);
    if (gt < QT) {
      lse_s[st][gt] = nlse * 1.44269504088896340736f;
      del_s[st][gt] = ndel;
    }
  };

  if (score) {
    const unsigned short* K = (const unsigned short*)a.K + base;
    const unsigned short* V = (const unsigned short*)a.V + base;
    bf16x8 kf[NKD], vf[NKD];
#pragma unroll
    for (int kk = 0; kk < NKD; ++kk) {
      kf[kk] = global_frag<VEC>(K + (long)key * rs, kk * 16 + 8 * g, dh, key < T);
      vf[kk] = global_frag<VEC>(V + (long)key * rs, kk * 16 + 8 * g, dh, key < T);
    }
    unsigned short* dsrow = nullptr;
    if (a.dSt) {
      const int s0 = ds_block_start(ktile, off, a.causal);
      dsrow = (unsigned short*)a.dSt + ((long)b * a.H + h) * a.ds_per + ds_block_offset(ktile, a.ds_ld, off, a.causal) +
              (long)(blk * 32 + r) * (a.ds_ld - s0) - s0 + 4 * g;
    }
    const float sc = a.scale * 1.44269504088896340736f;
    for (int it = 0; it <= n; ++it) {
      __syncthreads();
      if (it == n) break;
      const int q0 = qbeg + it * QT;
      const unsigned short* Qr = tiles + (it % NST) * STAGE;
      const unsigned short* Gr = Qr + QT * LD;
      f32x16 S, dP;
#pragma unroll
      for (int i = 0; i < 16; ++i) S[i] = dP[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKD; ++kk) {
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowfrag(&Qr[r * LD + kk * 16 + 8 * g]), kf[kk], S, 0, 0, 0);
        dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowfrag(&Gr[r * LD + kk * 16 + 8 * g]), vf[kk], dP, 0, 0, 0);
      }
      float p[16], ds[16];
      const float* Ls = lse_s[it % NST];
      const float* Ds = del_s[it % NST];
      // wave-uniform: most tiles lie wholly inside the visible region and need no per-element test
      const bool need_mask = q0 + QT > Tq || wk_first + 32 > T || (a.causal && wk_first + 31 > q0 + off);
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const float4 L = *(const float4*)&Ls[8 * i4 + 4 * g];
        const float4 D = *(const float4*)&Ds[8 * i4 + 4 * g];
        const float Lv[4] = {L.x, L.y, L.z, L.w}, Dv[4] = {D.x, D.y, D.z, D.w};
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const int i = 4 * i4 + t;
          float arg = fmaf(S[i], sc, -Lv[t]);
          if (need_mask) {
            const int qq = q0 + 8 * i4 + 4 * g + t;
            const bool vis = qq < Tq && key < T && (!a.causal || key <= qq + off);
            arg = fminf(arg, vis ? INFINITY : -INFINITY);   // exp2(-inf) = 0
          }
          const float pv = __builtin_amdgcn_exp2f(arg);
          p[i] = pv;
          ds[i] = pv * (dP[i] - Dv[t]);
        }
      }
      uint4* hd = hand[it & 1][blk][0] + lane;
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        union {
          bf16x8 v;
          uint4 q;
          uint2 hh[2];
        } up, ud;
        up.v = pack8(&p[8 * st]);
        ud.v = pack8(&ds[8 * st]);
        hd[st * 64] = up.q;
        hd[(2 + st) * 64] = ud.q;
        if (dsrow) {   // uniform.  Elements 0..3 / 4..7: queries q0 + 16 st + 4 g + {0..3} / + 8 + {0..3} of this lane's key
          *(uint2*)(dsrow + q0 + 16 * st) = ud.hh[0];
          *(uint2*)(dsrow + q0 + 16 * st + 8) = ud.hh[1];
        }
      }
    }
  } else {
    f32x16 accK[NDB], accV[NDB];
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
      for (int i = 0; i < 16; ++i) accK[d][i] = accV[d][i] = 0.f;
    if (n > 0) {
      prefetch(qbeg);
      stage(0);
      if (n > 1) prefetch(qbeg + QT);
    }
    for (int it = 0; it <= n; ++it) {
      __syncthreads();
      // the tile it + 1 (requested a trip ago) goes into its stage and the tile it + 2 starts to travel
      if (it + 1 < n) {
        stage((it + 1) % NST);
        if (it + 2 < n) prefetch(qbeg + (it + 2) * QT);
      }
      if (it == 0) continue;
      const unsigned short* Qt = tiles + ((it - 1) % NST) * STAGE;
      const unsigned short* Gt = Qt + QT * LD;
      const uint4* hd = hand[(it - 1) & 1][blk][0] + lane;
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        union {
          uint4 q;
          bf16x8 v;
        } up, ud;
        up.q = hd[st * 64];
        ud.q = hd[(2 + st) * 64];
        const int kb0 = 16 * st + 4 * g;
#pragma unroll
        for (int d = 0; d < NDB; ++d) {
          accV[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trfrag(Gt, LD, kb0, kb0 + 8, d * 32, lane), up.v, accV[d], 0, 0, 0);
          accK[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trfrag(Qt, LD, kb0, kb0 + 8, d * 32, lane), ud.v, accK[d], 0, 0, 0);
        }
      }
    }
    if (key < T) {
      store_rows_T<NDB>((unsigned short*)a.dK + base + (long)key * rs, accK, a.scale, g, dh);
      store_rows_T<NDB>((unsigned short*)a.dV + base + (long)key * rs, accV, 1.f, g, dh);
    }
  }
}

// ----------------------------------------------------------------------------------------
// backward, dQ: block = 4 waves x 32 queries (Q and dO rows of a wave live in registers);
// key tiles of K (both read patterns) and V are staged in LDS.
//   S^T[key][q] = K Q^T, dP^T[key][q] = V dO^T, dS^T = P^T (dP^T - delta),
//   dQ^T[d][q] += K^T[d][key] dS^T[key][q]
// ----------------------------------------------------------------------------------------
template <int DH, int VEC>
__global__ __launch_bounds__(256, DH <= 128 ? 2 : 1) void mfma_attn_dq_kernel(AttnBwdArgs a) {
  constexpr int KT = DH > 128 ? 32 : 64;
  constexpr bool SEP = DH <= 128;
  constexpr int LDR = SEP ? DH + 8 : ld_tr(DH), LDT = ld_tr(DH);
  constexpr int NKD = DH / 16, NDB = DH / 32;
  __shared__ __attribute__((aligned(16))) unsigned short Kr[KT * LDR];
  __shared__ __attribute__((aligned(16))) unsigned short Vr[KT * LDR];
  __shared__ __attribute__((aligned(16))) unsigned short Kt_[SEP ? KT * LDT : 8];
  unsigned short* Kt = SEP ? Kt_ : Kr;

  int b, h, qt;
  const int T = a.T, dh = a.dh, Tq = a.Tq > 0 ? a.Tq : a.T;
  const int off = T - Tq;   // position of query 0 among the keys
  attn_block_map(blockIdx.x, (Tq + 127) / 128, a.B * a.H, a.H, a.causal, true, DH <= 128 ? 2 : 1, b, h, qt);
  const int q0 = qt * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const long rs = (long)a.H * dh;
  const long base = ((long)b * T) * rs + (long)h * dh;
  const long qbase = ((long)b * Tq) * rs + (long)h * dh;
  const unsigned short* Q = (const unsigned short*)a.Q + qbase;
  const unsigned short* K = (const unsigned short*)a.K + base;
  const unsigned short* V = (const unsigned short*)a.V + base;
  const unsigned short* dO = (const unsigned short*)a.dO + qbase;

  const int q = q0 + wave * 32 + r;
  const int qpos = q + off;
  const int wq_last = q0 + wave * 32 + 31 + off;
  bf16x8 qf[NKD], gf[NKD];
#pragma unroll
  for (int kk = 0; kk < NKD; ++kk) {
    qf[kk] = global_frag<VEC>(Q + (long)q * rs, kk * 16 + 8 * g, dh, q < Tq);
    gf[kk] = global_frag<VEC>(dO + (long)q * rs, kk * 16 + 8 * g, dh, q < Tq);
  }
  const float lse2 = q < Tq ? a.lse[((long)b * a.H + h) * Tq + q] * 1.44269504088896340736f : 0.f;
  const float del = q < Tq ? a.delta[((long)b * Tq + q) * a.H + h] : 0.f;
  f32x16 acc[NDB];
#pragma unroll
  for (int d = 0; d < NDB; ++d)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[d][i] = 0.f;
  const float sc = a.scale * 1.44269504088896340736f;

  const int kend = a.causal ? min(T, q0 + 128 + off) : T;
  RowTile<DH, VEC, KT> tk, tv;
  tk.load(K, rs, T, dh, tid);
  tv.load(V, rs, T, dh, tid);
  for (int k0 = 0; k0 < kend; k0 += KT) {
    __syncthreads();
    tk.store(Kr, LDR, Kt, LDT, tid, dh);
    tv.store(Vr, LDR, Vr, LDR, tid, dh);
    __syncthreads();
    if (k0 + KT < kend) {
      tk.load(K + (long)(k0 + KT) * rs, rs, T - k0 - KT, dh, tid);
      tv.load(V + (long)(k0 + KT) * rs, rs, T - k0 - KT, dh, tid);
    }
    if (a.causal && k0 > wq_last) continue;
#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb) {
      f32x16 S, dP;
#pragma unroll
      for (int i = 0; i < 16; ++i) S[i] = dP[i] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKD; ++kk) {
        S = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowfrag(&Kr[(kb * 32 + r) * LDR + kk * 16 + 8 * g]), qf[kk], S, 0, 0, 0);
        dP = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rowfrag(&Vr[(kb * 32 + r) * LDR + kk * 16 + 8 * g]), gf[kk], dP, 0, 0, 0);
      }
      float ds[16];
      // key of element i = k0 + kb*32 + 4g + (8*(i/4) + i%4): visible iff that constant offset is at most
      // `lim` (one compare per element); the mask caps the exponent's argument, exp2(-inf) = 0
      const int lim = (a.causal ? min(T - 1, qpos) : T - 1) - (k0 + kb * 32 + 4 * g);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const bool vis = 8 * (i >> 2) + (i & 3) <= lim;
        const float pv = __builtin_amdgcn_exp2f(fminf(fmaf(S[i], sc, -lse2), vis ? INFINITY : -INFINITY));
        ds[i] = pv * (dP[i] - del);
      }
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        const bf16x8 db = pack8(&ds[8 * st]);
        const int kb0 = kb * 32 + 16 * st + 4 * g;
#pragma unroll
        for (int d = 0; d < NDB; ++d)
          acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trfrag(Kt, LDT, kb0, kb0 + 8, d * 32, lane), db, acc[d], 0, 0, 0);
      }
    }
  }
  if (q < Tq) store_rows_T<NDB>((unsigned short*)a.dQ + qbase + (long)q * rs, acc, a.scale, g, dh);
}

// ----------------------------------------------------------------------------------------
// backward, dQ from the stored score gradient: dQ[q][:] = scale * sum_key dS[q][key] K[key][:], a plain product.
// block = 4 waves x 64 queries; key tiles of KT rows of K and of dS^T (as the dK / dV kernel left it, [key][query])
// are staged in LDS and both read with transposing loads:
//   dQ^T[d][q] += K^T[d][key] dS^T[key][q]
// The dK / dV work-group of 128 keys starting at kt0 wrote the queries from (max(kt0 - off, 0) / DKV_QT) * DKV_QT on (every
// earlier query sees none of its keys); what lies before that in a row was never written and is replaced by zeros here.
// ----------------------------------------------------------------------------------------
template <int DH, int VEC, int QB>
__global__ __launch_bounds__(256, 2) void mfma_attn_dq_ds_kernel(AttnBwdArgs a) {
  // keys per trip.  Under a causal mask the last query tile of a sequence walks all keys while its light partner on the
  // CU is long done, one wave per SIMD and a barrier pair per trip: fewer, longer trips shorten that chain (T = 4096:
  // 101 -> 90 us with 128 keys; two work-groups per CU either way).  The 256-query tile has no LDS left for it.
  constexpr int KT = QB == 128 ? 128 : 64;
  constexpr int LDT = ld_tr(DH), LDD = ld_tr(QB);
  constexpr int NDB = DH / 32;
  // QB = 256: a wave owns 64 queries and all of d.  QB = 128 (twice the work-groups: short sequence counts fill the chip
  // and heavy and light causal tiles pair up): 64 queries and half of d.
  constexpr int DSPLIT = QB == 128 ? 2 : 1;
  static_assert(NDB % DSPLIT == 0, "d blocks split evenly");
  constexpr int ND = NDB / DSPLIT;
  constexpr int CPRD = QB / 8, NP = KT * CPRD / 256, RSTEP = 256 / CPRD;   // dS^T tile: 16-byte pieces per row, per thread
  __shared__ __attribute__((aligned(16))) unsigned short Kt[KT * LDT];
  __shared__ __attribute__((aligned(16))) unsigned short Dt[KT * LDD];

  int b, h, qt;
  const int T = a.T, dh = a.dh, Tq = a.Tq > 0 ? a.Tq : a.T;
  const int off = T - Tq;
  attn_block_map(blockIdx.x, (Tq + QB - 1) / QB, a.B * a.H, a.H, a.causal, true, 2, b, h, qt);
  const int q0 = qt * QB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int wq = (DSPLIT == 2 ? (wave & 1) : wave) * 64;   // the wave's first query in the tile
  const int d0 = DSPLIT == 2 ? (wave >> 1) * ND : 0;       // its first d block
  const long rs = (long)a.H * dh;
  const unsigned short* K = (const unsigned short*)a.K + ((long)b * T) * rs + (long)h * dh;
  const unsigned short* D = (const unsigned short*)a.dSt + ((long)b * a.H + h) * a.ds_per;
  const int wq_last = q0 + wq + 63 + off;

  f32x16 acc[2][ND];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int d = 0; d < ND; ++d)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[j][d][i] = 0.f;

  const int kend = a.causal ? min(T, q0 + QB + off) : T;
  RowTile<DH, VEC, KT> tk;
  // the dS^T tile: KT rows of QB queries: rows tid / CPRD + RSTEP i, queries 8 (tid % CPRD) ..
  uint4 td[NP];
  const int dq8 = (tid % CPRD) * 8;
  // the tile's block of 128 keys: its start within D and its first kept query; load_d is called with rising k0
  int blk_t = 0, blk_s = 0;
  long blk_off = 0;
  auto load_d = [&](int k0) {
    while (blk_t < (k0 >> 7)) {
      blk_off += 128L * (a.ds_ld - blk_s);
      ++blk_t;
      blk_s = ds_block_start(blk_t, off, a.causal);
    }
    const int ldt = a.ds_ld - blk_s;   // q0 >= blk_s: the block's keys are visible to this tile's queries or it is not read
    const char* p = (const char*)(D + blk_off + (long)(k0 & 127) * ldt + (q0 - blk_s));
    const unsigned voff = (unsigned)(((tid / CPRD) * ldt + dq8) * 2);
#pragma unroll
    for (int i = 0; i < NP; ++i) td[i] = *(const uint4*)(p + (unsigned)(RSTEP * i * ldt * 2) + voff);
  };
  tk.load(K, rs, T, dh, tid);
  load_d(0);
  for (int k0 = 0; k0 < kend; k0 += KT) {
    // first query the writer of this tile's keys covered
    const int written = a.causal ? (max((k0 / 128) * 128 - off, 0) / DKV_QT) * DKV_QT : 0;
    const bool keep = q0 + dq8 >= written;
    __syncthreads();
    tk.store(Kt, LDT, Kt, LDT, tid, dh);
#pragma unroll
    for (int i = 0; i < NP; ++i) *(uint4*)(&Dt[(tid / CPRD + RSTEP * i) * LDD + dq8]) = keep ? td[i] : make_uint4(0, 0, 0, 0);
    __syncthreads();
    if (k0 + KT < kend) {
      tk.load(K + (long)(k0 + KT) * rs, rs, T - k0 - KT, dh, tid);
      load_d(k0 + KT);
    }
    if (a.causal && k0 > wq_last) continue;   // wave-uniform: nothing visible to this wave's queries
#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        const int kr = kb * 32 + 16 * st + 4 * g;
        bf16x8 bq[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) bq[j] = trfrag(Dt, LDD, kr, kr + 8, wq + j * 32, lane);
#pragma unroll
        for (int d = 0; d < ND; ++d) {
          const bf16x8 ka = trfrag(Kt, LDT, kr, kr + 8, (d0 + d) * 32, lane);
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[j][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, bq[j], acc[j][d], 0, 0, 0);
        }
      }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int q = q0 + wq + j * 32 + r;
    if (q < Tq)
      store_rows_T<ND>((unsigned short*)a.dQ + ((long)b * Tq) * rs + (long)h * dh + (long)q * rs + d0 * 32, acc[j], a.scale, g, dh - d0 * 32);
  }
}

// The score-gradient scratch is used for head widths of 64 .. 128 (one work-group per CU otherwise, and the recomputing
// kernel is already the smaller part there).
bool attn_ds_dims(int T, int Tq, int dh, int causal, int* ld, long* per) {
  if (Tq <= 0) Tq = T;
  if (dh < 64 || dh > 128 || dh % 8 != 0) return false;
  *ld = (Tq + 255) / 256 * 256;
  *per = ds_block_offset((T + 127) / 128, *ld, T - Tq, causal);
  return true;
}

static int attn_vec(int dh) { return dh % 8 == 0 ? 8 : (dh % 4 == 0 ? 4 : 0); }

bool mfma_attn_supported(int T, int dh) { return T >= 1 && dh >= 4 && dh <= 256 && attn_vec(dh) != 0; }

template <int DH>
static void launch_dh(const AttnArgs* f, const AttnBwdArgs* bw, hipStream_t s) {
  if (f) {
    dim3 g((((f->Tq > 0 ? f->Tq : f->T) + 127) / 128) * f->H * f->B);
    // long sequences: two wave groups per work-group split the key tiles of a query tile between them
    const bool split = DH <= 128 && DH >= 64 && f->T >= 1024;
    if constexpr (DH <= 128 && DH >= 64) {
      if (split) {
        if (attn_vec(f->dh) == 8)
          mfma_attn_fwd_kernel<DH, 8, 2><<<g, 512, 0, s>>>(*f);
        else
          mfma_attn_fwd_kernel<DH, 4, 2><<<g, 512, 0, s>>>(*f);
        return;
      }
    }
    if (attn_vec(f->dh) == 8)
      mfma_attn_fwd_kernel<DH, 8><<<g, 256, 0, s>>>(*f);
    else
      mfma_attn_fwd_kernel<DH, 4><<<g, 256, 0, s>>>(*f);
  } else {
    dim3 g((((bw->Tq > 0 ? bw->Tq : bw->T) + 127) / 128) * bw->H * bw->B);
    prof_mark(s, "bwd.attention_dkv");
    // four waves (128 keys) per work-group; two-wave work-groups (two per CU where the registers
    // leave one wave per SIMD) were measured 7 % slower: the Q / dO staging doubles
    constexpr int NW = 4;
    constexpr int QT = DKV_QT;
    static_assert(32 * NW == 128, "the dQ-from-dS kernel and attn_ds_dims assume work-groups of 128 keys");
    dim3 gk(((bw->T + 32 * NW - 1) / (32 * NW)) * bw->H * bw->B);
    if constexpr (DH >= 64 && DH <= 128) {
      if (attn_vec(bw->dh) == 8)
        mfma_attn_dkv_ws_kernel<DH, 8><<<gk, 512, 0, s>>>(*bw);
      else
        mfma_attn_dkv_ws_kernel<DH, 4><<<gk, 512, 0, s>>>(*bw);
    } else if (attn_vec(bw->dh) == 8)
      mfma_attn_dkv_kernel<DH, 8, NW, QT><<<gk, 64 * NW, 0, s>>>(*bw);
    else
      mfma_attn_dkv_kernel<DH, 4, NW, QT><<<gk, 64 * NW, 0, s>>>(*bw);
    prof_mark(s, "bwd.attention_dq");
    if constexpr (DH >= 64 && DH <= 128) {
      if (bw->dSt) {
        const int tq = bw->Tq > 0 ? bw->Tq : bw->T;
        // 128-query tiles (half of d per wave) unless 256-query tiles already make three work-groups per CU
        constexpr bool can_split = (DH / 32) % 2 == 0;
        const long big = (long)((tq + 255) / 256) * bw->H * bw->B;
        if (can_split && big < 3 * 256) {
          if constexpr (can_split) mfma_attn_dq_ds_kernel<DH, 8, 128><<<dim3(((tq + 127) / 128) * bw->H * bw->B), 256, 0, s>>>(*bw);
        } else {
          mfma_attn_dq_ds_kernel<DH, 8, 256><<<dim3((unsigned)big), 256, 0, s>>>(*bw);
        }
        return;
      }
    }
    if (attn_vec(bw->dh) == 8)
      mfma_attn_dq_kernel<DH, 8><<<g, 256, 0, s>>>(*bw);
    else
      mfma_attn_dq_kernel<DH, 4><<<g, 256, 0, s>>>(*bw);
  }
}

static void dispatch_dh(int dh, const AttnArgs* f, const AttnBwdArgs* bw, hipStream_t s) {
  if (dh <= 32)
    launch_dh<32>(f, bw, s);
  else if (dh <= 64)
    launch_dh<64>(f, bw, s);
  else if (dh <= 96)
    launch_dh<96>(f, bw, s);
  else if (dh <= 128)
    launch_dh<128>(f, bw, s);
  else if (dh <= 192)
    launch_dh<192>(f, bw, s);
  else
    launch_dh<256>(f, bw, s);
}

void launch_mfma_attn_fwd(const AttnArgs& a, hipStream_t s) { dispatch_dh(a.dh, &a, nullptr, s); }
void launch_mfma_attn_bwd(const AttnBwdArgs& a, hipStream_t s) { dispatch_dh(a.dh, nullptr, &a, s); }

}  // namespace sh
