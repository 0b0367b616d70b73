// Fused attention on bf16 matrix cores for the SwitchHead layer (arXiv 2312.07987):
// A^h = softmax(Q^h K^h^T / sqrt(d_head)) and the read-out A^h V^h of Sec. 2.1, one
// attention matrix per head, computed tile by tile with a running maximum so that the
// T x T matrix never exists in memory; plus the matching backward kernels.
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

// copies `nrows` rows of `dh` bf16 (zero padded to DH columns and beyond `valid_rows`) into
// an LDS tile with row stride ld.  VEC = 8 or 4 elements per load.
template <int DH, int VEC>
__device__ __forceinline__ void stage_rows(unsigned short* tile, int ld, const unsigned short* src, long row_stride,
                                           int nrows, int valid_rows, int dh, int tid) {
  constexpr int CPR = DH / VEC;
  for (int c = tid; c < nrows * CPR; c += 256) {
    const int r = c / CPR, d = (c % CPR) * VEC;
    if constexpr (VEC == 8) {
      uint4 v = make_uint4(0, 0, 0, 0);
      if (r < valid_rows && d < dh) v = *(const uint4*)(src + (long)r * row_stride + d);
      *(uint4*)(tile + r * ld + d) = v;
    } else {
      uint2 v = make_uint2(0, 0);
      if (r < valid_rows && d < dh) v = *(const uint2*)(src + (long)r * row_stride + d);
      *(uint2*)(tile + r * ld + d) = v;
    }
  }
}

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

// ----------------------------------------------------------------------------------------
// forward: block = 4 waves x 32 queries, key tiles of KT keys
// ----------------------------------------------------------------------------------------
template <int DH, int VEC>
__global__ __launch_bounds__(256) void mfma_attn_fwd_kernel(AttnArgs a) {
  constexpr int KT = DH > 128 ? 32 : 64;
  constexpr int LDK = DH + 8, LDV = ld_tr(DH);
  constexpr int NKD = DH / 16;   // k steps of Q K^T
  constexpr int NDB = DH / 32;   // 32-wide d blocks of the output
  __shared__ __attribute__((aligned(16))) unsigned short Ks[KT * LDK];
  __shared__ __attribute__((aligned(16))) unsigned short Vs[KT * LDV];

  const int b = blockIdx.z, h = blockIdx.y;
  const int qt = a.causal ? (gridDim.x - 1 - blockIdx.x) : blockIdx.x;   // heavy tiles first
  const int q0 = qt * 128;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 31, g = lane >> 5;
  const int T = a.T, dh = a.dh;
  const long rs = (long)a.H * dh;
  const long base = ((long)b * T) * rs + (long)h * dh;
  const unsigned short* Q = (const unsigned short*)a.Q + base;
  const unsigned short* K = (const unsigned short*)a.K + base;
  const unsigned short* V = (const unsigned short*)a.V + base;

  const int q = q0 + wave * 32 + r;             // this lane's query
  const int wq_last = q0 + wave * 32 + 31;
  bf16x8 qf[NKD];
#pragma unroll
  for (int kk = 0; kk < NKD; ++kk) qf[kk] = global_frag<VEC>(Q + (long)q * rs, kk * 16 + 8 * g, dh, q < T);

  f32x16 o[NDB];
#pragma unroll
  for (int d = 0; d < NDB; ++d)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[d][i] = 0.f;
  float m = -INFINITY, l = 0.f;
  const float sc = a.scale * 1.44269504088896340736f;   // logits in log2 units

  const int kend = a.causal ? min(T, q0 + 128) : T;
  for (int k0 = 0; k0 < kend; k0 += KT) {
    __syncthreads();
    stage_rows<DH, VEC>(Ks, LDK, K + (long)k0 * rs, rs, KT, T - k0, dh, tid);
    stage_rows<DH, VEC>(Vs, LDV, V + (long)k0 * rs, rs, KT, T - k0, dh, tid);
    __syncthreads();
    if (a.causal && k0 > wq_last) continue;      // wave-uniform: nothing visible to this wave

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
      for (int i = 0; i < 16; ++i) s[kb][i] = acc[i] * sc;
    }
    const bool need_mask = (a.causal && k0 + KT - 1 > q0 + wave * 32) || (k0 + KT > T);
    if (need_mask) {
#pragma unroll
      for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = k0 + kb * 32 + 8 * (i >> 2) + 4 * g + (i & 3);
          if (key >= T || (a.causal && key > q)) s[kb][i] = -INFINITY;
        }
    }
    float mt = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) mt = fmaxf(mt, s[kb][i]);
    mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
    const float mn = fmaxf(m, mt);
    const float alpha = exp2f(m - mn);           // m = -inf on the first tile -> 0
    m = mn;
    float ps = 0.f;
#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        s[kb][i] = exp2f(s[kb][i] - mn);
        ps += s[kb][i];
      }
    l = l * alpha + ps;
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[d][i] *= alpha;

#pragma unroll
    for (int kb = 0; kb < KT / 32; ++kb)
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        const bf16x8 pb = pack8(&s[kb][8 * st]);
        const int kb0 = kb * 32 + 16 * st + 4 * g;
#pragma unroll
        for (int d = 0; d < NDB; ++d)
          o[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(trfrag(Vs, LDV, kb0, kb0 + 8, d * 32, lane), pb, o[d], 0, 0, 0);
      }
  }

  l += __shfl_xor(l, 32, 64);
  if (q < T) {
    const float inv = 1.f / l;
    unsigned short* O = (unsigned short*)a.O + base + (long)q * rs;
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const int dd = d * 32 + 8 * i4 + 4 * g;
        if (dd < dh) {
          uint2 w;
          w.x = (unsigned)f32_to_bf16(o[d][4 * i4] * inv) | ((unsigned)f32_to_bf16(o[d][4 * i4 + 1] * inv) << 16);
          w.y = (unsigned)f32_to_bf16(o[d][4 * i4 + 2] * inv) | ((unsigned)f32_to_bf16(o[d][4 * i4 + 3] * inv) << 16);
          *(uint2*)(O + dd) = w;
        }
      }
    if (g == 0) a.lse[((long)b * a.H + h) * T + q] = (m + log2f(l)) * 0.69314718055994530942f;
  }
}

static int attn_vec(int H, int dh) {
  if (dh % 8 == 0) return 8;
  if (dh % 4 == 0) return 4;
  (void)H;
  return 0;
}

bool mfma_attn_supported(int T, int dh) { return T >= 1 && dh >= 4 && dh <= 256 && attn_vec(1, dh) != 0; }

template <int DH>
static void launch_fwd_dh(const AttnArgs& a, hipStream_t s) {
  dim3 g((a.T + 127) / 128, a.H, a.B);
  if (attn_vec(a.H, a.dh) == 8)
    mfma_attn_fwd_kernel<DH, 8><<<g, 256, 0, s>>>(a);
  else
    mfma_attn_fwd_kernel<DH, 4><<<g, 256, 0, s>>>(a);
}

void launch_mfma_attn_fwd(const AttnArgs& a, hipStream_t s) {
  const int dh = a.dh;
  if (dh <= 32)
    launch_fwd_dh<32>(a, s);
  else if (dh <= 64)
    launch_fwd_dh<64>(a, s);
  else if (dh <= 96)
    launch_fwd_dh<96>(a, s);
  else if (dh <= 128)
    launch_fwd_dh<128>(a, s);
  else if (dh <= 192)
    launch_fwd_dh<192>(a, s);
  else
    launch_fwd_dh<256>(a, s);
}

void launch_mfma_attn_bwd(const AttnBwdArgs& a, hipStream_t s) { launch_simt_attn_bwd(a, 1, s); }

}  // namespace sh
