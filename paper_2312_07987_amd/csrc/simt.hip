// Plain fp32 kernels for every step of the layer (no matrix cores).  They serve the fp32
// storage type and any shape the MFMA kernels do not take, and they are the on-device
// cross-check of the MFMA family.  Storage type T is float or bf16; arithmetic is fp32.
//
//   row GEMM   value / output expert projections of Sec. 2.2 (V^h and y equations), the
//              dense Q, K projections of Sec. 2.1, and their data gradients
//   wgrad      weight gradients (reduction over the tokens routed to an expert)
//   attention  A^h = softmax(Q K^T / sqrt(d_head)), A^h V^h (Sec. 2.1), one wave per query
//              row with a running maximum, and the matching backward kernels
#include "common.h"

namespace sh {

// ----------------------------------------------------------------------------------------
// row GEMM, 64x64 tile, 16x16 threads, 4x4 outputs per thread
// ----------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void simt_row_gemm_kernel(RowGemmArgs a) {
  __shared__ int ids[64];
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const int h = blockIdx.z;
  int e = 0, row0, rows;
  if (a.perm) {
    if (!find_tile(a.offsets + (long)h * (a.E + 1), a.E, 64, blockIdx.x, e, row0, rows)) return;
  } else {
    row0 = blockIdx.x * 64;
    if (row0 >= a.M) return;
    rows = a.M - row0 < 64 ? a.M - row0 : 64;
  }
  const int tid = threadIdx.x;
  if (tid < 64) ids[tid] = tid < rows ? (a.perm ? a.perm[(long)h * a.M + row0 + tid] : row0 + tid) : -1;
  __syncthreads();

  const T* A = (const T*)a.A;
  const T* B = (const T*)a.B + (long)h * a.b_hstride + (long)e * a.b_estride;
  const int n0 = blockIdx.y * 64;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int k0 = 0; k0 < a.K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int t = tid + i * 256;
      int r = t >> 4, kk = t & 15;
      int id = ids[r];
      float v = 0.f;
      if (id >= 0 && k0 + kk < a.K) v = ld(A, (long)(id / a.a_div) * a.lda + (long)h * a.a_hoff + k0 + kk);
      As[kk][r] = v;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int t = tid + i * 256;
      int kk, n;
      if (a.sbk == 1) {
        kk = t & 15;
        n = t >> 4;
      } else {
        kk = t >> 6;
        n = t & 63;
      }
      float v = 0.f;
      if (k0 + kk < a.K && n0 + n < a.Nc) v = ld(B, (long)(k0 + kk) * a.sbk + (long)(n0 + n) * a.sbn);
      Bs[kk][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int id = ids[ty * 4 + i];
    if (id < 0) continue;
    float sc = a.gate ? a.gate[(long)h * a.gate_hstride + id] : 1.f;
    long crow = (long)(id / a.c_div) * a.ldc + (long)h * a.c_hoff;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= a.Nc) continue;
      float v = acc[i][j] * sc;
      if (a.mode == STORE_T)
        st((T*)a.C, crow + n, v);
      else if (a.mode == STORE_F32)
        ((float*)a.C)[crow + n] = v;
      else
        atomicAdd((float*)a.C + crow + n, v);
    }
  }
}

void launch_simt_row_gemm(const RowGemmArgs& a, int bf16, hipStream_t s) {
  if (a.M <= 0 || a.Nc <= 0) return;
  dim3 g((a.M + 63) / 64 + (a.perm ? a.E : 0), (a.Nc + 63) / 64, a.heads);
  if (bf16)
    simt_row_gemm_kernel<bf16_t><<<g, 256, 0, s>>>(a);
  else
    simt_row_gemm_kernel<float><<<g, 256, 0, s>>>(a);
}

// ----------------------------------------------------------------------------------------
// wgrad, 64x64 output tile, reduction over `chunk` rows per block, fp32 atomic add
// ----------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void simt_wgrad_kernel(WgradArgs a) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  __shared__ int ids[16];
  __shared__ float gs[16];
  const int h = blockIdx.z;
  int e = 0, row0, rows;
  if (a.perm) {
    if (!find_tile(a.offsets + (long)h * (a.E + 1), a.E, a.chunk, blockIdx.y, e, row0, rows)) return;
  } else {
    row0 = blockIdx.y * a.chunk;
    if (row0 >= a.M) return;
    rows = a.M - row0 < a.chunk ? a.M - row0 : a.chunk;
  }
  const int tj = (a.Kb + 63) / 64;
  const int i0 = (blockIdx.x / tj) * 64, j0 = (blockIdx.x % tj) * 64;
  const T* A = (const T*)a.A;
  const T* Bm = (const T*)a.Bm;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int r0 = 0; r0 < rows; r0 += 16) {
    if (tid < 16) {
      int id = -1;
      float g = 0.f;
      if (r0 + tid < rows) {
        id = a.perm ? a.perm[(long)h * a.M + row0 + r0 + tid] : row0 + r0 + tid;
        g = a.gate ? a.gate[(long)h * a.gate_hstride + id] : 1.f;
      }
      ids[tid] = id;
      gs[tid] = g;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int t = tid + i * 256;
      int r = t >> 6, c = t & 63;
      int id = ids[r];
      float va = 0.f, vb = 0.f;
      if (id >= 0) {
        if (i0 + c < a.Ka) va = (a.scale_b ? 1.f : gs[r]) * ld(A, (long)(id / a.a_div) * a.lda + (long)h * a.a_hoff + i0 + c);
        if (j0 + c < a.Kb) vb = (a.scale_b ? gs[r] : 1.f) * ld(Bm, (long)(id / a.b_div) * a.ldb + (long)h * a.b_hoff + j0 + c);
      }
      As[r][c] = va;
      Bs[r][c] = vb;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float av[4], bv[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) av[i] = As[r][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) bv[j] = Bs[r][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
  float* dW = a.dW + (long)h * a.w_hstride + (long)e * a.w_estride;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int ii = i0 + ty * 4 + i;
    if (ii >= a.Ka) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int jj = j0 + tx * 4 + j;
      if (jj < (a.kb_store ? a.kb_store : a.Kb)) atomicAdd(dW + (long)ii * a.swa + jj, acc[i][j]);
    }
  }
}

void launch_simt_wgrad(const WgradArgs& a, int bf16, hipStream_t s) {
  if (a.M <= 0) return;
  int ti = (a.Ka + 63) / 64, tj = (a.Kb + 63) / 64;
  dim3 g(ti * tj, (a.M + a.chunk - 1) / a.chunk + (a.perm ? a.E : 0), a.heads);
  if (bf16)
    simt_wgrad_kernel<bf16_t><<<g, 256, 0, s>>>(a);
  else
    simt_wgrad_kernel<float><<<g, 256, 0, s>>>(a);
}

// ----------------------------------------------------------------------------------------
// attention: one wave per query (forward, dQ) or per key (dK, dV).  A tile of KT rows of
// the other side is staged in LDS; lane = part*KT + row, the d_head sum of a row is split
// over `parts` = 64/KT lanes and combined with xor shuffles.
// ----------------------------------------------------------------------------------------
static constexpr int QPW = 4;          // rows handled by one wave
static constexpr int RPB = 4 * QPW;    // rows handled by one block (4 waves)

__device__ __forceinline__ float wsum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wmax(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float part_sum(float v, int KT) {
  for (int o = KT; o < 64; o <<= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// dynamic LDS layout (floats): t0[KT][dh+1], t1[KT][dh+1], rowv[4][dh] (per-wave row), ps[4][64], aux
template <typename T>
__global__ __launch_bounds__(256) void simt_attn_fwd_kernel(AttnArgs a, int KT) {
  extern __shared__ float lds[];
  const int dh = a.dh, ldt = dh + 1;
  float* Ks = lds;
  float* Vs = Ks + KT * ldt;
  float* qs = Vs + KT * ldt;  // [4][dh]
  float* ps = qs + 4 * dh;    // [4][64]
  const int b = blockIdx.z, h = blockIdx.y;
  const int q0 = blockIdx.x * RPB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int parts = 64 / KT, key_l = lane % KT, part = lane / KT;
  const long rs = (long)a.H * dh;  // row stride
  const int Tq = a.Tq > 0 ? a.Tq : a.T, off = a.T - Tq;   // query i sits at key position off + i
  const T* Q = (const T*)a.Q + ((long)b * Tq) * rs + (long)h * dh;
  const T* K = (const T*)a.K + ((long)b * a.T) * rs + (long)h * dh;
  const T* V = (const T*)a.V + ((long)b * a.T) * rs + (long)h * dh;
  T* O = (T*)a.O + ((long)b * Tq) * rs + (long)h * dh;

  float m[QPW], l[QPW], acc[QPW][4];
#pragma unroll
  for (int i = 0; i < QPW; ++i) {
    m[i] = -INFINITY;
    l[i] = 0.f;
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[i][c] = 0.f;
  }
  const int qlast = min(q0 + RPB, Tq) - 1;
  const int kend = a.causal ? qlast + off + 1 : a.T;

  for (int k0 = 0; k0 < kend; k0 += KT) {
    __syncthreads();
    for (int t = tid; t < KT * dh; t += 256) {
      int r = t / dh, d = t % dh;
      bool ok = k0 + r < a.T;
      Ks[r * ldt + d] = ok ? ld(K, (long)(k0 + r) * rs + d) : 0.f;
      Vs[r * ldt + d] = ok ? ld(V, (long)(k0 + r) * rs + d) : 0.f;
    }
#pragma unroll
    for (int i = 0; i < QPW; ++i) {
      const int q = q0 + wave * QPW + i;  // block-uniform control flow below
      __syncthreads();
      for (int d = lane; d < dh; d += 64) qs[wave * dh + d] = q < Tq ? ld(Q, (long)q * rs + d) : 0.f;
      __syncthreads();
      float s = 0.f;
      for (int d = part; d < dh; d += parts) s = fmaf(qs[wave * dh + d], Ks[key_l * ldt + d], s);
      s = part_sum(s, KT) * a.scale;
      const int key = k0 + key_l;
      const bool vis = key < a.T && q < Tq && (!a.causal || key <= q + off);
      float sm = vis ? s : -INFINITY;
      float mn = fmaxf(m[i], wmax(sm));
      float p = (vis && mn > -INFINITY) ? __expf(sm - mn) : 0.f;
      float alpha = (m[i] > -INFINITY) ? __expf(m[i] - mn) : 0.f;
      l[i] = l[i] * alpha + wsum(part == 0 ? p : 0.f);
      m[i] = mn;
      if (part == 0) ps[wave * 64 + key_l] = p;
      __syncthreads();
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int d = lane + 64 * c;
        if (d < dh) {
          float v = acc[i][c] * alpha;
          for (int r = 0; r < KT; ++r) v = fmaf(ps[wave * 64 + r], Vs[r * ldt + d], v);
          acc[i][c] = v;
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < QPW; ++i) {
    const int q = q0 + wave * QPW + i;
    if (q >= Tq) continue;
    float inv = 1.f / l[i];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int d = lane + 64 * c;
      if (d < dh) st(O, (long)q * rs + d, acc[i][c] * inv);
    }
    if (lane == 0) a.lse[((long)b * a.H + h) * Tq + q] = m[i] + logf(l[i]);
  }
}

// dQ: one wave per query; stages K and V tiles.
template <typename T>
__global__ __launch_bounds__(256) void simt_attn_dq_kernel(AttnBwdArgs a, int KT) {
  extern __shared__ float lds[];
  const int dh = a.dh, ldt = dh + 1;
  float* Ks = lds;
  float* Vs = Ks + KT * ldt;
  float* qs = Vs + KT * ldt;   // [4][dh]  query row
  float* gs = qs + 4 * dh;     // [4][dh]  dO row
  float* ps = gs + 4 * dh;     // [4][64]
  const int b = blockIdx.z, h = blockIdx.y;
  const int q0 = blockIdx.x * RPB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int parts = 64 / KT, key_l = lane % KT, part = lane / KT;
  const long rs = (long)a.H * dh;
  const int Tq = a.Tq > 0 ? a.Tq : a.T, off = a.T - Tq;
  const long base = ((long)b * a.T) * rs + (long)h * dh;
  const long qbase = ((long)b * Tq) * rs + (long)h * dh;
  const T* Q = (const T*)a.Q + qbase;
  const T* K = (const T*)a.K + base;
  const T* V = (const T*)a.V + base;
  const T* dO = (const T*)a.dO + qbase;
  T* dQ = (T*)a.dQ + qbase;

  float acc[QPW][4];
#pragma unroll
  for (int i = 0; i < QPW; ++i)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[i][c] = 0.f;
  const int qlast = min(q0 + RPB, Tq) - 1;
  const int kend = a.causal ? qlast + off + 1 : a.T;

  for (int k0 = 0; k0 < kend; k0 += KT) {
    __syncthreads();
    for (int t = tid; t < KT * dh; t += 256) {
      int r = t / dh, d = t % dh;
      bool ok = k0 + r < a.T;
      Ks[r * ldt + d] = ok ? ld(K, (long)(k0 + r) * rs + d) : 0.f;
      Vs[r * ldt + d] = ok ? ld(V, (long)(k0 + r) * rs + d) : 0.f;
    }
#pragma unroll
    for (int i = 0; i < QPW; ++i) {
      const int q = q0 + wave * QPW + i;
      const bool qok = q < Tq;
      __syncthreads();
      for (int d = lane; d < dh; d += 64) {
        qs[wave * dh + d] = qok ? ld(Q, (long)q * rs + d) : 0.f;
        gs[wave * dh + d] = qok ? ld(dO, (long)q * rs + d) : 0.f;
      }
      __syncthreads();
      float s = 0.f, dp = 0.f;
      for (int d = part; d < dh; d += parts) {
        s = fmaf(qs[wave * dh + d], Ks[key_l * ldt + d], s);
        dp = fmaf(gs[wave * dh + d], Vs[key_l * ldt + d], dp);
      }
      s = part_sum(s, KT) * a.scale;
      dp = part_sum(dp, KT);
      const int key = k0 + key_l;
      const bool vis = key < a.T && qok && (!a.causal || key <= q + off);
      float ds = 0.f;
      if (vis) {
        float lse = a.lse[((long)b * a.H + h) * Tq + q];
        float dl = a.delta[((long)b * Tq + q) * a.H + h];
        ds = __expf(s - lse) * (dp - dl) * a.scale;
      }
      if (part == 0) ps[wave * 64 + key_l] = ds;
      __syncthreads();
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int d = lane + 64 * c;
        if (d < dh) {
          float v = acc[i][c];
          for (int r = 0; r < KT; ++r) v = fmaf(ps[wave * 64 + r], Ks[r * ldt + d], v);
          acc[i][c] = v;
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < QPW; ++i) {
    const int q = q0 + wave * QPW + i;
    if (q >= Tq) continue;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int d = lane + 64 * c;
      if (d < dh) st(dQ, (long)q * rs + d, acc[i][c]);
    }
  }
}

// dK, dV: one wave per key; stages Q and dO tiles (KT queries).
template <typename T>
__global__ __launch_bounds__(256) void simt_attn_dkv_kernel(AttnBwdArgs a, int KT) {
  extern __shared__ float lds[];
  const int dh = a.dh, ldt = dh + 1;
  float* Qs = lds;
  float* Gs = Qs + KT * ldt;
  float* ks = Gs + KT * ldt;   // [4][dh] key row
  float* vs = ks + 4 * dh;     // [4][dh] value row
  float* ps = vs + 4 * dh;     // [4][64] p
  float* ds_ = ps + 4 * 64;    // [4][64] ds
  float* ls = ds_ + 4 * 64;    // [KT] lse
  float* dl = ls + 64;         // [KT] delta
  const int b = blockIdx.z, h = blockIdx.y;
  const int u0 = blockIdx.x * RPB;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int parts = 64 / KT, q_l = lane % KT, part = lane / KT;
  const long rs = (long)a.H * dh;
  const int Tq = a.Tq > 0 ? a.Tq : a.T, off = a.T - Tq;
  const long base = ((long)b * a.T) * rs + (long)h * dh;
  const long qbase = ((long)b * Tq) * rs + (long)h * dh;
  const T* Q = (const T*)a.Q + qbase;
  const T* K = (const T*)a.K + base;
  const T* V = (const T*)a.V + base;
  const T* dO = (const T*)a.dO + qbase;
  T* dK = (T*)a.dK + base;
  T* dV = (T*)a.dV + base;

  float ak[QPW][4], av[QPW][4];
#pragma unroll
  for (int i = 0; i < QPW; ++i)
#pragma unroll
    for (int c = 0; c < 4; ++c) ak[i][c] = av[i][c] = 0.f;
  const int qbeg = a.causal ? (max(u0 - off, 0) / KT) * KT : 0;

  for (int qt = qbeg; qt < Tq; qt += KT) {
    __syncthreads();
    for (int t = tid; t < KT * dh; t += 256) {
      int r = t / dh, d = t % dh;
      bool ok = qt + r < Tq;
      Qs[r * ldt + d] = ok ? ld(Q, (long)(qt + r) * rs + d) : 0.f;
      Gs[r * ldt + d] = ok ? ld(dO, (long)(qt + r) * rs + d) : 0.f;
    }
    if (tid < KT) {
      bool ok = qt + tid < Tq;
      ls[tid] = ok ? a.lse[((long)b * a.H + h) * Tq + qt + tid] : 0.f;
      dl[tid] = ok ? a.delta[((long)b * Tq + qt + tid) * a.H + h] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < QPW; ++i) {
      const int u = u0 + wave * QPW + i;
      const bool uok = u < a.T;
      __syncthreads();
      for (int d = lane; d < dh; d += 64) {
        ks[wave * dh + d] = uok ? ld(K, (long)u * rs + d) : 0.f;
        vs[wave * dh + d] = uok ? ld(V, (long)u * rs + d) : 0.f;
      }
      __syncthreads();
      float s = 0.f, dp = 0.f;
      for (int d = part; d < dh; d += parts) {
        s = fmaf(Qs[q_l * ldt + d], ks[wave * dh + d], s);
        dp = fmaf(Gs[q_l * ldt + d], vs[wave * dh + d], dp);
      }
      s = part_sum(s, KT) * a.scale;
      dp = part_sum(dp, KT);
      const int q = qt + q_l;
      const bool vis = q < Tq && uok && (!a.causal || u <= q + off);
      float p = 0.f, ds = 0.f;
      if (vis) {
        p = __expf(s - ls[q_l]);
        ds = p * (dp - dl[q_l]) * a.scale;
      }
      if (part == 0) {
        ps[wave * 64 + q_l] = p;
        ds_[wave * 64 + q_l] = ds;
      }
      __syncthreads();
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        int d = lane + 64 * c;
        if (d < dh) {
          float v1 = av[i][c], v2 = ak[i][c];
          for (int r = 0; r < KT; ++r) {
            v1 = fmaf(ps[wave * 64 + r], Gs[r * ldt + d], v1);
            v2 = fmaf(ds_[wave * 64 + r], Qs[r * ldt + d], v2);
          }
          av[i][c] = v1;
          ak[i][c] = v2;
        }
      }
    }
  }
#pragma unroll
  for (int i = 0; i < QPW; ++i) {
    const int u = u0 + wave * QPW + i;
    if (u >= a.T) continue;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      int d = lane + 64 * c;
      if (d < dh) {
        st(dK, (long)u * rs + d, ak[i][c]);
        st(dV, (long)u * rs + d, av[i][c]);
      }
    }
  }
}

static int attn_kt(int dh) { return dh > 128 ? 16 : 32; }

void launch_simt_attn_fwd(const AttnArgs& a, int bf16, hipStream_t s) {
  const int KT = attn_kt(a.dh);
  size_t lds = sizeof(float) * ((size_t)2 * KT * (a.dh + 1) + 4 * a.dh + 4 * 64);
  dim3 g(((a.Tq > 0 ? a.Tq : a.T) + RPB - 1) / RPB, a.H, a.B);
  if (bf16)
    simt_attn_fwd_kernel<bf16_t><<<g, 256, lds, s>>>(a, KT);
  else
    simt_attn_fwd_kernel<float><<<g, 256, lds, s>>>(a, KT);
}

void launch_simt_attn_bwd(const AttnBwdArgs& a, int bf16, hipStream_t s) {
  const int KT = attn_kt(a.dh);
  dim3 g((a.T + RPB - 1) / RPB, a.H, a.B);                             // keys
  dim3 gq(((a.Tq > 0 ? a.Tq : a.T) + RPB - 1) / RPB, a.H, a.B);       // queries
  size_t lds_q = sizeof(float) * ((size_t)2 * KT * (a.dh + 1) + 8 * a.dh + 4 * 64);
  size_t lds_kv = sizeof(float) * ((size_t)2 * KT * (a.dh + 1) + 8 * a.dh + 8 * 64 + 128);
  if (bf16) {
    simt_attn_dq_kernel<bf16_t><<<gq, 256, lds_q, s>>>(a, KT);
    simt_attn_dkv_kernel<bf16_t><<<g, 256, lds_kv, s>>>(a, KT);
  } else {
    simt_attn_dq_kernel<float><<<gq, 256, lds_q, s>>>(a, KT);
    simt_attn_dkv_kernel<float><<<g, 256, lds_kv, s>>>(a, KT);
  }
}

}  // namespace sh
