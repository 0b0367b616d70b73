// Small memory-bound kernels around the GEMMs: fills, casts, the gate-weighted sum over a
// token's k expert slots (the weighted average of Sec. 2.2's V^h equation and its mirror
// image in the backward pass) and the router's backward step.
#include "common.h"

namespace sh {

__global__ void fill_f32_kernel(float* p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

template <typename T>
__global__ void cast_from_f32_kernel(const float* __restrict__ src, T* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) st(dst, (long)i, src[i]);
}

template <typename T>
__global__ void cast_to_f32_kernel(const T* __restrict__ src, float* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = ld(src, (long)i);
}

static unsigned grid_for(size_t n, int block) {
  size_t g = (n + block - 1) / block;
  return (unsigned)(g < 1 ? 1 : (g > 65536 ? 65536 : g));
}

__global__ void zero4_f32_kernel(float* p0, size_t n0, float* p1, size_t n1, float* p2, size_t n2, float* p3, size_t n3) {
  float* p = blockIdx.y == 0 ? p0 : blockIdx.y == 1 ? p1 : blockIdx.y == 2 ? p2 : p3;
  const size_t n = blockIdx.y == 0 ? n0 : blockIdx.y == 1 ? n1 : blockIdx.y == 2 ? n2 : n3;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0.f;
}

// clears up to four arrays (NULL / 0 entries are skipped) with one launch
void launch_zero4_f32(float* p0, size_t n0, float* p1, size_t n1, float* p2, size_t n2, float* p3, size_t n3, hipStream_t s) {
  size_t mx = n0 > n1 ? n0 : n1;
  mx = mx > n2 ? mx : n2;
  mx = mx > n3 ? mx : n3;
  if (!mx) return;
  dim3 g(grid_for(mx, 256), 4);
  zero4_f32_kernel<<<g, 256, 0, s>>>(p0, n0, p1, n1, p2, n2, p3, n3);
}

void launch_fill_f32(float* p, size_t n, float v, hipStream_t s) {
  if (n) fill_f32_kernel<<<grid_for(n, 256), 256, 0, s>>>(p, n, v);
}

void launch_cast_from_f32(const float* src, void* dst, size_t n, int bf16, hipStream_t s) {
  if (!n) return;
  if (bf16)
    cast_from_f32_kernel<bf16_t><<<grid_for(n, 256), 256, 0, s>>>(src, (bf16_t*)dst, n);
  else
    cast_from_f32_kernel<float><<<grid_for(n, 256), 256, 0, s>>>(src, (float*)dst, n);
}

void launch_cast_to_f32(const void* src, float* dst, size_t n, int bf16, hipStream_t s) {
  if (!n) return;
  if (bf16)
    cast_to_f32_kernel<bf16_t><<<grid_for(n, 256), 256, 0, s>>>((const bf16_t*)src, dst, n);
  else
    cast_to_f32_kernel<float><<<grid_for(n, 256), 256, 0, s>>>((const float*)src, dst, n);
}

// out[i] = sum_h part[h][i] (+ add32[i]); part and out are bf16, 8 elements per thread.
__global__ __launch_bounds__(256) void sum_heads_kernel(const unsigned short* __restrict__ part, const float* __restrict__ add32,
                                                        unsigned short* __restrict__ out, size_t n8, size_t hstride, int H) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n8) return;
  float acc[8];
  if (add32) {
    const float4 a0 = *(const float4*)(add32 + i * 8), a1 = *(const float4*)(add32 + i * 8 + 4);
    acc[0] = a0.x; acc[1] = a0.y; acc[2] = a0.z; acc[3] = a0.w;
    acc[4] = a1.x; acc[5] = a1.y; acc[6] = a1.z; acc[7] = a1.w;
  } else {
#pragma unroll
    for (int t = 0; t < 8; ++t) acc[t] = 0.f;
  }
  for (int h = 0; h < H; ++h) {
    const uint4 v = *(const uint4*)(part + (size_t)h * hstride + i * 8);
    const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      acc[2 * t] += __uint_as_float(w[t] << 16);
      acc[2 * t + 1] += __uint_as_float(w[t] & 0xffff0000u);
    }
  }
  uint4 o;
  o.x = pack_bf16x2(acc[0], acc[1]);
  o.y = pack_bf16x2(acc[2], acc[3]);
  o.z = pack_bf16x2(acc[4], acc[5]);
  o.w = pack_bf16x2(acc[6], acc[7]);
  *(uint4*)(out + i * 8) = o;
}

void launch_sum_heads(const void* part, const float* add32, void* out, size_t n, size_t hstride, int H, hipStream_t s) {
  const size_t n8 = n / 8;
  if (n8) sum_heads_kernel<<<(unsigned)((n8 + 255) / 256), 256, 0, s>>>((const unsigned short*)part, add32, (unsigned short*)out, n8, hstride, H);
}

// ---- rotary position embedding of queries and keys (App. A.4 "RoPE Positional Encodings" of the paper; method of Su et al.) ----
// tab[t][i] = (cos, sin) of t * 10000^(-2i/d), d = 2*half: evaluated in fp64, stored in fp32
__global__ __launch_bounds__(256) void rope_table_kernel(float2* __restrict__ tab, int T, int half) {
  const long id = (long)blockIdx.x * 256 + threadIdx.x;
  if (id >= (long)T * half) return;
  const int t = (int)(id / half), i = (int)(id % half);
  const double theta = pow(10000.0, -2.0 * (double)i / (double)(2 * half));
  double sn, cs;
  sincos((double)t * theta, &sn, &cs);
  tab[id] = make_float2((float)cs, (float)sn);
}

// In place on up to two [N, H, dh] tensors: the pair (2i, 2i+1) of the row of token n (position n % T)
// turns by +angle (sign = 1) or -angle (sign = -1, the transpose: what a gradient takes).
template <typename TT>
__global__ __launch_bounds__(256) void rope_apply_kernel(TT* __restrict__ P0, TT* __restrict__ P1, const float2* __restrict__ tab,
                                                         long rows, int T, int pos0, int H, int dh, int half, float sign) {
  const long id = (long)blockIdx.x * 256 + threadIdx.x;
  if (id >= rows * half) return;
  TT* P = blockIdx.y ? P1 : P0;
  const long row = id / half;
  const int i = (int)(id % half);
  const int t = pos0 + (int)((row / H) % T);
  const float2 cs = tab[(long)t * half + i];
  const float c = cs.x, sn = sign * cs.y;
  const long o = row * dh + 2 * i;
  const float a = ld(P, o), b = ld(P, o + 1);
  st(P, o, a * c - b * sn);
  st(P, o + 1, a * sn + b * c);
}

// bf16 rows with dh % 8 == 0: 16 bytes (four pairs) per thread
__global__ __launch_bounds__(256) void rope_apply_vec_kernel(unsigned short* __restrict__ P0, unsigned short* __restrict__ P1,
                                                             const float2* __restrict__ tab, long rows, int T, int pos0, int H,
                                                             int dh, float sign) {
  const int per_row = dh / 8;
  const long id = (long)blockIdx.x * 256 + threadIdx.x;
  if (id >= rows * per_row) return;
  unsigned short* P = blockIdx.y ? P1 : P0;
  const long row = id / per_row;
  const int q = (int)(id % per_row);
  const int t = pos0 + (int)((row / H) % T);
  const float4* tp = (const float4*)(tab + (long)t * (dh / 2) + q * 4);
  const float4 t0 = tp[0], t1 = tp[1];
  const float c[4] = {t0.x, t0.z, t1.x, t1.z};
  const float sn[4] = {sign * t0.y, sign * t0.w, sign * t1.y, sign * t1.w};
  uint4* ptr = (uint4*)(P + row * dh + q * 8);
  const uint4 v = *ptr;
  const unsigned w[4] = {v.x, v.y, v.z, v.w};
  unsigned o[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    const float a = __uint_as_float(w[u] << 16), b = __uint_as_float(w[u] & 0xffff0000u);
    o[u] = pack_bf16x2(a * c[u] - b * sn[u], a * sn[u] + b * c[u]);
  }
  *ptr = make_uint4(o[0], o[1], o[2], o[3]);
}

// T [dm][ld] (fp32) holds x^T dz for both routers side by side (side s in columns s*HEp .. s*HEp+HE-1):
// the two router weight gradients are its column blocks.
__global__ __launch_bounds__(256) void router_wgrad_split_kernel(const float* __restrict__ T, float* __restrict__ dW0,
                                                                 float* __restrict__ dW1, int dm, int ld, int HE, int HEp,
                                                                 const float* __restrict__ dbpart, int nblk, int E,
                                                                 float* __restrict__ db0, float* __restrict__ db1) {
  const long id = (long)blockIdx.x * 256 + threadIdx.x;
  if (dbpart && id < 2L * HE * 64) {
    // bias gradients, one wave per column: column c of side s = head c / E, expert c % E; every lane adds
    // the block sums b = lane, lane + 64, ... in that order, a butterfly adds the lanes (a fixed order)
    const int col = (int)(id >> 6), lane = (int)(id & 63);
    const int side = col / HE, c = col % HE;
    float* db = side ? db1 : db0;
    if (db) {   // wave-uniform
      const float* p = dbpart + ((long)(side * (HE / E) + c / E) * nblk) * E + c % E;
      float s = 0.f;
      for (int b = lane; b < nblk; b += 64) s += p[(long)b * E];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
      if (lane == 0) db[c] = s;
    }
  }
  if (id >= (long)dm * HE) return;
  const long i = id / HE;
  const int c = (int)(id % HE);
  if (dW0) dW0[id] = T[i * ld + c];
  if (dW1) dW1[id] = T[i * ld + HEp + c];
}

void launch_router_wgrad_split(const float* T, float* dW0, float* dW1, int dm, int ld, int HE, int HEp, const float* dbpart,
                               int nblk, int E, float* db0, float* db1, hipStream_t s) {
  long n = (long)dm * HE;
  if (dbpart && n < 128L * HE) n = 128L * HE;   // one wave per bias-gradient column
  if (n) router_wgrad_split_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(T, dW0, dW1, dm, ld, HE, HEp, dbpart, nblk, E, db0, db1);
}

void launch_rope_table(float2* tab, int T, int dh, hipStream_t s) {
  const int half = dh / 2;
  const long n = (long)T * half;
  if (n) rope_table_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(tab, T, half);
}

void launch_rope_apply(void* P0, void* P1, const float2* tab, long N, int T, int pos0, int H, int dh, int inverse, int bf16,
                       hipStream_t s) {
  const int half = dh / 2;
  const long rows = N * H;
  if (!half || !rows) return;
  const float sign = inverse ? -1.f : 1.f;
  const unsigned ny = P1 ? 2 : 1;
  if (bf16 && dh % 8 == 0) {
    dim3 g((unsigned)((rows * (dh / 8) + 255) / 256), ny);
    rope_apply_vec_kernel<<<g, 256, 0, s>>>((unsigned short*)P0, (unsigned short*)P1, tab, rows, T, pos0, H, dh, sign);
    return;
  }
  dim3 g((unsigned)((rows * half + 255) / 256), ny);
  if (bf16)
    rope_apply_kernel<bf16_t><<<g, 256, 0, s>>>((bf16_t*)P0, (bf16_t*)P1, tab, rows, T, pos0, H, dh, half, sign);
  else
    rope_apply_kernel<float><<<g, 256, 0, s>>>((float*)P0, (float*)P1, tab, rows, T, pos0, H, dh, half, sign);
}

// out[(n / Tq) * T + (T - Tq) + n % Tq][:] += add[n][:] for the B*Tq rows of `add` (fp32): the rows of
// the last Tq positions of every sequence take one more term.  One thread per element.
template <typename TT>
__global__ __launch_bounds__(256) void add_query_rows_kernel(TT* __restrict__ out, const float* __restrict__ add, long rows, int T,
                                                             int Tq, int dm) {
  const long id = (long)blockIdx.x * 256 + threadIdx.x;
  if (id >= rows * dm) return;
  const long n = id / dm;
  const int c = (int)(id % dm);
  const long o = ((n / Tq) * T + (T - Tq) + n % Tq) * dm + c;
  st(out, o, ld(out, o) + add[id]);
}

void launch_add_query_rows(void* out, const float* add, long rows, int T, int Tq, int dm, int bf16, hipStream_t s) {
  const long n = rows * dm;
  if (!n) return;
  const unsigned g = (unsigned)((n + 255) / 256);
  if (bf16)
    add_query_rows_kernel<bf16_t><<<g, 256, 0, s>>>((bf16_t*)out, add, rows, T, Tq, dm);
  else
    add_query_rows_kernel<float><<<g, 256, 0, s>>>((float*)out, add, rows, T, Tq, dm);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wave per (token, head); lane handles elements lane, lane+64, ... of the d_head row.
template <typename T>
__global__ __launch_bounds__(256) void slot_combine_kernel(SlotArgs a) {
  const int lane = threadIdx.x & 63;
  const long pair = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (pair >= (long)a.N * a.H) return;
  const int n = (int)(pair / a.H), h = (int)(pair % a.H);
  const int dh = a.dh, k = a.k;
  const T* other = (const T*)a.other;
  T* out = (T*)a.out;
  float acc[4] = {0.f, 0.f, 0.f, 0.f}, oth[4] = {0.f, 0.f, 0.f, 0.f};
  const long row = ((long)n * a.H + h) * dh;
  if (other) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int d = lane + 64 * i;
      if (d < dh) oth[i] = ld(other, row + d);
    }
  }
  for (int j = 0; j < k; ++j) {
    const long aid = (long)h * a.N * k + (long)n * k + j;
    const T* sl = (const T*)a.slots + aid * dh;
    const float g = a.gate[aid];
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int d = lane + 64 * i;
      if (d < dh) {
        float v = ld(sl, d);
        acc[i] += g * v;
        dot += oth[i] * v;
      }
    }
    if (a.dots) {
      dot = wave_sum(dot);
      if (lane == 0) a.dots[aid] = a.dots_add ? a.dots[aid] + dot : dot;
    }
  }
  if (out) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int d = lane + 64 * i;
      if (d < dh) st(out, row + d, acc[i]);
    }
  }
  if (a.delta) {
    // the row sum uses the values as stored (rounded to the storage type): the attention backward
    // multiplies those, and its dS = P (dP - delta) cancels exactly only if both see the same numbers
    float dd = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float v = acc[i];
      if (out && sizeof(T) == 2) v = bf16_to_f32(f32_to_bf16(v));
      dd += v * oth[i];
    }
    dd = wave_sum(dd);
    if (lane == 0) a.delta[pair] = dd;
  }
}

// VW (8 or 4) consecutive bf16 -> floats
template <int VW>
__device__ __forceinline__ void load_bf16_vec(const unsigned short* p, float* f) {
  unsigned w[VW / 2];
  if constexpr (VW == 8) {
    const uint4 v = *(const uint4*)p;
    w[0] = v.x, w[1] = v.y, w[2] = v.z, w[3] = v.w;
  } else {
    const uint2 v = *(const uint2*)p;
    w[0] = v.x, w[1] = v.y;
  }
#pragma unroll
  for (int t = 0; t < VW / 2; ++t) {
    f[2 * t] = __uint_as_float(w[t] << 16);
    f[2 * t + 1] = __uint_as_float(w[t] & 0xffff0000u);
  }
}

// bf16 rows whose length is a multiple of VW (8 or 4): 16 or 8 bytes per thread, dh/VW threads per
// (token, head) row rounded up to a power of two <= 64 (a row never straddles a wave), shuffles inside
// that lane group.
template <int TPR, int VW>
__global__ __launch_bounds__(256) void slot_combine_vec_kernel(SlotArgs a) {
  const int lane_in = threadIdx.x % TPR;
  const long pair = ((long)blockIdx.x * 256 + threadIdx.x) / TPR;
  const bool valid = pair < (long)a.N * a.H;
  const int n = valid ? (int)(pair / a.H) : 0, h = valid ? (int)(pair % a.H) : 0;
  const int dh = a.dh, k = a.k, d0 = lane_in * VW;
  const bool act = valid && d0 < dh;
  const unsigned short* other = (const unsigned short*)a.other;
  const long row = ((long)n * a.H + h) * dh + d0;
  float oth[VW], acc[VW];
#pragma unroll
  for (int t = 0; t < VW; ++t) oth[t] = acc[t] = 0.f;
  if (other && act) load_bf16_vec<VW>(other + row, oth);
  for (int j = 0; j < k; ++j) {
    const long aid = (long)h * a.N * k + (long)n * k + j;
    float dot = 0.f;
    if (act) {
      const float g = a.gate[aid];
      float v[VW];
      load_bf16_vec<VW>((const unsigned short*)a.slots + aid * dh + d0, v);
#pragma unroll
      for (int t = 0; t < VW; ++t) {
        acc[t] += g * v[t];
        dot += oth[t] * v[t];
      }
    }
    if (a.dots) {
#pragma unroll
      for (int o = TPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, 64);
      if (valid && lane_in == 0) a.dots[aid] = a.dots_add ? a.dots[aid] + dot : dot;
    }
  }
  if (a.out && act) {
    unsigned o[VW / 2];
#pragma unroll
    for (int t = 0; t < VW / 2; ++t) o[t] = pack_bf16x2(acc[2 * t], acc[2 * t + 1]);
    if constexpr (VW == 8)
      *(uint4*)((unsigned short*)a.out + row) = make_uint4(o[0], o[1], o[2], o[3]);
    else
      *(uint2*)((unsigned short*)a.out + row) = make_uint2(o[0], o[1]);
  }
  if (a.delta) {
    // from the values as stored (rounded to bf16): the attention backward multiplies those, and its
    // dS = P (dP - delta) cancels exactly only if both see the same numbers
    float dd = 0.f;
#pragma unroll
    for (int t = 0; t < VW; ++t) dd += (a.out ? bf16_to_f32(f32_to_bf16(acc[t])) : acc[t]) * oth[t];
#pragma unroll
    for (int o = TPR / 2; o > 0; o >>= 1) dd += __shfl_xor(dd, o, 64);
    if (valid && lane_in == 0) a.delta[pair] = dd;
  }
}

template <int VW>
static void launch_slot_combine_vec(const SlotArgs& a, hipStream_t s) {
  const long pairs = (long)a.N * a.H;
  int tpr = 1;
  while (tpr * VW < a.dh) tpr *= 2;   // threads per row, power of two
  const unsigned g = (unsigned)((pairs * tpr + 255) / 256);
  switch (tpr) {
    case 1: slot_combine_vec_kernel<1, VW><<<g, 256, 0, s>>>(a); return;
    case 2: slot_combine_vec_kernel<2, VW><<<g, 256, 0, s>>>(a); return;
    case 4: slot_combine_vec_kernel<4, VW><<<g, 256, 0, s>>>(a); return;
    case 8: slot_combine_vec_kernel<8, VW><<<g, 256, 0, s>>>(a); return;
    case 16: slot_combine_vec_kernel<16, VW><<<g, 256, 0, s>>>(a); return;
    case 32: slot_combine_vec_kernel<32, VW><<<g, 256, 0, s>>>(a); return;
    default: slot_combine_vec_kernel<64, VW><<<g, 256, 0, s>>>(a); return;
  }
}

void launch_slot_combine(const SlotArgs& a, int bf16, hipStream_t s) {
  long pairs = (long)a.N * a.H;
  if (bf16 && a.dh % 8 == 0) return launch_slot_combine_vec<8>(a, s);
  if (bf16 && a.dh % 4 == 0) return launch_slot_combine_vec<4>(a, s);   // rows are 8-byte aligned
  unsigned g = (unsigned)((pairs + 3) / 4);
  if (bf16)
    slot_combine_kernel<bf16_t><<<g, 256, 0, s>>>(a);
  else
    slot_combine_kernel<float><<<g, 256, 0, s>>>(a);
}

// One thread per (token, side, head): writes the E logit-gradient entries it owns.
template <typename T>
__global__ __launch_bounds__(256) void router_bwd_kernel(RouterBwdArgs a) {
  __shared__ float wsum[4][64];   // per wave and expert: the sum of the wave's logit gradients
  const int sh_ = blockIdx.y;  // side*H + h over the sides that own a router
  const int side = sh_ / a.H, h = sh_ % a.H;
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int E = a.E, k = a.k, HE = a.H * a.E;
  if (sizeof(T) == 2 && a.wide_out) {
    const long tot = (long)a.dm * a.wide_width, nthr = (long)gridDim.x * gridDim.y * 256;
    for (long i = ((long)blockIdx.y * gridDim.x + blockIdx.x) * 256 + threadIdx.x; i < tot; i += nthr) {
      const int c = (int)(i % a.wide_width);
      const long row = i / a.wide_width;
      const int ws = c / a.side_stride, cc = c % a.side_stride;
      unsigned short v = 0;
      if (ws < a.sides && cc < HE) v = ((const unsigned short*)a.W[ws])[row * HE + cc];
      ((unsigned short*)a.wide_out)[i] = v;
    }
  }
  int es[8];     // this token's experts and their logit gradients
  float vs[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    es[j] = -1;
    vs[j] = 0.f;
  }
  if (n < a.N) {
    T* dz = (T*)a.dz;
    const long base = (long)n * a.ld + (long)side * a.side_stride + (long)h * E;
    for (int e = 0; e < E; ++e) st(dz, base + e, 0.f);
    if (h == a.H - 1) {   // padding columns of this side, and after the last side
      for (int c = HE; c < a.side_stride; ++c) st(dz, (long)n * a.ld + (long)side * a.side_stride + c, 0.f);
      if (side == a.sides - 1) {
        int c = a.sides * a.side_stride;
        if (sizeof(T) == 2 && a.side_stride % 8 == 0 && a.ld % 8 == 0)   // 16-byte pieces of zeros
          for (; c + 8 <= a.pad_to; c += 8) *(uint4*)((unsigned short*)a.dz + (long)n * a.ld + c) = make_uint4(0, 0, 0, 0);
        for (; c < a.pad_to; ++c) st(dz, (long)n * a.ld + c, 0.f);
      }
    }
    const long o = ((long)sh_ * a.N + n) * k;  // side-major layout [side][H][N][k]
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < k) {
        int e = a.idx[o + j];
        float g = a.gate[o + j];
        float dg = a.dgate[o + j];
        if (a.shared) dg += a.dgate[(long)a.H * a.N * k + o + j];
        float v = dg * g * (1.f - g);
        st(dz, base + e, v);
        es[j] = e;
        vs[j] = v;
      }
  }
  // bias gradient of this block: per expert a butterfly over the lanes, then the waves in order (no
  // atomics inside the block: the sum has one fixed order)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int e = 0; e < E; ++e) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < 8; ++j) v += es[j] == e ? vs[j] : 0.f;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if (lane == 0) wsum[wave][e] = v;
  }
  __syncthreads();
  if (threadIdx.x < E) {
    const float bs = ((wsum[0][threadIdx.x] + wsum[1][threadIdx.x]) + wsum[2][threadIdx.x]) + wsum[3][threadIdx.x];
    if (a.dbpart)
      a.dbpart[((long)sh_ * gridDim.x + blockIdx.x) * E + threadIdx.x] = bs;
    else if (a.db[side])
      atomicAdd(&a.db[side][h * E + threadIdx.x], bs);
  }
}

int router_bwd_blocks(int N) { return (N + 255) / 256; }

void launch_router_bwd(const RouterBwdArgs& a, int bf16, hipStream_t s) {
  dim3 g((a.N + 255) / 256, a.sides * a.H);
  if (bf16)
    router_bwd_kernel<bf16_t><<<g, 256, 0, s>>>(a);
  else
    router_bwd_kernel<float><<<g, 256, 0, s>>>(a);
}

}  // namespace sh
