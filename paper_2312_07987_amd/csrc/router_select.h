// Device code of the exact router's selection, shared by the logits GEMM (which runs it as its
// epilogue) and routing.hip.  See the comment on the two-stage router in routing.hip for the bound.
#pragma once
#include "common.h"

namespace sh {

// Second stage of the exact router for one (side, head, token) entry, run by one wave: recomputes the
// head's E logits in fp64 and redoes the selection.  Lane l sums the products of input features
// 16 l .. 16 l + 15 (per 1024-feature slab) against the head's column vectors, the lanes' sums are added
// by a butterfly, lane 0 adds the bias and selects.  zs: 64 doubles of LDS owned by the wave.
//
// The blocked sum is not the canonical one (one accumulator, i = 0 .. d_model-1 ascending, bias last), but
// both are fp64 sums of the same exact products, so each lies within d_model * 2^-53 * sum|x_i w_i| of the
// true value and the two differ by at most twice that.  `reorder` is an upper bound of that difference
// (Cauchy-Schwarz on sum|x_i w_i|, with slack); any two logits of the head that the blocked sum puts
// further apart than `reorder` are ordered the same way by the canonical sum.  If some pair is closer
// (every exact tie is), lane 0 evaluates the canonical sum itself and selects from that, so the indices
// are those of the canonical logits in every case.
__device__ __forceinline__ void recheck_entry(const unsigned short* __restrict__ xrow, const unsigned short* __restrict__ wt0,
                                              const float* __restrict__ bh, double* __restrict__ zs, double* __restrict__ zout,
                                              int* __restrict__ idx_out, float* __restrict__ gate_out, int dm, int dmp, int E,
                                              int k, int lane, double reorder) {
  // eight experts at a time: the token's features are loaded once per slab and the eight columns'
  // loads are in flight together (one expert after the other pays one memory round trip each)
  for (int e0 = 0; e0 < E; e0 += 8) {
    double acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = 0.0;
    for (int s0 = 0; s0 < dmp; s0 += 1024) {
      const int i0 = s0 + lane * 16;
      uint2 xv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        xv[q] = make_uint2(0, 0);
        if (i0 + 4 * q < dm) xv[q] = *(const uint2*)(xrow + i0 + 4 * q);   // dm % 4 == 0: 8-byte aligned rows
      }
      uint4 wv[8][2];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int e = e0 + u < E ? e0 + u : E - 1;   // past the last expert: a repeat, never stored
        wv[u][0] = *(const uint4*)(wt0 + (long)e * dmp + i0);
        wv[u][1] = *(const uint4*)(wt0 + (long)e * dmp + i0 + 8);
      }
      const unsigned xw[8] = {xv[0].x, xv[0].y, xv[1].x, xv[1].y, xv[2].x, xv[2].y, xv[3].x, xv[3].y};
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const unsigned ww[8] = {wv[u][0].x, wv[u][0].y, wv[u][0].z, wv[u][0].w, wv[u][1].x, wv[u][1].y, wv[u][1].z, wv[u][1].w};
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          acc[u] = fma((double)__uint_as_float(xw[q] << 16), (double)__uint_as_float(ww[q] << 16), acc[u]);
          acc[u] = fma((double)__uint_as_float(xw[q] & 0xffff0000u), (double)__uint_as_float(ww[q] & 0xffff0000u), acc[u]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      double v = acc[u];
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      if (lane == 0 && e0 + u < E) zs[e0 + u] = v + (bh ? (double)bh[e0 + u] : 0.0);
    }
  }
  if (lane == 0) {
    bool close = false;
    for (int e = 1; e < E; ++e)
      for (int f = 0; f < e; ++f) close = close || !(fabs(zs[e] - zs[f]) > reorder);
    if (close) {
      for (int e = 0; e < E; ++e) {
        const unsigned short* w = wt0 + (long)e * dmp;
        double acc = 0.0;
        for (int i = 0; i < dm; ++i)
          acc = fma((double)__uint_as_float((unsigned)xrow[i] << 16), (double)__uint_as_float((unsigned)w[i] << 16), acc);
        zs[e] = acc + (bh ? (double)bh[e] : 0.0);
      }
    }
    for (int e = 0; e < E; ++e) zout[e] = zs[e];
    unsigned long long sel = 0ull;
    for (int j = 0; j < k; ++j) {
      int best = -1;
      double bv = 0.0;
      for (int e = 0; e < E; ++e) {
        if ((sel >> e) & 1ull) continue;
        const double v = zs[e];
        if (best < 0 || v > bv) {
          best = e;
          bv = v;
        }
      }
      sel |= 1ull << best;
      idx_out[j] = best;
      gate_out[j] = (float)(1.0 / (1.0 + exp(-bv)));
    }
  }
}

// First-stage selection of the (token, head) items of one tile of tokens, then the fp64 recheck of the
// items whose margins do not clear the error bound (a fraction of a percent, and every exact tie), one
// wave per item.  Called by all 256 threads of a work-group.
//   zt    LDS, [rows][HEp]: the tile's stage-1 logits of one side (fp64 sums of fp32 K-step sums)
//   rs    LDS, [rows]: the sum of squares of each token's input features
//   ids   LDS, [rows]: token index of each row, -1 past the end
//   zs, flist, nflag: LDS scratch (4 x 64 doubles, 256 ints, 1 int; nflag = 0 on entry)
__device__ __forceinline__ void router_select_tile(const RouterSelect& r, int side, const double* zt, int HEp, const float* rs,
                                                   const int* ids, int rows, double (*zs)[64], int* flist, int* nflag) {
  const int H = r.H, E = r.E, k = r.k, N = r.N;
  const float* b = r.b[side];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int item0 = 0; item0 < rows * H; item0 += 256) {
    const int item = item0 + threadIdx.x;
    const int nl = item / H, h = item % H;
    const int n = item < rows * H ? ids[nl] : -1;
    if (n >= 0) {
      const int sh_ = side * H + h;
      const double* z = zt + nl * HEp + h * E;
      float w2 = 0.f;   // largest squared column norm of this head's router
      for (int e = 0; e < E; ++e) w2 = fmaxf(w2, r.wnorm2[(long)sh_ * E + e]);
      const double bound0 = 4.0 * (double)r.kstep * 5.9604645e-8 * (double)(sqrtf(rs[nl]) * 1.0001f) * (double)(sqrtf(w2) * 1.0001f);
      unsigned long long sel = 0ull;
      const long o = ((long)sh_ * N + n) * k;
      double prev = 0.0, bprev = 0.0;
      bool flag = false;
      const int passes = k < E ? k + 1 : k;
      for (int j = 0; j < passes; ++j) {
        int best = -1;
        double bv = 0.0;
        for (int e = 0; e < E; ++e) {
          if ((sel >> e) & 1ull) continue;
          double v = z[e] + (b ? (double)b[h * E + e] : 0.0);
          if (best < 0 || v > bv) {
            best = e;
            bv = v;
          }
        }
        const double bb = bound0 + 1e-13 * (fabs(bv) + 1.0);
        if (j > 0 && !(prev - bv > bprev + bb)) flag = true;
        prev = bv;
        bprev = bb;
        sel |= 1ull << best;
        if (j < k) {
          r.idx[o + j] = best;
          r.gate[o + j] = (float)(1.0 / (1.0 + exp(-bv)));
        }
      }
      if (flag) flist[atomicAdd(nflag, 1)] = item;
    }
    __syncthreads();
    // the recheck overwrites what the first stage wrote for its items (same work-group, after the barrier)
    const int HE = H * E;
    const int nf = *nflag;
    for (int f = wave; f < nf; f += 4) {
      const int it = flist[f];
      const int fl = it / H, h = it % H, n = ids[fl];
      const int sh_ = side * H + h;
      const long o = ((long)sh_ * N + n) * k;
      float w2 = 0.f;
      for (int e = 0; e < E; ++e) w2 = fmaxf(w2, r.wnorm2[(long)sh_ * E + e]);
      // twice d_model * 2^-53 * |x| * max|w|, doubled again for the rounding of the norms themselves
      const double reorder = 4.0 * (double)r.dm * 1.1102230246251565e-16 * (double)sqrtf(rs[fl]) * (double)sqrtf(w2);
      recheck_entry((const unsigned short*)r.x + (long)n * r.dm, r.Wt + ((long)side * HE + h * E) * r.dmp, b ? b + h * E : nullptr,
                    zs[wave], r.Z + ((long)side * N + n) * HE + (long)h * E, r.idx + o, r.gate + o, r.dm, r.dmp, E, k, lane, reorder);
    }
    __syncthreads();
    if (threadIdx.x == 0) *nflag = 0;
    __syncthreads();
  }
}

}  // namespace sh
