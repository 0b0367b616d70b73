// Router of the SwitchHead layer (arXiv 2312.07987, Sec. 2.2: s = sigmoid(x W), argtopk)
// and the expert-sorted permutation of the token->expert assignments (the "sorting and
// top-k steps" of Sec. 3.5).
//
//   router_logits  z = x W (+ b) in fp64, summed over i = 0..d_model-1 in that order with
//                  one accumulator per logit, so the selection is a fixed function of the
//                  stored inputs (products of bf16/fp32 inputs are exact in fp64)
//   topk_hist      per (side, head, token): k passes of "largest remaining logit, lowest
//                  index on ties"; gate = sigmoid(logit); per-block expert histogram from
//                  wave ballots
//   scan           exclusive scan over (expert major, token block minor)
//   scatter        stable placement: rank inside the block from ballots + popcounts, so
//                  no atomics decide an order and the result is deterministic
#include "common.h"

namespace sh {

static constexpr int RT_TOK = 64;    // tokens per block of the logits kernel
static constexpr int RT_COL = 64;    // logit columns per block
static constexpr int RT_KC = 32;     // d_model chunk staged in LDS
static constexpr int RB = 256;       // tokens per block of topk/scatter kernels

int router_blocks(int N) { return (N + RB - 1) / RB; }

template <typename T>
__global__ __launch_bounds__(256) void router_logits_kernel(const T* __restrict__ x, const T* __restrict__ W0,
                                                            const T* __restrict__ W1, const float* __restrict__ b0,
                                                            const float* __restrict__ b1, double* __restrict__ Z,
                                                            int N, int dm, int HE) {
  __shared__ double xs[RT_TOK][RT_KC + 1];
  __shared__ double ws[RT_KC][RT_COL];
  const int side = blockIdx.y;
  const T* W = side ? W1 : W0;
  const float* b = side ? b1 : b0;
  const int tok0 = blockIdx.x * RT_TOK;
  const int col0 = blockIdx.z * RT_COL;
  const int tid = threadIdx.x;
  const int tok = tid % RT_TOK;
  const int cg = tid / RT_TOK;  // 0..3 -> 16 columns each

  double acc[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) acc[c] = 0.0;

  for (int k0 = 0; k0 < dm; k0 += RT_KC) {
    for (int t = tid; t < RT_TOK * RT_KC; t += 256) {
      int r = t / RT_KC, i = t % RT_KC;
      int n = tok0 + r, kk = k0 + i;
      xs[r][i] = (n < N && kk < dm) ? (double)ld(x, (long)n * dm + kk) : 0.0;
    }
    for (int t = tid; t < RT_KC * RT_COL; t += 256) {
      int i = t / RT_COL, c = t % RT_COL;
      int kk = k0 + i, col = col0 + c;
      ws[i][c] = (kk < dm && col < HE) ? (double)ld(W, (long)kk * HE + col) : 0.0;
    }
    __syncthreads();
    // strictly ascending i; the zero padding beyond d_model adds exact zeros
#pragma unroll 4
    for (int i = 0; i < RT_KC; ++i) {
      double xv = xs[tok][i];
#pragma unroll
      for (int c = 0; c < 16; ++c) acc[c] = fma(xv, ws[i][cg * 16 + c], acc[c]);
    }
    __syncthreads();
  }
  int n = tok0 + tok;
  if (n < N) {
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      int col = col0 + cg * 16 + c;
      if (col < HE) {
        double z = acc[c];
        if (b) z += (double)b[col];
        Z[((long)side * N + n) * HE + col] = z;
      }
    }
  }
}

__global__ __launch_bounds__(RB) void topk_hist_kernel(const double* __restrict__ Z, int* __restrict__ idx,
                                                       float* __restrict__ gate, int* __restrict__ blockcnt, int N,
                                                       int H, int E, int k, int nblk) {
  __shared__ int cnt[64];
  const int sh_ = blockIdx.y;  // side*H + h
  const int side = sh_ / H, h = sh_ % H;
  const int n = blockIdx.x * RB + threadIdx.x;
  const bool valid = n < N;
  if (threadIdx.x < 64) cnt[threadIdx.x] = 0;
  __syncthreads();

  unsigned long long sel = 0ull;
  if (valid) {
    const double* z = Z + ((long)side * N + n) * (long)(H * E) + (long)h * E;
    long o = ((long)sh_ * N + n) * k;
    for (int j = 0; j < k; ++j) {
      int best = -1;
      double bv = 0.0;
      for (int e = 0; e < E; ++e) {
        if ((sel >> e) & 1ull) continue;
        double v = z[e];
        if (best < 0 || v > bv) {  // strict: the lower index keeps a tie
          best = e;
          bv = v;
        }
      }
      sel |= 1ull << best;
      idx[o + j] = best;
      gate[o + j] = (float)(1.0 / (1.0 + exp(-bv)));
    }
  }
  const int lane = threadIdx.x & 63;
  for (int e = 0; e < E; ++e) {
    unsigned long long bal = __ballot(valid && ((sel >> e) & 1ull));
    if (lane == 0 && bal) atomicAdd(&cnt[e], __popcll(bal));
  }
  __syncthreads();
  if (threadIdx.x < E) blockcnt[((long)sh_ * nblk + blockIdx.x) * E + threadIdx.x] = cnt[threadIdx.x];
}

// One block per (side, head).  blockcnt[sh][blk][e] (counts) -> in place: first position of
// expert e for token block blk; offsets[sh][0..E].
__global__ __launch_bounds__(128) void scan_kernel(int* __restrict__ blockcnt, int* __restrict__ offsets, int E,
                                                  int nblk) {
  __shared__ int tot[129];
  const int sh_ = blockIdx.x;
  const int e = threadIdx.x;
  int* c = blockcnt + (long)sh_ * nblk * E;
  int sum = 0;
  if (e < E)
    for (int b = 0; b < nblk; ++b) sum += c[(long)b * E + e];
  tot[e] = e < E ? sum : 0;
  __syncthreads();
  if (e == 0) {
    int run = 0;
    for (int i = 0; i < E; ++i) {
      int t = tot[i];
      tot[i] = run;
      run += t;
    }
    tot[E] = run;
    for (int i = 0; i <= E; ++i) offsets[(long)sh_ * (E + 1) + i] = tot[i];
  }
  __syncthreads();
  if (e < E) {
    int run = tot[e];
    for (int b = 0; b < nblk; ++b) {
      int t = c[(long)b * E + e];
      c[(long)b * E + e] = run;
      run += t;
    }
  }
}

__global__ __launch_bounds__(RB) void scatter_kernel(const int* __restrict__ idx, const int* __restrict__ base,
                                                     int* __restrict__ perm, int N, int E, int k, int nblk) {
  __shared__ int wcnt[RB / 64][64];
  const int sh_ = blockIdx.y;
  const int n = blockIdx.x * RB + threadIdx.x;
  const bool valid = n < N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  int ej[8], rk[8];
  unsigned long long sel = 0ull;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    ej[j] = -1;
    rk[j] = 0;
    if (valid && j < k) {
      ej[j] = idx[((long)sh_ * N + n) * k + j];
      sel |= 1ull << ej[j];
    }
  }
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int e = 0; e < E; ++e) {
    unsigned long long bal = __ballot(valid && ((sel >> e) & 1ull));
    int r = __popcll(bal & lt);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (ej[j] == e) rk[j] = r;
    if (lane == 0) wcnt[wave][e] = __popcll(bal);
  }
  __syncthreads();
  if (!valid) return;
  const int* bs = base + ((long)sh_ * nblk + blockIdx.x) * E;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (j < k) {
      int e = ej[j];
      int pos = bs[e] + rk[j];
      for (int w = 0; w < wave; ++w) pos += wcnt[w][e];
      perm[(long)sh_ * N * k + pos] = n * k + j;
    }
  }
}

__global__ void dense_routing_kernel(int* idx, float* gate, int* perm, int* offsets, int N, int H) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long tot = (long)H * N;
  if (i < tot) {
    idx[i] = 0;
    gate[i] = 1.0f;
    perm[i] = (int)(i % N);
  }
  if (i < H) {
    offsets[2 * i] = 0;
    offsets[2 * i + 1] = N;
  }
}

void launch_router(const RouterArgs& a, hipStream_t s) {
  const int HE = a.H * a.E;
  dim3 g((a.N + RT_TOK - 1) / RT_TOK, a.sides, (HE + RT_COL - 1) / RT_COL);
  if (a.bf16)
    router_logits_kernel<bf16_t><<<g, 256, 0, s>>>((const bf16_t*)a.x, (const bf16_t*)a.W[0], (const bf16_t*)a.W[1],
                                                   a.b[0], a.b[1], a.Z, a.N, a.dm, HE);
  else
    router_logits_kernel<float><<<g, 256, 0, s>>>((const float*)a.x, (const float*)a.W[0], (const float*)a.W[1],
                                                  a.b[0], a.b[1], a.Z, a.N, a.dm, HE);
  const int nblk = router_blocks(a.N);
  dim3 g2(nblk, a.sides * a.H);
  topk_hist_kernel<<<g2, RB, 0, s>>>(a.Z, a.idx, a.gate, a.blockcnt, a.N, a.H, a.E, a.k, nblk);
  scan_kernel<<<a.sides * a.H, 128, 0, s>>>(a.blockcnt, a.offsets, a.E, nblk);
  scatter_kernel<<<g2, RB, 0, s>>>(a.idx, a.blockcnt, a.perm, a.N, a.E, a.k, nblk);
}

// ----------------------------------------------------------------------------------------
// Expert-SET sorting.  A token's k experts of one head form one of C(E,k) sets; tokens that
// share a set share all k weight matrices, so the k gate-weighted products of Sec. 2.2's
// output equation can be summed inside one matrix-core accumulator.  Set id = rank of the
// ascending combination (combinatorial number system), tokens are counting-sorted by it.
// ----------------------------------------------------------------------------------------
__device__ __forceinline__ int binom(int n, int r) {
  if (r < 0 || r > n) return 0;
  long v = 1;
  for (int i = 1; i <= r; ++i) v = v * (n - r + i) / i;
  return (int)v;
}

__global__ __launch_bounds__(RB) void set_hist_kernel(const int* __restrict__ idx, const float* __restrict__ gate,
                                                      int* __restrict__ setid, float* __restrict__ gset,
                                                      int* __restrict__ blockcnt, int N, int k, int nsets, int nblk) {
  __shared__ int cnt[128];
  const int sh_ = blockIdx.y;
  const int n = blockIdx.x * RB + threadIdx.x;
  const bool valid = n < N;
  if (threadIdx.x < 128) cnt[threadIdx.x] = 0;
  __syncthreads();
  int sid = -1;
  if (valid) {
    int e[8];
    float g[8];
    const long o = ((long)sh_ * N + n) * k;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      e[j] = j < k ? idx[o + j] : 0x7fffffff;
      g[j] = j < k ? gate[o + j] : 0.f;
    }
    // ascending experts (k <= 8: odd-even transposition sort with static indexing)
#pragma unroll
    for (int pass = 0; pass < 8; ++pass)
#pragma unroll
      for (int j = pass & 1; j + 1 < 8; j += 2)
        if (e[j] > e[j + 1]) {
          int te = e[j];
          e[j] = e[j + 1];
          e[j + 1] = te;
          float tg = g[j];
          g[j] = g[j + 1];
          g[j + 1] = tg;
        }
    sid = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < k) {
        sid += binom(e[j], j + 1);
        gset[o + j] = g[j];
      }
    setid[(long)sh_ * N + n] = sid;
  }
  const int lane = threadIdx.x & 63;
  for (int s = 0; s < nsets; ++s) {
    unsigned long long bal = __ballot(sid == s);
    if (lane == 0 && bal) atomicAdd(&cnt[s], __popcll(bal));
  }
  __syncthreads();
  if (threadIdx.x < nsets) blockcnt[((long)sh_ * nblk + blockIdx.x) * nsets + threadIdx.x] = cnt[threadIdx.x];
}

__global__ __launch_bounds__(RB) void set_scatter_kernel(const int* __restrict__ setid, const int* __restrict__ base,
                                                         int* __restrict__ setperm, int N, int nsets, int nblk) {
  __shared__ int wcnt[RB / 64][128];
  const int sh_ = blockIdx.y;
  const int n = blockIdx.x * RB + threadIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sid = n < N ? setid[(long)sh_ * N + n] : -1;
  const unsigned long long lt = (1ull << lane) - 1ull;
  int rk = 0;
  for (int s = 0; s < nsets; ++s) {
    unsigned long long bal = __ballot(sid == s);
    if (sid == s) rk = __popcll(bal & lt);
    if (lane == 0) wcnt[wave][s] = __popcll(bal);
  }
  __syncthreads();
  if (sid < 0) return;
  int pos = base[((long)sh_ * nblk + blockIdx.x) * nsets + sid] + rk;
  for (int w = 0; w < wave; ++w) pos += wcnt[w][sid];
  setperm[(long)sh_ * N + pos] = n;
}

void launch_set_sort(const SetSortArgs& a, hipStream_t s) {
  const int nblk = router_blocks(a.N);
  dim3 g(nblk, a.sides * a.H);
  set_hist_kernel<<<g, RB, 0, s>>>(a.idx, a.gate, a.setid, a.gset, a.blockcnt, a.N, a.k, a.nsets, nblk);
  scan_kernel<<<a.sides * a.H, 128, 0, s>>>(a.blockcnt, a.setoff, a.nsets, nblk);
  set_scatter_kernel<<<g, RB, 0, s>>>(a.setid, a.blockcnt, a.setperm, a.N, a.nsets, nblk);
}

void launch_dense_routing(int* idx, float* gate, int* perm, int* offsets, int N, int H, hipStream_t s) {
  long tot = (long)H * N;
  dense_routing_kernel<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>(idx, gate, perm, offsets, N, H);
}

}  // namespace sh
