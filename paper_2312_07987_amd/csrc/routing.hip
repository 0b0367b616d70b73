// Router of the SwitchHead layer (arXiv 2312.07987, Sec. 2.2: s = sigmoid(x W), argtopk)
// and the expert-sorted permutation of the token->expert assignments (the "sorting and
// top-k steps" of Sec. 3.6 "Shared Selection").
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
// bin e for token block blk; offsets[sh][0..E].  One wave per bin, lanes over token blocks.
__device__ __forceinline__ void scan_body(int* __restrict__ blockcnt, int* __restrict__ offsets, int E, int nblk) {
  __shared__ int tot[129];
  const int sh_ = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int* c = blockcnt + (long)sh_ * nblk * E;
  for (int e = wave; e < E; e += 4) {
    int sum = 0;
    for (int b = lane; b < nblk; b += 64) sum += c[(long)b * E + e];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (lane == 0) tot[e] = sum;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < E; ++i) {
      int t = tot[i];
      tot[i] = run;
      run += t;
    }
    tot[E] = run;
  }
  __syncthreads();
  for (int i = threadIdx.x; i <= E; i += 256) offsets[(long)sh_ * (E + 1) + i] = tot[i];
  for (int e = wave; e < E; e += 4) {
    int run = tot[e];
    for (int b0 = 0; b0 < nblk; b0 += 64) {
      const int b = b0 + lane;
      const int v = b < nblk ? c[(long)b * E + e] : 0;
      int inc = v;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        int u = __shfl_up(inc, o, 64);
        if (lane >= o) inc += u;
      }
      if (b < nblk) c[(long)b * E + e] = run + inc - v;
      run += __shfl(inc, 63, 64);
    }
  }
}
__global__ __launch_bounds__(256) void scan_kernel(int* __restrict__ blockcnt, int* __restrict__ offsets, int E,
                                                   int nblk) {
  scan_body(blockcnt, offsets, E, nblk);
}
// the expert table (blockIdx.y == 0) and the set table (blockIdx.y == 1) in one launch
__global__ __launch_bounds__(256) void scan2_kernel(int* __restrict__ blockcnt, int* __restrict__ offsets, int E,
                                                    int* __restrict__ setcnt, int* __restrict__ setoff, int nsets,
                                                    int nblk) {
  if (blockIdx.y == 0)
    scan_body(blockcnt, offsets, E, nblk);
  else
    scan_body(setcnt, setoff, nsets, nblk);
}

// What scan_body would leave for this token block, computed by the block itself from the raw counts
// cnt[sh][blk][bin] (for tables small enough that every block can read them whole): sbase[bin] = first
// position of bin `bin` for token block blockIdx.x; token block 0 also writes offsets[sh][0..nbins].
// One wave per bin, lanes over token blocks.  Called by all RB threads; ends with a barrier.
__device__ __forceinline__ void block_bases(const int* __restrict__ cnt, int* __restrict__ offsets, int nbins, int nblk,
                                            int* __restrict__ sbase /* LDS [2 * 128 + 1] */) {
  const int sh_ = blockIdx.y, blk = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int* c = cnt + (long)sh_ * nblk * nbins;
  int* tot = sbase + 128;
  for (int e = wave; e < nbins; e += RB / 64) {
    int all = 0, pre = 0;
    for (int b = lane; b < nblk; b += 64) {
      const int v = c[(long)b * nbins + e];
      all += v;
      pre += b < blk ? v : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      all += __shfl_xor(all, o, 64);
      pre += __shfl_xor(pre, o, 64);
    }
    if (lane == 0) {
      tot[e] = all;
      sbase[e] = pre;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < nbins; ++i) {
      const int t = tot[i];
      tot[i] = run;
      sbase[i] += run;
      run += t;
    }
    tot[nbins] = run;
  }
  __syncthreads();
  if (blk == 0)
    for (int i = threadIdx.x; i <= nbins; i += RB) offsets[(long)sh_ * (nbins + 1) + i] = tot[i];
}

// LOCAL: the block's bases are in LDS (sbase, from block_bases) instead of the scanned table `base`
template <bool LOCAL = false>
__device__ __forceinline__ void scatter_body(const int* __restrict__ idx, const int* __restrict__ base,
                                             int* __restrict__ perm, int N, int E, int k, int nblk,
                                             const int* sbase = nullptr) {
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
  if (valid) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (j < k) {
        int e = ej[j];
        int pos = rk[j];
        if constexpr (LOCAL)
          pos += sbase[e];
        else
          pos += base[((long)sh_ * nblk + blockIdx.x) * E + e];
        for (int w = 0; w < wave; ++w) pos += wcnt[w][e];
        perm[(long)sh_ * N * k + pos] = n * k + j;
      }
    }
  }
}
__global__ __launch_bounds__(RB) void scatter_kernel(const int* __restrict__ idx, const int* __restrict__ base,
                                                     int* __restrict__ perm, int N, int E, int k, int nblk) {
  scatter_body(idx, base, perm, N, E, k, nblk);
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

// ----------------------------------------------------------------------------------------
// Two-stage router for bf16 storage.  Stage 1 takes the logits from a matrix-core GEMM whose
// fp32 accumulator only ever holds the sum of one K step (KS = 64 exact bf16 x bf16 products)
// and is added to an fp64 accumulator after every step.  Their distance from the canonical
// fp64 logits is bounded by
//   bound = 4 * KS * 2^-24 * |x_n|_2 * max_c |W[:,c]|_2  (+ 1e-13 relative for the fp64 adds),
// a Cauchy-Schwarz bound on sum_i |x_i w_i| times the fp32 error of a KS-term sum, with a
// factor 4 of slack for the adder tree of the matrix core.  If every gap between consecutive sorted
// logits down to the (k+1)-th exceeds 2*bound, the ordered top-k list is provably the one
// the fp64 logits give, and it is written directly.  Otherwise stage 2 (same kernel, one wave per
// such (token, side, head)) re-evaluates its E logits in fp64 and selects from those.  Stage 2 adds
// the products in a fixed blocked order (16 per lane, then a butterfly over the lanes), which
// differs from the sequential fp64 sum by a few ulp of fp64 -- twelve orders of magnitude below
// the fp32-level gaps that send an entry here -- and gives bit-identical sums for identical
// columns, so ties still resolve to the lower index.
// ----------------------------------------------------------------------------------------
// Per (side, head, expert) work-group: the squared norm of that router column (the error bound takes
// the largest of a head's), the column copied out as a contiguous
// vector Wt[side][h*E + e][dmp] (zero padded to dmp, a multiple of 1024) for the fp64 recheck and into
// the padded matrix Wp[side][i][HEp] the logits GEMM reads (the last column also zeroes the padding).
__global__ __launch_bounds__(256) void router_prep_kernel(const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1,
                                                          float* __restrict__ wnorm2, unsigned short* __restrict__ Wt, unsigned short* __restrict__ Wp,
                                                          int dm, int dmp, int H, int E, int HEp) {
  __shared__ float red[4];
  const int HE = H * E;
  const int side = blockIdx.x / HE, col = blockIdx.x % HE;   // col = h*E + e
  const unsigned short* W = (const unsigned short*)(side ? W1 : W0);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned short* wp = Wp + (long)side * dm * HEp;
  if (col == HE - 1)
    for (int t = threadIdx.x; t < dm * (HEp - HE); t += 256) wp[(long)(t / (HEp - HE)) * HEp + HE + t % (HEp - HE)] = 0;
  float s = 0.f;
  unsigned short* wt = Wt + ((long)side * HE + col) * dmp;
  for (int i = threadIdx.x; i < dmp; i += 256) {
    unsigned short v = 0;
    if (i < dm) {
      v = W[(long)i * HE + col];
      wp[(long)i * HEp + col] = v;
    }
    wt[i] = v;
    const float f = __uint_as_float((unsigned)v << 16);
    s = fmaf(f, f, s);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if (lane == 0) red[wave] = s;
  __syncthreads();
  if (threadIdx.x == 0) wnorm2[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

__device__ __forceinline__ void hist_body(const int* __restrict__ idx, int* __restrict__ blockcnt, int N, int E, int k,
                                          int nblk) {
  __shared__ int cnt[64];
  const int sh_ = blockIdx.y;
  const int n = blockIdx.x * RB + threadIdx.x;
  if (threadIdx.x < 64) cnt[threadIdx.x] = 0;
  __syncthreads();
  unsigned long long sel = 0ull;
  if (n < N)
    for (int j = 0; j < k; ++j) sel |= 1ull << idx[((long)sh_ * N + n) * k + j];
  const int lane = threadIdx.x & 63;
  for (int e = 0; e < E; ++e) {
    unsigned long long bal = __ballot((sel >> e) & 1ull);
    if (lane == 0 && bal) atomicAdd(&cnt[e], __popcll(bal));
  }
  __syncthreads();
  if (threadIdx.x < E) blockcnt[((long)sh_ * nblk + blockIdx.x) * E + threadIdx.x] = cnt[threadIdx.x];
}
__global__ __launch_bounds__(RB) void hist_kernel(const int* __restrict__ idx, int* __restrict__ blockcnt, int N, int E,
                                                  int k, int nblk) {
  hist_body(idx, blockcnt, N, E, k, nblk);
}

// The expert histogram, and along the same pass over the top-k tables the dense gate rows of the
// gated-concatenation GEMMs: gtab[sh / H][n][(sh % H) * E + e] = the token's gate of expert e, 0 if not selected.
__device__ __forceinline__ void gate_row_body(const int* __restrict__ idx, const float* __restrict__ gate,
                                              float* __restrict__ gtab, int N, int H, int E, int k) {
  const int sh_ = blockIdx.y, n = blockIdx.x * RB + threadIdx.x;
  if (n >= N) return;
  float* out = gtab + ((long)(sh_ / H) * N + n) * (H * E) + (long)(sh_ % H) * E;
  const long o = ((long)sh_ * N + n) * k;
  for (int e = 0; e < E; ++e) {
    float g = 0.f;
    for (int j = 0; j < k; ++j) g = idx[o + j] == e ? gate[o + j] : g;
    out[e] = g;
  }
}
__global__ __launch_bounds__(RB) void hist_gate_table_kernel(const int* __restrict__ idx, const float* __restrict__ gate,
                                                             int* __restrict__ blockcnt, float* __restrict__ gtab, int N, int H,
                                                             int E, int k, int nblk) {
  hist_body(idx, blockcnt, N, E, k, nblk);
  gate_row_body(idx, gate, gtab, N, H, E, k);
}

// expert scatter whose blocks scan the (small) count table for themselves: one launch instead of scan + scatter
__global__ __launch_bounds__(RB) void scan_scatter1_kernel(const int* __restrict__ idx, const int* __restrict__ cnt,
                                                           int* __restrict__ offsets, int* __restrict__ perm, int N, int E, int k,
                                                           int nblk) {
  __shared__ int sb[2 * 128 + 1];
  block_bases(cnt, offsets, E, nblk, sb);
  scatter_body<true>(idx, nullptr, perm, N, E, k, nblk, sb);
}

// Wp[side][i][c] = W_side[i][c] for c < HE, 0 for HE <= c < HEp (rows padded to 16 bytes)
__global__ void pack_router_kernel(const bf16_t* __restrict__ W0, const bf16_t* __restrict__ W1, bf16_t* __restrict__ Wp,
                                   int dm, int HE, int HEp, int sides) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long tot = (long)sides * dm * HEp;
  if (i >= tot) return;
  int c = (int)(i % HEp);
  long r = i / HEp;
  int side = (int)(r / dm);
  long row = r % dm;
  const bf16_t* W = side ? W1 : W0;
  bf16_t v;
  v.v = 0;
  if (c < HE) v = W[row * HE + c];
  Wp[i] = v;
}

void launch_pack_router(const void* W0, const void* W1, void* Wp, int dm, int HE, int HEp, int sides, hipStream_t s) {
  const long tot = (long)sides * dm * HEp;
  pack_router_kernel<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>((const bf16_t*)W0, (const bf16_t*)W1, (bf16_t*)Wp, dm, HE, HEp, sides);
}

size_t router_hybrid_bytes(int N, int dm, int H, int E, size_t* off) {
  const size_t HEp = ((size_t)H * E + 7) / 8 * 8;
  size_t o = 0;
  auto take = [&](size_t b) {
    size_t r = o;
    o += (b + 255) & ~(size_t)255;
    return r;
  };
  off[0] = take(2 * (size_t)dm * HEp * 2);   // Wp
  off[1] = off[2] = 0;                       // (unused: the stage-1 logits and the row norms stay on the CU)
  (void)N;
  off[3] = take(2 * (size_t)H * E * 4);      // squared column norms
  off[4] = off[5] = 0;                       // (unused)
  off[6] = take(2 * (size_t)H * E * (((size_t)dm + 1023) / 1024 * 1024) * 2);   // Wt: router columns as vectors
  return o;
}

// Dense gate table for the gated-concatenation GEMMs: gtab[side][n][h*E + e] = the gate of expert e of head h
// for token n if the token selected it (Sec. 2.2: e in E^h), else 0.  One thread per (side, head, token).
__global__ __launch_bounds__(256) void gate_table_kernel(const int* __restrict__ idx, const float* __restrict__ gate,
                                                         float* __restrict__ gtab, int N, int H, int E, int k, long side_stride_in,
                                                         long side_stride_out) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  const int h = blockIdx.y, side = blockIdx.z;
  if (n >= N) return;
  float* out = gtab + side * side_stride_out + ((long)n * H + h) * E;
  for (int e = 0; e < E; ++e) out[e] = 0.f;
  const long o = side * side_stride_in + ((long)h * N + n) * k;
  for (int j = 0; j < k; ++j) out[idx[o + j]] = gate[o + j];
}

void launch_gate_table(const int* idx, const float* gate, float* gtab, int N, int H, int E, int k, int sides, long side_stride_in,
                       hipStream_t s) {
  dim3 g((N + 255) / 256, H, sides);
  gate_table_kernel<<<g, 256, 0, s>>>(idx, gate, gtab, N, H, E, k, side_stride_in, (long)N * H * E);
}

bool router_hybrid_supported(const RouterArgs& a) {
  return a.bf16 && a.dm % 4 == 0 && ((uintptr_t)a.x % 16) == 0 && a.H * a.E <= 32;
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
  scan_kernel<<<a.sides * a.H, 256, 0, s>>>(a.blockcnt, a.offsets, a.E, nblk);
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

__device__ __forceinline__ void set_hist_body(const int* __restrict__ idx, const float* __restrict__ gate,
                                              int* __restrict__ setid, float* __restrict__ gset,
                                              int* __restrict__ setexp, int* __restrict__ blockcnt, int N, int k, int E,
                                              int nsets, int nblk) {
  __shared__ int cnt[128];
  const int sh_ = blockIdx.y;
  const int n = blockIdx.x * RB + threadIdx.x;
  const bool valid = n < N;
  if (threadIdx.x < 128) cnt[threadIdx.x] = 0;
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < nsets) {
    // the table set id -> ascending experts (combinadic unranking), for the GEMMs that follow
    int rank = threadIdx.x;
    for (int p = k - 1; p >= 0; --p) {
      int x = p;
      while (x + 1 < E && binom(x + 1, p + 1) <= rank) ++x;
      rank -= binom(x, p + 1);
      setexp[threadIdx.x * 8 + p] = x;
    }
  }
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
__global__ __launch_bounds__(RB) void set_hist_kernel(const int* __restrict__ idx, const float* __restrict__ gate,
                                                      int* __restrict__ setid, float* __restrict__ gset,
                                                      int* __restrict__ setexp, int* __restrict__ blockcnt, int N, int k,
                                                      int E, int nsets, int nblk) {
  set_hist_body(idx, gate, setid, gset, setexp, blockcnt, N, k, E, nsets, nblk);
}
// both histograms of a forward pass in one launch
__global__ __launch_bounds__(RB) void hist2_kernel(const int* __restrict__ idx, const float* __restrict__ gate,
                                                   int* __restrict__ blockcnt, int* __restrict__ setid,
                                                   float* __restrict__ gset, int* __restrict__ setexp,
                                                   int* __restrict__ setcnt, int N, int k, int E, int nsets, int nblk) {
  hist_body(idx, blockcnt, N, E, k, nblk);
  set_hist_body(idx, gate, setid, gset, setexp, setcnt, N, k, E, nsets, nblk);
}

template <bool LOCAL = false>
__device__ __forceinline__ void set_scatter_body(const int* __restrict__ setid, const int* __restrict__ base,
                                                 int* __restrict__ setperm, const float* __restrict__ gset,
                                                 float* __restrict__ gsort, int N, int k, int nsets, int nblk,
                                                 const int* sbase = nullptr) {
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
  int pos = rk;
  if constexpr (LOCAL)
    pos += sbase[sid];
  else
    pos += base[((long)sh_ * nblk + blockIdx.x) * nsets + sid];
  for (int w = 0; w < wave; ++w) pos += wcnt[w][sid];
  setperm[(long)sh_ * N + pos] = n;
  for (int j = 0; j < k; ++j) gsort[((long)sh_ * N + pos) * k + j] = gset[((long)sh_ * N + n) * k + j];
}
__global__ __launch_bounds__(RB) void set_scatter_kernel(const int* __restrict__ setid, const int* __restrict__ base,
                                                         int* __restrict__ setperm, const float* __restrict__ gset,
                                                         float* __restrict__ gsort, int N, int k, int nsets, int nblk) {
  set_scatter_body(setid, base, setperm, gset, gsort, N, k, nsets, nblk);
}
// both scatters of a forward pass in one launch (the set scatter last: it may leave early)
__global__ __launch_bounds__(RB) void scatter2_kernel(const int* __restrict__ idx, const int* __restrict__ base,
                                                      int* __restrict__ perm, const int* __restrict__ setid,
                                                      const int* __restrict__ setbase, int* __restrict__ setperm,
                                                      const float* __restrict__ gset, float* __restrict__ gsort, int N, int E,
                                                      int k, int nsets, int nblk) {
  scatter_body(idx, base, perm, N, E, k, nblk);
  __syncthreads();
  set_scatter_body(setid, setbase, setperm, gset, gsort, N, k, nsets, nblk);
}
// the same with the scans done by every block for itself (small tables): `cnt` and `setcnt` hold the raw
// per-block counts, the offsets tables are written here
__global__ __launch_bounds__(RB) void scan_scatter2_kernel(const int* __restrict__ idx, const int* __restrict__ cnt,
                                                           int* __restrict__ offsets, int* __restrict__ perm,
                                                           const int* __restrict__ setid, const int* __restrict__ setcnt,
                                                           int* __restrict__ setoff, int* __restrict__ setperm,
                                                           const float* __restrict__ gset, float* __restrict__ gsort, int N,
                                                           int E, int k, int nsets, int nblk) {
  __shared__ int sb[2][2 * 128 + 1];
  block_bases(cnt, offsets, E, nblk, sb[0]);
  block_bases(setcnt, setoff, nsets, nblk, sb[1]);
  scatter_body<true>(idx, nullptr, perm, N, E, k, nblk, sb[0]);
  __syncthreads();
  set_scatter_body<true>(setid, nullptr, setperm, gset, gsort, N, k, nsets, nblk, sb[1]);
}

void launch_set_sort(const SetSortArgs& a, hipStream_t s) {
  const int nblk = router_blocks(a.N);
  dim3 g(nblk, a.sides * a.H);
  set_hist_kernel<<<g, RB, 0, s>>>(a.idx, a.gate, a.setid, a.gset, a.setexp, a.blockcnt, a.N, a.k, a.E, a.nsets, nblk);
  scan_kernel<<<a.sides * a.H, 256, 0, s>>>(a.blockcnt, a.setoff, a.nsets, nblk);
  set_scatter_kernel<<<g, RB, 0, s>>>(a.setid, a.blockcnt, a.setperm, a.gset, a.gsort, a.N, a.k, a.nsets, nblk);
}

void launch_dense_routing(int* idx, float* gate, int* perm, int* offsets, int N, int H, hipStream_t s) {
  long tot = (long)H * N;
  dense_routing_kernel<<<(unsigned)((tot + 255) / 256), 256, 0, s>>>(idx, gate, perm, offsets, N, H);
}

void launch_router_hybrid(const RouterArgs& a, char* scratch, hipStream_t s) {
  size_t off[7];
  router_hybrid_bytes(a.N, a.dm, a.H, a.E, off);
  const int HE = a.H * a.E, HEp = (HE + 7) / 8 * 8;
  bf16_t* Wp = (bf16_t*)(scratch + off[0]);
  float* wmax = (float*)(scratch + off[3]);
  unsigned short* Wt = (unsigned short*)(scratch + off[6]);
  const int dmp = (a.dm + 1023) / 1024 * 1024;

  // per (side, head): largest column norm, columns copied out as vectors and
  // into the padded matrix the GEMM reads
  router_prep_kernel<<<a.sides * a.H * a.E, 256, 0, s>>>((const bf16_t*)a.W[0], (const bf16_t*)a.W[1], wmax, Wt,
                                                   (unsigned short*)Wp, a.dm, dmp, a.H, a.E, HEp);
  // stage 1: z32 = x W on the matrix cores, fp32 accumulation, both sides in one launch; the selection
  // (and the fp64 recheck of its doubtful entries) is that kernel's epilogue
  RowGemmArgs g{};
  g.heads = a.sides;
  g.E = 1;
  g.M = a.N;
  g.a_div = 1;
  g.c_div = 1;
  g.A = a.x;
  g.lda = a.dm;
  g.B = Wp;
  g.b_hstride = (long)a.dm * HEp;
  g.sbk = HEp;
  g.sbn = 1;
  g.C = nullptr;   // nothing is stored: the selection consumes the logits inside the kernel
  g.K = a.dm;
  g.Nc = HEp;
  g.mode = STORE_F64;
  g.tag = TAG_ROUTER;
  g.rsel.b[0] = a.b[0];
  g.rsel.b[1] = a.b[1];
  g.rsel.wnorm2 = wmax;
  g.rsel.idx = a.idx;
  g.rsel.gate = a.gate;
  g.rsel.x = a.x;
  g.rsel.Wt = Wt;
  g.rsel.Z = a.Z;
  g.rsel.N = a.N;
  g.rsel.kstep = rg_kstep();
  g.rsel.H = a.H;
  g.rsel.E = a.E;
  g.rsel.k = a.k;
  g.rsel.dm = a.dm;
  g.rsel.dmp = dmp;
  launch_mfma_row_gemm(g, s);

  const int nblk = router_blocks(a.N);
  dim3 g2(nblk, a.sides * a.H);
  if (a.sets && a.sets->sides == a.sides) {
    // the expert sort and the expert-set sort share their passes over the top-k tables
    const SetSortArgs& t = *a.sets;
    hist2_kernel<<<g2, RB, 0, s>>>(a.idx, a.gate, a.blockcnt, t.setid, t.gset, t.setexp, t.blockcnt, a.N, a.k, a.E, t.nsets,
                                   nblk);
    if ((long)nblk * (a.E > t.nsets ? a.E : t.nsets) <= 8192) {
      // small tables: every scatter block scans the counts it needs itself, one launch less
      scan_scatter2_kernel<<<g2, RB, 0, s>>>(a.idx, a.blockcnt, a.offsets, a.perm, t.setid, t.blockcnt, t.setoff, t.setperm,
                                             t.gset, t.gsort, a.N, a.E, a.k, t.nsets, nblk);
      return;
    }
    scan2_kernel<<<dim3(a.sides * a.H, 2), 256, 0, s>>>(a.blockcnt, a.offsets, a.E, t.blockcnt, t.setoff, t.nsets, nblk);
    scatter2_kernel<<<g2, RB, 0, s>>>(a.idx, a.blockcnt, a.perm, t.setid, t.blockcnt, t.setperm, t.gset, t.gsort, a.N, a.E,
                                      a.k, t.nsets, nblk);
    return;
  }
  if (a.gtab)
    hist_gate_table_kernel<<<g2, RB, 0, s>>>(a.idx, a.gate, a.blockcnt, a.gtab, a.N, a.H, a.E, a.k, nblk);
  else
    hist_kernel<<<g2, RB, 0, s>>>(a.idx, a.blockcnt, a.N, a.E, a.k, nblk);
  if ((long)nblk * a.E <= 8192) {
    scan_scatter1_kernel<<<g2, RB, 0, s>>>(a.idx, a.blockcnt, a.offsets, a.perm, a.N, a.E, a.k, nblk);
    return;
  }
  scan_kernel<<<a.sides * a.H, 256, 0, s>>>(a.blockcnt, a.offsets, a.E, nblk);
  scatter_kernel<<<g2, RB, 0, s>>>(a.idx, a.blockcnt, a.perm, a.N, a.E, a.k, nblk);
}

}  // namespace sh
