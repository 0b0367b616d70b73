// bf16 matrix-core (MFMA) kernels for the projections of the SwitchHead layer (arXiv
// 2312.07987, Sec. 2.2): the grouped conditional expert GEMMs of the V^h and y equations,
// the dense per-head Q/K projections of Sec. 2.1, their data gradients and their weight
// gradients.  gfx950 only: v_mfma_f32_32x32x16_bf16, 64-wide waves, LDS-staged tiles,
// ds_read_b64_tr_b16 for operands whose reduction index is the slow one in memory.
//
// Fragment layouts of v_mfma_f32_32x32x16_bf16 (lane = 32*g + r, g in {0,1}):
//   A operand: A[row r][k = 8g .. 8g+7]      B operand: B[k = 8g .. 8g+7][col r]
//   D: register q (0..15) holds D[8*(q/4) + 4g + q%4][col r]
#include "common.h"
#include "mfma_util.h"
#include "router_select.h"
#include <cstdlib>

namespace sh {

// ----------------------------------------------------------------------------------------
// Row GEMM.  4 waves per work-group arranged WM x WN, each wave owns MI x NJ MFMA blocks of
// 32 x 32.  Two shapes of use:
//   small   128 x 128 tile, wave 64 x 64, K step 64, one LDS stage (the next K step waits in
//           registers), three work-groups per CU; gathered rows, small or ragged problems
//   medium  256 x 128 (wave 128 x 64) and wide 128 x 256 (wave 64 x 128), K step 64, one stage, two
//           work-groups per CU; dense rows.  The larger wave tile reads 0.75 KB of LDS per MFMA
//           instead of 1 KB, and a K step of 64 takes whole 128-byte lines from every row (a step of
//           32 with two stages moved half lines and measured 5 % slower).
// LDS is dynamic: [stages][A tile | B tile] bf16, then row ids, row scales, segment offsets.
// ----------------------------------------------------------------------------------------
template <int WM_, int WN_, int MI_, int NJ_, int BK_, int STAGES_, int MINB_ = 1>
struct TileCfg {
  static constexpr int WM = WM_, WN = WN_, MI = MI_, NJ = NJ_, BK = BK_, STAGES = STAGES_, MINB = MINB_;
  static constexpr int BM = WM * MI * 32, BN = WN * NJ * 32;
  static constexpr int LDA = BK + 8;        // A tile [BM][LDA], k contiguous
  static constexpr int LDB_NT = BK + 8;     // B tile [BN][LDB_NT] when k is contiguous in memory
  // B tile [BK][LDB_NN] when n is contiguous in memory: rows 16 banks (mod 64) apart for the transposing reads
  static constexpr int LDB_NN = BN == 96 ? 160 : BN + 32;
  static constexpr int A_ELEMS = BM * LDA;
  static constexpr int B_ELEMS = (BN * LDB_NT > BK * LDB_NN) ? BN * LDB_NT : BK * LDB_NN;
  static constexpr int STAGE_ELEMS = A_ELEMS + B_ELEMS;
  static constexpr int LDC = NJ * 32 + 8;   // staged output: 32 rows per wave at a time
  static_assert(4 * 32 * LDC <= STAGES * STAGE_ELEMS, "output staging must fit in the operand tiles");
  static constexpr size_t lds_bytes(bool sets) {
    return (size_t)STAGES * STAGE_ELEMS * 2 + (size_t)BM * 4 + (size_t)BM * (sets ? 8 : 1) * 4 + 64;
  }
};
typedef TileCfg<2, 2, 2, 2, 64, 1> CfgSmall;    // 128 x 128
typedef TileCfg<2, 2, 2, 2, 80, 1> CfgSmall80;  // the same with an 80-wide K step: a reduction of 65..80 (a head width of 76
                                                // or 80) then takes one step per segment instead of one and a mostly empty second
typedef TileCfg<4, 1, 1, 3, 64, 1> CfgN96;      // 128 x 96, wave tile 32 x 96: outputs 65..96 wide (head widths 76, 80, 96)
                                                // waste a fifth of a 96-wide tile instead of two fifths of a 128-wide one
typedef TileCfg<2, 2, 1, 1, 64, 1> CfgRouter;   // 64 x 64: the router logits have <= 32 columns and want many work-groups (a K step of
                                                // 256, four times the bytes per load round trip but one work-group per CU: 35 -> 50 us at c2)
typedef TileCfg<2, 2, 2, 4, 64, 1, 2> CfgWide;     // 128 x 256, wave tile 64 x 128, two work-groups per CU
typedef TileCfg<2, 2, 4, 2, 64, 1, 2> CfgMed;   // 256 x 128, wave tile 128 x 64, two work-groups per CU

template <class Cfg, int VEC, bool BNT, int TAG, int SEG>
__global__ __launch_bounds__(256, Cfg::MINB) void mfma_row_gemm_kernel(RowGemmArgs a) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NJ = Cfg::NJ;
  constexpr int LDA = Cfg::LDA, LDB_NT = Cfg::LDB_NT, LDB_NN = Cfg::LDB_NN;
  typedef typename Chunk<VEC>::type chunk_t;
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int* ids = (int*)(smem + Cfg::STAGES * Cfg::STAGE_ELEMS);
  float* gsc = (float*)(ids + BM);                         // SEG 1: [row][segment]
  long* bseg = (long*)(gsc + BM * (SEG == 1 ? 8 : 1));     // SEG 1: B offset of each segment's expert

  // ---- which tile ------------------------------------------------------------------------
  const int ncol = (a.Nc + BN - 1) / BN;
  int h, e = 0, row0, rows, ct, w, slot;
  if constexpr (SEG == 1) {
    decode_block(blockIdx.x, ncol, w, slot);
    ct = slot;
    const int tph = (a.M + BM - 1) / BM + a.E;   // upper bound of the row tiles of one head
    h = w / tph;
    if (h >= a.heads) return;
    if (!find_tile_wave(a.offsets + (long)h * (a.E + 1), a.E, BM, w % tph, threadIdx.x & 63, e, row0, rows)) return;
  } else {
    decode_block(blockIdx.x, a.heads * a.E * ncol, w, slot);
    const int grp = slot / ncol;
    ct = slot % ncol;
    h = grp / a.E;
    e = grp % a.E;
    if (a.perm) {
      const int* off = a.offsets + (long)h * (a.E + 1);
      row0 = off[e] + w * BM;
      const int end = off[e + 1];
      if (row0 >= end) return;
      rows = end - row0 < BM ? end - row0 : BM;
    } else {
      row0 = w * BM;
      if (row0 >= a.M) return;
      rows = a.M - row0 < BM ? a.M - row0 : BM;
    }
  }
  const bool second = a.hsplit > 0 && h >= a.hsplit;
  const int hh = second ? h - a.hsplit : h;
  const unsigned inv_adiv = div_magic(a.a_div), inv_cdiv = div_magic(a.c_div);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nseg = SEG ? a.nseg : 1;
  if constexpr (SEG == 1) {
    // the rows' ids, their gates and the segments' experts are independent loads: all are requested
    // before the first is waited for
    constexpr int GS = (BM * 8 + 255) / 256;
    float gv[GS];
#pragma unroll
    for (int u = 0; u < GS; ++u) {
      const int t = tid + u * 256, rr = t / nseg, p = t % nseg;
      gv[u] = 0.f;
      if (t < BM * nseg && rr < rows) gv[u] = a.segate[(long)h * a.gate_hstride + (long)(row0 + rr) * nseg + p];
    }
    static_assert(BM <= 256, "one row id per thread");
    int idv = -1;
    if (tid < rows) idv = a.perm ? a.perm[(long)h * a.M + row0 + tid] : row0 + tid;
    long bs = 0;
    if (tid < nseg) bs = (long)hh * a.b_hstride + (long)a.set_experts[e * 8 + tid] * a.b_estride;
    if (tid < BM) ids[tid] = idv;
#pragma unroll
    for (int u = 0; u < GS; ++u) {
      const int t = tid + u * 256;
      if (t < BM * nseg) gsc[(t / nseg) * 8 + t % nseg] = gv[u];
    }
    if (tid < nseg) bseg[tid] = bs;
  } else {
    for (int t = tid; t < BM; t += 256) {
      int id = -1;
      float g = 0.f;
      if (t < rows) {
        id = a.perm ? a.perm[(long)h * a.M + row0 + t] : row0 + t;
        g = a.gate ? a.gate[(long)h * a.gate_hstride + id] : 1.f;
      }
      ids[t] = id;
      gsc[t] = g;
    }
  }
  __syncthreads();

  const unsigned short* A = (const unsigned short*)a.A;
  const unsigned short* Bbase = (const unsigned short*)(second ? a.B2 : a.B);
  const unsigned short* B = Bbase + (SEG ? 0 : (long)hh * a.b_hstride + (long)e * a.b_estride);
  const int n0 = ct * BN;
  const int K = a.K, Nc = a.Nc;

  // ---- per-thread load plan -----------------------------------------------------------
  constexpr int A_CPR = BK / VEC;                 // chunks per A row
  constexpr int A_N = BM * A_CPR / 256;           // chunks per thread
  constexpr int B_N = (BK * BN / VEC) / 256;
  long a_off[A_N];
  int a_kc[A_N], a_lds[A_N];
#pragma unroll
  for (int i = 0; i < A_N; ++i) {
    int c = tid + i * 256;
    int rr = c / A_CPR, kc = (c % A_CPR) * VEC;
    int id = ids[rr];
    a_off[i] = id >= 0 ? (long)div_by(id, inv_adiv) * a.lda + (long)hh * a.a_hoff + kc : -1;
    a_kc[i] = kc;
    a_lds[i] = rr * LDA + kc;
  }
  long b_off[B_N];
  int b_kc[B_N], b_lds[B_N];
  bool b_ok[B_N];
#pragma unroll
  for (int i = 0; i < B_N; ++i) {
    int c = tid + i * 256;
    if constexpr (BNT) {
      constexpr int CPR = BK / VEC;
      int n = c / CPR, kc = (c % CPR) * VEC;
      b_ok[i] = n0 + n < Nc;
      b_off[i] = (long)(n0 + n) * a.sbn + kc;
      b_kc[i] = kc;
      b_lds[i] = n * LDB_NT + kc;
    } else {
      constexpr int CPR = BN / VEC;
      int kr = c / CPR, nc = (c % CPR) * VEC;
      b_ok[i] = n0 + nc < Nc;
      b_off[i] = (long)kr * a.sbk + n0 + nc;
      b_kc[i] = kr;
      b_lds[i] = kr * LDB_NN + nc;
    }
  }

  chunk_t ra[A_N], rb[B_N];
  const int nks = (K + BK - 1) / BK;   // K steps per segment
  float sumsq[TAG == TAG_ROUTER ? A_N : 1] = {};
  int staged_seg = 0;   // segment of the K step that sits in ra / rb
  auto load_global = [&](int it) {
    const int seg = SEG ? it / nks : 0;
    const int k0 = (SEG ? it % nks : it) * BK;
    staged_seg = seg;
    const unsigned short* Ap = A;
    const unsigned short* Bp = B;
    if constexpr (SEG == 1) Bp = B + bseg[seg];
    if constexpr (SEG == 2) {
      const int which = seg / a.seg_split, sh_ = seg % a.seg_split;
      Ap = A + (long)which * a.a_wstride + (long)sh_ * a.a_sstride;
      Bp = (const unsigned short*)(which == 0 ? a.B : which == 1 ? a.B2 : a.B3) + (long)sh_ * a.b_sstride;
    }
#pragma unroll
    for (int i = 0; i < A_N; ++i) {
      ra[i] = zero_chunk<VEC>();
      if (a_off[i] >= 0 && k0 + a_kc[i] < K) ra[i] = *(const chunk_t*)(Ap + a_off[i] + k0);
    }
#pragma unroll
    for (int i = 0; i < B_N; ++i) {
      rb[i] = zero_chunk<VEC>();
      if (b_ok[i] && k0 + b_kc[i] < K) {
        if constexpr (BNT)
          rb[i] = *(const chunk_t*)(Bp + b_off[i] + k0);
        else
          rb[i] = *(const chunk_t*)(Bp + b_off[i] + (long)k0 * a.sbk);
      }
    }
  };
  auto store_lds = [&](int stage) {
    unsigned short* As = smem + stage * Cfg::STAGE_ELEMS;
    unsigned short* Bs = As + Cfg::A_ELEMS;
#pragma unroll
    for (int i = 0; i < A_N; ++i) {
      // expert-set mode: the gate is applied here, not at the load, so that the load stays in
      // flight while the previous step is multiplied
      if constexpr (SEG == 1) ra[i] = scale_chunk(ra[i], gsc[(a_lds[i] / LDA) * 8 + staged_seg]);
      *(chunk_t*)(&As[a_lds[i]]) = ra[i];
      if constexpr (TAG == TAG_ROUTER) sumsq[i] += chunk_sumsq(ra[i]);   // row norms ride along (see epilogue)
    }
#pragma unroll
    for (int i = 0; i < B_N; ++i) *(chunk_t*)(&Bs[b_lds[i]]) = rb[i];
  };

  const int wm = (wave / Cfg::WN) * (MI * 32), wn = (wave % Cfg::WN) * (NJ * 32);
  const int r = lane & 31, g = lane >> 5;
  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  constexpr bool ACC64 = TAG == TAG_ROUTER;
  const bool active = !ACC64 || n0 + wn < Nc;   // router: at most 32 columns, held by the waves with wn == 0
  double acc64[ACC64 ? MI : 1][16];
  if constexpr (ACC64) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc64[i][q] = 0.0;
  }

  auto compute = [&](int stage) {
    const unsigned short* As = smem + stage * Cfg::STAGE_ELEMS;
    const unsigned short* Bs = As + Cfg::A_ELEMS;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 fa[MI], fb[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i] = frag_rowmajor(&As[(wm + i * 32 + r) * LDA + kk + 8 * g]);
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        if constexpr (BNT)
          fb[j] = frag_rowmajor(&Bs[(wn + j * 32 + r) * LDB_NT + kk + 8 * g]);
        else
          fb[j] = frag_transposed(Bs, LDB_NN, kk + 8 * g, wn + j * 32, lane);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
          if (!ACC64 || j == 0) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      if constexpr (ACC64) {
        // router logits: the fp32 accumulator only ever holds the sum of 64 terms
        if ((kk & 63) == 48) {
#pragma unroll
          for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int q = 0; q < 16; ++q) {
              acc64[i][q] += (double)acc[i][0][q];
              acc[i][0][q] = 0.f;
            }
        }
      }
    }
  };

  const int nk = nks * nseg;
  if constexpr (Cfg::STAGES == 1) {
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      if (kt + 1 < nk) load_global(kt + 1);
      if (active) compute(0);
      __syncthreads();
      if (kt + 1 < nk) {
        store_lds(0);
        __syncthreads();
      }
    }
  } else {
    // two LDS stages: K step kt is multiplied from stage kt&1 while step kt+2 travels
    // global -> registers; it is written into the stage just consumed
    load_global(0);
    store_lds(0);
    if (nk > 1) {
      load_global(1);
      store_lds(1);
    }
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      if (kt + 2 < nk) load_global(kt + 2);
      compute(kt & 1);
      __syncthreads();
      if (kt + 2 < nk) store_lds(kt & 1);
    }
    __syncthreads();
  }

  // ---- epilogue -------------------------------------------------------------------------
  char* Cb = (char*)(second ? a.C2 : a.C);
  if constexpr (ACC64) {
    // Router: the tile's logits never leave the CU.  They go to LDS (the operand tiles are dead) next to
    // the rows' sums of squares (the error bound needs |x_n|, and every chunk of the A rows went through
    // this block's registers: 8 threads share a row), and the selection runs on them right here.
    static_assert(BM * 32 * 8 + BM * 4 + 4 * 64 * 8 + 256 * 4 + 16 <= Cfg::STAGES * Cfg::STAGE_ELEMS * 2, "router epilogue needs the LDS");
    double* zt = (double*)smem;                  // [BM][Nc], Nc <= 32
    double(*zs)[64] = (double(*)[64])(zt + BM * 32);
    float* rs = (float*)(zs + 4);
    int* flist = (int*)(rs + BM);
    int* nflag = flist + 256;
    __syncthreads();
    for (int t = tid; t < BM; t += 256) rs[t] = 0.f;
    if (tid == 0) *nflag = 0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < A_N; ++i) atomicAdd(&rs[a_lds[i] / LDA], sumsq[i]);
    if (active) {
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const int row = wm + i * 32 + 8 * (q >> 2) + 4 * g + (q & 3);
          const int n = n0 + wn + r;
          if (n < Nc) zt[row * Nc + n] = acc64[i][q];
        }
    }
    __syncthreads();
    router_select_tile(a.rsel, h, zt, Nc, rs, ids, BM, zs, flist, nflag);
    return;
  }
  if (a.mode == STORE_T) {   // the host checks Nc % VEC == 0 for this mode
    // bf16 output: each wave stages 32 rows of its tile in LDS (the operand tiles are dead: the
    // main loop ends with a barrier), then stores them as 16-byte (8-byte) pieces along the rows.  The
    // staging area is the wave's own and a wave's LDS operations complete in order, so no
    // work-group barrier is needed here, only a fixed instruction order.
    constexpr int LDC = Cfg::LDC;
    unsigned short* Cs = smem + wave * 32 * LDC;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int lr = 8 * (q >> 2) + 4 * g + (q & 3);
        const float sc = SEG == 1 ? 1.f : gsc[wm + i * 32 + lr];
#pragma unroll
        for (int j = 0; j < NJ; ++j) Cs[lr * LDC + j * 32 + r] = f32_to_bf16(acc[i][j][q] * sc);
      }
      __builtin_amdgcn_wave_barrier();
      constexpr int PPR = NJ * 32 / VEC;   // pieces per staged row
#pragma unroll
      for (int u = 0; u < 32 * PPR / 64; ++u) {
        const int c = lane + u * 64;
        const int lr = c / PPR, cc = (c % PPR) * VEC;
        const int id = ids[wm + i * 32 + lr];
        if (id < 0 || n0 + wn + cc >= Nc) continue;
        const long crow = (long)div_by(id, inv_cdiv) * a.ldc + (long)hh * a.c_hoff;
        *(chunk_t*)((unsigned short*)Cb + crow + n0 + wn + cc) = *(const chunk_t*)(&Cs[lr * LDC + cc]);
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int row = wm + i * 32 + 8 * (q >> 2) + 4 * g + (q & 3);
      const int id = ids[row];
      if (id < 0) continue;
      const float sc = SEG == 1 ? 1.f : gsc[row];
      const long crow = (long)div_by(id, inv_cdiv) * a.ldc + (long)hh * a.c_hoff;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int n = n0 + wn + j * 32 + r;
        if (n >= Nc) continue;
        const float v = acc[i][j][q] * sc;
        if (a.mode == STORE_T)
          ((unsigned short*)Cb)[crow + n] = f32_to_bf16(v);
        else if (a.mode == STORE_F32)
          ((float*)Cb)[crow + n] = v;
        else
          atomicAdd((float*)Cb + crow + n, v);
      }
    }
  }
}

int rg_kstep() { return 64; }   // terms the router logits GEMM sums in fp32 before it flushes to fp64

static bool aligned_to(const void* p, size_t b) { return ((uintptr_t)p % b) == 0; }

// vector width (bf16 elements) all loads of a row GEMM can use, 0 if none
static int row_gemm_vec(const RowGemmArgs& a) {
  const bool nt = a.sbk == 1;
  if (!nt && a.sbn != 1) return 0;
  for (int vec = 8; vec >= 4; vec -= 4) {
    const size_t bytes = vec * 2;
    bool ok = aligned_to(a.A, bytes) && aligned_to(a.B, bytes) && a.lda % vec == 0 && a.a_hoff % vec == 0 &&
              a.K % vec == 0 && a.b_hstride % vec == 0 && a.b_estride % vec == 0;
    if (a.hsplit > 0 || a.seg_mode == 2) ok = ok && aligned_to(a.B2, bytes);
    if (a.seg_mode == 2 && a.nseg > 2 * a.seg_split) ok = ok && a.B3 && aligned_to(a.B3, bytes) && a.nseg <= 3 * a.seg_split;
    if (a.seg_mode == 2) ok = ok && a.a_sstride % vec == 0 && a.a_wstride % vec == 0 && a.b_sstride % vec == 0;
    if (a.mode == STORE_T) ok = ok && aligned_to(a.C, bytes) && a.ldc % vec == 0 && a.c_hoff % vec == 0 && a.Nc % vec == 0;
    if (nt)
      ok = ok && a.sbn % vec == 0;
    else
      ok = ok && a.sbk % vec == 0 && a.Nc % vec == 0;
    if (ok) return vec;
  }
  return 0;
}

bool mfma_row_gemm_supported(const RowGemmArgs& a) {
  if (a.seg_mode == 1 && (a.nseg < 1 || a.nseg > 8 || a.E > 128)) return false;   // the tile lookup covers 128 groups
  if (a.tag == TAG_ROUTER && (a.Nc > 32 || a.mode != STORE_F64 || a.seg_mode != 0 || a.perm || a.E != 1 || a.hsplit != 0 ||
                              a.a_div != 1 || a.Nc < a.rsel.H * a.rsel.E))
    return false;
  // row ids stay below M; the multiply-high division needs id * divisor < 2^32
  if ((long)a.M * (a.a_div > a.c_div ? a.a_div : a.c_div) >= (1L << 32)) return false;
  return row_gemm_vec(a) != 0;
}

template <class Cfg, int VEC, bool BNT, int TAG, int SEG>
static void launch_cfg(const RowGemmArgs& a, hipStream_t s) {
  const int ncol = (a.Nc + Cfg::BN - 1) / Cfg::BN;
  dim3 g;
  if (SEG == 1) {
    const int tph = (a.M + Cfg::BM - 1) / Cfg::BM + a.E;
    g = dim3(grid_windows(a.heads * tph, ncol));
  } else {
    const int group_rows = a.perm ? a.max_group_rows : a.M;
    g = dim3(grid_windows((group_rows + Cfg::BM - 1) / Cfg::BM, a.heads * a.E * ncol));
  }
  const size_t lds = Cfg::lds_bytes(SEG == 1);
  auto kern = mfma_row_gemm_kernel<Cfg, VEC, BNT, TAG, SEG>;
  if (lds > 64 * 1024) {
    static bool raised = false;   // per instantiation
    if (!raised) {
      (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      raised = true;
    }
  }
  kern<<<g, 256, lds, s>>>(a);
}

// tile shape for a launch: the big tiles pay off when a group has enough rows to fill them
enum { SHAPE_SMALL, SHAPE_WIDE, SHAPE_MED };
static int pick_shape(const RowGemmArgs& a) {
  const int group_rows = a.perm ? a.max_group_rows : a.M;
  if (a.tag == TAG_ROUTER || a.tag == TAG_GENERIC) return SHAPE_SMALL;
  // measured on MI355X: the 256 x 128 tile with two work-groups per CU wins where the rows are
  // dense (its operand traffic per flop is 25 % lower); expert-gathered rows do better with
  // the small tile (more work-groups in flight per CU)
  if (!a.perm && group_rows >= 4096 && a.Nc >= 512 && a.seg_mode == 2) return SHAPE_WIDE;   // concatenated-K dgrad
  if (!a.perm && group_rows >= 4096 && a.Nc >= 128) return SHAPE_MED;
  return SHAPE_SMALL;
}

// Only the (step tag, segment mode) pairs the layer uses get a kernel of their own name;
// everything else runs under the generic tag with the small tile.
template <bool BNT, int TAG, int SEG>
static void launch_tagged(const RowGemmArgs& a, hipStream_t s) {
  switch (pick_shape(a)) {
    case SHAPE_WIDE: launch_cfg<CfgWide, 8, BNT, TAG, SEG>(a, s); break;
    case SHAPE_MED: launch_cfg<CfgMed, 8, BNT, TAG, SEG>(a, s); break;
    default:
      if (a.K > 64 && a.K <= 80)
        launch_cfg<CfgSmall80, 8, BNT, TAG, SEG>(a, s);
      else if (a.Nc > 64 && a.Nc <= 96)
        launch_cfg<CfgN96, 8, BNT, TAG, SEG>(a, s);
      else
        launch_cfg<CfgSmall, 8, BNT, TAG, SEG>(a, s);
      break;
  }
}

template <class Cfg, int VEC, bool BNT>
static void launch_generic_cfg(const RowGemmArgs& a, hipStream_t s) {
  if (a.seg_mode == 1)
    launch_cfg<Cfg, VEC, BNT, TAG_GENERIC, 1>(a, s);
  else if (a.seg_mode == 2)
    launch_cfg<Cfg, VEC, BNT, TAG_GENERIC, 2>(a, s);
  else
    launch_cfg<Cfg, VEC, BNT, TAG_GENERIC, 0>(a, s);
}
template <int VEC, bool BNT>
static void launch_generic(const RowGemmArgs& a, hipStream_t s) {
  if (a.K > 64 && a.K <= 80)
    launch_generic_cfg<CfgSmall80, VEC, BNT>(a, s);
  else if (a.Nc > 64 && a.Nc <= 96)
    launch_generic_cfg<CfgN96, VEC, BNT>(a, s);
  else
    launch_generic_cfg<CfgSmall, VEC, BNT>(a, s);
}

void launch_mfma_row_gemm(const RowGemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.Nc <= 0) return;
  if (pp_row_gemm_supported(a)) return launch_pp_row_gemm(a, s);
  const int vec = row_gemm_vec(a);
  const bool nt = a.sbk == 1;
  if (vec == 8) {
    const int key = a.tag * 4 + a.seg_mode;
    if (nt) {
      switch (key) {
        case TAG_O_DGRAD * 4 + 0: return launch_tagged<true, TAG_O_DGRAD, 0>(a, s);
        case TAG_V_DGRAD * 4 + 0: return launch_tagged<true, TAG_V_DGRAD, 0>(a, s);
        case TAG_V_DGRAD * 4 + 1: return launch_tagged<true, TAG_V_DGRAD, 1>(a, s);
        case TAG_QK_DGRAD * 4 + 0: return launch_tagged<true, TAG_QK_DGRAD, 0>(a, s);
        case TAG_QK_DGRAD * 4 + 2: return launch_tagged<true, TAG_QK_DGRAD, 2>(a, s);
        default: return launch_generic<8, true>(a, s);
      }
    } else {
      switch (key) {
        case TAG_QK_PROJ * 4 + 0: return launch_tagged<false, TAG_QK_PROJ, 0>(a, s);
        case TAG_V_EXPERTS * 4 + 0: return launch_tagged<false, TAG_V_EXPERTS, 0>(a, s);
        case TAG_O_EXPERTS * 4 + 0: return launch_tagged<false, TAG_O_EXPERTS, 0>(a, s);
        case TAG_O_EXPERTS * 4 + 1: return launch_tagged<false, TAG_O_EXPERTS, 1>(a, s);
        case TAG_ROUTER * 4 + 0: return launch_cfg<CfgRouter, 8, false, TAG_ROUTER, 0>(a, s);
        default: return launch_generic<8, false>(a, s);
      }
    }
  }
  if (nt)
    return launch_generic<4, true>(a, s);
  if (a.tag == TAG_ROUTER) return launch_cfg<CfgRouter, 4, false, TAG_ROUTER, 0>(a, s);
  return launch_generic<4, false>(a, s);
}

// ----------------------------------------------------------------------------------------
// Weight-gradient GEMM: dW[i, j] += sum_rows g * A[row, i] * Bm[row, j].  The reduction runs
// over gathered rows, so both tiles are stored [row][feature] and read with transposing
// loads.  Block tile 128 (i) x 128 (j), 32 rows per step, `chunk` rows per block, fp32
// atomic add of the block's partial sum.
// ----------------------------------------------------------------------------------------
// Output tile BM (features of A) x BN (features of Bm), 4 waves as WM x WN with MI x NJ MFMA
// blocks each, BK rows per step, two LDS stages (one barrier per step).  Dynamic LDS:
// [2][A tile [BK][BM+32] | B tile [BK][BN+32]] bf16, then the chunk's row ids and gates.
template <int WM_, int WN_, int MI_, int NJ_, int MINB_>
struct WgCfg {
  static constexpr int WM = WM_, WN = WN_, MI = MI_, NJ = NJ_, MINB = MINB_, BK = 32;
  static constexpr int BM = WM * MI * 32, BN = WN * NJ * 32;
  static constexpr int LDA = BM + 32, LDB = BN + 32;      // row strides 16 banks (mod 64) apart
  static constexpr int STAGE_ELEMS = BK * (LDA + LDB);
  static constexpr int MAX_CHUNK = 2048;
  static constexpr int ROW_CAP = MAX_CHUNK + 4 * BK;   // the row tables reach past the chunk as far as the prefetch does
  static constexpr size_t lds_bytes() { return (size_t)2 * STAGE_ELEMS * 2 + (size_t)ROW_CAP * 8; }
};
typedef WgCfg<2, 2, 2, 2, 1> WgSmall;   // 128 x 128
typedef WgCfg<1, 4, 4, 2, 2> WgWide;    // 128 x 256, wave tile 128 x 64, two work-groups per CU
typedef WgCfg<4, 1, 2, 4, 2> WgTall;    // 256 x 128, wave tile 64 x 128, two work-groups per CU

// FULL: every load is issued without a condition (rows past the chunk repeat its last row, feature
// pieces past Ka / Kb repeat the last piece; both are zeroed on their way into LDS).  With the loads of a
// step a fixed number, the wait before a step is staged names exactly the loads of that step and
// leaves the younger ones of the next step in flight; a branch around a load makes it wait for all.
// MODE 0 is the general form; 1..3 are FULL with the gate fixed at compile time (1 none, 2 on the rows
// of A, 3 on the rows of Bm) and with the operand row (the row id divided by the shared a_div = b_div)
// kept in LDS instead of the id, which takes the division out of every load's address.
template <class Cfg, int VEC, int TAG, int MODE = 0>
__global__ __launch_bounds__(256, Cfg::MINB) void mfma_wgrad_kernel(WgradArgs a) {
  constexpr bool FULL = MODE != 0;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, MI = Cfg::MI, NJ = Cfg::NJ;
  constexpr int LDA = Cfg::LDA, LDB = Cfg::LDB;
  typedef typename Chunk<VEC>::type chunk_t;
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int* ids = (int*)(smem + 2 * Cfg::STAGE_ELEMS);
  float* gsc = (float*)(ids + Cfg::ROW_CAP);

  // unit = (chunk window, group); the output tiles of a unit share an XCD (they read the same rows).  Which XCD
  // a unit runs on: see the window-major placement below.
  const int ti_ = (a.Ka + BM - 1) / BM, tj = (a.Kb + BN - 1) / BN;
  const int ntile = ti_ * tj;
  const int G = a.heads * a.E;
  int w, grp, tile;
  int g_first = 0, g_rows = 0;   // the group's first row in the sorted order, its row count
  if (G <= 64) {
    // Window-major placement.  The chunk windows of all groups cover about the same tokens (the w-th chunk of every
    // expert's sorted rows lies near the same token range), so the work-groups of one window should meet in one L2:
    // the non-empty (window, group) units are counted window by window, and XCD x (work-group ids x, x + 8, ...) takes
    // the x-th eighth of that list, i.e. one or two windows, instead of every eighth unit of all windows.  Every wave
    // derives the list from the group sizes by itself (lane g holds the rows of group g).
    const int lane_ = threadIdx.x & 63;
    int grows = 0, gstart = 0;
    if (lane_ < G) {
      const int gh = lane_ / a.E, ge = lane_ % a.E;
      if (a.perm) {
        gstart = a.offsets[(long)gh * (a.E + 1) + ge];
        grows = a.offsets[(long)gh * (a.E + 1) + ge + 1] - gstart;
      } else {
        grows = a.M;
      }
    }
    long units = 0;
    for (int ww = 0;; ++ww) {
      const int cw = __popcll(__ballot(grows > ww * a.chunk));
      if (cw == 0) break;
      units += cw;
    }
    const long total = units * ntile, share = (total + 7) / 8;
    const long slot = blockIdx.x >> 3, q = (long)(blockIdx.x & 7) * share + slot;
    if (slot >= share || q >= total) return;
    long u = q / ntile;
    tile = (int)(q % ntile);
    int ww = 0;
    unsigned long long m = 0;
    for (;; ++ww) {
      m = __ballot(grows > ww * a.chunk);
      const int cw = __popcll(m);
      if (u < cw) break;
      u -= cw;
    }
    for (long t = 0; t < u; ++t) m &= m - 1;   // drop the u lowest groups of the window
    w = ww;
    grp = __ffsll((long long)m) - 1;
    // the group's first row and row count sit in lane grp: no second trip to the offsets
    g_first = __shfl(gstart, grp);
    g_rows = __shfl(grows, grp);
  } else {
    int unit;
    decode_block(blockIdx.x, ntile, unit, tile);
    w = unit / G;
    grp = unit % G;
    if (w * a.chunk >= (a.perm ? a.max_group_rows : a.M)) return;
    if (a.perm) {
      const int* off = a.offsets + (long)(grp / a.E) * (a.E + 1);
      g_first = off[grp % a.E];
      g_rows = off[grp % a.E + 1] - g_first;
    } else {
      g_rows = a.M;
    }
  }
  const int h = grp / a.E, e = grp % a.E;
  if (w * a.chunk >= g_rows) return;
  const int row0 = g_first + w * a.chunk;
  const int rows = g_rows - w * a.chunk < a.chunk ? g_rows - w * a.chunk : a.chunk;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the chunk's row ids, then their gates: every thread requests all of its ids before it waits for one, and
  // likewise the gates (two round trips; a loop over the rows would make two per 256 rows, and every work-group
  // of the launch stands in this prologue at the same time)
  {
    constexpr int PR = Cfg::MAX_CHUNK / 256;
    int idv[PR];
    float gv[PR];
    // (clamped indices instead of tests: a test around a load costs a branch and a wait for every load before it)
    if (a.perm) {
      const int* pp = a.perm + (long)h * a.M + row0;
#pragma unroll
      for (int i = 0; i < PR; ++i) idv[i] = pp[min(tid + 256 * i, rows - 1)];
    } else {
#pragma unroll
      for (int i = 0; i < PR; ++i) idv[i] = row0 + min(tid + 256 * i, rows - 1);
    }
    if (a.gate) {
      const float* gp = a.gate + (long)h * a.gate_hstride;
#pragma unroll
      for (int i = 0; i < PR; ++i) gv[i] = gp[idv[i]];
    } else {
#pragma unroll
      for (int i = 0; i < PR; ++i) gv[i] = 1.f;
    }
#pragma unroll
    for (int i = 0; i < PR; ++i) {
      const int t = tid + 256 * i;
      if (t < rows) {
        ids[t] = FULL ? div_by(idv[i], div_magic(a.a_div)) : idv[i];
        gsc[t] = gv[i];
      }
    }
  }
  // rows past the chunk that a step can touch (the loop rounds the step count up to an even number and requests
  // rows two steps ahead): a zero gate, and in the FULL modes the row of the chunk's last entry, so that the
  // loads need no clamp
  __syncthreads();
  {
    const int last = ids[rows - 1];
    for (int t = rows + tid; t < rows + 4 * BK && t < Cfg::ROW_CAP; t += 256) {
      gsc[t] = 0.f;
      if (FULL) ids[t] = last;
    }
  }
  __syncthreads();

  const int i0 = (tile / tj) * BM, j0 = (tile % tj) * BN;
  const int which = a.hsplit > 0 ? h / a.hsplit : 0;   // operand set of this head
  const bool second = which == 1;
  const int hh = a.hsplit > 0 ? h % a.hsplit : h;
  const unsigned short* A = (const unsigned short*)a.A;
  const unsigned short* Bm = (const unsigned short*)(which == 0 ? a.Bm : which == 1 ? a.Bm2 : a.Bm3);
  const bool scaled = a.gate != nullptr;

  constexpr int A_CPR = BM / VEC, B_CPR = BN / VEC;     // chunks per tile row
  constexpr int A_N = BK * A_CPR / 256, B_N = BK * B_CPR / 256;
  // row id -> operand row: ids are divided by a small constant (the k slots of a token share a row);
  // multiply-high by ceil(2^32 / d) is exact for ids below 2^32 / d
  const unsigned inv_a = div_magic(a.a_div), inv_b = div_magic(a.b_div);
  auto row_of = [](int id, unsigned inv) { return FULL ? id : div_by(id, inv); };   // FULL: already divided
  // two register sets: a step's rows are requested two steps before they are multiplied, so a
  // load has two steps of the work-group (and of its neighbour on the CU) to arrive
  chunk_t ra0[A_N], rb0[B_N], ra1[A_N], rb1[B_N];
  // FULL: a load's address is the operand's base (uniform) plus a 32-bit byte offset, row * stride + this thread's
  // column, one 24-bit multiply-add (the launcher checks that rows and strides stay below 2^24 and the operand
  // below 4 GiB); the row comes from the padded table, so nothing is clamped
  const char* Ab = (const char*)(A + (long)hh * a.a_hoff);
  const char* Bb = (const char*)(Bm + (long)hh * a.b_hoff);
  const unsigned lda2 = (unsigned)a.lda * 2, ldb2 = (unsigned)a.ldb * 2;
  const unsigned col_a2 = (unsigned)min(i0 + (tid % A_CPR) * VEC, a.Ka - VEC) * 2;
  const unsigned col_b2 = (unsigned)min(j0 + (tid % B_CPR) * VEC, a.Kb - VEC) * 2;
  auto load_global = [&](chunk_t (&ra)[A_N], chunk_t (&rb)[B_N], int r0) {
    if constexpr (FULL) {
      const int* ia = ids + r0 + tid / A_CPR;
      const int* ib = ids + r0 + tid / B_CPR;
#pragma unroll
      for (int i = 0; i < A_N; ++i) ra[i] = *(const chunk_t*)(Ab + (__umul24((unsigned)ia[i * (256 / A_CPR)], lda2) + col_a2));
#pragma unroll
      for (int i = 0; i < B_N; ++i) rb[i] = *(const chunk_t*)(Bb + (__umul24((unsigned)ib[i * (256 / B_CPR)], ldb2) + col_b2));
      return;
    }
#pragma unroll
    for (int i = 0; i < A_N; ++i) {
      const int c = tid + i * 256;
      const int rr = c / A_CPR, fc = (c % A_CPR) * VEC;
      ra[i] = zero_chunk<VEC>();
      if (r0 + rr < rows && i0 + fc < a.Ka) {
        ra[i] = *(const chunk_t*)(A + (long)row_of(ids[r0 + rr], inv_a) * a.lda + (long)hh * a.a_hoff + i0 + fc);
      }
    }
#pragma unroll
    for (int i = 0; i < B_N; ++i) {
      const int c = tid + i * 256;
      const int rr = c / B_CPR, fc = (c % B_CPR) * VEC;
      rb[i] = zero_chunk<VEC>();
      if (r0 + rr < rows && j0 + fc < a.Kb) {
        rb[i] = *(const chunk_t*)(Bm + (long)row_of(ids[r0 + rr], inv_b) * a.ldb + (long)hh * a.b_hoff + j0 + fc);
      }
    }
  };
  auto store_lds = [&](int stage, chunk_t (&ra)[A_N], chunk_t (&rb)[B_N], int staged_r0) {
    unsigned short* As = smem + stage * Cfg::STAGE_ELEMS;
    unsigned short* Bs = As + BK * LDA;
    // the gate is applied here, not at the load, so that the load stays in flight while the
    // previous steps are multiplied (rows past the chunk hold zeros and a zero gate)
    if constexpr (FULL) {
      // every row of the step lies in the chunk (a uniform test): nothing to zero.  Columns past the last feature of a
      // ragged tile hold a repeat of the last piece here; they only reach output elements that are never stored.
      if (staged_r0 + BK <= rows) {
        const float* ga = gsc + staged_r0 + tid / A_CPR;
        const float* gb = gsc + staged_r0 + tid / B_CPR;
#pragma unroll
        for (int i = 0; i < A_N; ++i) {
          chunk_t v = ra[i];
          if (MODE == 2) v = scale_chunk(v, ga[i * (256 / A_CPR)]);
          *(chunk_t*)(&As[(tid / A_CPR + i * (256 / A_CPR)) * LDA + (tid % A_CPR) * VEC]) = v;
        }
#pragma unroll
        for (int i = 0; i < B_N; ++i) {
          chunk_t v = rb[i];
          if (MODE == 3) v = scale_chunk(v, gb[i * (256 / B_CPR)]);
          *(chunk_t*)(&Bs[(tid / B_CPR + i * (256 / B_CPR)) * LDB + (tid % B_CPR) * VEC]) = v;
        }
        return;
      }
    }
#pragma unroll
    for (int i = 0; i < A_N; ++i) {
      const int c = tid + i * 256;
      chunk_t v = ra[i];   // a copy: the register sets themselves are only ever written by the loads
      if (MODE == 2 || (MODE == 0 && scaled && !a.scale_b)) v = scale_chunk(v, gsc[min(staged_r0 + c / A_CPR, Cfg::ROW_CAP - 1)]);
      if constexpr (FULL) v = i0 + (c % A_CPR) * VEC < a.Ka ? v : zero_chunk<VEC>();   // pieces past the last feature
      *(chunk_t*)(&As[(c / A_CPR) * LDA + (c % A_CPR) * VEC]) = v;
    }
#pragma unroll
    for (int i = 0; i < B_N; ++i) {
      const int c = tid + i * 256;
      chunk_t v = rb[i];
      if (MODE == 3 || (MODE == 0 && scaled && a.scale_b)) v = scale_chunk(v, gsc[min(staged_r0 + c / B_CPR, Cfg::ROW_CAP - 1)]);
      if constexpr (FULL) v = staged_r0 + c / B_CPR < rows && j0 + (c % B_CPR) * VEC < a.Kb ? v : zero_chunk<VEC>();   // repeats count for nothing
      *(chunk_t*)(&Bs[(c / B_CPR) * LDB + (c % B_CPR) * VEC]) = v;
    }
  };

  const int wm = (wave / Cfg::WN) * (MI * 32), wn = (wave % Cfg::WN) * (NJ * 32);
  const int r = lane & 31, g = lane >> 5;
  f32x16 acc[MI][NJ];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  const int nk = (rows + BK - 1) / BK;
  auto compute = [&](int stage) {
    const unsigned short* As = smem + stage * Cfg::STAGE_ELEMS;
    const unsigned short* Bs = As + BK * LDA;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 fa[MI], fb[NJ];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i] = frag_transposed(As, LDA, kk + 8 * g, wm + i * 32, lane);
#pragma unroll
      for (int j = 0; j < NJ; ++j) fb[j] = frag_transposed(Bs, LDB, kk + 8 * g, wn + j * 32, lane);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  };
  // the loop body is two steps, straight-line: an odd step count is rounded up (rows past the
  // chunk load as zeros)
  const int nk2 = (nk + 1) & ~1;
  load_global(ra0, rb0, 0);
  load_global(ra1, rb1, BK);
  store_lds(0, ra0, rb0, 0);
  __syncthreads();
  for (int kt = 0; kt < nk2; kt += 2) {
    // even step: its rows sit in stage 0; set 0 is free for step kt + 2, set 1 holds step kt + 1
    load_global(ra0, rb0, (kt + 2) * BK);
    compute(0);
    store_lds(1, ra1, rb1, (kt + 1) * BK);
    __syncthreads();
    load_global(ra1, rb1, (kt + 3) * BK);
    compute(1);
    store_lds(0, ra0, rb0, (kt + 2) * BK);
    __syncthreads();
  }

  if (a.partial) {
    // this chunk's partial sum, plain stores; launch_wgrad_reduce adds the chunks up
    float* P = a.partial + ((long)(h * a.E + e) * a.max_chunks + w) * ((long)a.Ka * a.Kb);
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int ii = i0 + wm + i * 32 + 8 * (q >> 2) + 4 * g + (q & 3);
        if (ii >= a.Ka) continue;
#pragma unroll
        for (int j = 0; j < NJ; ++j) {
          const int jj = j0 + wn + j * 32 + r;
          if (jj < a.Kb) P[(long)ii * a.Kb + jj] = acc[i][j][q];
        }
      }
    return;
  }
  float* dW = (second ? a.dW2 : a.dW) + (long)hh * a.w_hstride + (long)e * a.w_estride;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int ii = i0 + wm + i * 32 + 8 * (q >> 2) + 4 * g + (q & 3);
      if (ii >= a.Ka) continue;
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        int jj = j0 + wn + j * 32 + r;
        float* out = dW;
        if (a.col_split > 0 && jj >= a.col_split) {   // the right-hand block of columns has its own output
          jj -= a.col_split;
          out = a.dW2;
        }
        if (jj < (a.kb_store ? a.kb_store : a.Kb)) atomicAdd(out + (long)ii * a.swa + jj, acc[i][j][q]);
      }
    }
}

// dW_g = sum over the chunks of group g of its partial sums (4 consecutive j per thread)
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(WgradArgs a) {
  const int grp = blockIdx.y;
  const int h = grp / a.E, e = grp % a.E;
  const long per = (long)a.Ka * a.Kb;
  const long i4 = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i4 >= per) return;
  int rows = a.M;
  if (a.perm) {
    const int* off = a.offsets + (long)h * (a.E + 1);
    rows = off[e + 1] - off[e];
  }
  const int nch = (rows + a.chunk - 1) / a.chunk;
  const float* P = a.partial + (long)grp * a.max_chunks * per + i4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int c = 0; c < nch; ++c) {
    const float4 v = *(const float4*)(P + (long)c * per);
    s.x += v.x;
    s.y += v.y;
    s.z += v.z;
    s.w += v.w;
  }
  const int which = a.hsplit > 0 ? h / a.hsplit : 0;
  const int hh = a.hsplit > 0 ? h % a.hsplit : h;
  float* dW = (which == 0 ? a.dW : which == 1 ? a.dW2 : a.dW3) + (long)hh * a.w_hstride + (long)e * a.w_estride;
  const long ii = i4 / a.Kb, jj = i4 % a.Kb;   // Kb % 4 == 0: the 4 elements share a row
  *(float4*)(dW + ii * a.swa + jj) = s;
}

void launch_wgrad_reduce(const WgradArgs& a, hipStream_t s) {
  const long per = (long)a.Ka * a.Kb;
  dim3 g((unsigned)((per / 4 + 255) / 256), a.heads * a.E);
  wgrad_reduce_kernel<<<g, 256, 0, s>>>(a);
}

static int wgrad_vec(const WgradArgs& a) {
  if (a.chunk > WgSmall::MAX_CHUNK || a.chunk % 32 != 0) return 0;
  for (int vec = 8; vec >= 4; vec -= 4) {
    const size_t bytes = vec * 2;
    if (aligned_to(a.A, bytes) && aligned_to(a.Bm, bytes) && a.lda % vec == 0 && a.a_hoff % vec == 0 &&
        a.ldb % vec == 0 && a.b_hoff % vec == 0 && a.Ka % vec == 0 && a.Kb % vec == 0 &&
        (a.hsplit == 0 || aligned_to(a.Bm2, bytes)) && (a.hsplit == 0 || a.heads <= 2 * a.hsplit || (a.partial && aligned_to(a.Bm3, bytes))) &&
        (!a.partial || (a.swa % 4 == 0 && aligned_to(a.dW, 16))))
      return vec;
  }
  return 0;
}

bool mfma_wgrad_supported(const WgradArgs& a) { return wgrad_vec(a) != 0; }

template <class Cfg, int VEC, int TAG>
static void launch_wg(const WgradArgs& a, hipStream_t s) {
  const int ti = (a.Ka + Cfg::BM - 1) / Cfg::BM, tj = (a.Kb + Cfg::BN - 1) / Cfg::BN;
  const int group_rows = a.perm ? a.max_group_rows : a.M;
  dim3 g(grid_windows(((group_rows + a.chunk - 1) / a.chunk) * a.heads * a.E, ti * tj));
  const size_t lds = Cfg::lds_bytes();
  // the unconditional-load modes address both operands by 32-bit byte offsets made by a 24-bit multiply
  const size_t op_rows = ((size_t)a.M + (a.a_div > 0 ? a.a_div : 1) - 1) / (a.a_div > 0 ? a.a_div : 1);
  const size_t ldmax = (size_t)(a.lda > a.ldb ? a.lda : a.ldb);
  const bool small_offsets = op_rows < ((size_t)1 << 24) && ldmax * 2 < ((size_t)1 << 24) && op_rows * ldmax * 2 < ((size_t)1 << 32);
  const bool full = a.a_div == a.b_div && a.Ka >= VEC && a.Kb >= VEC && small_offsets;
  // the gate scales the rows of the narrower side of the tile (the same product, half the elements to scale); square
  // tiles take the side the caller names
  constexpr bool can_a = Cfg::BM <= Cfg::BN, can_b = Cfg::BM >= Cfg::BN;
  const bool on_b = !can_a || (can_b && a.scale_b);
  const int mode = !full ? 0 : (a.gate == nullptr ? 1 : (on_b ? 3 : 2));
  void (*kern)(WgradArgs) = mfma_wgrad_kernel<Cfg, VEC, TAG, 0>;
  if (mode == 1) kern = mfma_wgrad_kernel<Cfg, VEC, TAG, 1>;
  if constexpr (can_a)
    if (mode == 2) kern = mfma_wgrad_kernel<Cfg, VEC, TAG, 2>;
  if constexpr (can_b)
    if (mode == 3) kern = mfma_wgrad_kernel<Cfg, VEC, TAG, 3>;
  if (lds > 64 * 1024) {
    static bool raised = false;
    if (!raised) {
      (void)hipFuncSetAttribute((const void*)mfma_wgrad_kernel<Cfg, VEC, TAG, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      (void)hipFuncSetAttribute((const void*)mfma_wgrad_kernel<Cfg, VEC, TAG, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if constexpr (can_a)
        (void)hipFuncSetAttribute((const void*)mfma_wgrad_kernel<Cfg, VEC, TAG, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if constexpr (can_b)
        (void)hipFuncSetAttribute((const void*)mfma_wgrad_kernel<Cfg, VEC, TAG, 3>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      raised = true;
    }
  }
  kern<<<g, 256, lds, s>>>(a);
}

template <int TAG, int VEC = 8>
static void launch_wg_tagged(const WgradArgs& a, hipStream_t s) {
  // wide outputs get the 128 x 256 tile, tall ones the 256 x 128 tile
  int shape = a.Kb >= 256 && a.Ka <= 128 ? 1 : (a.Ka >= 256 && a.Kb >= 64 ? 2 : 0);
  if (shape == 1)
    launch_wg<WgWide, VEC, TAG>(a, s);
  else if (shape == 2)
    launch_wg<WgTall, VEC, TAG>(a, s);
  else
    launch_wg<WgSmall, VEC, TAG>(a, s);
}

void launch_mfma_wgrad(const WgradArgs& a, hipStream_t s) {
  if (a.M <= 0) return;
  const int vec = wgrad_vec(a);
  if (vec == 8) {
    switch (a.tag) {
      case TAG_O_WGRAD: return launch_wg_tagged<TAG_O_WGRAD>(a, s);
      case TAG_V_WGRAD: return launch_wg_tagged<TAG_V_WGRAD>(a, s);
      case TAG_QK_WGRAD: return launch_wg_tagged<TAG_QK_WGRAD>(a, s);
      default: return launch_wg<WgSmall, 8, TAG_GENERIC>(a, s);
    }
  }
  launch_wg_tagged<TAG_GENERIC, 4>(a, s);
}

}  // namespace sh
