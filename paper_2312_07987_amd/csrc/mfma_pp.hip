// Row GEMM of the SwitchHead projections (arXiv 2312.07987, Sec. 2.1 - 2.2) on 256 x 256 output tiles with
// eight waves per work-group, two per SIMD, that alternate roles ("ping-pong"): while the four waves of one
// group multiply (16 MFMAs on operand fragments they already hold in registers), the four waves of the other
// group do the memory work of their next half step (fragment reads from LDS, the LDS stores of the next
// K step's global data, the global loads of the step after).  A work-group barrier ends every phase, the second
// group runs one phase behind the first, so each SIMD always has one wave in a multiply phase and one in a
// memory phase.  One work-group per CU (147 KB of LDS for two stages of a 256 x 64 A tile and a 64 x 256 B tile).
//
// Same arguments and arithmetic as mfma_row_gemm_kernel (mfma_gemm.hip), for the launches whose shapes fill
// such tiles: reduction lengths that are multiples of 64, outputs 256 columns wide (or two adjacent heads of
// 128 columns), dense rows, expert-set rows (segment mode 1) and concatenated reductions (segment mode 2).
#include "common.h"
#include "mfma_util.h"

namespace sh {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));   // staging registers: native vectors stay in registers

__device__ __forceinline__ u32x4 scale_chunk4(u32x4 c, float g) {
  u32x4 o;
  o.x = scale_pair(c.x, g);
  o.y = scale_pair(c.y, g);
  o.z = scale_pair(c.z, g);
  o.w = scale_pair(c.w, g);
  return o;
}

struct PpCfg {
  static constexpr int BM = 256, BN = 256, BK = 64;
  static constexpr int LDA = BK + 8;
  static constexpr int LDB_NT = BK + 8, LDB_NN = BN + 32;
  static constexpr int A_ELEMS = BM * LDA;
  static constexpr int B_ELEMS = BN * LDB_NT;   // == BK * LDB_NN
  static constexpr int STAGE = A_ELEMS + B_ELEMS;
  static constexpr size_t lds_bytes() { return (size_t)2 * STAGE * 2 + BM * 4 + BM * 8 * 4 + 8 * 8; }
};
static_assert(PpCfg::BN * PpCfg::LDB_NT == PpCfg::BK * PpCfg::LDB_NN, "both B layouts fill the same area");

// PAIR: the tile's 256 columns are two adjacent heads of 128 columns each (dense queries / keys)
template <bool BNT, int TAG, int SEG>
__global__ __launch_bounds__(512, 1) void pp_row_gemm_kernel(RowGemmArgs a) {
  constexpr int BM = PpCfg::BM, BN = PpCfg::BN, BK = PpCfg::BK;
  constexpr int LDA = PpCfg::LDA, LDB = BNT ? PpCfg::LDB_NT : PpCfg::LDB_NN;
  constexpr int A_ELEMS = PpCfg::A_ELEMS, STAGE = PpCfg::STAGE;
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  int* ids = (int*)(smem + 2 * STAGE);
  float* gsc = (float*)(ids + BM);        // SEG 1: [row][segment]
  long* bseg = (long*)(gsc + BM * 8);     // SEG 1: B offset of each segment's expert

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int grp = wave >> 2;
  const int wm = grp * 128, wn = (wave & 3) * 64;
  const int r = lane & 31, g = lane >> 5;
  const bool pair = a.Nc < BN;            // two heads of 128 columns side by side

  // ---- which tile ------------------------------------------------------------------------
  const int ncol = pair ? 1 : a.Nc / BN;
  int h, e = 0, row0, rows, ct, w, slot;
  if constexpr (SEG == 1) {
    decode_block(blockIdx.x, ncol, w, slot);
    ct = slot;
    const int tph = (a.M + BM - 1) / BM + a.E;
    h = w / tph;
    if (h >= a.heads) return;
    if (!find_tile_wave(a.offsets + (long)h * (a.E + 1), a.E, BM, w % tph, lane, e, row0, rows)) return;
  } else {
    const int hunits = pair ? a.heads / 2 : a.heads;
    decode_block(blockIdx.x, hunits * ncol, w, slot);
    h = (slot / ncol) * (pair ? 2 : 1);
    ct = slot % ncol;
    row0 = w * BM;
    if (row0 >= a.M) return;
    rows = a.M - row0 < BM ? a.M - row0 : BM;
  }
  const bool second = a.hsplit > 0 && h >= a.hsplit;
  const int hh = second ? h - a.hsplit : h;
  const int nseg = SEG ? a.nseg : 1;

  if constexpr (SEG == 1) {
    float gv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = tid + u * 512, rr = t / nseg, p = t % nseg;
      gv[u] = 0.f;
      if (t < BM * nseg && rr < rows) gv[u] = a.segate[(long)h * a.gate_hstride + (long)(row0 + rr) * nseg + p];
    }
    int idv = -1;
    if (tid < rows) idv = a.perm[(long)h * a.M + row0 + tid];
    long bs = 0;
    if (tid < nseg) bs = (long)hh * a.b_hstride + (long)a.set_experts[e * 8 + tid] * a.b_estride;
    if (tid < BM) ids[tid] = idv;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int t = tid + u * 512;
      if (t < BM * nseg) gsc[(t / nseg) * 8 + t % nseg] = gv[u];
    }
    if (tid < nseg) bseg[tid] = bs;
  } else {
    if (tid < BM) ids[tid] = tid < rows ? row0 + tid : -1;
  }
  __syncthreads();

  const unsigned short* A = (const unsigned short*)a.A;
  const unsigned short* B0 = (const unsigned short*)(second ? a.B2 : a.B) + (SEG ? 0 : (long)hh * a.b_hstride);
  const int n0 = ct * BN;
  const int nks = a.K / BK;            // K steps per segment
  const int nk = nks * nseg;

  // ---- load plan: 4 A pieces and 4 B pieces of 16 bytes per thread and K step ------------
  // A: piece i is row (tid / 8) + 64 i, k piece tid % 8; rows past the tile's end repeat its first row
  // (their products are never stored).  One 32-bit byte offset per piece, the K step moves a uniform base.
  unsigned a_voff[4];
  const int a_lds0 = (tid >> 3) * LDA + (tid & 7) * 8;
  {
    const unsigned inv_adiv = div_magic(a.a_div);
    const int first = ids[0];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int id = ids[(tid >> 3) + 64 * i];
      id = id < 0 ? first : id;
      a_voff[i] = (unsigned)(((long)div_by(id, inv_adiv) * a.lda + (long)hh * a.a_hoff + (tid & 7) * 8) * 2);
    }
  }
  // B: n contiguous (k rows (tid / 32) + 16 i, column piece tid % 32) or k contiguous (like A).
  unsigned b_voff;
  int b_lds0;
  long b_istep;   // elements between a thread's consecutive pieces
  if constexpr (BNT) {
    b_voff = (unsigned)(((long)(n0 + (tid >> 3)) * a.sbn + (tid & 7) * 8) * 2);
    b_lds0 = (tid >> 3) * LDB + (tid & 7) * 8;
    b_istep = 64l * a.sbn;
  } else {
    const int nc = (tid & 31) * 8;
    const long col = pair ? (long)(nc >> 7) * a.b_hstride + (nc & 127) : (long)(n0 + nc);
    b_voff = (unsigned)(((long)(tid >> 5) * a.sbk + col) * 2);
    b_lds0 = (tid >> 5) * LDB + nc;
    b_istep = 16l * a.sbk;
  }

  // uniform operand bases of K step `it`
  auto a_base = [&](int it) -> const unsigned short* {
    const int seg = SEG ? it / nks : 0, k0 = (SEG ? it % nks : it) * BK;
    if constexpr (SEG == 2) return A + (long)(seg / a.seg_split) * a.a_wstride + (long)(seg % a.seg_split) * a.a_sstride + k0;
    if constexpr (SEG == 3) return (const unsigned short*)a.segd[seg].A + k0;
    return A + k0;
  };
  auto b_base = [&](int it) -> const unsigned short* {
    const int seg = SEG ? it / nks : 0, k0 = (SEG ? it % nks : it) * BK;
    const unsigned short* Bp = B0;
    if constexpr (SEG == 1) {   // the same value in every lane: make it a scalar
      const long o = bseg[seg];
      const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)o), hi = __builtin_amdgcn_readfirstlane((unsigned)(o >> 32));
      Bp = B0 + (long)(((unsigned long)hi << 32) | lo);
    }
    if constexpr (SEG == 2) {
      const int which = seg / a.seg_split;
      Bp = (const unsigned short*)(which == 0 ? a.B : which == 1 ? a.B2 : a.B3) + (long)(seg % a.seg_split) * a.b_sstride;
    }
    if constexpr (SEG == 3) Bp = (const unsigned short*)a.segd[seg].B;
    return BNT ? Bp + k0 : Bp + (long)k0 * a.sbk;
  };
  // SEG 3: the gates of the step's segment for the thread's four rows travel with the A pieces
  const unsigned g_voff = SEG == 3 ? (unsigned)(((long)(row0 + (tid >> 3)) * a.gld) * 4) : 0u;
  auto load_a = [&](u32x4 (&ra)[4], float (&rg)[4], int it) {
    const char* p = (const char*)a_base(it);
#pragma unroll
    for (int i = 0; i < 4; ++i) ra[i] = *(const u32x4*)(p + a_voff[i]);
    if constexpr (SEG == 3) {
      const int gcol = a.segd[it / nks].gcol;
      if (gcol >= 0) {
        const char* gp = (const char*)(a.gtab + gcol);
#pragma unroll
        for (int i = 0; i < 4; ++i) rg[i] = *(const float*)(gp + (long)i * 64 * a.gld * 4 + g_voff);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) rg[i] = 1.f;
      }
    }
  };
  auto load_b = [&](u32x4 (&rb)[4], int it) {
    const unsigned short* p = b_base(it);
#pragma unroll
    for (int i = 0; i < 4; ++i) rb[i] = *(const u32x4*)((const char*)(p + i * b_istep) + b_voff);
  };
  auto store_a = [&](const u32x4 (&ra)[4], const float (&rg)[4], int stage, int it) {
    unsigned short* As = smem + stage * STAGE;
    const int seg = SEG == 1 ? it / nks : 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      u32x4 v = ra[i];
      // expert sets: the row's gate for this segment's expert, applied on the way into LDS
      if constexpr (SEG == 1) v = scale_chunk4(v, gsc[((tid >> 3) + 64 * i) * 8 + seg]);
      if constexpr (SEG == 3) v = scale_chunk4(v, rg[i]);
      *(u32x4*)(&As[a_lds0 + i * 64 * LDA]) = v;
    }
  };
  auto store_b = [&](const u32x4 (&rb)[4], int stage) {
    unsigned short* Bs = smem + stage * STAGE + A_ELEMS;
#pragma unroll
    for (int i = 0; i < 4; ++i) *(u32x4*)(&Bs[b_lds0 + i * (BNT ? 64 : 16) * LDB]) = rb[i];
  };

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.f;

  bf16x8 fa[2][4], fb[2][2];
  auto read_frags = [&](int stage, int half) {
    const unsigned short* As = smem + stage * STAGE;
    const unsigned short* Bs = As + A_ELEMS;
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      const int kk = half * 32 + k2 * 16;
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[k2][i] = frag_rowmajor(&As[(wm + i * 32 + r) * LDA + kk + 8 * g]);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if constexpr (BNT)
          fb[k2][j] = frag_rowmajor(&Bs[(wn + j * 32 + r) * LDB + kk + 8 * g]);
        else
          fb[k2][j] = frag_transposed(Bs, LDB, kk + 8 * g, wn + j * 32, lane);
      }
    }
  };
  auto mma = [&]() {
    __builtin_amdgcn_s_setprio(2);
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[k2][i], fb[k2][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
  };
  // end of a phase: LDS traffic of this wave done, every wave of the work-group arrives (global loads stay in flight)
  auto phase_end = [&]() {
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    __builtin_amdgcn_sched_barrier(0);
  };

  // Every wave passes the same number of barriers: 1 + 4 nk + 1, the extra one before the loop for the second
  // group and after it for the first.  Stage (it+1)&1 is written in the two memory phases of step `it`
  // (A in the first, B in the second), a phase after the last read of its previous content (step it-1's
  // second memory phase of the second group) and a phase before the first read of the new one.
  u32x4 ra[4], rb[4];
  float rg[4] = {1.f, 1.f, 1.f, 1.f};
  load_a(ra, rg, 0);
  load_b(rb, 0);
  store_a(ra, rg, 0, 0);
  store_b(rb, 0);
  if (nk > 1) {
    load_a(ra, rg, 1);
    load_b(rb, 1);
  }
  __syncthreads();
  if (grp == 1) phase_end();
  for (int it = 0; it < nk; ++it) {
    const int st = it & 1;
    read_frags(st, 0);
    if (it + 1 < nk) store_a(ra, rg, st ^ 1, it + 1);
    if (it + 2 < nk) load_a(ra, rg, it + 2);
    phase_end();
    mma();
    phase_end();
    read_frags(st, 1);
    if (it + 1 < nk) store_b(rb, st ^ 1);
    if (it + 2 < nk) load_b(rb, it + 2);
    phase_end();
    mma();
    phase_end();
  }
  if (grp == 0) phase_end();

  // ---- epilogue -------------------------------------------------------------------------
  const unsigned inv_cdiv = div_magic(a.c_div);
  char* Cb = (char*)(second ? a.C2 : a.C);
  if (a.mode == STORE_T) {
    // each wave stages 32 rows x 64 columns of its tile in LDS (the operand stages are dead: the loop ends with
    // a barrier of all waves), then stores 16-byte pieces along the rows; the staging area is the wave's own
    constexpr int LDC = 64 + 8;
    unsigned short* Cs = smem + wave * 32 * LDC;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int lr = 8 * (q >> 2) + 4 * g + (q & 3);
#pragma unroll
        for (int j = 0; j < 2; ++j) Cs[lr * LDC + j * 32 + r] = f32_to_bf16(acc[i][j][q]);
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = lane + u * 64;
        const int lr = c >> 3, cc = (c & 7) * 8;
        const int id = ids[wm + i * 32 + lr];
        if (id < 0) continue;
        const long crow = (long)div_by(id, inv_cdiv) * a.ldc + (long)hh * a.c_hoff;
        *(uint4*)((unsigned short*)Cb + crow + n0 + wn + cc) = *(const uint4*)(&Cs[lr * LDC + cc]);
      }
    }
    return;
  }
  // fp32 output
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int id = ids[wm + i * 32 + 8 * (q >> 2) + 4 * g + (q & 3)];
      if (id < 0) continue;
      const long crow = (long)div_by(id, inv_cdiv) * a.ldc + (long)hh * a.c_hoff;
#pragma unroll
      for (int j = 0; j < 2; ++j) ((float*)Cb)[crow + n0 + wn + j * 32 + r] = acc[i][j][q];
    }
}

static bool pp_aligned(const void* p) { return ((uintptr_t)p % 16) == 0; }

bool pp_row_gemm_supported(const RowGemmArgs& a) {
  const bool nt = a.sbk == 1;
  if (!nt && a.sbn != 1) return false;
  if (a.perm && a.seg_mode != 1) return false;   // gathered rows only as expert sets
  if (a.gate) return false;
  if (a.mode != STORE_T && a.mode != STORE_F32) return false;
  if (a.K < 64 || a.K % 64 != 0 || a.a_div != 1 || a.c_div != 1) return false;
  const bool pair = a.Nc == 128 && a.seg_mode == 0 && !nt && a.E == 1 && a.heads % 2 == 0 && a.hsplit % 2 == 0 && a.c_hoff == 128;
  if (!pair && a.Nc % 256 != 0) return false;
  // 16-byte pieces everywhere
  bool ok = (a.seg_mode == 3 || (pp_aligned(a.A) && pp_aligned(a.B))) && pp_aligned(a.C) && a.lda % 8 == 0 && a.a_hoff % 8 == 0 && a.b_hstride % 8 == 0 &&
            a.b_estride % 8 == 0 && a.ldc % 8 == 0 && a.c_hoff % 8 == 0;
  ok = ok && (nt ? a.sbn % 8 == 0 : a.sbk % 8 == 0);
  if (a.hsplit > 0) ok = ok && pp_aligned(a.B2) && pp_aligned(a.C2);
  if (a.seg_mode == 2) {
    ok = ok && a.B2 && pp_aligned(a.B2) && a.a_sstride % 8 == 0 && a.a_wstride % 8 == 0 && a.b_sstride % 8 == 0 && a.seg_split > 0 &&
         a.nseg <= 3 * a.seg_split && (a.nseg <= 2 * a.seg_split || (a.B3 && pp_aligned(a.B3))) && a.heads == 1 && a.E == 1;
  }
  if (a.seg_mode == 3) {
    ok = ok && a.nseg >= 1 && a.nseg <= MAX_SEGD && a.heads == 1 && a.E == 1 && a.M % 256 == 0 && a.hsplit == 0;
    for (int p = 0; ok && p < a.nseg; ++p)
      ok = a.segd[p].A && a.segd[p].B && pp_aligned(a.segd[p].A) && pp_aligned(a.segd[p].B) && (a.segd[p].gcol < 0 || (a.gtab && a.segd[p].gcol < a.gld));
  }
  if (a.seg_mode == 1) {
    ok = ok && a.nseg >= 1 && a.nseg <= 8 && a.E <= 128 && a.perm && a.segate && a.set_experts;
    // 256-row tiles pay off when a set's rows fill several of them
    ok = ok && (long)a.M >= 1024l * a.E;
  } else {
    ok = ok && a.M >= 2048;
  }
  if (!ok) return false;
  // one 32-bit byte offset per piece: every operand element the launch can touch lies below 4 GiB
  const long a_elems = (long)a.M * a.lda + (long)a.heads * a.a_hoff + (a.seg_mode == 2 ? 3 * a.a_wstride + a.seg_split * a.a_sstride : 0) + a.K;
  const long b_elems = nt ? (long)a.Nc * a.sbn + a.K + 2 * a.b_hstride : (long)a.K * a.sbk + a.Nc + 2 * a.b_hstride;
  if (a_elems * 2 >= (1l << 32) || b_elems * 2 >= (1l << 32)) return false;
  switch (a.tag * 4 + a.seg_mode) {
    case TAG_QK_PROJ * 4 + 0: return !nt;
    case TAG_O_EXPERTS * 4 + 1: return !nt;
    case TAG_V_DGRAD * 4 + 1: return nt;
    case TAG_QK_DGRAD * 4 + 2: return nt;
    case TAG_O_EXPERTS * 4 + 3: return !nt;
    case TAG_QK_DGRAD * 4 + 3: return nt;
    default: return false;
  }
}

template <bool BNT, int TAG, int SEG>
static void launch_pp(const RowGemmArgs& a, hipStream_t s) {
  const bool pair = a.Nc < PpCfg::BN;
  const int ncol = pair ? 1 : a.Nc / PpCfg::BN;
  dim3 g;
  if (SEG == 1) {
    const int tph = (a.M + PpCfg::BM - 1) / PpCfg::BM + a.E;
    g = dim3(grid_windows(a.heads * tph, ncol));
  } else {
    g = dim3(grid_windows((a.M + PpCfg::BM - 1) / PpCfg::BM, (pair ? a.heads / 2 : a.heads) * ncol));
  }
  auto kern = pp_row_gemm_kernel<BNT, TAG, SEG>;
  static bool raised = false;   // per instantiation
  if (!raised) {
    (void)hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)PpCfg::lds_bytes());
    raised = true;
  }
  kern<<<g, 512, PpCfg::lds_bytes(), s>>>(a);
}

void launch_pp_row_gemm(const RowGemmArgs& a, hipStream_t s) {
  switch (a.tag * 4 + a.seg_mode) {
    case TAG_QK_PROJ * 4 + 0: return launch_pp<false, TAG_QK_PROJ, 0>(a, s);
    case TAG_O_EXPERTS * 4 + 1: return launch_pp<false, TAG_O_EXPERTS, 1>(a, s);
    case TAG_V_DGRAD * 4 + 1: return launch_pp<true, TAG_V_DGRAD, 1>(a, s);
    case TAG_QK_DGRAD * 4 + 2: return launch_pp<true, TAG_QK_DGRAD, 2>(a, s);
    case TAG_O_EXPERTS * 4 + 3: return launch_pp<false, TAG_O_EXPERTS, 3>(a, s);
    case TAG_QK_DGRAD * 4 + 3: return launch_pp<true, TAG_QK_DGRAD, 3>(a, s);
    default: return;
  }
}

}  // namespace sh
