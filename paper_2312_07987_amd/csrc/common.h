// Internal declarations shared by the HIP translation units of libswitchhead.
// Nothing here is part of the C ABI (that is include/switchhead.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sh {

// ----------------------------------------------------------------------------------------
// storage types
// ----------------------------------------------------------------------------------------
struct bf16_t {
  unsigned short v;
};

__device__ __forceinline__ float bf16_to_f32(unsigned short v) { return __uint_as_float(((unsigned)v) << 16); }

// round-to-nearest-even (the hardware conversion of gfx950)
__device__ __forceinline__ unsigned short f32_to_bf16(float f) { return __builtin_bit_cast(unsigned short, (__bf16)f); }
// two floats -> packed bf16 pair (lo in bits 0..15)
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  bf16x2_t v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(unsigned, v);
}

__device__ __forceinline__ float ld(const float* p, long i) { return p[i]; }
__device__ __forceinline__ float ld(const bf16_t* p, long i) { return bf16_to_f32(p[i].v); }
__device__ __forceinline__ void st(float* p, long i, float v) { p[i] = v; }
__device__ __forceinline__ void st(bf16_t* p, long i, float v) { p[i].v = f32_to_bf16(v); }

// ----------------------------------------------------------------------------------------
// Grouped row GEMM:   C[crow, n] (op)= scale * sum_k A[arow, k] * B_g[k, n]
//
// Rows come either from an expert-sorted permutation (perm != NULL: head h owns positions
// [h*M, (h+1)*M) of perm; expert e of head h owns positions offsets[h*(E+1)+e] ..
// offsets[h*(E+1)+e+1]; a position holds an assignment id a = token*k + slot) or from the
// identity (perm == NULL: every head covers rows a = 0..M-1, E must be 1).
//   arow = a / a_div,  crow = a / c_div,  scale = gate ? gate[h*gate_hstride + a] : 1
//   A[arow*lda + h*a_hoff + k],  B[h*b_hstride + e*b_estride + k*sbk + n*sbn],
//   C[crow*ldc + h*c_hoff + n]
// ----------------------------------------------------------------------------------------
enum { STORE_T = 0, STORE_F32 = 1, ATOMIC_F32 = 2, STORE_F64 = 3 };

// Which step of the layer a launch serves.  The MFMA kernels are instantiated once per tag so
// that a profiler shows one kernel name per step; the arithmetic is the same for every tag.
enum {
  TAG_GENERIC = 0,
  TAG_QK_PROJ, TAG_V_EXPERTS, TAG_O_EXPERTS,   // forward row GEMMs
  TAG_O_DGRAD, TAG_V_DGRAD, TAG_QK_DGRAD,      // backward row GEMMs
  TAG_O_WGRAD, TAG_V_WGRAD, TAG_QK_WGRAD,      // weight gradients
  TAG_ROUTER                                   // router logits: fp32 partial sums of 64 terms, added up in fp64
};

// Epilogue of the router logits GEMM (TAG_ROUTER): the selection of Sec. 2.2's router equations on the
// tile's logits, see router_select.h.  Launch head h is router side h.
struct RouterSelect {
  const float* b[2];            // logit bias per side or NULL
  const float* wnorm2;          // [side][H*E] squared column norms
  int* idx;                     // [side][H][N][k]
  float* gate;
  const void* x;                // bf16 [N][dm]
  const unsigned short* Wt;     // [side][H*E][dmp] router columns as vectors
  double* Z;                    // [side][N][H*E] fp64 logits of the rechecked entries
  int N, kstep, H, E, k, dm, dmp;
};

// One segment of a concatenated reduction with per-row gates (segment mode 3): the segment's A columns start at
// A (rows lda apart, shared by all segments), its B matrix at B (strides sbk / sbn shared), and row n of A
// is scaled by gtab[n * gld + gcol] before it is multiplied (gcol < 0: not scaled).
struct SegDesc {
  const void* A;
  const void* B;
  int gcol;
  int pad_;
};
enum { MAX_SEGD = 40 };

struct RowGemmArgs {
  const int* perm;
  const int* offsets;
  int heads, E, M;
  int a_div, c_div;
  const void* A;
  long lda, a_hoff;
  const void* B;
  long b_hstride, b_estride;
  int sbk, sbn;
  void* C;
  long ldc, c_hoff;
  const float* gate;
  long gate_hstride;
  int K, Nc;
  int mode;
  int tag;
  int max_group_rows;   // upper bound of the rows of one group (tokens per call)
  // Second operand set: heads h >= hsplit (hsplit > 0) use B2 / C2 with head index h - hsplit
  // (queries and keys projected by one launch).
  const void* B2;
  const void* B3;
  void* C2;
  int hsplit;
  // Segmented reduction, seg_mode:
  //  1  expert sets: perm holds token ids sorted by expert set, offsets the nsets+1 set
  //     boundaries per head (E = nsets); the reduction runs over nseg = k segments of length
  //     K: segment p reads the A row of sorted position r scaled by
  //     segate[h*gate_hstride + r*nseg + p] against B of expert set_experts[set*8 + p].
  //  2  concatenation: segment p reads A columns (p/seg_split)*a_wstride + (p%seg_split)*a_sstride
  //     against (B, B2 or B3 for p/seg_split = 0, 1, 2) + (p%seg_split)*b_sstride.
  int seg_mode, nseg, experts;
  const int* set_experts;
  // TAG_ROUTER only: the selection that consumes the logits in the kernel's epilogue (C is not written)
  RouterSelect rsel;
  const float* segate;
  int seg_split;
  long a_sstride, a_wstride, b_sstride;
  //  3  gated concatenation (token-ordered rows, M a multiple of 256): nseg segments of length K described by
  //     segd[]; the expert projections whose experts sit on the reduction side (Sec. 2.2, the y equation, and
  //     the value experts' input gradient) run over ALL experts of every head this way, an unselected expert
  //     having gate 0, so that heads and experts are summed in one accumulator and the output is written once.
  const float* gtab;
  int gld;
  SegDesc segd[MAX_SEGD];
};

// ----------------------------------------------------------------------------------------
// Grouped weight-gradient GEMM (reduction over the rows of a group):
//   dW_g[i, j] += sum_{rows a of group g} scale * A[arow, i] * Bm[brow, j]
//   A[arow*lda + h*a_hoff + i] (i < Ka),  Bm[brow*ldb + h*b_hoff + j] (j < Kb),
//   dW[h*w_hstride + e*w_estride + i*swa + j]   fp32, atomic add (zeroed by the caller).
// ----------------------------------------------------------------------------------------
struct WgradArgs {
  const int* perm;
  const int* offsets;
  int heads, E, M;
  int a_div, b_div;
  const void* A;
  long lda, a_hoff;
  int Ka;
  const void* Bm;
  long ldb, b_hoff;
  int Kb;
  float* dW;
  long w_hstride, w_estride;
  int swa;
  const float* gate;
  long gate_hstride;
  int chunk;  // rows reduced by one block
  int tag;
  int max_group_rows;  // upper bound of the rows of one group (tokens per call)
  // Further operand sets (hsplit > 0): head h belongs to set h / hsplit with head index h % hsplit;
  // set 1 uses Bm2 / dW2, set 2 (MFMA kernel with partial sums only) Bm3 / dW3.
  const void* Bm2;
  float* dW2;
  int hsplit;
  const void* Bm3;
  float* dW3;
  // Deterministic reduction (MFMA kernel): if partial != NULL every block stores the partial
  // sum of its chunk to partial[((h*E + e)*max_chunks + chunk)*Ka*Kb + i*Kb + j] and
  // launch_wgrad_reduce adds the chunks of each group into dW (plain stores, no zero fill).
  float* partial;
  int max_chunks;
  int scale_b;   // apply the gate to the rows of Bm instead of A (same product, fewer elements to scale)
  // Atomic path only: columns j >= kb_store are computed (Bm rows are read Kb wide, e.g. zero padded
  // to a multiple of 8) but not stored; 0 means Kb.
  int kb_store;
  // Atomic path of the MFMA kernel only (hsplit must be 0): columns j >= col_split belong to a second
  // output dW2 (same shape and swa), as its columns j - col_split; kb_store bounds each block.
  int col_split;
};
void launch_wgrad_reduce(const WgradArgs& a, hipStream_t s);

// Finds the tile `tile` (of `bm` rows) among the E groups of one head.  Returns false when
// `tile` lies beyond the last tile.  off points at the head's E+1 offsets.
__device__ __forceinline__ bool find_tile(const int* off, int E, int bm, int tile, int& e, int& row0, int& rows) {
  for (e = 0; e < E; ++e) {
    int beg = off[e], end = off[e + 1];
    int nt = (end - beg + bm - 1) / bm;
    if (tile < nt) {
      row0 = beg + tile * bm;
      rows = end - row0 < bm ? end - row0 : bm;
      return true;
    }
    tile -= nt;
  }
  return false;
}

// ----------------------------------------------------------------------------------------
// Attention
//   Q, K, V, O: [N, H, dh] with N = B*T (row stride H*dh); lse: [B, H, T] fp32.
// ----------------------------------------------------------------------------------------
struct AttnArgs {
  const void *Q, *K, *V;
  void* O;
  float* lse;
  int B, T, H, dh, causal;
  float scale;  // 1/sqrt(dh)
  // queries per sequence; 0 = T.  With Tq < T the queries are the last Tq positions (cached context in
  // front): Q, O, lse have Tq rows per sequence, K, V have T, and query i sees keys <= i + (T - Tq).
  int Tq;
};

struct AttnBwdArgs {
  const void *Q, *K, *V, *dO;
  const float *lse, *delta;  // delta[N, H] = <dO, O>
  void *dQ, *dK, *dV;
  int B, T, H, dh, causal;
  float scale;
  int Tq;   // as in AttnArgs: Q, dO, dQ, lse, delta have Tq rows per sequence, K, V, dK, dV have T
  // Optional scratch for the score gradient dS^T[b][h][key][query] in bf16 (layout: attn_ds_dims).  If not NULL the
  // dK / dV kernel leaves dS there and dQ = dS K is a plain product that reads it back instead of recomputing the
  // scores and probabilities.  ds_ld: queries rounded up to 256; ds_per: elements per (b, h).
  void* dSt;
  int ds_ld;
  long ds_per;
};

// ----------------------------------------------------------------------------------------
// launchers (defined in routing.hip, simt.hip, mfma_*.hip); all enqueue on `s`
// ----------------------------------------------------------------------------------------
struct SetSortArgs;
struct RouterArgs {
  const void* x;          // [N, dm]
  const void* W[2];       // per side [dm, HE]; W[1] == NULL -> one side only
  const float* b[2];      // per side [HE] or NULL
  double* Z;              // [sides, N, HE] fp64 logits (scratch)
  int* idx;               // [sides, H, N, k]
  float* gate;            // [sides, H, N, k]
  int* perm;              // [sides, H, N*k]
  int* offsets;           // [sides, H, E+1]
  int* blockcnt;          // [sides*H, nblk, E] scratch
  int N, dm, H, E, k, sides;
  int bf16;
  // if not NULL (and for as many sides), launch_router_hybrid also sorts the tokens by expert set,
  // sharing the passes of the expert sort; the caller then skips launch_set_sort
  const SetSortArgs* sets;
  // if not NULL (launch_router_hybrid without `sets`, both sides routed on the same N tokens): the dense gate table
  // [sides][N][H*E] is written along the histogram pass
  float* gtab;
};
void launch_router(const RouterArgs& a, hipStream_t s);
// bf16 storage: fp32 matrix-core logits with an fp64 re-evaluation of every decision that
// is not provably safe (see routing.hip).  `scratch` needs router_hybrid_bytes() bytes.
size_t router_hybrid_bytes(int N, int dm, int H, int E, size_t* off7);
bool router_hybrid_supported(const RouterArgs& a);
void launch_router_hybrid(const RouterArgs& a, char* scratch, hipStream_t s);
void launch_dense_routing(int* idx, float* gate, int* perm, int* offsets, int N, int H, hipStream_t s);
int router_blocks(int N);  // token blocks used by the histogram/scatter kernels
// gtab[side][n][h*E+e] = gate of the selected experts, 0 elsewhere (idx, gate: [side][H][N][k], sides side_stride_in apart)
void launch_gate_table(const int* idx, const float* gate, float* gtab, int N, int H, int E, int k, int sides, long side_stride_in,
                       hipStream_t s);

// Sorting of tokens by expert set (see routing.hip).  nsets = C(E,k) <= 128.
struct SetSortArgs {
  const int* idx;      // [sides, H, N, k]
  const float* gate;   // [sides, H, N, k]
  int* setid;          // [sides, H, N] scratch
  float* gset;         // [sides, H, N, k] scratch: gates in ascending-expert order, by token
  float* gsort;        // [sides, H, N, k] the same gates in sorted (setperm) order
  int* setexp;         // [nsets, 8] the ascending experts of every set
  int* setperm;        // [sides, H, N] token ids sorted by set id (stable)
  int* setoff;         // [sides, H, nsets+1]
  int* blockcnt;       // [sides*H, nblk, nsets] scratch
  int N, H, k, E, nsets, sides;
};
void launch_set_sort(const SetSortArgs& a, hipStream_t s);

void launch_fill_f32(float* p, size_t n, float v, hipStream_t s);
void launch_zero4_f32(float* p0, size_t n0, float* p1, size_t n1, float* p2, size_t n2, float* p3, size_t n3, hipStream_t s);
void launch_cast_from_f32(const float* src, void* dst, size_t n, int bf16, hipStream_t s);
void launch_cast_to_f32(const void* src, float* dst, size_t n, int bf16, hipStream_t s);
// out[i] = sum_h part[h*hstride + i] (+ add32[i]) for bf16 part/out; n must be a multiple of 8
// Rotary position embedding (App. A.4 "RoPE Positional Encodings"; Su et al.): tab [T][dh/2] of (cos, sin); apply turns the pairs
// (2i, 2i+1) of every row of up to two [N, H, dh] tensors in place, position = n % T.
void launch_rope_table(float2* tab, int T, int dh, hipStream_t s);
// (T rows per sequence, the first of them at position pos0)
void launch_rope_apply(void* P0, void* P1, const float2* tab, long N, int T, int pos0, int H, int dh, int inverse, int bf16,
                       hipStream_t s);
// out [B, T, dm] (storage type) += add [B, Tq, dm] (fp32) on the last Tq rows of every sequence
void launch_add_query_rows(void* out, const float* add, long rows, int T, int Tq, int dm, int bf16, hipStream_t s);
// dW0[i][c] = T[i*ld + c], dW1[i][c] = T[i*ld + HEp + c] for c < HE (either output may be NULL)
// Also, if dbpart is not NULL: db_side[h*E + e] = the sum over the `nblk` block partials router_bwd left there.
void launch_router_wgrad_split(const float* T, float* dW0, float* dW1, int dm, int ld, int HE, int HEp, const float* dbpart,
                               int nblk, int E, float* db0, float* db1, hipStream_t s);
int router_bwd_blocks(int N);   // token blocks of launch_router_bwd
void launch_sum_heads(const void* part, const float* add32, void* out, size_t n, size_t hstride, int H, hipStream_t s);

// out[n,h,:] = sum_j gate[h][n*k+j] * slots[h][n*k+j][:]   (slots [H, N*k, dh], storage type T)
// dots[h][n*k+j] = <other[n,h,:], slots[h][n*k+j][:]>        (if dots != NULL)
// delta[n,h]     = <out[n,h,:], other[n,h,:]>                (if delta != NULL)
// out may be NULL (dots only).  out/other have storage type T, layout [N, H, dh].
struct SlotArgs {
  const void* slots;
  const float* gate;
  const void* other;
  void* out;
  float* dots;
  float* delta;
  int N, H, k, dh;
  int dots_add;   // 1: dots[] += the row dots instead of being overwritten
};
void launch_slot_combine(const SlotArgs& a, int bf16, hipStream_t s);

// dz[n, side*HE + h*E + e] = dg*g*(1-g) at selected entries, 0 elsewhere.  With `shared`
// there is one side and dg = dgate[0] + dgate[1].  dz has storage type T, [N, sides*HE];
// the bias gradients are summed from the unrounded fp32 values.
struct RouterBwdArgs {
  const int* idx;       // [2 or 1, H, N, k]
  const float* gate;    // same
  const float* dgate;   // [2, H, N, k]
  void* dz;             // [N][ld]: side s owns columns s*side_stride .. +HE, the rest of its stride is zeroed
  float* db[2];         // per side [HE] or NULL, atomic add (zeroed by caller)
  float* dbpart;        // if not NULL: no atomics; block b of (side, head) sh stores its E sums at
                        // dbpart[(sh * blocks + b) * E + e] and launch_router_wgrad_split adds them up
  int N, H, E, k, sides, shared;
  int ld, side_stride;
  int pad_to;   // columns sides*side_stride .. pad_to-1 of every row are zeroed too (0: none)
  // Rides along (bf16 only, if wide_out is not NULL): both routers' weights side by side as
  // wide_out[d_model][wide_width], column side*side_stride + c = W_side[i][c], zeros elsewhere
  // (what launch_pack_router_wide writes), spread over the launch's threads.
  const void* W[2];
  void* wide_out;
  int dm, wide_width;
};
void launch_router_bwd(const RouterBwdArgs& a, int bf16, hipStream_t s);

// Step profiler (host.hip): when enabled, records an event on `st`; the time up to the next mark is
// booked under `label` (a string literal; NULL closes the last step).
void prof_mark(hipStream_t st, const char* label);
// both routers' weights as bf16 [side][d_model][HEp], columns HE..HEp-1 zero (W1 unused when sides == 1)
void launch_pack_router(const void* W0, const void* W1, void* Wp, int dm, int HE, int HEp, int sides, hipStream_t s);

void launch_simt_row_gemm(const RowGemmArgs& a, int bf16, hipStream_t s);
void launch_simt_wgrad(const WgradArgs& a, int bf16, hipStream_t s);
void launch_simt_attn_fwd(const AttnArgs& a, int bf16, hipStream_t s);
void launch_simt_attn_bwd(const AttnBwdArgs& a, int bf16, hipStream_t s);

// MFMA family (bf16 storage only).  *_supported() say whether a launch can be served.
bool mfma_row_gemm_supported(const RowGemmArgs& a);
int rg_kstep();  // terms summed in fp32 by one K step of the row GEMM
void launch_mfma_row_gemm(const RowGemmArgs& a, hipStream_t s);
// 256 x 256 tiles, eight waves in two alternating groups (mfma_pp.hip); launch_mfma_row_gemm routes to it
bool pp_row_gemm_supported(const RowGemmArgs& a);
void launch_pp_row_gemm(const RowGemmArgs& a, hipStream_t s);
bool mfma_wgrad_supported(const WgradArgs& a);
void launch_mfma_wgrad(const WgradArgs& a, hipStream_t s);
bool mfma_attn_supported(int T, int dh);
// The score-gradient scratch of launch_mfma_attn_bwd: per (sequence, head) the blocks of 128 keys follow each other; block t
// holds, for each of its keys, the queries from ds_block_start(t) on (under a causal mask earlier queries see none of the
// block's keys), i.e. rows of ld - ds_block_start(t) elements.  Returns ld (queries rounded up to 256) and the elements
// per (sequence, head); false if this head width does not use the scratch.
bool attn_ds_dims(int T, int Tq, int dh, int causal, int* ld, long* per);
void launch_mfma_attn_fwd(const AttnArgs& a, hipStream_t s);
void launch_mfma_attn_bwd(const AttnBwdArgs& a, hipStream_t s);

}  // namespace sh
