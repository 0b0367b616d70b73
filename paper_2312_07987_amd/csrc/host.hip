// C ABI of libswitchhead (declared in include/switchhead.h): argument checks, workspace
// carving and the launch sequence of the forward and backward passes of the SwitchHead
// layer (arXiv 2312.07987, Sec. 2.2).  Nothing here allocates or synchronises.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <initializer_list>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/switchhead.h"
#include "common.h"

using namespace sh;

// Workspace of switchhead_forward_static: device memory that exists from the moment the code object is
// loaded on a GPU until the process ends, one copy per GPU.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels and copies get the address that call returns (static_scratch below).
static __device__ __align__(256) unsigned char scratch[SWITCHHEAD_STATIC_WORKSPACE_BYTES];

namespace {

thread_local char g_err[512] = "";
std::atomic<int> g_family{0};

sh_status fail(sh_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

// ---- per-step timing for benchmarks: one HIP event per mark on the launch stream ----------
struct ProfMark {
  const char* label;  // NULL closes the previous step
  hipEvent_t ev;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfMark> g_marks;
std::vector<hipEvent_t> g_event_pool;

void prof_mark_impl(hipStream_t st, const char* label) {
  if (!g_prof_on) return;
  std::lock_guard<std::mutex> lk(g_prof_mu);
  hipEvent_t ev;
  if (!g_event_pool.empty()) {
    ev = g_event_pool.back();
    g_event_pool.pop_back();
  } else if (hipEventCreate(&ev) != hipSuccess) {
    return;
  }
  if (hipEventRecord(ev, st) != hipSuccess) {
    g_event_pool.push_back(ev);
    return;
  }
  g_marks.push_back({label, ev});
}

}  // namespace

void sh::prof_mark(hipStream_t st, const char* label) { prof_mark_impl(st, label); }

namespace {

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

struct Layout {
  size_t total = 0, kept = 0;   // kept: bytes forward leaves for backward; the rest is scratch of one pass
  size_t idx, gate, perm, offsets, Q, K, V, ctx, lse, pV;          // saved by forward
  size_t pQ, pK;                                                   // per-slot query / key rows (expert Q/K only)
  size_t rope;                                                     // (cos, sin) table [T][dh/2] (rotary embedding only)
  size_t xq, accq;   // fewer queries than keys only: the query tokens' rows of x; their fp32 share of dx
  size_t Z, blockcnt, acc32;                                       // forward scratch
  size_t setid, gset, gsort, setexp, setperm, setoff, setcnt, yh;
  size_t gtab;                                                     // dense gate table [2][N][H*E] fp32 (gated-concatenation GEMMs)
  size_t wrt;                                                      // x^T dz of both routers [dm, dh] fp32 (fused with the Q/K weight gradient)
  size_t dR, wr3;                                                  // wide router dz rows [N, H*dh], routers packed [dm, dh]                 // expert-set path (bf16 only)
  size_t rh;                                                       // two-stage router scratch (bf16 only)
  size_t wpart;                                                    // per-chunk weight-gradient partial sums (bf16 only)
  size_t u, dctx, dQ, dK, dV, delta, dgate, dz;                    // backward scratch
  size_t dst;                                                      // score gradient dS^T of the attention backward (0: recomputed)
};

// number of k-subsets of E experts, saturating at MAX_SETS + 1
constexpr int MAX_SETS = 128;
// Rows reduced by one weight-gradient block.  Each block writes a partial sum of its output tile
// that a second kernel adds up, so chunks should be long, but short enough that the launch still
// fills the chip: about 480 blocks (256 CUs x 2 resident work-groups, a little slack for ragged
// groups), output tiles of 256 x 128, chunks of 256 .. 2048 rows in multiples of 64.
static int wgrad_chunk(size_t total_rows, size_t dm, size_t dh) {
  const size_t tiles = ((dm + 255) / 256) * ((dh + 127) / 128);
  const size_t units = 480 / tiles > 0 ? 480 / tiles : 1;
  size_t chunk = (total_rows + units - 1) / units;
  chunk = (chunk + 63) / 64 * 64;
  return (int)(chunk < 256 ? 256 : chunk > 2048 ? 2048 : chunk);
}
int count_sets(int E, int k) {
  long v = 1;
  for (int i = 1; i <= k; ++i) {
    v = v * (E - k + i) / i;
    if (v > MAX_SETS) return MAX_SETS + 1;
  }
  return (int)v;
}

sh_status check_shape(const sh_shape* s) {
  if (!s) return fail(SH_ERR_INVALID_ARG, "shape is NULL");
  if (s->B < 1 || s->T < 1 || s->d_model < 1 || s->nheads < 1 || s->d_head < 1 || s->E < 1 || s->k < 1)
    return fail(SH_ERR_INVALID_ARG, "every dimension must be >= 1 (B=%d T=%d d_model=%d nheads=%d d_head=%d E=%d k=%d)",
                s->B, s->T, s->d_model, s->nheads, s->d_head, s->E, s->k);
  if (s->k > s->E) return fail(SH_ERR_INVALID_ARG, "k=%d exceeds E=%d", s->k, s->E);
  if (s->dtype != SH_F32 && s->dtype != SH_BF16) return fail(SH_ERR_INVALID_ARG, "unknown dtype %d", s->dtype);
  if (s->causal != 0 && s->causal != 1) return fail(SH_ERR_INVALID_ARG, "causal must be 0 or 1");
  if (s->qk_experts != 0 && s->qk_experts != 1) return fail(SH_ERR_INVALID_ARG, "qk_experts must be 0 or 1");
  if (s->rope != 0 && s->rope != 1) return fail(SH_ERR_INVALID_ARG, "rope must be 0 or 1");
  if (s->T_q < 0 || s->T_q > s->T) return fail(SH_ERR_INVALID_ARG, "T_q=%d must lie in 0..T=%d", s->T_q, s->T);
  if (s->E > 64) return fail(SH_ERR_UNSUPPORTED, "E=%d exceeds the limit of 64", s->E);
  if (s->k > 8) return fail(SH_ERR_UNSUPPORTED, "k=%d exceeds the limit of 8", s->k);
  if (s->d_head > 256) return fail(SH_ERR_UNSUPPORTED, "d_head=%d exceeds the limit of 256", s->d_head);
  if (s->B > 65535 || s->nheads > 4096) return fail(SH_ERR_UNSUPPORTED, "B > 65535 or nheads > 4096");
  const long long N = (long long)s->B * s->T;
  if (N * s->k >= (1ll << 31) || N * s->d_model >= (1ll << 40) || N * s->nheads * s->d_head >= (1ll << 40))
    return fail(SH_ERR_UNSUPPORTED, "problem too large (B*T*k must stay below 2^31)");
  return SH_OK;
}

// Shapes whose output experts and input gradient run as gated concatenation (see gated_concat below): a property
// of the shape alone, so that the workspace layout and both passes agree on it.  Such shapes have no expert-set tables.
bool gated_shape(const sh_shape* s) {
  const long long N = (long long)s->B * s->T;
  const bool rect = s->T_q > 0 && s->T_q < s->T;
  return s->dtype == SH_BF16 && !rect && !s->qk_experts && s->d_head % 64 == 0 && s->d_model % 256 == 0 && N % 256 == 0 &&
         N >= 2048 && s->nheads * s->E + 2 * s->nheads + 1 <= MAX_SEGD && s->E <= 2 * s->k;
}

Layout make_layout(const sh_shape* s) {
  Layout L;
  const size_t N = (size_t)s->B * s->T, H = s->nheads, E = s->E, k = s->k, dh = s->d_head, dm = s->d_model;
  const size_t esz = s->dtype == SH_BF16 ? 2 : 4;
  size_t off = 0, kept = 0;
  // keep = true: forward leaves it for backward (and for get_routing / get_intermediates); false: scratch of one pass
  auto take = [&](size_t bytes, bool keep = false) {
    size_t o = off;
    off += align_up(bytes);
    if (keep) kept += align_up(bytes);
    return o;
  };
  L.idx = take(2 * H * N * k * 4, true);
  L.gate = take(2 * H * N * k * 4, true);
  L.perm = take(2 * H * N * k * 4, true);
  L.offsets = take(2 * H * (E + 1) * 4, true);
  L.Q = take(N * H * dh * esz, true);
  L.K = take(N * H * dh * esz, true);
  L.V = take(N * H * dh * esz, true);
  L.ctx = take(N * H * dh * esz, true);
  L.lse = take(N * H * 4, true);
  L.pV = take(H * N * k * dh * esz, true);   // the per-slot value rows: what the gates' gradient costs (the only kept part that grows with k)
  L.pQ = L.pK = 0;
  L.rope = s->rope ? take((size_t)s->T * (dh / 2 > 0 ? dh / 2 : 1) * 8, true) : 0;
  L.xq = L.accq = 0;
  if (s->T_q > 0 && s->T_q < s->T) {
    const size_t Nq = (size_t)s->B * s->T_q;
    L.xq = take(Nq * dm * esz, true);
    L.accq = take(Nq * dm * 4);
  }
  if (s->qk_experts) {
    L.pQ = take(H * N * k * dh * esz, true);
    L.pK = take(H * N * k * dh * esz, true);
  }
  L.Z = take(2 * N * H * E * 8);
  L.blockcnt = take(2 * H * (size_t)router_blocks((int)N) * E * 4);
  L.acc32 = take(N * dm * 4);
  L.u = take(H * N * k * dh * esz);
  L.dctx = take(N * H * dh * esz);
  L.dQ = take(N * H * dh * esz);
  L.dK = take(N * H * dh * esz);
  L.dR = take(N * H * dh * esz);   // directly behind dK, same size: a third operand set for the Q/K dgrad GEMM
  L.dV = take(N * H * dh * esz);
  L.wr3 = take(dm * dh * esz);
  L.wrt = take(dm * dh * 4);
  L.delta = take(N * H * 4);
  L.dgate = take(2 * H * N * k * 4);
  L.dz = take(N * 2 * ((H * E + 7) / 8 * 8) * esz);   // each side padded to a multiple of 8 columns
  if (s->dtype == SH_BF16 && count_sets(s->E, s->k) <= MAX_SETS && !gated_shape(s)) {
    const size_t ns = count_sets(s->E, s->k);
    L.setid = take(2 * H * N * 4);
    L.gset = take(2 * H * N * k * 4);
    L.gsort = take(2 * H * N * k * 4, true);
    L.setexp = take((size_t)MAX_SETS * 8 * 4, true);
    L.setperm = take(2 * H * N * 4, true);
    L.setoff = take(2 * H * (ns + 1) * 4, true);
    L.setcnt = take(2 * H * (size_t)router_blocks((int)N) * ns * 4);
    // partial sums of dx (y in the forward pass): one per head from the value experts, then either one
    // for the dense Q/K pair or one per head for each of the query and key experts, one for the routers
    L.yh = take(((s->qk_experts ? 3 * H : H + 1) + 1) * N * dm * esz);
  } else {
    L.setid = L.gset = L.gsort = L.setexp = L.setperm = L.setoff = L.setcnt = L.yh = 0;
  }
  L.rh = L.wpart = L.gtab = 0;
  if (s->dtype == SH_BF16) {
    L.gtab = take(2 * N * H * E * 4, true);
    // groups x chunks-per-group x one expert matrix, fp32 (the dense Q/K pair counts as 2H groups)
    const size_t groups = H * E > 2 * H + 1 ? H * E : 2 * H + 1;   // expert Q/K banks: H * E groups each, one at a time
    const size_t ce = wgrad_chunk(H * N * k, dm, dh), cd = wgrad_chunk(2 * H * N, dm, dh);
    const size_t cmin = ce < cd ? ce : cd;
    L.wpart = take(groups * ((N + cmin - 1) / cmin) * dm * dh * 4);
    size_t o7[7];
    L.rh = take(router_hybrid_bytes((int)N, (int)dm, (int)H, (int)E, o7));
  }
  // The score gradient of the attention backward, [B][H][keys][queries] bf16: the dK / dV kernel leaves it for the
  // dQ product instead of that kernel recomputing scores and probabilities.  Quadratic in T, so only up to 1 GiB.
  L.dst = 0;
  {
    int ld = 0;
    long per = 0;
    if (s->dtype == SH_BF16 && attn_ds_dims(s->T, s->T_q, (int)dh, s->causal, &ld, &per)) {
      const size_t bytes = (size_t)s->B * H * (size_t)per * 2;
      // It lives from the dK / dV kernel to the dQ product.  The fp32 accumulator of dx (first written after the
      // attention backward) and the per-slot rows of the output experts' dgrad (consumed before it), which lie next to
      // each other, are dead in between: the score gradient takes their place if it fits.
      if (L.u == L.acc32 + align_up(N * dm * 4) && bytes <= align_up(N * dm * 4) + align_up(H * N * k * dh * esz))
        L.dst = L.acc32;
      else if (bytes <= ((size_t)1 << 30))
        L.dst = take(bytes);
    }
  }
  L.total = off;
  L.kept = kept;
  return L;
}

struct Ctx {
  const sh_shape* s;
  Layout L;
  char* ws;
  hipStream_t st;
  int N, H, E, k, dh, dm, bf16;
  int Tq, Nq;   // queries per sequence and in all; Tq < T: only the last Tq positions are destinations
  bool rect;    // Tq < T
  bool dense, shared, qk_experts;
  bool aligned = true;   // every tensor pointer of the call is 16-byte aligned (the matrix-core kernels need it)
  int n(int side) const { return side ? Nq : N; }   // tokens of the source (0) / destination (1) side
  template <typename T>
  T* p(size_t off) const {
    return (T*)(ws + off);
  }
  // per-side routing tables (side 0 = source, 1 = destination)
  int* idx(int side) const { return p<int>(L.idx) + (size_t)side * H * N * k; }
  float* gate(int side) const { return p<float>(L.gate) + (size_t)side * H * N * k; }
  int* perm(int side) const { return p<int>(L.perm) + (size_t)side * H * N * k; }
  int* offsets(int side) const { return p<int>(L.offsets) + (size_t)side * H * (E + 1); }
};

sh_status make_ctx(Ctx& c, const sh_shape* s, const void* W_S, const void* W_D, const void* ws, size_t ws_bytes,
                   void* stream) {
  sh_status r = check_shape(s);
  if (r != SH_OK) return r;
  c.s = s;
  c.L = make_layout(s);
  if (!ws) return fail(SH_ERR_INVALID_ARG, "workspace is NULL");
  if (((uintptr_t)ws & 255) != 0) return fail(SH_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  if (ws_bytes < c.L.total)
    return fail(SH_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, c.L.total);
  c.ws = (char*)ws;
  c.st = (hipStream_t)stream;
  c.N = s->B * s->T;
  c.Tq = s->T_q > 0 ? s->T_q : s->T;
  c.Nq = s->B * c.Tq;
  c.rect = c.Tq != s->T;
  c.H = s->nheads;
  c.E = s->E;
  c.k = s->k;
  c.dh = s->d_head;
  c.dm = s->d_model;
  c.bf16 = s->dtype == SH_BF16;
  c.qk_experts = s->qk_experts != 0;
  c.dense = W_S == nullptr;
  c.shared = W_S != nullptr && W_D == nullptr;
  if (c.dense && (s->E != 1 || s->k != 1))
    return fail(SH_ERR_INVALID_ARG, "W_S is NULL (dense attention) but E=%d, k=%d; both must be 1", s->E, s->k);
  return SH_OK;
}

sh_status check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(SH_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return SH_OK;
}

bool use_mfma(const Ctx& c) { return c.bf16 && c.aligned && g_family.load() == 0; }

// the matrix-core kernels move 16-byte pieces: NULL counts as aligned
bool all_aligned16(std::initializer_list<const void*> ps) {
  for (const void* q : ps)
    if (((uintptr_t)q & 15) != 0) return false;
  return true;
}

void row_gemm(const Ctx& c, const RowGemmArgs& a) {
  if (use_mfma(c) && mfma_row_gemm_supported(a))
    launch_mfma_row_gemm(a, c.st);
  else
    launch_simt_row_gemm(a, c.bf16, c.st);
}

// Weight gradient of one step.  MFMA family: per-chunk partial sums + a reduction (deterministic,
// the outputs need no zero fill); otherwise atomic adds into zeroed outputs.
void wgrad(const Ctx& c, WgradArgs a, bool deterministic = true, bool zero = true) {
  if (use_mfma(c)) {
    WgradArgs b = a;
    if (deterministic) {
      b.partial = c.p<float>(c.L.wpart);
      b.max_chunks = (int)(((a.perm ? a.max_group_rows : a.M) + a.chunk - 1) / a.chunk);
    }
    if (b.partial && mfma_wgrad_supported(b)) {
      launch_mfma_wgrad(b, c.st);
      prof_mark(c.st, "bwd.wgrad_reduce");
      launch_wgrad_reduce(b, c.st);
      return;
    }
  }
  // atomic paths add into zeroed outputs
  const int h1 = a.hsplit > 0 ? a.hsplit : a.heads;
  const size_t kb = a.kb_store ? a.kb_store : a.Kb;
  if (zero) {
    launch_fill_f32(a.dW, (size_t)h1 * a.E * a.Ka * kb, 0.f, c.st);
    if (a.hsplit > 0) launch_fill_f32(a.dW2, (size_t)(a.heads - a.hsplit) * a.E * a.Ka * kb, 0.f, c.st);
  }
  if (use_mfma(c) && mfma_wgrad_supported(a)) {
    launch_mfma_wgrad(a, c.st);
    return;
  }
  if (a.hsplit > 0) {   // the plain kernels take one operand set at a time
    WgradArgs a1 = a, a2 = a;
    a1.heads = a.hsplit;
    a1.hsplit = 0;
    a2.heads = a.heads - a.hsplit;
    a2.hsplit = 0;
    a2.Bm = a.Bm2;
    a2.dW = a.dW2;
    launch_simt_wgrad(a1, c.bf16, c.st);
    launch_simt_wgrad(a2, c.bf16, c.st);
    return;
  }
  launch_simt_wgrad(a, c.bf16, c.st);
}

// rows taken through the expert-sorted permutation of one side
RowGemmArgs perm_rows(const Ctx& c, int side) {
  RowGemmArgs a{};
  a.perm = c.perm(side);
  a.offsets = c.offsets(side);
  a.heads = c.H;
  a.E = c.E;
  a.M = c.n(side) * c.k;
  a.max_group_rows = c.n(side);
  a.a_div = c.k;
  a.c_div = 1;
  return a;
}

// rows taken through the expert-set permutation of one side (one row per token and head)
RowGemmArgs set_rows(const Ctx& c, int side) {
  RowGemmArgs a{};
  const int ns = count_sets(c.E, c.k);
  a.perm = c.p<int>(c.L.setperm) + (size_t)side * c.H * c.N;
  a.offsets = c.p<int>(c.L.setoff) + (size_t)side * c.H * (ns + 1);
  a.heads = c.H;
  a.E = ns;
  a.M = c.n(side);
  a.a_div = 1;
  a.c_div = 1;
  a.max_group_rows = c.n(side);
  a.seg_mode = 1;
  a.nseg = c.k;
  a.experts = c.E;
  a.segate = c.p<float>(c.L.gsort) + (size_t)side * c.H * c.N * c.k;
  a.set_experts = c.p<int>(c.L.setexp);
  a.gate_hstride = (long)c.n(side) * c.k;
  return a;
}

// Whether the shape has expert-set tables at all.  Forward builds them whenever this holds, whichever
// kernel family runs, so that a backward call under another family (or with differently aligned
// pointers) never finds tables its forward call did not write.
// (shapes that run the gated concatenation sum heads and experts inside one accumulator: they have neither
// expert-set tables nor per-head partial sums, in the workspace layout as here)
bool set_tables(const Ctx& c) {
  return c.bf16 && !gated_shape(c.s) && count_sets(c.E, c.k) <= MAX_SETS && c.dm % 4 == 0 && c.dh % 4 == 0 &&
         ((size_t)c.N * c.dm) % 8 == 0 && ((size_t)c.Nq * c.dm) % 8 == 0;
}
bool sets_usable(const Ctx& c) { return use_mfma(c) && set_tables(c); }

// Whether the projections whose experts sit on the reduction side (output experts; the value experts' input
// gradient) run as ONE token-ordered GEMM over all E experts of every head, an unselected expert having gate 0:
// heads and experts are then summed inside the accumulator and y / dx are written once, instead of one bf16
// partial per head that another kernel adds up.  It multiplies E/k times the selected experts' work, so it is
// taken where that factor is at most 2 (and the shape fills the 256 x 256 tiles); else the expert-set path.
bool gated_concat(const Ctx& c) { return use_mfma(c) && gated_shape(c.s); }

RowGemmArgs identity_rows(const Ctx& c, int heads, int side = 0) {
  RowGemmArgs a{};
  a.heads = heads;
  a.E = 1;
  a.M = c.n(side);
  a.a_div = 1;
  a.c_div = 1;
  return a;
}

}  // namespace

extern "C" {

const char* switchhead_last_error(void) { return g_err; }
const char* switchhead_version(void) { return "0.1"; }

int32_t switchhead_set_kernel_family(int32_t family) { return g_family.exchange(family ? 1 : 0); }

sh_status switchhead_profile_enable(int32_t on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  g_prof_on = on != 0;
  for (auto& m : g_marks) g_event_pool.push_back(m.ev);
  g_marks.clear();
  return SH_OK;
}

int32_t switchhead_profile_read(char* labels, size_t labels_bytes, float* total_ms, int32_t* launches,
                                int32_t max_entries) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  std::vector<std::string> names;
  std::vector<float> ms;
  std::vector<int> cnt;
  for (size_t i = 0; i + 1 < g_marks.size(); ++i) {
    if (!g_marks[i].label) continue;
    if (hipEventSynchronize(g_marks[i + 1].ev) != hipSuccess) break;
    float t = 0.f;
    if (hipEventElapsedTime(&t, g_marks[i].ev, g_marks[i + 1].ev) != hipSuccess) continue;
    size_t j = 0;
    for (; j < names.size(); ++j)
      if (names[j] == g_marks[i].label) break;
    if (j == names.size()) {
      names.push_back(g_marks[i].label);
      ms.push_back(0.f);
      cnt.push_back(0);
    }
    ms[j] += t;
    cnt[j] += 1;
  }
  for (auto& m : g_marks) g_event_pool.push_back(m.ev);
  g_marks.clear();
  int32_t n = 0;
  size_t used = 0;
  if (labels && labels_bytes) labels[0] = 0;
  for (size_t j = 0; j < names.size() && n < max_entries; ++j) {
    if (labels) {
      if (used + names[j].size() + 2 > labels_bytes) break;
      memcpy(labels + used, names[j].c_str(), names[j].size());
      used += names[j].size();
      labels[used++] = '\n';
      labels[used] = 0;
    }
    if (total_ms) total_ms[n] = ms[j];
    if (launches) launches[n] = cnt[j];
    ++n;
  }
  return n;
}

size_t switchhead_workspace_bytes(const sh_shape* shape) {
  if (check_shape(shape) != SH_OK) return 0;
  return make_layout(shape).total;
}

sh_status switchhead_workspace_parts(const sh_shape* shape, size_t* kept_bytes, size_t* scratch_bytes) {
  sh_status r = check_shape(shape);
  if (r != SH_OK) return r;
  const Layout L = make_layout(shape);
  if (kept_bytes) *kept_bytes = L.kept;
  if (scratch_bytes) *scratch_bytes = L.total - L.kept;
  return SH_OK;
}

sh_status switchhead_forward(const sh_shape* shape, const void* x, const void* W_Q, const void* W_K, const void* W_V,
                             const void* W_O, const void* W_S, const void* W_D, const float* b_S, const float* b_D,
                             void* y, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Ctx c;
  sh_status r = make_ctx(c, shape, W_S, W_D, workspace, workspace_bytes, hip_stream);
  if (r != SH_OK) return r;
  if (!x || !W_Q || !W_K || !W_V || !W_O || !y) return fail(SH_ERR_INVALID_ARG, "x, W_Q, W_K, W_V, W_O, y must not be NULL");
  if (c.dense && W_D) return fail(SH_ERR_INVALID_ARG, "W_D given without W_S");
  c.aligned = all_aligned16({x, W_Q, W_K, W_V, W_O, W_S, W_D, y});
  const int N = c.N, H = c.H, E = c.E, k = c.k, dh = c.dh, dm = c.dm;
  const long hd = (long)H * dh;

  // step 1: routers, top-k, expert-sorted permutation (and, where the shape has them, the set-sorted
  // one: `tables`; `sets` says whether this call's kernels use them)
  const bool tables = set_tables(c);
  const bool sets = sets_usable(c);
  const bool gated = gated_concat(c);
  bool gtab_done = false;
  // the tables a path uses must have a place in the workspace layout (offset 0 is the top-k indices)
  if ((tables && (c.L.setperm == 0 || c.L.setid == 0 || c.L.gsort == 0)) || (gated && c.L.gtab == 0) || (sets && c.L.yh == 0))
    return fail(SH_ERR_UNSUPPORTED, "switchhead_forward: internal error, the workspace layout lacks a table this shape's path uses");
  bool sets_sorted = false;
  SetSortArgs sa{};
  if (tables) {
    sa.idx = c.idx(0);
    sa.gate = c.gate(0);
    sa.setid = c.p<int>(c.L.setid);
    sa.gset = c.p<float>(c.L.gset);
    sa.gsort = c.p<float>(c.L.gsort);
    sa.setexp = c.p<int>(c.L.setexp);
    sa.setperm = c.p<int>(c.L.setperm);
    sa.setoff = c.p<int>(c.L.setoff);
    sa.blockcnt = c.p<int>(c.L.setcnt);
    sa.N = N;
    sa.H = H;
    sa.k = k;
    sa.E = E;
    sa.nsets = count_sets(E, k);
    sa.sides = 2;
  }
  prof_mark(c.st, "fwd.router");
  const void* xq = x;   // the destination (query) tokens' rows of x
  if (c.rect) {
    // Fewer queries than keys: the query tokens' rows (the last T_q of every sequence) are copied into
    // one block, and each side is routed on its own tokens.  Shared selection evaluates the one router
    // on the query rows again, which gives the source side's numbers for those tokens.
    const size_t esz = c.bf16 ? 2 : 4, rowb = (size_t)dm * esz;
    xq = c.p<void>(c.L.xq);
    if (hipMemcpy2DAsync(c.p<void>(c.L.xq), (size_t)c.Tq * rowb, (const char*)x + (size_t)(shape->T - c.Tq) * rowb,
                         (size_t)shape->T * rowb, (size_t)c.Tq * rowb, (size_t)shape->B, hipMemcpyDeviceToDevice,
                         c.st) != hipSuccess)
      return fail(SH_ERR_HIP, "switchhead_forward: copy of the query rows failed");
    const int nblk = router_blocks(N), ns = count_sets(E, k);
    for (int side = 0; side < 2; ++side) {
      const int n = c.n(side);
      // this side's expert-set tables (the set sort of each side runs on its own tokens)
      SetSortArgs s1 = sa;
      if (tables) {
        s1.idx = c.idx(side);
        s1.gate = c.gate(side);
        s1.setid = sa.setid + (size_t)side * H * N;
        s1.gset = sa.gset + (size_t)side * H * N * k;
        s1.gsort = sa.gsort + (size_t)side * H * N * k;
        s1.setperm = sa.setperm + (size_t)side * H * N;
        s1.setoff = sa.setoff + (size_t)side * H * (ns + 1);
        s1.blockcnt = sa.blockcnt + (size_t)side * H * nblk * ns;
        s1.N = n;
        s1.sides = 1;
      }
      if (c.dense) {
        // (dense attention has one expert set, but the kernels of the set path still read its tables)
        launch_dense_routing(c.idx(side), c.gate(side), c.perm(side), c.offsets(side), n, H, c.st);
        if (tables) launch_set_sort(s1, c.st);
        continue;
      }
      const bool own = side == 1 && !c.shared;   // the destination side's own router
      RouterArgs ra{};
      ra.x = side ? xq : x;
      ra.W[0] = own ? W_D : W_S;
      ra.b[0] = own ? b_D : b_S;
      ra.Z = c.p<double>(c.L.Z) + (size_t)side * N * H * E;
      ra.idx = c.idx(side);
      ra.gate = c.gate(side);
      ra.perm = c.perm(side);
      ra.offsets = c.offsets(side);
      ra.blockcnt = c.p<int>(c.L.blockcnt) + (size_t)side * H * nblk * E;
      ra.N = n;
      ra.dm = dm;
      ra.H = H;
      ra.E = E;
      ra.k = k;
      ra.sides = 1;
      ra.bf16 = c.bf16;
      if (use_mfma(c) && router_hybrid_supported(ra)) {
        if (tables) ra.sets = &s1;
        launch_router_hybrid(ra, c.p<char>(c.L.rh), c.st);
      } else {
        launch_router(ra, c.st);
        if (tables) launch_set_sort(s1, c.st);
      }
    }
    sets_sorted = true;
  } else if (c.dense) {
    launch_dense_routing(c.idx(0), c.gate(0), c.perm(0), c.offsets(0), N, H, c.st);
  } else {
    RouterArgs ra{};
    ra.x = x;
    ra.W[0] = W_S;
    ra.W[1] = W_D;
    ra.b[0] = b_S;
    ra.b[1] = b_D;
    ra.Z = c.p<double>(c.L.Z);
    ra.idx = c.idx(0);
    ra.gate = c.gate(0);
    ra.perm = c.perm(0);
    ra.offsets = c.offsets(0);
    ra.blockcnt = c.p<int>(c.L.blockcnt);
    ra.N = N;
    ra.dm = dm;
    ra.H = H;
    ra.E = E;
    ra.k = k;
    ra.sides = c.shared ? 1 : 2;
    ra.bf16 = c.bf16;
    if (use_mfma(c) && router_hybrid_supported(ra)) {
      if (tables && !c.shared) {   // both sorts in the same launches
        ra.sets = &sa;
        sets_sorted = true;
      } else if (gated && !c.shared && !c.dense) {   // the dense gate table rides along the histogram pass
        ra.gtab = c.p<float>(c.L.gtab);
        gtab_done = true;
      }
      launch_router_hybrid(ra, c.p<char>(c.L.rh), c.st);
    } else {
      launch_router(ra, c.st);
    }
  }
  if ((c.dense || c.shared) && !c.rect) {
    // one selection serves both sides: the destination tables repeat the source tables
    const size_t n1 = (size_t)H * N * k * 4;
    (void)hipMemcpyAsync(c.idx(1), c.idx(0), n1, hipMemcpyDeviceToDevice, c.st);
    (void)hipMemcpyAsync(c.gate(1), c.gate(0), n1, hipMemcpyDeviceToDevice, c.st);
    (void)hipMemcpyAsync(c.perm(1), c.perm(0), n1, hipMemcpyDeviceToDevice, c.st);
    (void)hipMemcpyAsync(c.offsets(1), c.offsets(0), (size_t)H * (E + 1) * 4, hipMemcpyDeviceToDevice, c.st);
  }

  if (tables && !sets_sorted) {
    prof_mark(c.st, "fwd.set_sort");
    sa.idx = c.idx(0);
    sa.gate = c.gate(0);
    sa.setid = c.p<int>(c.L.setid);
    sa.gset = c.p<float>(c.L.gset);
    sa.gsort = c.p<float>(c.L.gsort);
    sa.setexp = c.p<int>(c.L.setexp);
    sa.E = E;
    sa.setperm = c.p<int>(c.L.setperm);
    sa.setoff = c.p<int>(c.L.setoff);
    sa.blockcnt = c.p<int>(c.L.setcnt);
    sa.N = N;
    sa.H = H;
    sa.k = k;
    sa.nsets = count_sets(E, k);
    sa.sides = 2;
    launch_set_sort(sa, c.st);
  }

  if (gated && !c.dense && !gtab_done) {
    prof_mark(c.st, "fwd.gate_table");
    launch_gate_table(c.idx(0), c.gate(0), c.p<float>(c.L.gtab), N, H, E, k, 2, (long)H * N * k, c.st);
  }

  // step 2, all-expert form: queries mix the destination side's experts, keys the source side's,
  // each like the value projection of step 3 (per-slot rows, then the gate-weighted sum)
  if (c.qk_experts) {
    for (int which = 0; which < 2; ++which) {
      const int side = which ? 0 : 1;
      prof_mark(c.st, which ? "fwd.k_experts" : "fwd.q_experts");
      RowGemmArgs a = perm_rows(c, side);
      a.tag = TAG_V_EXPERTS;
      a.A = x;
      a.lda = dm;
      a.B = which ? W_K : W_Q;
      a.b_hstride = (long)E * dm * dh;
      a.b_estride = (long)dm * dh;
      a.sbk = dh;
      a.sbn = 1;
      a.A = side ? xq : x;
      a.C = c.p<void>(which ? c.L.pK : c.L.pQ);
      a.ldc = dh;
      a.c_hoff = (long)c.n(side) * k * dh;
      a.K = dm;
      a.Nc = dh;
      a.mode = STORE_T;
      row_gemm(c, a);
      prof_mark(c.st, which ? "fwd.k_combine" : "fwd.q_combine");
      SlotArgs sl{};
      sl.slots = a.C;
      sl.gate = c.gate(side);
      sl.out = c.p<void>(which ? c.L.K : c.L.Q);
      sl.N = c.n(side);
      sl.H = H;
      sl.k = k;
      sl.dh = dh;
      launch_slot_combine(sl, c.bf16, c.st);
    }
  } else
  // step 2: dense queries and keys (one launch for both when the MFMA kernel takes it)
  {
    RowGemmArgs a = identity_rows(c, 2 * H);
    a.tag = TAG_QK_PROJ;
    a.A = x;
    a.lda = dm;
    a.a_hoff = 0;
    a.B = W_Q;
    a.B2 = W_K;
    a.hsplit = H;
    a.b_hstride = (long)dm * dh;
    a.sbk = dh;
    a.sbn = 1;
    a.C = c.p<void>(c.L.Q);
    a.C2 = c.p<void>(c.L.K);
    a.ldc = hd;
    a.c_hoff = dh;
    a.K = dm;
    a.Nc = dh;
    a.mode = STORE_T;
    if (!c.rect && use_mfma(c) && mfma_row_gemm_supported(a)) {
      prof_mark(c.st, "fwd.qk_proj");
      launch_mfma_row_gemm(a, c.st);
    } else {
      a.heads = H;
      a.hsplit = 0;
      for (int which = 0; which < 2; ++which) {
        prof_mark(c.st, which ? "fwd.k_proj" : "fwd.q_proj");
        a.A = which ? x : xq;              // keys from every token, queries from the destination tokens
        a.M = c.n(which ? 0 : 1);
        a.B = which ? W_K : W_Q;
        a.C = c.p<void>(which ? c.L.K : c.L.Q);
        row_gemm(c, a);
      }
    }
  }

  // rotary position embedding of queries and keys (App. A.4 "RoPE Positional Encodings")
  if (shape->rope) {
    prof_mark(c.st, "fwd.rope");
    launch_rope_table(c.p<float2>(c.L.rope), shape->T, dh, c.st);
    if (c.rect) {   // query i of a sequence sits at position (T - T_q) + i
      launch_rope_apply(c.p<void>(c.L.Q), nullptr, c.p<float2>(c.L.rope), c.Nq, c.Tq, shape->T - c.Tq, H, dh, 0, c.bf16, c.st);
      launch_rope_apply(c.p<void>(c.L.K), nullptr, c.p<float2>(c.L.rope), N, shape->T, 0, H, dh, 0, c.bf16, c.st);
    } else {
      launch_rope_apply(c.p<void>(c.L.Q), c.p<void>(c.L.K), c.p<float2>(c.L.rope), N, shape->T, 0, H, dh, 0, c.bf16, c.st);
    }
  }

  // step 3: value experts, unscaled per-slot results, then the gate-weighted sum over slots
  {
    prof_mark(c.st, "fwd.v_experts");
    RowGemmArgs a = perm_rows(c, 0);
    a.tag = TAG_V_EXPERTS;
    a.A = x;
    a.lda = dm;
    a.B = W_V;
    a.b_hstride = (long)E * dm * dh;
    a.b_estride = (long)dm * dh;
    a.sbk = dh;
    a.sbn = 1;
    a.C = c.p<void>(c.L.pV);
    a.ldc = dh;
    a.c_hoff = (long)N * k * dh;
    a.K = dm;
    a.Nc = dh;
    a.mode = STORE_T;
    row_gemm(c, a);
    prof_mark(c.st, "fwd.v_combine");
    SlotArgs sa{};
    sa.slots = c.p<void>(c.L.pV);
    sa.gate = c.gate(0);
    sa.out = c.p<void>(c.L.V);
    sa.N = N;
    sa.H = H;
    sa.k = k;
    sa.dh = dh;
    launch_slot_combine(sa, c.bf16, c.st);
  }

  // step 4: one attention matrix per head
  {
    prof_mark(c.st, "fwd.attention");
    AttnArgs a{};
    a.Q = c.p<void>(c.L.Q);
    a.K = c.p<void>(c.L.K);
    a.V = c.p<void>(c.L.V);
    a.O = c.p<void>(c.L.ctx);
    a.lse = c.p<float>(c.L.lse);
    a.B = shape->B;
    a.T = shape->T;
    a.H = H;
    a.dh = dh;
    a.causal = shape->causal;
    a.scale = 1.0f / sqrtf((float)dh);
    a.Tq = c.Tq;
    if (use_mfma(c) && mfma_attn_supported(shape->T, dh))
      launch_mfma_attn_fwd(a, c.st);
    else
      launch_simt_attn_fwd(a, c.bf16, c.st);
  }

  // step 5: output experts.  Gated concatenation: one GEMM over the H*E (head, expert) segments, rows scaled by
  // the dense gate table, y written once.
  bool y_done = false;
  if (gated) {
    RowGemmArgs a = identity_rows(c, 1, 1);
    a.tag = TAG_O_EXPERTS;
    a.seg_mode = 3;
    a.nseg = H * E;
    a.lda = hd;
    a.sbk = dm;
    a.sbn = 1;
    a.C = y;
    a.ldc = dm;
    a.K = dh;
    a.Nc = dm;
    a.mode = STORE_T;
    a.gtab = c.dense ? nullptr : c.p<float>(c.L.gtab) + (size_t)N * H * E;   // the destination side's gates
    a.gld = H * E;
    for (int s_ = 0; s_ < H * E; ++s_) {
      a.segd[s_].A = c.p<bf16_t>(c.L.ctx) + (size_t)(s_ / E) * dh;
      a.segd[s_].B = (const bf16_t*)W_O + (size_t)s_ * dh * dm;
      a.segd[s_].gcol = c.dense ? -1 : s_;
    }
    if (pp_row_gemm_supported(a)) {
      prof_mark(c.st, "fwd.o_experts");
      launch_pp_row_gemm(a, c.st);
      y_done = true;
    }
  }
  // Expert-set path: per head one GEMM whose reduction runs over the
  // k gate-scaled copies of the token's read-out row, then the sum over heads.
  if (y_done) {
  } else if (sets) {
    prof_mark(c.st, "fwd.o_experts");
    RowGemmArgs a = set_rows(c, 1);
    a.tag = TAG_O_EXPERTS;
    a.A = c.p<void>(c.L.ctx);
    a.lda = hd;
    a.a_hoff = dh;
    a.B = W_O;
    a.b_hstride = (long)E * dh * dm;
    a.b_estride = (long)dh * dm;
    a.sbk = dm;
    a.sbn = 1;
    a.C = H == 1 ? y : c.p<void>(c.L.yh);
    a.ldc = dm;
    a.c_hoff = (long)c.Nq * dm;
    a.K = dh;
    a.Nc = dm;
    a.mode = STORE_T;
    launch_mfma_row_gemm(a, c.st);
    if (H > 1) {
      prof_mark(c.st, "fwd.y_sum");
      launch_sum_heads(c.p<void>(c.L.yh), nullptr, y, (size_t)c.Nq * dm, (size_t)c.Nq * dm, H, c.st);
    }
  } else
  // fallback: expert-sorted rows, gate-scaled, summed over heads and slots with fp32 atomics
  {
    prof_mark(c.st, "fwd.y_zero");
    float* acc = c.bf16 ? c.p<float>(c.L.acc32) : (float*)y;
    launch_fill_f32(acc, (size_t)c.Nq * dm, 0.f, c.st);
    prof_mark(c.st, "fwd.o_experts");
    RowGemmArgs a = perm_rows(c, 1);
    a.tag = TAG_O_EXPERTS;
    a.c_div = k;
    a.A = c.p<void>(c.L.ctx);
    a.lda = hd;
    a.a_hoff = dh;
    a.B = W_O;
    a.b_hstride = (long)E * dh * dm;
    a.b_estride = (long)dh * dm;
    a.sbk = dm;
    a.sbn = 1;
    a.C = acc;
    a.ldc = dm;
    a.c_hoff = 0;
    a.gate = c.gate(1);
    a.gate_hstride = (long)c.Nq * k;
    a.K = dh;
    a.Nc = dm;
    a.mode = ATOMIC_F32;
    row_gemm(c, a);
    prof_mark(c.st, "fwd.y_cast");
    if (c.bf16) launch_cast_from_f32(acc, y, (size_t)c.Nq * dm, 1, c.st);
  }
  prof_mark(c.st, nullptr);
  return check_launch("switchhead_forward");
}

sh_status switchhead_forward_static(const sh_shape* shape, const void* x, const void* W_Q, const void* W_K,
                                    const void* W_V, const void* W_O, const void* W_S, const void* W_D, const float* b_S,
                                    const float* b_D, void* y, void* hip_stream) {
  // the size test needs no GPU and comes first: a shape that does not fit touches nothing
  sh_status r = check_shape(shape);
  if (r != SH_OK) return r;
  const size_t need = make_layout(shape).total;
  if (need > (size_t)SWITCHHEAD_STATIC_WORKSPACE_BYTES)
    return fail(SH_ERR_WORKSPACE_TOO_SMALL, "switchhead_forward_static: this shape needs %zu bytes of workspace, the built-in one has %zu",
                need, (size_t)SWITCHHEAD_STATIC_WORKSPACE_BYTES);
  // the array's device address on the current GPU, looked up once per GPU
  static std::mutex mu;
  static void* addr[64] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64)
    return fail(SH_ERR_HIP, "switchhead_forward_static: no current device (or its index is above 63)");
  void* ws = nullptr;
  {
    std::lock_guard<std::mutex> lk(mu);
    if (!addr[dev]) {
      void* q = nullptr;
      const hipError_t e = hipGetSymbolAddress(&q, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !q) return fail(SH_ERR_HIP, "switchhead_forward_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
      addr[dev] = q;
    }
    ws = addr[dev];
  }
  return switchhead_forward(shape, x, W_Q, W_K, W_V, W_O, W_S, W_D, b_S, b_D, y, ws, (size_t)SWITCHHEAD_STATIC_WORKSPACE_BYTES,
                            hip_stream);
}

sh_status switchhead_backward(const sh_shape* shape, const void* x, const void* W_Q, const void* W_K, const void* W_V,
                              const void* W_O, const void* W_S, const void* W_D, const void* dy, void* workspace,
                              size_t workspace_bytes, void* dx, float* dW_Q, float* dW_K, float* dW_V, float* dW_O,
                              float* dW_S, float* dW_D, float* db_S, float* db_D, void* hip_stream) {
  Ctx c;
  sh_status r = make_ctx(c, shape, W_S, W_D, workspace, workspace_bytes, hip_stream);
  if (r != SH_OK) return r;
  if (!x || !W_Q || !W_K || !W_V || !W_O || !dy || !dx || !dW_Q || !dW_K || !dW_V || !dW_O)
    return fail(SH_ERR_INVALID_ARG, "x, W_Q, W_K, W_V, W_O, dy, dx, dW_Q, dW_K, dW_V, dW_O must not be NULL");
  c.aligned = all_aligned16({x, W_Q, W_K, W_V, W_O, W_S, W_D, dy, dx, dW_Q, dW_K, dW_V, dW_O, dW_S, dW_D});
  const int N = c.N, H = c.H, E = c.E, k = c.k, dh = c.dh, dm = c.dm;
  const long hd = (long)H * dh;
  const int chunk = wgrad_chunk((size_t)H * N * k, dm, dh);         // expert-sorted operands
  const int chunk_dense = wgrad_chunk((size_t)2 * H * N, dm, dh);   // fused dense Q/K
  // ... with the routers' x^T dz as one more head: sized for 2H + 1 groups, or the launch spills into a second round
  // (c2: 540 work-groups for 512 places with the chunk of 2H groups, 468 with this one)
  const int chunk_dense_r = wgrad_chunk((size_t)(2 * H + 1) * N, dm, dh);
  const bool sets = sets_usable(c);
  if ((sets && (c.L.yh == 0 || c.L.setperm == 0)) || (gated_concat(c) && c.L.gtab == 0))
    return fail(SH_ERR_UNSUPPORTED, "switchhead_backward: internal error, the workspace layout lacks a table this shape's path uses");
  const int Nq = c.Nq;
  const void* xq = c.rect ? c.p<void>(c.L.xq) : x;   // the query tokens' rows of x (copied by forward)

  // output experts: u[h][a][:] = dy[n] W_O[h,e]^T (unscaled), then dctx, d(gate_D), delta
  {
    prof_mark(c.st, "bwd.o_dgrad");
    RowGemmArgs a = perm_rows(c, 1);
    a.tag = TAG_O_DGRAD;
    a.A = dy;
    a.lda = dm;
    a.B = W_O;
    a.b_hstride = (long)E * dh * dm;
    a.b_estride = (long)dh * dm;
    a.sbk = 1;
    a.sbn = dm;
    a.C = c.p<void>(c.L.u);
    a.ldc = dh;
    a.c_hoff = (long)Nq * k * dh;
    a.K = dm;
    a.Nc = dh;
    a.mode = STORE_T;
    row_gemm(c, a);
    prof_mark(c.st, "bwd.dctx_combine");
    SlotArgs sa{};
    sa.slots = c.p<void>(c.L.u);
    sa.gate = c.gate(1);
    sa.other = c.p<void>(c.L.ctx);
    sa.out = c.p<void>(c.L.dctx);
    sa.dots = c.p<float>(c.L.dgate) + (size_t)H * N * k;
    sa.delta = c.p<float>(c.L.delta);
    sa.N = Nq;
    sa.H = H;
    sa.k = k;
    sa.dh = dh;
    launch_slot_combine(sa, c.bf16, c.st);
  }
  {
    prof_mark(c.st, "bwd.o_wgrad");
    WgradArgs w{};
    w.tag = TAG_O_WGRAD;
    w.perm = c.perm(1);
    w.offsets = c.offsets(1);
    w.heads = H;
    w.E = E;
    w.M = Nq * k;
    w.max_group_rows = Nq;
    w.a_div = k;
    w.b_div = k;
    w.A = c.p<void>(c.L.ctx);
    w.lda = hd;
    w.a_hoff = dh;
    w.Ka = dh;
    w.Bm = dy;
    w.ldb = dm;
    w.b_hoff = 0;
    w.Kb = dm;
    w.dW = dW_O;
    w.w_hstride = (long)E * dh * dm;
    w.w_estride = (long)dh * dm;
    w.swa = dm;
    w.gate = c.gate(1);
    w.gate_hstride = (long)Nq * k;
    w.chunk = chunk;
    wgrad(c, w);
  }

  // attention
  {
    AttnBwdArgs a{};
    a.Q = c.p<void>(c.L.Q);
    a.K = c.p<void>(c.L.K);
    a.V = c.p<void>(c.L.V);
    a.dO = c.p<void>(c.L.dctx);
    a.lse = c.p<float>(c.L.lse);
    a.delta = c.p<float>(c.L.delta);
    a.dQ = c.p<void>(c.L.dQ);
    a.dK = c.p<void>(c.L.dK);
    a.dV = c.p<void>(c.L.dV);
    a.B = shape->B;
    a.T = shape->T;
    a.H = H;
    a.dh = dh;
    a.causal = shape->causal;
    a.scale = 1.0f / sqrtf((float)dh);
    a.Tq = c.Tq;
    if (c.L.dst != 0 && attn_ds_dims(shape->T, c.Tq, dh, shape->causal, &a.ds_ld, &a.ds_per)) a.dSt = c.p<void>(c.L.dst);
    if (use_mfma(c) && mfma_attn_supported(shape->T, dh))
      launch_mfma_attn_bwd(a, c.st);   // marks its two kernels itself
    else {
      prof_mark(c.st, "bwd.attention");
      launch_simt_attn_bwd(a, c.bf16, c.st);
    }
  }

  // back through the rotation of queries and keys: gradients take the opposite turn
  if (shape->rope) {
    prof_mark(c.st, "bwd.rope");
    if (c.rect) {
      launch_rope_apply(c.p<void>(c.L.dQ), nullptr, c.p<float2>(c.L.rope), c.Nq, c.Tq, shape->T - c.Tq, H, dh, 1, c.bf16, c.st);
      launch_rope_apply(c.p<void>(c.L.dK), nullptr, c.p<float2>(c.L.rope), N, shape->T, 0, H, dh, 1, c.bf16, c.st);
    } else {
      launch_rope_apply(c.p<void>(c.L.dQ), c.p<void>(c.L.dK), c.p<float2>(c.L.rope), N, shape->T, 0, H, dh, 1, c.bf16, c.st);
    }
  }

  // dense queries and keys: weight gradients, then dx = dQ W_Q^T + dK W_K^T.  With the MFMA
  // kernel this is one GEMM whose reduction runs over the 2*nheads (projection, head) segments
  // and that overwrites the fp32 dx accumulator; otherwise the accumulator is zeroed and every
  // head adds its part atomically.
  float* dxacc = c.bf16 ? c.p<float>(c.L.acc32) : (float*)dx;
  bool qk_partial = false;    // the Q/K share of dx sits in a bf16 partial, not in dxacc
  bool acc_written = false;   // dxacc holds (part of) dx
  // dW_Q, dW_K = x^T dQ, x^T dK as one launch over the 2H (projection, head) pairs; with_router: the
  // routers' x^T dz rides along as one more head (dz sits in rows shaped like a dQ / dK row)
  auto qk_wgrad_args = [&](bool with_router) {
    WgradArgs w{};
    w.tag = TAG_QK_WGRAD;
    w.heads = 2 * H + (with_router ? 1 : 0);
    w.Bm3 = c.p<void>(c.L.dR);
    w.dW3 = c.p<float>(c.L.wrt);
    w.hsplit = H;
    w.E = 1;
    w.M = N;
    w.a_div = 1;
    w.b_div = 1;
    w.A = x;
    w.lda = dm;
    w.a_hoff = 0;
    w.Ka = dm;
    w.Bm = c.p<void>(c.L.dQ);
    w.Bm2 = c.p<void>(c.L.dK);
    w.ldb = hd;
    w.b_hoff = dh;
    w.Kb = dh;
    w.dW = dW_Q;
    w.dW2 = dW_K;
    w.w_hstride = (long)dm * dh;
    w.swa = dh;
    w.chunk = with_router ? chunk_dense_r : chunk_dense;
    return w;
  };
  auto run_qk_wgrad = [&](bool with_router) {
    prof_mark(c.st, "bwd.qk_wgrad");
    WgradArgs w = qk_wgrad_args(with_router);
    if (!c.rect) {
      wgrad(c, w);
    } else {   // queries and keys come from different token sets: one launch each
      w.heads = H;
      w.hsplit = 0;
      w.A = xq;
      w.M = Nq;
      wgrad(c, w);
      prof_mark(c.st, "bwd.qk_wgrad");
      w.A = x;
      w.M = N;
      w.Bm = c.p<void>(c.L.dK);
      w.dW = dW_K;
      wgrad(c, w);
    }
  };
  // the query tokens' own share of dx (fewer queries than keys): fp32, added to their rows at the end
  float* accq = c.rect ? c.p<float>(c.L.accq) : nullptr;
  bool accq_set = false;
  if (c.rect && !c.qk_experts) {
    // dQ W_Q^T as one GEMM over the H concatenated head segments that overwrites the accumulator
    RowGemmArgs a = identity_rows(c, 1, 1);
    a.tag = TAG_QK_DGRAD;
    a.A = c.p<void>(c.L.dQ);
    a.lda = hd;
    a.seg_mode = 2;
    a.nseg = H;
    a.seg_split = H;
    a.a_sstride = dh;
    a.B = W_Q;
    a.b_sstride = (long)dm * dh;
    a.sbk = 1;
    a.sbn = dh;
    a.C = accq;
    a.ldc = dm;
    a.K = dh;
    a.Nc = dm;
    a.mode = STORE_F32;
    if (use_mfma(c) && mfma_row_gemm_supported(a)) {
      prof_mark(c.st, "bwd.q_dgrad");
      launch_mfma_row_gemm(a, c.st);
      accq_set = true;
    }
  }
  if (c.rect && !accq_set) {
    prof_mark(c.st, "bwd.dx_zero");
    launch_fill_f32(accq, (size_t)Nq * dm, 0.f, c.st);
    if (!c.qk_experts) {
      prof_mark(c.st, "bwd.q_dgrad");
      RowGemmArgs b = identity_rows(c, H, 1);
      b.tag = TAG_QK_DGRAD;
      b.A = c.p<void>(c.L.dQ);
      b.lda = hd;
      b.a_hoff = dh;
      b.B = W_Q;
      b.b_hstride = (long)dm * dh;
      b.sbk = 1;
      b.sbn = dh;
      b.C = accq;
      b.ldc = dm;
      b.K = dh;
      b.Nc = dm;
      b.mode = ATOMIC_F32;
      row_gemm(c, b);
    }
  }
  // dx += dQ W_Q^T + dK W_K^T (one GEMM over the 2H concatenated segments).  Where the routers' dz fits
  // into rows of the same shape it rides along as one more segment (dz_S W_S^T + dz_D W_D^T), and the
  // launch moves behind the router backward kernel.
  const int HE_r = H * E, HEp_r = (HE_r + 7) / 8 * 8, sides_r = c.shared ? 1 : 2;
  const bool wide_dz = !c.dense && sides_r * HEp_r <= dh && (c.L.dR - c.L.dK) == (c.L.dK - c.L.dQ);
  // All of dx as ONE token-ordered GEMM (gated concatenation, see gated_concat): the value experts' input gradient
  // over all E experts of every head with the source side's dense gates, the 2H query / key segments and, where
  // the routers' dz rows have the shape of a dQ row, the routers' segment; dx is written once, in bf16.
  auto merged_dx_args = [&](bool with_router) {
    RowGemmArgs a = identity_rows(c, 1);
    a.tag = TAG_QK_DGRAD;
    a.seg_mode = 3;
    a.lda = hd;
    a.sbk = 1;
    a.sbn = dh;
    a.C = dx;
    a.ldc = dm;
    a.K = dh;
    a.Nc = dm;
    a.mode = STORE_T;
    a.gtab = c.dense ? nullptr : c.p<float>(c.L.gtab);   // the source side's gates
    a.gld = H * E;
    int n = 0;
    for (int s_ = 0; s_ < H * E && n < MAX_SEGD; ++s_, ++n) {
      a.segd[n].A = c.p<bf16_t>(c.L.dV) + (size_t)(s_ / E) * dh;
      a.segd[n].B = (const bf16_t*)W_V + (size_t)s_ * dm * dh;
      a.segd[n].gcol = c.dense ? -1 : s_;
    }
    for (int which = 0; which < 2; ++which)
      for (int h_ = 0; h_ < H && n < MAX_SEGD; ++h_, ++n) {
        a.segd[n].A = c.p<bf16_t>(which ? c.L.dK : c.L.dQ) + (size_t)h_ * dh;
        a.segd[n].B = (const bf16_t*)(which ? W_K : W_Q) + (size_t)h_ * dm * dh;
        a.segd[n].gcol = -1;
      }
    if (with_router && n < MAX_SEGD) {
      a.segd[n].A = c.p<bf16_t>(c.L.dR);
      a.segd[n].B = c.p<bf16_t>(c.L.wr3);
      a.segd[n].gcol = -1;
      ++n;
    }
    a.nseg = n;
    return a;
  };
  const bool merged_dx = gated_concat(c) && (c.dense || wide_dz) && pp_row_gemm_supported(merged_dx_args(!c.dense));
  const bool fuse_router = wide_dz && (sets || merged_dx) && c.bf16 && use_mfma(c) && !c.qk_experts && !c.rect;
  bool router_fused = false;
  // the routers' weight gradients ride along with the Q/K weight gradient under the same conditions,
  // if the three-set launch is one the matrix-core kernel takes (it has no other implementation)
  bool fuse_router_w = false;
  if (fuse_router && dW_S && (c.shared || dW_D)) {
    WgradArgs probe = qk_wgrad_args(true);
    probe.partial = c.p<float>(c.L.wpart);
    probe.max_chunks = (probe.M + probe.chunk - 1) / probe.chunk;
    fuse_router_w = mfma_wgrad_supported(probe);
  }
  if (!c.qk_experts && !fuse_router_w) run_qk_wgrad(false);
  auto run_qk_dgrad = [&](bool with_router) {
    RowGemmArgs a = identity_rows(c, 1);
    a.tag = TAG_QK_DGRAD;
    a.A = c.p<void>(c.L.dQ);
    a.lda = hd;
    a.seg_mode = 2;
    a.nseg = 2 * H + (with_router ? 1 : 0);
    a.B3 = c.p<void>(c.L.wr3);
    a.seg_split = H;
    a.a_sstride = dh;
    a.a_wstride = (long)((c.L.dK - c.L.dQ) / (c.bf16 ? 2 : 4));
    a.B = W_Q;
    a.B2 = W_K;
    if (c.rect) {   // the keys' segments alone: the queries' share went to the query rows' accumulator
      a.A = c.p<void>(c.L.dK);
      a.nseg = H;
      a.B = W_K;
    }
    a.b_sstride = (long)dm * dh;
    a.sbk = 1;
    a.sbn = dh;
    a.C = dxacc;
    a.ldc = dm;
    a.K = dh;
    a.Nc = dm;
    a.mode = STORE_F32;
    if (sets && c.bf16) {
      // with the expert-set path dx is a sum of bf16 partials anyway: this one goes to slot H
      RowGemmArgs p = a;
      p.C = c.p<char>(c.L.yh) + (size_t)H * N * dm * 2;
      p.mode = STORE_T;
      if (mfma_row_gemm_supported(p)) {
        a = p;
        qk_partial = true;
      }
    }
    if (use_mfma(c) && mfma_row_gemm_supported(a)) {
      prof_mark(c.st, "bwd.qk_dgrad");
      launch_mfma_row_gemm(a, c.st);
      acc_written = !qk_partial;
      router_fused = with_router;
    } else {
      acc_written = true;
      prof_mark(c.st, "bwd.dx_zero");
      launch_fill_f32(dxacc, (size_t)N * dm, 0.f, c.st);
      for (int which = c.rect ? 1 : 0; which < 2; ++which) {
        prof_mark(c.st, which ? "bwd.k_dgrad" : "bwd.q_dgrad");
        RowGemmArgs b = identity_rows(c, H);
        b.tag = TAG_QK_DGRAD;
        b.A = c.p<void>(which ? c.L.dK : c.L.dQ);
        b.lda = hd;
        b.a_hoff = dh;
        b.B = which ? W_K : W_Q;
        b.b_hstride = (long)dm * dh;
        b.sbk = 1;
        b.sbn = dh;
        b.C = dxacc;
        b.ldc = dm;
        b.K = dh;
        b.Nc = dm;
        b.mode = ATOMIC_F32;
        row_gemm(c, b);
      }
    }
  };
  if (c.qk_experts) {
    if (!sets) {   // the expert input gradients below add into the accumulator
      prof_mark(c.st, "bwd.dx_zero");
      launch_fill_f32(dxacc, (size_t)N * dm, 0.f, c.st);
      acc_written = true;
    }
  } else if (!fuse_router && !merged_dx) {
    run_qk_dgrad(false);
  }

  // A projection P[n,h] = sum_j g[n,h,j] x[n] W[h,e_j] (values; queries and keys in the all-expert
  // form) given dP: the gates' gradient <x W[h,e_j], dP> from the per-slot rows the forward pass
  // kept, dW[h,e] = sum_n g x[n]^T dP[n,h], and the projection's share of dx.
  int yh_used = 0;   // bf16 partials of dx written so far (expert-set path)
  const bool sets_path = sets;
  auto expert_proj_bwd = [&](int side, const void* W, size_t dP, size_t slots, float* dW, bool dots_add,
                             const char* l_gate, const char* l_wgrad, const char* l_dgrad) {
    prof_mark(c.st, l_gate);
    SlotArgs sa{};
    sa.slots = c.p<void>(slots);
    sa.gate = c.gate(side);
    sa.other = c.p<void>(dP);
    sa.dots = c.p<float>(c.L.dgate) + (size_t)side * H * N * k;
    sa.dots_add = dots_add;
    sa.N = c.n(side);
    sa.H = H;
    sa.k = k;
    sa.dh = dh;
    launch_slot_combine(sa, c.bf16, c.st);
    prof_mark(c.st, l_wgrad);
    WgradArgs w{};
    w.tag = TAG_V_WGRAD;
    w.scale_b = 1;   // gate on the d_head-wide dP rows instead of the d_model-wide x rows
    w.perm = c.perm(side);
    w.offsets = c.offsets(side);
    w.heads = H;
    w.E = E;
    w.M = c.n(side) * k;
    w.max_group_rows = c.n(side);
    w.a_div = k;
    w.b_div = k;
    w.A = side ? xq : x;
    w.lda = dm;
    w.a_hoff = 0;
    w.Ka = dm;
    w.Bm = c.p<void>(dP);
    w.ldb = hd;
    w.b_hoff = dh;
    w.Kb = dh;
    w.dW = dW;
    w.w_hstride = (long)E * dm * dh;
    w.w_estride = (long)dm * dh;
    w.swa = dh;
    w.gate = c.gate(side);
    w.gate_hstride = (long)c.n(side) * k;
    w.chunk = chunk;
    wgrad(c, w);
    if (merged_dx) return;   // this projection's share of dx is part of the one GEMM that writes dx
    prof_mark(c.st, l_dgrad);
    const bool to_accq = c.rect && side == 1;   // rows of the query tokens: their own fp32 accumulator
    const bool sets = sets_path && !to_accq;
    RowGemmArgs a = sets ? set_rows(c, side) : perm_rows(c, side);
    a.tag = TAG_V_DGRAD;
    a.A = c.p<void>(dP);
    a.lda = hd;
    a.a_hoff = dh;
    a.B = W;
    a.b_hstride = (long)E * dm * dh;
    a.b_estride = (long)dm * dh;
    a.sbk = 1;
    a.sbn = dh;
    a.K = dh;
    a.Nc = dm;
    if (sets) {
      // per-head partial sums of dx in bf16; they are added to the rest of dx at the end
      a.C = c.p<char>(c.L.yh) + (size_t)yh_used * N * dm * 2;
      a.ldc = dm;
      a.c_hoff = (long)N * dm;
      a.mode = STORE_T;
      launch_mfma_row_gemm(a, c.st);
      yh_used += H;
    } else {
      a.c_div = k;
      a.C = to_accq ? accq : dxacc;
      a.ldc = dm;
      a.gate = c.gate(side);
      a.gate_hstride = (long)c.n(side) * k;
      a.mode = ATOMIC_F32;
      row_gemm(c, a);
    }
  };
  expert_proj_bwd(0, W_V, c.L.dV, c.L.pV, dW_V, false, "bwd.dgate_s", "bwd.v_wgrad", "bwd.v_dgrad");
  if (c.qk_experts) {
    // keys add to the source side's gate gradients, queries to the destination side's (written by
    // the output experts' step above)
    expert_proj_bwd(0, W_K, c.L.dK, c.L.pK, dW_K, true, "bwd.dgate_k", "bwd.k_wgrad_e", "bwd.k_dgrad_e");
    expert_proj_bwd(1, W_Q, c.L.dQ, c.L.pQ, dW_Q, true, "bwd.dgate_q", "bwd.q_wgrad_e", "bwd.q_dgrad_e");
  }
  // slots of the partial-sum buffer taken so far: the experts' above, or the value experts' H and
  // (once its GEMM has run) the dense Q/K pair's one right behind them
  auto yh_taken = [&] { return c.qk_experts ? yh_used : H + (qk_partial ? 1 : 0); };

  // routers
  bool router_partial = false;
  if (!c.dense && c.rect) {
    // fewer queries than keys: each side has its own tokens, so every step runs once per side; the
    // destination side's input gradient goes to the query rows' accumulator
    prof_mark(c.st, "bwd.router");
    const int HE = H * E, HEp = (HE + 7) / 8 * 8;
    const size_t esz = c.bf16 ? 2 : 4;
    launch_zero4_f32(db_S, db_S ? (size_t)HE : 0, c.shared ? nullptr : db_D, (!c.shared && db_D) ? (size_t)HE : 0, nullptr, 0,
                     nullptr, 0, c.st);
    for (int side = 0; side < 2; ++side) {
      const bool own = side == 1 && !c.shared;
      const void* W = own ? W_D : W_S;
      float* dW = own ? dW_D : dW_S;
      char* dzs = c.p<char>(c.L.dz) + (size_t)side * N * HEp * esz;
      RouterBwdArgs rb{};
      rb.idx = c.idx(side);
      rb.gate = c.gate(side);
      rb.dgate = c.p<float>(c.L.dgate) + (size_t)side * H * N * k;
      rb.dz = dzs;
      rb.db[0] = own ? db_D : db_S;
      rb.N = c.n(side);
      rb.H = H;
      rb.E = E;
      rb.k = k;
      rb.sides = 1;
      rb.shared = 0;
      rb.ld = HEp;
      rb.side_stride = HEp;
      rb.pad_to = 0;
      launch_router_bwd(rb, c.bf16, c.st);
      if (dW) {
        prof_mark(c.st, "bwd.router_wgrad");
        WgradArgs w{};
        w.heads = 1;
        w.E = 1;
        w.M = c.n(side);
        w.a_div = 1;
        w.b_div = 1;
        w.A = side ? xq : x;
        w.lda = dm;
        w.Ka = dm;
        w.Bm = dzs;
        w.ldb = HEp;
        w.Kb = HEp;
        w.kb_store = HE;
        w.swa = HE;
        w.chunk = 256;
        w.dW = dW;
        wgrad(c, w, false, /*zero=*/!(c.shared && side == 1));   // shared selection: both sides add into dW_S
      }
      prof_mark(c.st, "bwd.router_dgrad");
      RowGemmArgs a = identity_rows(c, 1, side);
      a.A = dzs;
      a.lda = HEp;
      a.B = W;
      a.sbk = 1;
      a.sbn = HE;
      a.ldc = dm;
      a.K = HE;
      a.Nc = dm;
      a.mode = ATOMIC_F32;
      if (side == 1) {
        a.C = accq;
      } else {
        if (sets && c.bf16 && use_mfma(c)) {
          // the router packed as [d_model][HEp]: one GEMM, stored as one more bf16 partial of dx
          bf16_t* Wp = (bf16_t*)(c.p<char>(c.L.rh));
          RowGemmArgs p = a;
          p.tag = TAG_QK_DGRAD;
          p.seg_mode = 2;
          p.nseg = 1;
          p.seg_split = 1;
          p.a_wstride = HEp;
          p.B = Wp;
          p.sbn = HEp;
          p.K = HEp;
          p.C = c.p<char>(c.L.yh) + (size_t)yh_taken() * N * dm * esz;
          p.mode = STORE_T;
          if (mfma_row_gemm_supported(p)) {
            launch_pack_router(W, nullptr, Wp, dm, HE, HEp, 1, c.st);
            launch_mfma_row_gemm(p, c.st);
            router_partial = true;
            continue;
          }
        }
        if (!acc_written) {
          launch_fill_f32(dxacc, (size_t)N * dm, 0.f, c.st);
          acc_written = true;
        }
        a.C = dxacc;
      }
      row_gemm(c, a);
    }
  } else if (!c.dense) {
    prof_mark(c.st, "bwd.router");
    const int sides = c.shared ? 1 : 2;
    const int HE = H * E;
    float* dWs[2] = {dW_S, c.shared ? nullptr : dW_D};
    float* dbs[2] = {db_S, c.shared ? nullptr : db_D};
    // the small outputs that are accumulated with atomics are cleared by one launch
    const bool both_w = sides == 2 && dWs[0] && dWs[1] && !fuse_router_w;
    // fused weight gradient: the bias gradients go through per-block sums that the split kernel adds up
    // (no atomics, nothing to clear); the dz region proper is free then (the rows sit in dR)
    const size_t esz_r = c.bf16 ? 2 : 4;
    const int rblk = router_bwd_blocks(N);
    const bool db_partial = fuse_router_w && wide_dz && (dbs[0] || dbs[1]) &&
                            (size_t)sides * H * rblk * E * 4 <= (size_t)N * 2 * ((H * E + 7) / 8 * 8) * esz_r;
    if (!db_partial)
      launch_zero4_f32(dbs[0], dbs[0] ? (size_t)HE : 0, dbs[1], dbs[1] ? (size_t)HE : 0, both_w ? dWs[0] : nullptr,
                       both_w ? (size_t)dm * HE : 0, both_w ? dWs[1] : nullptr, both_w ? (size_t)dm * HE : 0, c.st);
    RouterBwdArgs rb{};
    rb.idx = c.idx(0);
    rb.gate = c.gate(0);
    rb.dgate = c.p<float>(c.L.dgate);
    rb.dz = c.p<void>(wide_dz ? c.L.dR : c.L.dz);
    rb.db[0] = dbs[0];
    rb.db[1] = dbs[1];
    rb.dbpart = db_partial ? c.p<float>(c.L.dz) : nullptr;
    rb.N = N;
    rb.H = H;
    rb.E = E;
    rb.k = k;
    rb.sides = sides;
    rb.shared = c.shared;
    const int HEp = (HE + 7) / 8 * 8;
    rb.ld = wide_dz ? (int)hd : sides * HEp;   // wide rows: the shape of a dQ / dK row
    rb.side_stride = HEp;
    rb.pad_to = wide_dz ? dh : 0;
    if (fuse_router) {   // the packed routers for the Q/K dgrad launch below ride along
      rb.W[0] = W_S;
      rb.W[1] = c.shared ? nullptr : W_D;
      rb.wide_out = c.p<void>(c.L.wr3);
      rb.dm = dm;
      rb.wide_width = dh;
    }
    launch_router_bwd(rb, c.bf16, c.st);
    const size_t esz = c.bf16 ? 2 : 4;
    const char* dz0 = c.p<char>(wide_dz ? c.L.dR : c.L.dz);
    if (fuse_router && merged_dx) {
      prof_mark(c.st, "bwd.dx_gemm");
      launch_pp_row_gemm(merged_dx_args(true), c.st);
      router_fused = true;
    } else if (fuse_router) {
      run_qk_dgrad(true);
    }
    if (fuse_router_w) {
      run_qk_wgrad(true);
      prof_mark(c.st, "bwd.router_wsplit");
      launch_router_wgrad_split(c.p<float>(c.L.wrt), dWs[0], dWs[1], dm, dh, HE, HEp, db_partial ? c.p<float>(c.L.dz) : nullptr,
                                rblk, E, dbs[0], dbs[1], c.st);
    } else
    // dW_S / dW_D = x^T dz: one launch for both sides when both are wanted
    {
      WgradArgs w{};
      w.E = 1;
      w.M = N;
      w.a_div = 1;
      w.b_div = 1;
      w.A = x;
      w.lda = dm;
      w.Ka = dm;
      w.ldb = rb.ld;
      w.Kb = HEp;        // the padded columns of dz are zero; reading them keeps the rows 16-byte wide
      w.kb_store = HE;
      w.swa = HE;
      w.chunk = 256;   // tiny output: many short chunks keep the GPU busy, atomics are few
      if (sides == 2 && dWs[0] && dWs[1]) {
        prof_mark(c.st, "bwd.router_wgrad");
        // one pass over x for both sides: the row of dz holds [side 0 | side 1], HEp columns each
        WgradArgs w2 = w;
        w2.heads = 1;
        w2.Bm = dz0;
        w2.Kb = 2 * HEp;
        w2.col_split = HEp;
        w2.dW = dWs[0];
        w2.dW2 = dWs[1];
        if (use_mfma(c) && mfma_wgrad_supported(w2)) {
          launch_mfma_wgrad(w2, c.st);   // outputs cleared above
        } else {
          w.heads = 2;
          w.hsplit = 1;
          w.Bm = dz0;
          w.Bm2 = dz0 + (size_t)HEp * esz;
          w.dW = dWs[0];
          w.dW2 = dWs[1];
          wgrad(c, w, false);
        }
      } else {
        for (int sd = 0; sd < sides; ++sd) {
          if (!dWs[sd]) continue;
          prof_mark(c.st, "bwd.router_wgrad");
          w.heads = 1;
          w.Bm = dz0 + (size_t)sd * HEp * esz;
          w.dW = dWs[sd];
          wgrad(c, w, false);
        }
      }
    }
    // dx += dz_S W_S^T + dz_D W_D^T, unless it went along with the Q/K input gradient above
    if (!router_fused) prof_mark(c.st, "bwd.router_dgrad");
    if (!router_fused && sets && c.bf16 && use_mfma(c)) {
      // both routers packed as [side][d_model][HEp]: one GEMM over the concatenated columns,
      // stored as one more partial of dx
      bf16_t* Wp = (bf16_t*)(c.p<char>(c.L.rh));
      RowGemmArgs a = identity_rows(c, 1);
      a.tag = TAG_QK_DGRAD;
      a.A = dz0;
      a.lda = rb.ld;
      a.seg_mode = 2;
      a.nseg = sides;
      a.seg_split = 1;
      a.a_wstride = HEp;
      a.B = Wp;
      a.B2 = Wp + (size_t)dm * HEp;
      a.sbk = 1;
      a.sbn = HEp;
      a.C = c.p<char>(c.L.yh) + (size_t)yh_taken() * N * dm * esz;
      a.ldc = dm;
      a.K = HEp;
      a.Nc = dm;
      a.mode = STORE_T;
      if (mfma_row_gemm_supported(a)) {
        launch_pack_router(W_S, c.shared ? nullptr : W_D, Wp, dm, HE, HEp, sides, c.st);
        launch_mfma_row_gemm(a, c.st);
        router_partial = true;
      }
    }
    if (!router_partial && !router_fused) {
      if (!acc_written) {
        launch_fill_f32(dxacc, (size_t)N * dm, 0.f, c.st);
        acc_written = true;
      }
      for (int sd = 0; sd < sides; ++sd) {
        RowGemmArgs a = identity_rows(c, 1);
        a.A = dz0 + (size_t)sd * HEp * esz;
        a.lda = rb.ld;
        a.B = sd ? W_D : W_S;
        a.sbk = 1;
        a.sbn = HE;
        a.C = dxacc;
        a.ldc = dm;
        a.K = HE;
        a.Nc = dm;
        a.mode = ATOMIC_F32;
        row_gemm(c, a);
      }
    }
  }
  if (merged_dx && c.dense) {
    prof_mark(c.st, "bwd.dx_gemm");
    launch_pp_row_gemm(merged_dx_args(false), c.st);
  }
  if (!merged_dx) prof_mark(c.st, "bwd.dx_cast");
  if (merged_dx) {
  } else if (sets)
    launch_sum_heads(c.p<void>(c.L.yh), acc_written ? dxacc : nullptr, dx, (size_t)N * dm, (size_t)N * dm,
                     yh_taken() + (router_partial ? 1 : 0), c.st);
  else if (c.bf16)
    launch_cast_from_f32(dxacc, dx, (size_t)N * dm, 1, c.st);
  if (c.rect) {
    prof_mark(c.st, "bwd.dx_query_rows");
    launch_add_query_rows(dx, accq, Nq, shape->T, c.Tq, dm, c.bf16, c.st);
  }
  prof_mark(c.st, nullptr);
  return check_launch("switchhead_backward");
}

sh_status switchhead_get_routing(const sh_shape* shape, const void* workspace, size_t workspace_bytes,
                                 int32_t* topk_idx, float* gate, int32_t* perm, int32_t* expert_offsets,
                                 void* hip_stream) {
  sh_status r = check_shape(shape);
  if (r != SH_OK) return r;
  Layout L = make_layout(shape);
  if (!workspace) return fail(SH_ERR_INVALID_ARG, "workspace is NULL");
  if (workspace_bytes < L.total) return fail(SH_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
  const char* ws = (const char*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t n1 = (size_t)2 * shape->nheads * shape->B * shape->T * shape->k;
  hipError_t e = hipSuccess;
  if (topk_idx) e = hipMemcpyAsync(topk_idx, ws + L.idx, n1 * 4, hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess && gate) e = hipMemcpyAsync(gate, ws + L.gate, n1 * 4, hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess && perm) e = hipMemcpyAsync(perm, ws + L.perm, n1 * 4, hipMemcpyDeviceToDevice, st);
  if (e == hipSuccess && expert_offsets)
    e = hipMemcpyAsync(expert_offsets, ws + L.offsets, (size_t)2 * shape->nheads * (shape->E + 1) * 4,
                       hipMemcpyDeviceToDevice, st);
  if (e != hipSuccess) return fail(SH_ERR_HIP, "switchhead_get_routing: %s", hipGetErrorString(e));
  return SH_OK;
}

sh_status switchhead_get_intermediates(const sh_shape* shape, const void* workspace, size_t workspace_bytes, float* Q,
                                       float* K, float* V, float* ctx, float* lse, void* hip_stream) {
  sh_status r = check_shape(shape);
  if (r != SH_OK) return r;
  Layout L = make_layout(shape);
  if (!workspace) return fail(SH_ERR_INVALID_ARG, "workspace is NULL");
  if (workspace_bytes < L.total) return fail(SH_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
  const char* ws = (const char*)workspace;
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t n = (size_t)shape->B * shape->T * shape->nheads * shape->d_head;
  const int bf = shape->dtype == SH_BF16;
  if (Q) launch_cast_to_f32(ws + L.Q, Q, n, bf, st);
  if (K) launch_cast_to_f32(ws + L.K, K, n, bf, st);
  if (V) launch_cast_to_f32(ws + L.V, V, n, bf, st);
  if (ctx) launch_cast_to_f32(ws + L.ctx, ctx, n, bf, st);
  if (lse) {
    hipError_t e = hipMemcpyAsync(lse, ws + L.lse, (size_t)shape->B * shape->T * shape->nheads * 4,
                                  hipMemcpyDeviceToDevice, st);
    if (e != hipSuccess) return fail(SH_ERR_HIP, "switchhead_get_intermediates: %s", hipGetErrorString(e));
  }
  return check_launch("switchhead_get_intermediates");
}

}  // extern "C"
