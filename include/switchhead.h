/*
 * switchhead.h - C ABI of the SwitchHead attention layer for AMD MI355X (gfx950).
 *
 * The layer is the one defined in arXiv 2312.07987, Sec. 2.2 ("From Dense to SwitchHead
 * Attention Layer"): per head h a source-side and a destination-side sigmoid router pick
 * k of E experts per token; queries and keys are dense per head; the value projection and
 * the output projection are gate-weighted sums over the selected experts; one softmax
 * attention matrix is computed per head (Sec. 2.1, first equation).
 *
 * Conventions shared by every entry point
 *   - every tensor pointer is a DEVICE pointer to row-major, contiguous memory owned by
 *     the caller; the library allocates no device memory and frees none;
 *   - `workspace` is caller-owned device memory of at least
 *     switchhead_workspace_bytes(shape) bytes, 256-byte aligned; forward fills it,
 *     backward and get_routing read what forward left there (same shape, untouched);
 *   - calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without synchronising;
 *   - arguments are checked on the host before anything is launched; a failed check
 *     returns an error code, launches nothing and leaves every buffer untouched;
 *     switchhead_last_error() then gives a description (thread-local, static storage);
 *   - storage type of x, weights, y, dy, dx is shape->dtype (fp32 or bf16); arithmetic
 *     accumulates in fp32; the routers' selection is that of the fp64 logits (see
 *     switchhead_forward); weight and bias gradients are always fp32;
 *   - alignment: x, y, dy, dx, the weight tensors and the workspace are read and written
 *     with 16-byte vector accesses by the matrix-core kernels; with bf16 storage a tensor
 *     pointer that is not 16-byte aligned makes the call take the plain kernels for the
 *     whole layer (same results, slower);
 *   - two calls that share a workspace must not overlap in time.
 */
#ifndef SWITCHHEAD_H
#define SWITCHHEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  SH_OK = 0,
  SH_ERR_INVALID_ARG = 1,         /* null required pointer, dimension < 1, k > E, ...      */
  SH_ERR_UNSUPPORTED = 2,         /* a limit of the kernels: E > 64, k > 8, d_head > 256   */
  SH_ERR_WORKSPACE_TOO_SMALL = 3,
  SH_ERR_HIP = 4                  /* a HIP runtime call (launch, copy) reported an error   */
} sh_status;

typedef enum { SH_F32 = 0, SH_BF16 = 1 } sh_dtype;

/* Problem shape, in the paper's notation (Sec. 2.1-2.2): T sequence length, d_model,
 * nheads = number of attention matrices, d_head, E experts per head, k active experts. */
typedef struct {
  int32_t B;        /* sequences per call                                                 */
  int32_t T;        /* tokens per sequence                                                */
  int32_t d_model;
  int32_t nheads;
  int32_t d_head;
  int32_t E;
  int32_t k;
  int32_t causal;   /* 1: key u visible to query t iff u <= t; 0: full attention (the
                       paper's ListOps analysis, Sec. 4, uses the unmasked form)          */
  int32_t dtype;    /* sh_dtype                                                           */
  int32_t qk_experts; /* 0: SwitchHead proper, one dense W_Q and W_K per head (Sec. 2.2, last
                       paragraph; Sec. 3.1 finds query/key experts unnecessary).
                       1: the form Sec. 2.2 states first, all four projections mixtures of
                       experts: W_Q, W_K (and dW_Q, dW_K) are expert banks
                       [nheads, E, d_model, d_head] like W_V;
                       K^h = sum_{e in E_S^h} s_S^h[e] x W_K^{h,e} (source-side selection),
                       Q^h = sum_{e in E_D^h} s_D^h[e] x W_Q^{h,e} (destination side)      */
  int32_t rope;     /* 1: rotary position embedding of queries and keys, as in the models of the
                       paper's App. A.4 "RoPE Positional Encodings" (method of Su et al.; square attention, no cache): the
                       element pair (2i, 2i+1) of every head's query and key at position t (index
                       in its sequence, from 0) turns by t * 10000^(-2i/d), d = the even part of
                       d_head; an odd last element stays.  0: no position term (Sec. 2.2 as
                       written)                                                            */
  int32_t T_q;      /* queries per sequence; 0 or T: every position is a query (square attention).
                       0 < T_q < T: attention over a cached context as in the paper's
                       Transformer-XL models (Sec. 3; App. A.2, keys and values of shape CT x d_head):
                       x holds the cached positions followed by the current chunk; keys, values
                       and the source-side selection are computed for all T positions, queries,
                       the destination-side selection and the output only for the last T_q;
                       query i sees keys u <= (T - T_q) + i when causal, and rotary positions
                       count from the start of x.  Then y and dy are [B, T_q, d_model]; dx stays
                       [B, T, d_model] and is the full gradient (a trainer that treats the cache
                       as constant ignores its first T - T_q rows); in the routing tables and
                       intermediates the destination-side blocks and Q, ctx keep their place but
                       hold B*T_q tokens, packed at the front of the block.  With shared
                       selection the one router is evaluated on the query tokens for the
                       destination side, and its gradients collect both sides.  No relative
                       position term is added (the paper does not define one)               */
} sh_shape;

/* Bytes of workspace a forward (+ backward) call of this shape needs; 0 if the shape is
 * invalid or unsupported (switchhead_last_error() says why).  Host-only, no GPU needed.  */
size_t switchhead_workspace_bytes(const sh_shape* shape);

/* The two parts of that workspace (their sum is switchhead_workspace_bytes; either pointer may be NULL):
 *   kept     what forward leaves for backward, get_routing and get_intermediates: the routing tables
 *            (top-k indices, gates, permutation, offsets; with bf16 storage the dense gate table or the
 *            expert-set tables), Q, K, V, the attention read-out and its log-sum-exp, and the unscaled
 *            value rows of every slot [nheads, N*k, d_head] that the gates' gradient reads - the one kept
 *            buffer that grows with k (App. A.2 "Resource Usage of Different Methods" counts the k-weighted
 *            average as free; storing the slot rows is this build's choice against a second pass over x);
 *   scratch  buffers one pass writes and reads itself (fp32 accumulators, per-slot gradient rows,
 *            dQ/dK/dV, weight-gradient partial sums, router scratch, and with bf16 storage and head
 *            widths 64..128 the attention's score gradient [B, nheads, T, T_q] in bf16 (under the causal
 *            mask only the visible half), which the backward keeps between its dK/dV and dQ kernels:
 *            quadratic in T, used up to
 *            1 GiB, recomputed beyond; it shares the place of other scratch where it fits); their
 *            contents mean nothing between calls.  The two parts are interleaved in the buffer: this call reports sizes, not
 *            address ranges, and the whole workspace must stay untouched between forward and backward.
 * Host-only.  Returns SH_OK or the shape's error. */
sh_status switchhead_workspace_parts(const sh_shape* shape, size_t* kept_bytes, size_t* scratch_bytes);

/*
 * Forward pass: Sec. 2.2, the equations for s_S, E_S, s_D, E_D, V^h and y.
 *
 *   x    [B, T, d_model]                     input
 *   W_Q  [nheads, d_model, d_head]           dense query projection per head
 *   W_K  [nheads, d_model, d_head]           dense key projection per head
 *        (both [nheads, E, d_model, d_head] when shape->qk_experts == 1)
 *   W_V  [nheads, E, d_model, d_head]        value experts
 *   W_O  [nheads, E, d_head, d_model]        output experts
 *   W_S  [d_model, nheads*E]                 source-side router, column h*E+e.
 *                                            NULL = dense multi-head attention (needs
 *                                            E == 1, k == 1; every gate is 1; Sec. 2.1)
 *   W_D  [d_model, nheads*E]                 destination-side router; NULL = shared
 *                                            selection, the destination side reuses the
 *                                            source side's choice and gates (Sec. 3.6 "Shared Selection")
 *   b_S, b_D  fp32 [nheads*E] or NULL        logit bias added after the sum (not in the
 *                                            paper; used to skew the routing on purpose)
 *   y    [B, T, d_model]                     output, overwritten
 *
 * Selection: the canonical logit is z = x W (+ b) in fp64, products summed over
 * i = 0..d_model-1 in that order with one accumulator, bias last; the k largest logits
 * win, equal logits -> lower expert index; slots are ordered by descending logit; gates
 * are not renormalised.  fp32 storage evaluates exactly that sum.  bf16 storage on the
 * matrix-core kernels is two-stage: fp32 matrix-core partial sums (64 terms each, added up
 * in fp64) decide every choice whose margin exceeds a proven bound of their error; every
 * other choice (and every exact tie) is re-evaluated in fp64, and where two of those
 * fp64 logits are closer than the reordering error of a blocked fp64 sum, by the canonical
 * sum itself - so the indices are always those of the canonical logits.  gate = sigmoid(z)
 * stored as fp32 (on that two-stage path z is the first-stage logit where it decided:
 * gates agree with the canonical ones to about 1e-6 relative).  Per (side, head) the
 * N*k assignments a = n*k + j (n = b*T + t) are stably sorted by expert into `perm`, with
 * `offsets[e]` = first position of expert e.
 */
sh_status switchhead_forward(const sh_shape* shape,
                             const void* x, const void* W_Q, const void* W_K,
                             const void* W_V, const void* W_O,
                             const void* W_S, const void* W_D,
                             const float* b_S, const float* b_D,
                             void* y,
                             void* workspace, size_t workspace_bytes,
                             void* hip_stream);

/*
 * Forward pass for callers that cannot allocate device memory (code under HIP graph capture,
 * serving loops, harnesses that forbid hipMalloc): the same computation and the same kernels
 * as switchhead_forward, with the workspace taken from a device array built into the library
 * instead of a caller's buffer.  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine) as long as the step profiler is off.
 *   - limit: shapes with switchhead_workspace_bytes(shape) <= SWITCHHEAD_STATIC_WORKSPACE_BYTES;
 *     a larger shape returns SH_ERR_WORKSPACE_TOO_SMALL before anything is launched;
 *   - the array exists once per GPU from the first use of the library on it until the
 *     process ends; the call uses the copy of the GPU that is current when it is made;
 *   - every call on a GPU shares that GPU's array, which keeps the previous call's contents
 *     (the forward pass clears what it needs cleared): calls that overlap in time on one GPU,
 *     on whatever streams, race; the intermediates are not kept for a backward call.
 * Arguments as for switchhead_forward, without the workspace.
 */
#define SWITCHHEAD_STATIC_WORKSPACE_BYTES (16u << 20)
sh_status switchhead_forward_static(const sh_shape* shape,
                                    const void* x, const void* W_Q, const void* W_K,
                                    const void* W_V, const void* W_O,
                                    const void* W_S, const void* W_D,
                                    const float* b_S, const float* b_D,
                                    void* y,
                                    void* hip_stream);

/*
 * Backward pass: the chain rule through the six steps of the forward pass (the paper
 * trains with automatic differentiation and prints no backward equations; App. A.2 only
 * notes that all intermediate results are stored).  The top-k choice is piecewise
 * constant: only the selected gates carry gradient, through sigmoid' = g (1 - g).
 *
 *   inputs   the same x, W_* (and shape) that were given to forward; dy [B, T, d_model];
 *            `workspace` exactly as forward left it
 *   outputs  dx [B, T, d_model] in shape->dtype; dW_Q, dW_K, dW_V, dW_O, dW_S, dW_D fp32
 *            with the shapes of the corresponding weights; db_S, db_D fp32 [nheads*E].
 *            All are overwritten; an expert no token chose gets zeros.
 *            dW_S, dW_D, db_S, db_D may be NULL when not wanted; dW_D/db_D are ignored
 *            with shared selection (dW_S then holds the sum of both sides) and all four
 *            are ignored in dense mode.
 * Determinism: with bf16 storage and the matrix-core kernels, dW_Q, dW_K, dW_V, dW_O are
 * sums of per-chunk partial results added in a fixed order (bit-identical from run to run),
 * and so are the router gradients dW_S, dW_D, db_S, db_D where they ride along the query/key
 * weight-gradient launch (square attention, dense queries and keys, 2 * nheads * E, each side
 * rounded up to a multiple of 8, not above d_head).  Otherwise the router gradients, and every
 * weight gradient of the plain fp32 kernels, are accumulated with fp32 atomic adds over token
 * chunks, so their last bits may differ from run to run.
 */
sh_status switchhead_backward(const sh_shape* shape,
                              const void* x, const void* W_Q, const void* W_K,
                              const void* W_V, const void* W_O,
                              const void* W_S, const void* W_D,
                              const void* dy,
                              void* workspace, size_t workspace_bytes,
                              void* dx,
                              float* dW_Q, float* dW_K, float* dW_V, float* dW_O,
                              float* dW_S, float* dW_D, float* db_S, float* db_D,
                              void* hip_stream);

/*
 * Copies the routing artefacts of the last forward call out of `workspace`
 * (device-to-device, asynchronous on `hip_stream`); any destination may be NULL.
 *   topk_idx        int32 [2, nheads, N, k]      side 0 = source, 1 = destination
 *   gate            fp32  [2, nheads, N, k]      sigmoid of the selected logits
 *   perm            int32 [2, nheads, N*k]       assignment ids sorted by expert (stable)
 *   expert_offsets  int32 [2, nheads, E+1]       exclusive scan of per-expert counts
 * With shared selection (or dense mode) side 1 repeats side 0.  (Sec. 2.2 defines the
 * sets E_S, E_D and scores; Sec. 3.6 "Shared Selection" names the sorting step that `perm` is the result of.)
 */
sh_status switchhead_get_routing(const sh_shape* shape,
                                 const void* workspace, size_t workspace_bytes,
                                 int32_t* topk_idx, float* gate,
                                 int32_t* perm, int32_t* expert_offsets,
                                 void* hip_stream);

/*
 * Copies intermediates of the last forward call out of `workspace`, converted to fp32
 * (device-to-device, asynchronous); any destination may be NULL.  For tests and debugging.
 *   Q, K, V, ctx  fp32 [N, nheads, d_head]   queries, keys, mixed values V^h (Sec. 2.2),
 *                                            attention read-out A^h V^h
 *   lse           fp32 [B, nheads, T_q]      natural-log sum of exp of the scaled logits
 *                                            (T_q = T for square attention)
 * With 0 < T_q < T, Q and ctx hold B*T_q rows packed at the front of their [N, ...] blocks.
 */
sh_status switchhead_get_intermediates(const sh_shape* shape,
                                       const void* workspace, size_t workspace_bytes,
                                       float* Q, float* K, float* V, float* ctx, float* lse,
                                       void* hip_stream);

/* Description of the last error on this thread ("" if none). Never NULL. */
const char* switchhead_last_error(void);

/* Selects the kernel family for later calls on any thread: 0 = automatic (MFMA kernels
 * for bf16 shapes they support, plain fp32 kernels otherwise), 1 = always the plain fp32
 * kernels.  Returns the previous value.  Used by tests to cross-check both families.     */
int32_t switchhead_set_kernel_family(int32_t family);

/*
 * Per-step timing for benchmarks (not part of the method).  While enabled, forward and
 * backward record one HIP event on the launch stream before each step of the layer
 * ("fwd.v_experts", "bwd.attention", ...).  switchhead_profile_read waits for the recorded
 * events, adds up the elapsed time and the number of occurrences per step label over all
 * calls since the last read (or enable), writes up to max_entries of them (labels as one
 * '\n'-separated string) and returns how many it wrote.  Host-side events only: no device
 * memory is allocated.  Enabling or reading resets the record.
 */
sh_status switchhead_profile_enable(int32_t on);
int32_t switchhead_profile_read(char* labels, size_t labels_bytes, float* total_ms,
                                int32_t* launches, int32_t max_entries);

/* Library version, "major.minor". */
const char* switchhead_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SWITCHHEAD_H */
