"""Float64 CPU oracle for the SwitchHead attention layer (arXiv 2312.07987).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg; never by the product path.  It shares no code with the HIP kernels.

What it computes, in the paper's notation (Sec. 2.1 and 2.2):

  s_S^h = sigmoid(x W_S^h),  E_S^h = argtopk(s_S^h, k)          source-side router
  s_D^h = sigmoid(x W_D^h),  E_D^h = argtopk(s_D^h, k)          destination-side router
  Q^h = x W_Q^h,  K^h = x W_K^h                                  dense, one copy per head
    (or, when W_Q and W_K are given as expert banks, the form Sec. 2.2 states before it
     settles on dense queries and keys:
     K^h = sum_{e in E_S^h} s_S^h[e] x W_K^{h,e},  Q^h = sum_{e in E_D^h} s_D^h[e] x W_Q^{h,e})
  V^h = sum_{e in E_S^h} s_S^h[e] x W_V^{h,e}                    value experts
  A^h = softmax(Q^h K^h^T / sqrt(d_head))                        Sec. 2.1, first equation
  y   = sum_h sum_{e in E_D^h} s_D^h[e] A^h V^h W_O^{h,e}        output experts

With `T_q` < T the attention is the rectangular one of the paper's Transformer-XL models
(Sec. 3; App. A.2: keys and values of shape CT x d_head): x holds the cached positions
followed by the current chunk; keys, values and the source-side selection exist for all T
positions, queries, the destination-side selection and the output only for the last T_q.

Everything is plain numpy float64, written as the definitions read: no blocking, no
fusion, no reordering.  The paper gives no backward pass; `backward` is the chain rule
applied to the six forward steps (the top-k selection is piecewise constant, so only the
selected gates carry gradient).

Readings where the paper is silent (all listed in the design notes of the repository):
  * selection is made on the pre-sigmoid logit (sigmoid is strictly increasing, so the
    chosen set is the same in exact arithmetic); equal logits -> the lower index wins;
    the k slots are ordered by descending logit;
  * the router logit is the float64 sum over i = 0..d_model-1 taken IN THAT ORDER with a
    single accumulator, bias (if any) added last;
  * gates are not renormalised (non-competitive selection, Sec. 2.2);
  * causal mask: key u is visible to query t iff u <= t; masked logits are -inf;
  * no dropout, bias or normalisation inside the layer; no positional encoding unless
    `rope` is asked for: then queries and keys are rotated as in the rotary position
    embedding the paper's App. A.4 "RoPE Positional Encodings" models use (Su et al., RoFormer): element pair
    (2i, 2i+1) of every head's query and key at position t (index in its sequence, from 0)
    turns by the angle t * 10000^(-2i/d), d = the even part of d_head; an odd last element
    is left as it is.  The paper cites the method without restating it; the adjacent-pair
    form and base 10000 are the cited paper's own.

Pinned by tests/test_oracle_pins.py against: a dense-masked brute force in pure Python
loops, the k=E dense mixture, the single-expert case against a textbook concat-form MHA,
closed forms (all gates 0.5), invariants (causality, T=1, batch equivariance, permutation
properties), exact ties, central finite differences and torch.autograd of an independent
dense-masked formulation for the backward pass.
"""
from __future__ import annotations

import numpy as np

__all__ = ["router_logits", "select_topk", "routing_tables", "rotary", "forward", "backward"]


def _f64(a):
    return None if a is None else np.asarray(a, dtype=np.float64)


def router_logits(x2, W, b=None):
    """z[n, c] = sum_i x2[n, i] * W[i, c] (+ b[c]); Sec. 2.2, argument of the sigmoid.

    The sum runs over i ascending with one accumulator per output, so that the value is
    a fixed function of the inputs (a BLAS call would block the sum in an unspecified way).
    """
    x2 = _f64(x2)
    W = _f64(W)
    z = np.zeros((x2.shape[0], W.shape[1]), dtype=np.float64)
    for i in range(x2.shape[1]):
        z += x2[:, i:i + 1] * W[i:i + 1, :]
    if b is not None:
        z += _f64(b)[None, :]
    return z


def select_topk(z, nheads, k):
    """argtopk of Sec. 2.2 per (token, head): indices of the k largest logits, in
    descending order of logit, equal logits -> lower index first; gates = sigmoid(logit).

    z: [N, nheads*E] -> idx int32 [nheads, N, k], gate float64 [nheads, N, k],
    margin float64 [nheads, N] (gap between the k-th and (k+1)-th logit; inf if k == E).
    """
    N = z.shape[0]
    E = z.shape[1] // nheads
    zh = z.reshape(N, nheads, E).transpose(1, 0, 2)          # [H, N, E]
    order = np.argsort(-zh, axis=-1, kind="stable")          # stable: ties keep index order
    idx = order[..., :k].astype(np.int32)
    zsel = np.take_along_axis(zh, idx.astype(np.int64), axis=-1)
    gate = 1.0 / (1.0 + np.exp(-zsel))
    if k < E:
        znext = np.take_along_axis(zh, order[..., k:k + 1], axis=-1)[..., 0]
        margin = zsel[..., k - 1] - znext
    else:
        margin = np.full((nheads, N), np.inf)
    return idx, gate, margin


def routing_tables(idx, E):
    """Expert-sorted permutation of the N*k assignments of one (side, head).

    idx: int [N, k].  Assignment id a = n*k + j.  Returns
      perm    int32 [N*k]  assignment ids sorted by expert, stable (ascending a inside an expert)
      offsets int32 [E+1]  exclusive scan of the per-expert counts
      inv     int32 [N*k]  inverse permutation: inv[perm[p]] = p
    (the "sorting and top-k steps" mentioned in Sec. 3.6 "Shared Selection").
    """
    flat = np.asarray(idx).reshape(-1)
    perm = np.argsort(flat, kind="stable").astype(np.int32)
    counts = np.bincount(flat, minlength=E)
    offsets = np.zeros(E + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size, dtype=np.int32)
    return perm, offsets, inv


def rotary(P, pos, inverse=False):
    """Rotary position embedding of query or key rows (App. A.4 "RoPE Positional Encodings" of the paper, method of
    Su et al.): P [..., n, d_head] with `pos` [n] the position of each row; the pair
    (P[2i], P[2i+1]) is turned by the angle pos * 10000^(-2i/d), d = 2*floor(d_head/2).
    `inverse` turns by the opposite angle (the transpose of the rotation: what the chain
    rule applies to a gradient)."""
    P = np.asarray(P, dtype=np.float64)
    dh = P.shape[-1]
    half = dh // 2
    theta = 10000.0 ** (-2.0 * np.arange(half) / (2 * half)) if half else np.zeros(0)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]        # [n, half]
    if inverse:
        ang = -ang
    c, s_ = np.cos(ang), np.sin(ang)
    out = P.copy()
    a, b = P[..., 0:2 * half:2], P[..., 1:2 * half:2]
    out[..., 0:2 * half:2] = a * c - b * s_
    out[..., 1:2 * half:2] = a * s_ + b * c
    return out


def _attention_matrix(Qbh, Kbh, causal):
    """A = softmax(Q K^T / sqrt(d_head)) for one (sequence, head); Sec. 2.1.  With fewer
    queries than keys the queries are the LAST positions of the sequence (cached context in
    front, App. A.2): query i sits at position (Tk - Tq) + i and, if causal, sees the keys up
    to and including its own position."""
    Tq, dh = Qbh.shape
    Tk = Kbh.shape[0]
    S = (Qbh @ Kbh.T) / np.sqrt(float(dh))
    if causal:
        S = np.where(np.arange(Tk)[None, :] <= (np.arange(Tq) + (Tk - Tq))[:, None], S, -np.inf)
    S = S - S.max(axis=-1, keepdims=True)
    P = np.exp(S)
    return P / P.sum(axis=-1, keepdims=True)


def forward(x, W_Q, W_K, W_V, W_O, W_S, W_D=None, b_S=None, b_D=None, *, k, causal=True, rope=False, T_q=None):
    """One SwitchHead layer call.

    x [B,T,dm]; W_Q, W_K [H,dm,dh]; W_V [H,E,dm,dh]; W_O [H,E,dh,dm];
    W_Q, W_K may instead be expert banks [H,E,dm,dh] (all four projections mixtures of
    experts, Sec. 2.2): keys mix by the source-side selection, queries by the
    destination-side selection.
    W_S, W_D [dm, H*E] (column h*E+e); b_S, b_D [H*E] or None.
    W_D None  -> shared selection: the destination side reuses the source side's choice
                 (Sec. 3.6 "Shared Selection").
    W_S None  -> dense multi-head attention (requires E == 1; every gate is exactly 1;
                 Sec. 2.1, per-head-sum form of the output).
    T_q (None = T): only the last T_q positions of every sequence are queries; y is
    [B,T_q,dm], the destination-side tables cover B*T_q tokens, the source side all B*T.
    Returns a dict with y and every intermediate the backward pass and the tests need.
    """
    x, W_Q, W_K, W_V, W_O = map(_f64, (x, W_Q, W_K, W_V, W_O))
    B, T, dm = x.shape
    H, E = W_V.shape[0], W_V.shape[1]
    dh = W_V.shape[3]
    N = B * T
    x2 = x.reshape(N, dm)
    Tq = T if T_q is None else int(T_q)
    assert 1 <= Tq <= T
    Nq = B * Tq
    xq2 = x[:, T - Tq:, :].reshape(Nq, dm)        # the destination (query) tokens

    # step 1: routers (Sec. 2.2): source side over every token, destination side over the queries
    if W_S is None:
        assert E == 1 and k == 1
        zS = zD = None
        idx_S, idx_D = np.zeros((H, N, 1), dtype=np.int32), np.zeros((H, Nq, 1), dtype=np.int32)
        g_S, g_D = np.ones((H, N, 1)), np.ones((H, Nq, 1))
        mar_S, mar_D = np.full((H, N), np.inf), np.full((H, Nq), np.inf)
    else:
        zS = router_logits(x2, W_S, b_S)
        idx_S, g_S, mar_S = select_topk(zS, H, k)
        if W_D is None and Tq == T:
            zD, idx_D, g_D, mar_D = zS, idx_S, g_S, mar_S
        else:
            # shared selection with fewer queries: the same router evaluated on the query tokens
            zD = router_logits(xq2, W_S if W_D is None else W_D, b_S if W_D is None else b_D)
            idx_D, g_D, mar_D = select_topk(zD, H, k)

    # step 2: queries and keys
    assert W_Q.ndim == W_K.ndim
    if W_Q.ndim == 3:
        # dense, one copy per head
        Q = np.stack([xq2 @ W_Q[h] for h in range(H)], axis=1)      # [Nq,H,dh]
        K = np.stack([x2 @ W_K[h] for h in range(H)], axis=1)       # [N,H,dh]
    else:
        # K^h = sum_{e in E_S} s_S[e] x W_K^{h,e};  Q^h = sum_{e in E_D} s_D[e] x W_Q^{h,e}
        Q, K = np.zeros((Nq, H, dh)), np.zeros((N, H, dh))
        for h in range(H):
            for j in range(k):
                for e in range(E):
                    rows = np.nonzero(idx_D[h, :, j] == e)[0]
                    if rows.size:
                        Q[rows, h, :] += g_D[h, rows, j][:, None] * (xq2[rows] @ W_Q[h, e])
                    rows = np.nonzero(idx_S[h, :, j] == e)[0]
                    if rows.size:
                        K[rows, h, :] += g_S[h, rows, j][:, None] * (x2[rows] @ W_K[h, e])

    # rotary position embedding of queries and keys (App. A.4 "RoPE Positional Encodings"), position = index in the sequence
    if rope:
        pos, posq = np.tile(np.arange(T), B), np.tile(np.arange(T - Tq, T), B)
        for h in range(H):
            Q[:, h, :] = rotary(Q[:, h, :], posq)
            K[:, h, :] = rotary(K[:, h, :], pos)

    # step 3: V^h = sum_{e in E_S} s_S[e] x W_V^{h,e}
    V = np.zeros((N, H, dh))
    for h in range(H):
        for j in range(k):
            for e in range(E):
                rows = np.nonzero(idx_S[h, :, j] == e)[0]
                if rows.size:
                    V[rows, h, :] += g_S[h, rows, j][:, None] * (x2[rows] @ W_V[h, e])

    # step 4: one attention matrix per (sequence, head)
    ctx = np.zeros((Nq, H, dh))
    for b in range(B):
        sl, sq = slice(b * T, (b + 1) * T), slice(b * Tq, (b + 1) * Tq)
        for h in range(H):
            A = _attention_matrix(Q[sq, h], K[sl, h], causal)
            ctx[sq, h, :] = A @ V[sl, h]

    # step 5: y = sum_h sum_{e in E_D} s_D[e] (A V) W_O^{h,e}
    y = np.zeros((Nq, dm))
    for h in range(H):
        for j in range(k):
            for e in range(E):
                rows = np.nonzero(idx_D[h, :, j] == e)[0]
                if rows.size:
                    y[rows] += g_D[h, rows, j][:, None] * (ctx[rows, h, :] @ W_O[h, e])

    # step 6: routing artefacts per (side, head)
    tabs = {}
    for name, idx in (("S", idx_S), ("D", idx_D)):
        pr, of, iv = zip(*(routing_tables(idx[h], E) for h in range(H)))
        tabs["perm_" + name] = np.stack(pr)
        tabs["offsets_" + name] = np.stack(of)
        tabs["inv_" + name] = np.stack(iv)

    out = dict(y=y.reshape(B, Tq, dm), T_q=Tq, Q=Q, K=K, V=V, ctx=ctx, zS=zS, zD=zD,
               idx_S=idx_S, idx_D=idx_D, gate_S=g_S, gate_D=g_D,
               margin_S=mar_S, margin_D=mar_D, k=k, causal=causal, rope=bool(rope),
               shared=(W_S is not None and W_D is None), dense=(W_S is None))
    # (with shared selection and T_q < T the destination tables are the source router's, evaluated on
    #  the query tokens: the same numbers as the source tables' rows of those tokens)
    out.update(tabs)
    return out


def backward(x, W_Q, W_K, W_V, W_O, W_S, W_D, fwd, dy):
    """Gradients of sum(y * dy) w.r.t. every input of `forward` (chain rule; the paper
    prints no backward equations, it trains with automatic differentiation, App. A.2).

    `fwd` is the dict returned by `forward` on the same inputs.  Returns dx [B,T,dm],
    dW_Q, dW_K, dW_V, dW_O, dW_S, dW_D, db_S, db_D (router entries None in dense mode;
    dW_D/db_D None with shared selection, whose dW_S collects both sides).
    """
    x, W_Q, W_K, W_V, W_O, dy = map(_f64, (x, W_Q, W_K, W_V, W_O, dy))
    W_S, W_D = _f64(W_S), _f64(W_D)
    B, T, dm = x.shape
    H, E = W_V.shape[0], W_V.shape[1]
    dh = W_V.shape[3]
    N = B * T
    k, causal = fwd["k"], fwd["causal"]
    Tq = fwd.get("T_q", T)
    Nq = B * Tq
    qrows = (np.arange(B)[:, None] * T + np.arange(T - Tq, T)[None, :]).reshape(-1)   # query tokens' rows of x
    x2, dy2 = x.reshape(N, dm), dy.reshape(Nq, dm)
    xq2 = x2[qrows]
    Q, K, V, ctx = fwd["Q"], fwd["K"], fwd["V"], fwd["ctx"]
    idx_S, idx_D, g_S, g_D = fwd["idx_S"], fwd["idx_D"], fwd["gate_S"], fwd["gate_D"]

    dx = np.zeros((N, dm))
    dW_Q, dW_K = np.zeros_like(W_Q), np.zeros_like(W_K)
    dW_V, dW_O = np.zeros_like(W_V), np.zeros_like(W_O)

    # output experts: y[n] = sum_h sum_j gD * ctx[n,h] W_O[h,e_j]
    dgD = np.zeros((H, Nq, k))
    dctx = np.zeros((Nq, H, dh))
    for h in range(H):
        for j in range(k):
            for e in range(E):
                rows = np.nonzero(idx_D[h, :, j] == e)[0]
                if not rows.size:
                    continue
                g = g_D[h, rows, j][:, None]
                P6 = ctx[rows, h, :] @ W_O[h, e]                       # [r, dm]
                dgD[h, rows, j] = np.sum(P6 * dy2[rows], axis=1)
                dctx[rows, h, :] += g * (dy2[rows] @ W_O[h, e].T)
                dW_O[h, e] += (g * ctx[rows, h, :]).T @ dy2[rows]

    # attention: ctx = A V, A = softmax(S), S = Q K^T / sqrt(dh)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    scale = 1.0 / np.sqrt(float(dh))
    for b in range(B):
        sl, sq = slice(b * T, (b + 1) * T), slice(b * Tq, (b + 1) * Tq)
        for h in range(H):
            A = _attention_matrix(Q[sq, h], K[sl, h], causal)
            dV[sl, h] = A.T @ dctx[sq, h]
            dA = dctx[sq, h] @ V[sl, h].T
            dS = A * (dA - np.sum(dA * A, axis=-1, keepdims=True))
            dQ[sq, h] = (dS @ K[sl, h]) * scale
            dK[sl, h] = (dS.T @ Q[sq, h]) * scale

    # back through the rotation of queries and keys: the transpose of a rotation is the opposite turn
    if fwd.get("rope"):
        pos, posq = np.tile(np.arange(T), B), np.tile(np.arange(T - Tq, T), B)
        for h in range(H):
            dQ[:, h, :] = rotary(dQ[:, h, :], posq, inverse=True)
            dK[:, h, :] = rotary(dK[:, h, :], pos, inverse=True)

    # value experts: V[n,h] = sum_j gS * x[n] W_V[h,e_j]
    dgS = np.zeros((H, N, k))
    for h in range(H):
        for j in range(k):
            for e in range(E):
                rows = np.nonzero(idx_S[h, :, j] == e)[0]
                if not rows.size:
                    continue
                g = g_S[h, rows, j][:, None]
                P3 = x2[rows] @ W_V[h, e]                              # [r, dh]
                dgS[h, rows, j] = np.sum(P3 * dV[rows, h, :], axis=1)
                dW_V[h, e] += (g * x2[rows]).T @ dV[rows, h, :]
                dx[rows] += g * (dV[rows, h, :] @ W_V[h, e].T)

    if W_Q.ndim == 3:
        # dense queries and keys
        for h in range(H):
            dW_Q[h] = xq2.T @ dQ[:, h, :]
            dW_K[h] = x2.T @ dK[:, h, :]
            dx += dK[:, h, :] @ W_K[h].T
            dx[qrows] += dQ[:, h, :] @ W_Q[h].T
    else:
        # expert queries (destination-side gates) and keys (source-side gates): same pattern as
        # the value experts; the gates collect one more term each
        allrows = np.arange(N)
        for W, dW, dP, idx, g_, dg, xs, xrow in ((W_Q, dW_Q, dQ, idx_D, g_D, dgD, xq2, qrows),
                                                 (W_K, dW_K, dK, idx_S, g_S, dgS, x2, allrows)):
            for h in range(H):
                for j in range(k):
                    for e in range(E):
                        rows = np.nonzero(idx[h, :, j] == e)[0]
                        if not rows.size:
                            continue
                        g = g_[h, rows, j][:, None]
                        P2 = xs[rows] @ W[h, e]                            # [r, dh]
                        dg[h, rows, j] += np.sum(P2 * dP[rows, h, :], axis=1)
                        dW[h, e] += (g * xs[rows]).T @ dP[rows, h, :]
                        dx[xrow[rows]] += g * (dP[rows, h, :] @ W[h, e].T)

    # routers: g = sigmoid(z) at the selected entries, nothing elsewhere
    dW_S = dW_D = db_S = db_D = None
    if not fwd["dense"]:
        def dz_of(idx, g, dg):
            n = idx.shape[1]
            dz = np.zeros((n, H * E))
            for h in range(H):
                for j in range(k):
                    dz[np.arange(n), h * E + idx[h, :, j]] += dg[h, :, j] * g[h, :, j] * (1.0 - g[h, :, j])
            return dz
        dzS = dz_of(idx_S, g_S, dgS)
        dzD = dz_of(idx_D, g_D, dgD)
        if fwd["shared"]:
            # one router serves both sides: its gradient collects both (the query tokens' rows twice)
            dW_S, db_S = x2.T @ dzS + xq2.T @ dzD, dzS.sum(axis=0) + dzD.sum(axis=0)
            dx += dzS @ W_S.T
            dx[qrows] += dzD @ W_S.T
        else:
            dW_S, db_S = x2.T @ dzS, dzS.sum(axis=0)
            dW_D, db_D = xq2.T @ dzD, dzD.sum(axis=0)
            dx += dzS @ W_S.T
            dx[qrows] += dzD @ W_D.T

    return dict(dx=dx.reshape(B, T, dm), dW_Q=dW_Q, dW_K=dW_K, dW_V=dW_V, dW_O=dW_O,
                dW_S=dW_S, dW_D=dW_D, db_S=db_S, db_D=db_D,
                dQ=dQ, dK=dK, dV=dV, dctx=dctx, dgate_S=dgS, dgate_D=dgD)
