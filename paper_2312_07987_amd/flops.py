"""Work model of the SwitchHead layer.

`macs_*`: the paper's multiply-accumulate counts per layer per sequence (App. A.2).
`layer_flops`: the algorithmic floating-point operations of one call of this library
(2 flop per MAC, causal attention counted on the unmasked half only), used by bench.py
to turn time into TFLOP/s.  Host logic only; nothing here runs on the GPU.
"""
from __future__ import annotations


def macs_dense_xl(nheads, d_head, d_model, T, C=2):
    """N_MAC^XL of App. A.2: H (4 T dh dm + 2 C T^2 dh + 2 C T dh dm)."""
    return nheads * (4 * T * d_head * d_model + 2 * C * T * T * d_head + 2 * C * T * d_head * d_model)


def mem_dense_xl(nheads, d_head, T, C=2):
    """N_mem^XL of App. A.2: H (4 T dh + 2 C T^2 + 2 C T dh)."""
    return nheads * (4 * T * d_head + 2 * C * T * T + 2 * C * T * d_head)


def macs_switchhead_printed(nheads, d_head, d_model, T, k, C=2):
    """N_MAC^SwitchHead exactly as printed in App. A.2 (two position-projection terms,
    no router term).  It does NOT reproduce the numbers in the paper's tables."""
    return nheads * (2 * T * d_head * d_model + 2 * T * k * d_head * (d_model + 1)
                     + 2 * C * T * T * d_head + 2 * C * T * d_head * d_model)


def macs_switchhead_tables(nheads, d_head, d_model, T, k, E, C=2):
    """The count that reproduces every SwitchHead MAC entry of the paper's tables:
    one position-projection term and the two routers (2 T dm E per head) added."""
    return nheads * (2 * T * d_head * d_model + 2 * T * k * d_head * (d_model + 1)
                     + 2 * C * T * T * d_head + C * T * d_head * d_model + 2 * T * d_model * E)


def mem_switchhead_tables(nheads, d_head, T, C=2):
    """Float count that reproduces the SwitchHead memory entries of the tables."""
    return nheads * (4 * T * d_head + 2 * C * T * T + C * T * d_head)


def layer_flops(B, T, d_model, nheads, d_head, E, k, causal=True, shared=False, dense=False, qk_experts=False, T_q=None):
    """Algorithmic flops of one forward / backward call of this library's layer (no
    positional term).  T_q < T: queries, destination-side routing and output only for the last
    T_q positions of every sequence (attention over a cached context).  Returns a dict of
    per-step and total counts."""
    Tq = T if not T_q else T_q
    N, Nq = B * T, B * Tq
    if dense:
        router = 0
    else:   # source router over every token, destination router (or the shared one again) over the queries
        router = 2 * d_model * nheads * E * ((N if shared and Tq == T else N + Nq))
    kq = k if qk_experts else 1   # k experts per token when queries and keys are banks
    qk = 2 * (N + Nq) * d_model * nheads * d_head * kq
    v = 2 * N * k * d_model * nheads * d_head
    o = 2 * Nq * k * d_model * nheads * d_head
    pairs = Tq * (T - Tq) + Tq * (Tq + 1) // 2 if causal else Tq * T
    attn = 4 * B * nheads * d_head * pairs
    fwd = router + qk + v + o + attn
    bwd = 2 * (router + qk + v + o) + (5 * attn) // 2
    return dict(router=router, qk=qk, v=v, o=o, attn=attn, fwd=fwd, bwd=bwd, fwd_bwd=fwd + bwd)
