"""Seeded synthetic inputs for the SwitchHead layer.

This module holds no arithmetic of the method itself: it only draws Gaussian tensors of
the shapes the paper trains with (hyper-parameter table of App. A.5 "Hyperparameters") and rounds them to
the storage type.  Both the float64 oracle (through the tests) and the HIP path consume
exactly the arrays produced here.

Recipe: x ~ N(0,1); W_Q, W_K, W_V ~ N(0, 1/d_model); W_O ~ N(0, 1/d_head);
W_S, W_D ~ N(0, 1/d_model); upstream gradient dy ~ N(0,1).  Drawn with
numpy.random.default_rng(seed).standard_normal(float32) in the fixed order
x, W_Q, W_K, W_V, W_O, W_S, W_D, dy.  bf16 workloads round every tensor to bf16
(round-to-nearest-even) once; the rounded values are what every consumer sees.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 20231207

# name, storage dtype, B, T, d_model, nheads, d_head, E, k, causal, bias on expert 0
CONFIGS = [
    dict(name="c0", dtype="f32", B=2, T=64, d_model=64, nheads=2, d_head=32, E=4, k=2, causal=1, bias0=0.0),
    dict(name="c1", dtype="bf16", B=64, T=256, d_model=412, nheads=2, d_head=76, E=5, k=3, causal=1, bias0=0.0),
    dict(name="c2", dtype="bf16", B=32, T=512, d_model=1024, nheads=4, d_head=128, E=5, k=3, causal=1, bias0=0.0),
    dict(name="c3", dtype="bf16", B=4, T=4096, d_model=1024, nheads=4, d_head=128, E=8, k=2, causal=1, bias0=0.0),
    dict(name="c4", dtype="bf16", B=32, T=512, d_model=1024, nheads=4, d_head=128, E=5, k=3, causal=1, bias0=3.0),
]


def config(name_or_index):
    if isinstance(name_or_index, int):
        return dict(CONFIGS[name_or_index])
    for c in CONFIGS:
        if c["name"] == name_or_index:
            return dict(c)
    raise KeyError(name_or_index)


def to_bf16_bits(a):
    """float32 array -> uint16 array of bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b):
    """uint16 array of bf16 bit patterns -> float32 array (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a):
    """float32 array -> float32 array whose values are all bf16-representable."""
    return from_bf16_bits(to_bf16_bits(a))


def make_inputs(cfg, seed=None, shared_router=False):
    """Draw every tensor of one layer call for `cfg` (a dict like the CONFIGS entries).

    Returns float32 arrays (already rounded to bf16-representable values when
    cfg['dtype'] == 'bf16'): x, W_Q, W_K, W_V, W_O, W_S, W_D, b_S, b_D, dy.
    b_S and b_D are None unless cfg['bias0'] != 0 (then +bias0 on column h*E+0).
    cfg['qk_experts'] (optional, default 0): W_Q and W_K are expert banks [H,E,dm,dh].
    """
    if seed is None:
        names = [c["name"] for c in CONFIGS]
        seed = BASE_SEED + (names.index(cfg["name"]) if cfg.get("name") in names else 0)
    rng = np.random.default_rng(seed)
    B, T, dm, H, dh, E = (cfg[s] for s in ("B", "T", "d_model", "nheads", "d_head", "E"))

    def draw(shape, std):
        return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)

    t = {}
    t["x"] = draw((B, T, dm), 1.0)
    qk_shape = (H, E, dm, dh) if cfg.get("qk_experts") else (H, dm, dh)
    t["W_Q"] = draw(qk_shape, dm ** -0.5)
    t["W_K"] = draw(qk_shape, dm ** -0.5)
    t["W_V"] = draw((H, E, dm, dh), dm ** -0.5)
    t["W_O"] = draw((H, E, dh, dm), dh ** -0.5)
    t["W_S"] = draw((dm, H * E), dm ** -0.5)
    t["W_D"] = draw((dm, H * E), dm ** -0.5)
    t["dy"] = draw((B, T, dm), 1.0)
    if cfg["dtype"] == "bf16":
        t = {n: round_to_bf16(a) for n, a in t.items()}
    if shared_router:
        t["W_D"] = None
    bias0 = float(cfg.get("bias0", 0.0))
    if bias0 != 0.0:
        b = np.zeros(H * E, dtype=np.float32)
        b[0::E] = bias0
        t["b_S"], t["b_D"] = b, (None if shared_router else b.copy())
    else:
        t["b_S"] = t["b_D"] = None
    return t
