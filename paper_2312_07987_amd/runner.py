"""Device-buffer plumbing around the C ABI for tests and bench.py: uploads one set of host
tensors, owns the workspace and the output buffers, and calls the library.  No arithmetic of
the layer happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding

_W = ("W_Q", "W_K", "W_V", "W_O", "W_S", "W_D")


class DeviceLayer:
    def __init__(self, cfg, host, device="cuda:0", dense=False):
        """cfg: dict with B, T, d_model, nheads, d_head, E, k, causal, dtype ('f32'|'bf16').
        host: dict of float32 numpy arrays as produced by inputs.make_inputs."""
        self.cfg = dict(cfg)
        self.dev = torch.device(device)
        self.tdtype = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        self.shape = binding.make_shape(cfg["B"], cfg["T"], cfg["d_model"], cfg["nheads"], cfg["d_head"],
                                        cfg["E"], cfg["k"], cfg.get("causal", 1), cfg["dtype"],
                                        cfg.get("qk_experts", 0), cfg.get("rope", 0), cfg.get("T_q", 0))
        up = lambda a, dt: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(self.dev).to(dt).contiguous()
        self.Tq = cfg.get("T_q", 0) or cfg["T"]      # queries per sequence (the last Tq positions)
        self.x = up(host["x"], self.tdtype)
        dy = host.get("dy")
        self.dy = up(None if dy is None else dy[:, cfg["T"] - self.Tq:], self.tdtype)
        self.W = {n: up(host.get(n), self.tdtype) for n in _W}
        if dense:
            self.W["W_S"] = self.W["W_D"] = None
        self.b_S = up(host.get("b_S"), torch.float32)
        self.b_D = up(host.get("b_D"), torch.float32)
        nbytes = binding.switchhead_workspace_bytes(self.shape)
        if nbytes == 0:
            raise binding.SwitchHeadError(-1, binding.switchhead_last_error())
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        self.y = torch.empty((cfg["B"], self.Tq, cfg["d_model"]), dtype=self.tdtype, device=self.dev)
        self.dx = torch.empty_like(self.x)
        f32 = lambda t: None if t is None else torch.empty(t.shape, dtype=torch.float32, device=self.dev)
        self.dW = {n: f32(self.W[n]) for n in _W}
        HE = cfg["nheads"] * cfg["E"]
        self.db_S = None if self.W["W_S"] is None else torch.empty(HE, dtype=torch.float32, device=self.dev)
        self.db_D = None if self.W["W_D"] is None else torch.empty(HE, dtype=torch.float32, device=self.dev)

    def forward(self, stream=None):
        W = self.W
        binding.switchhead_forward(self.shape, self.x, W["W_Q"], W["W_K"], W["W_V"], W["W_O"], W["W_S"], W["W_D"],
                                   self.b_S, self.b_D, self.y, self.ws, stream)

    def forward_static(self, stream=None):
        """The same forward pass on the library's built-in workspace (nothing of this object's `ws` is used)."""
        W = self.W
        binding.switchhead_forward_static(self.shape, self.x, W["W_Q"], W["W_K"], W["W_V"], W["W_O"], W["W_S"], W["W_D"],
                                          self.b_S, self.b_D, self.y, stream)

    def backward(self, stream=None):
        W, dW = self.W, self.dW
        binding.switchhead_backward(self.shape, self.x, W["W_Q"], W["W_K"], W["W_V"], W["W_O"], W["W_S"], W["W_D"],
                                    self.dy, self.ws, self.dx, dW["W_Q"], dW["W_K"], dW["W_V"], dW["W_O"],
                                    dW["W_S"], dW["W_D"], self.db_S, self.db_D, stream)

    def routing(self):
        c = self.cfg
        H, N, k, E = c["nheads"], c["B"] * c["T"], c["k"], c["E"]
        idx = torch.empty((2, H, N, k), dtype=torch.int32, device=self.dev)
        gate = torch.empty((2, H, N, k), dtype=torch.float32, device=self.dev)
        perm = torch.empty((2, H, N * k), dtype=torch.int32, device=self.dev)
        off = torch.empty((2, H, E + 1), dtype=torch.int32, device=self.dev)
        binding.switchhead_get_routing(self.shape, self.ws, idx, gate, perm, off)
        torch.cuda.synchronize()
        out = dict(idx=idx.cpu().numpy(), gate=gate.cpu().numpy(), perm=perm.cpu().numpy(), offsets=off.cpu().numpy())
        if self.Tq != c["T"]:
            # the destination side's block holds B*Tq tokens packed at its front
            Nq = c["B"] * self.Tq
            out["idx_D"] = out["idx"][1].reshape(-1)[:H * Nq * k].reshape(H, Nq, k)
            out["gate_D"] = out["gate"][1].reshape(-1)[:H * Nq * k].reshape(H, Nq, k)
            out["perm_D"] = out["perm"][1].reshape(-1)[:H * Nq * k].reshape(H, Nq * k)
        return out

    def intermediates(self):
        c = self.cfg
        H, N, dh = c["nheads"], c["B"] * c["T"], c["d_head"]
        bufs = {n: torch.empty((N, H, dh), dtype=torch.float32, device=self.dev) for n in ("Q", "K", "V", "ctx")}
        lse = torch.empty((c["B"], H, c["T"]), dtype=torch.float32, device=self.dev)
        binding.switchhead_get_intermediates(self.shape, self.ws, bufs["Q"], bufs["K"], bufs["V"], bufs["ctx"], lse)
        torch.cuda.synchronize()
        out = {n: t.cpu().numpy() for n, t in bufs.items()}
        if self.Tq != c["T"]:
            Nq = c["B"] * self.Tq
            for n in ("Q", "ctx"):
                out[n] = out[n].reshape(-1)[:Nq * H * dh].reshape(Nq, H, dh)
        out["lse"] = lse.cpu().numpy()
        return out

    def outputs(self):
        torch.cuda.synchronize()
        return self.y.float().cpu().numpy()

    def grads(self):
        torch.cuda.synchronize()
        g = {"dx": self.dx.float().cpu().numpy()}
        for n in _W:
            g["d" + n] = None if self.dW[n] is None else self.dW[n].cpu().numpy()
        g["db_S"] = None if self.db_S is None else self.db_S.cpu().numpy()
        g["db_D"] = None if self.db_D is None else self.db_D.cpu().numpy()
        return g
