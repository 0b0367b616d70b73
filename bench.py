#!/usr/bin/env python3
"""Benchmark of the SwitchHead attention layer on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2]

One step = one forward + backward pass of the whole layer (router, top-k, permutation, Q/K
projections, value experts, attention, output experts and every gradient) over one batch
of synthetic input that is already resident in HBM.  Prints ONE JSON line:
value = tokens/s of forward+backward; `extra` carries the forward-only figure and the
per-step times; `roofline` describes the step that takes the most time, measured with HIP
events recorded by the library on the launch stream; `cpu_baseline` is the float64 oracle
timed on the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_VEC_TFLOPS = 157.3  # MI355X fp32 vector ALU: what the plain fp32 kernels (fp32 storage) run on
PEAK_FP64_VEC_TFLOPS = 78.6   # MI355X fp64 vector ALU (256 CUs x 4 SIMD x 16 lanes x 2 x 2.4 GHz)
PEAK_HBM_GBS = 8000.0


def step_work(cfg):
    """Algorithmic flops (MFMA-bound steps) and bytes (HBM-bound steps) per launch of each step."""
    B, T, dm, H, dh, E, k = (cfg[s] for s in ("B", "T", "d_model", "nheads", "d_head", "E", "k"))
    N = B * T
    Tq = cfg.get("T_q") or T              # queries per sequence (destination-side tokens)
    Nq = B * Tq
    es = 2 if cfg["dtype"] == "bf16" else 4
    pairs = Tq * (T - Tq) + Tq * (Tq + 1) // 2 if cfg["causal"] else Tq * T
    proj = 2 * N * dm * H * dh
    proj_q = 2 * Nq * dm * H * dh
    expert = 2 * N * k * dm * H * dh
    expert_q = 2 * Nq * k * dm * H * dh
    attn = 4 * B * H * dh * pairs
    router = 2 * (N + Nq) * dm * H * E
    slots = N * H * k * dh * 4
    flops = {
        "fwd.q_proj": proj_q, "fwd.k_proj": proj, "fwd.qk_proj": 2 * proj, "bwd.qk_dgrad": proj + (proj if Tq == T else 0),
        "fwd.v_experts": expert, "fwd.o_experts": expert_q,
        "fwd.attention": attn, "bwd.attention": 5 * attn // 2,
        # backward attention = 5 matmuls of attn/2 flops each: S and dP (shared), dV, dK, dQ; the dK/dV
        # kernel is credited with four of them, the dQ kernel with dQ alone (it reads the score gradient the
        # dK/dV kernel left, or recomputes S and dP where that scratch is not used: not algorithmic work)
        "bwd.attention_dkv": 2 * attn, "bwd.attention_dq": attn // 2,
        "bwd.o_dgrad": expert_q, "bwd.o_wgrad": expert_q, "bwd.v_wgrad": expert, "bwd.v_dgrad": expert,
        "bwd.q_wgrad": proj_q, "bwd.k_wgrad": proj, "bwd.qk_wgrad": proj + proj_q, "bwd.q_dgrad": proj_q, "bwd.k_dgrad": proj,
        "bwd.router_wgrad": router, "bwd.router_dgrad": router,
        # all of dx as one GEMM: the value experts' input gradient, the queries' and keys', the routers'
        "bwd.dx_gemm": expert + proj + proj_q + router,
        # query / key expert banks (all-expert form): each step has the shape of its value-expert twin
        "fwd.q_experts": expert_q, "fwd.k_experts": expert, "bwd.q_wgrad_e": expert_q, "bwd.k_wgrad_e": expert,
        "bwd.q_dgrad_e": expert_q, "bwd.k_dgrad_e": expert,
    }
    alu = {"fwd.router": router}
    nbytes = {
        "fwd.v_combine": slots + N * H * dh * es + N * H * k * 4,
        "bwd.dctx_combine": slots + 2 * N * H * dh * es + 2 * N * H * k * 4,
        "bwd.dgate_s": slots + N * H * dh * es + N * H * k * 4,
        "fwd.y_zero": N * dm * 4, "bwd.dx_zero": N * dm * 4,
        "fwd.y_sum": N * dm * es * (H + 1), "fwd.set_sort": 2 * H * N * (k * 8 + 12),
        "fwd.y_cast": N * dm * (4 + es), "bwd.dx_cast": N * dm * (4 + es),
        "bwd.zero_dw": 4 * (2 * H * dm * dh + 2 * H * E * dm * dh),
        "bwd.router": 4 * H * N * k * 4 + N * 2 * H * E * es,
        "fwd.rope": 4 * N * H * dh * es, "bwd.rope": 4 * N * H * dh * es,   # Q and K (dQ and dK) read and written
        "fwd.gate_table": 2 * H * N * (k * 8 + E * 4),
    }
    return flops, alu, nbytes


# Which kernel a profiled step launches, as a pattern on the kernel name rocprofv3 reports
# (row GEMM: "..., <B transposed>, <tag>, <segment mode>>"; weight gradient: "..., <vec>, <tag>>").
STEP_KERNEL = {
    "fwd.qk_proj": r"(pp_row_gemm_kernel<false, 1, 0>|mfma_row_gemm_kernel<.*, 1, 0(, \w+)?>)",
    "fwd.v_experts": r"mfma_row_gemm_kernel<.*, 2, 0(, \w+)?>",
    "fwd.o_experts": r"(pp_row_gemm_kernel<false, 3, [13]>|mfma_row_gemm_kernel<.*, 3, 1(, \w+)?>)",
    "bwd.o_dgrad": r"mfma_row_gemm_kernel<.*, 4, 0(, \w+)?>",
    "bwd.v_dgrad": r"(pp_row_gemm_kernel<true, 5, 1>|mfma_row_gemm_kernel<.*, 5, 1(, \w+)?>)",
    "bwd.qk_dgrad": r"(pp_row_gemm_kernel<true, 6, 2>|mfma_row_gemm_kernel<.*, 6, 2(, \w+)?>)",
    "bwd.dx_gemm": r"pp_row_gemm_kernel<true, 6, 3>",
    "bwd.o_wgrad": r"mfma_wgrad_kernel<.*, 8, 7(, \w+)?>", "bwd.v_wgrad": r"mfma_wgrad_kernel<.*, 8, 8(, \w+)?>",
    "bwd.qk_wgrad": r"mfma_wgrad_kernel<.*, 8, 9(, \w+)?>", "bwd.wgrad_reduce": r"wgrad_reduce_kernel",
    "fwd.attention": r"mfma_attn_fwd_kernel", "bwd.attention_dkv": r"mfma_attn_dkv(_ws)?_kernel",
    "bwd.attention_dq": r"mfma_attn_dq(_ds)?_kernel", "fwd.y_sum": r"sum_heads_kernel", "bwd.dx_cast": r"sum_heads_kernel",
    "fwd.v_combine": r"slot_combine", "bwd.dctx_combine": r"slot_combine", "bwd.dgate_s": r"slot_combine",
}


def source_hash():
    """sha256 (first 16 hex digits) of the kernel sources: a counter summary under profiles/ names the hash it was
    taken with, and is only quoted while the sources are still those."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2312_07987_amd", "csrc")
    for n in sorted(os.listdir(d)):
        if n.endswith((".hip", ".h")):
            h.update(open(os.path.join(d, n), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(cfg_name, step):
    """(HBM bytes per launch of the step's kernel, note) from the committed rocprofv3 counter summary
    profiles/traffic_<cfg>.json; (None, why) if there is none for this kernel or it was taken from other sources."""
    import re
    path = os.path.join(ROOT, "profiles", "traffic_%s.json" % cfg_name)
    pat = STEP_KERNEL.get(step)
    if pat is None or not os.path.exists(path):
        return None, "no counter summary for this step"
    t = json.load(open(path))
    if t.get("source_sha16") != source_hash():
        return None, "profiles/traffic_%s.json was taken from other kernel sources (%s)" % (cfg_name, t.get("source_sha16"))
    for name, v in t["kernels"].items():
        if re.search(pat, name):
            return v["fetch_bytes"] + v["write_bytes"], "from the committed profiles/traffic_%s.json (same sources), not from this run" % cfg_name
    return None, "kernel not in profiles/traffic_%s.json" % cfg_name


def time_loop(fn, steps):
    """Wall-clock milliseconds per call over exactly `steps` calls, bracketed by device synchronisation."""
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def event_median(fn, steps):
    """Median over `steps` calls of the time between two HIP events recorded around each call on the launch
    stream (torch's current stream, the one the binding hands to the library)."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in ev)
    return ts[len(ts) // 2]


def profile_steps(layer, steps):
    """Per-step milliseconds from the HIP events the library records on the launch stream (separate pass, same work)."""
    import torch
    from paper_2312_07987_amd import binding
    binding.switchhead_profile_enable(True)
    for _ in range(steps):
        layer.forward()
        layer.backward()
    torch.cuda.synchronize()
    prof = binding.switchhead_profile_read()
    binding.switchhead_profile_enable(False)
    return {n: ms / c for n, (ms, c) in prof.items() if c}


def roofline_of(cfg, per_step):
    """The step with the largest time: its algorithmic work over its event-timed duration against the peak that bounds it."""
    flops, alu, nbytes = step_work(cfg)
    dom = max(per_step, key=per_step.get)
    if dom in flops:
        ach = flops[dom] / (per_step[dom] * 1e-3) / 1e12
        mfma = cfg["dtype"] == "bf16"   # fp32 storage runs the plain fp32 kernels: vector ALU, not MFMA
        peak = PEAK_BF16_TFLOPS if mfma else PEAK_FP32_VEC_TFLOPS
        roof = {"bound": "mfma" if mfma else "alu", "achieved": ach, "peak": peak, "unit": "TFLOP/s", "frac": ach / peak}
    elif dom in alu:
        ach = alu[dom] / (per_step[dom] * 1e-3) / 1e12
        roof = {"bound": "alu", "achieved": ach, "peak": PEAK_FP64_VEC_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_FP64_VEC_TFLOPS}
    else:
        ach = nbytes.get(dom, 0) / (per_step[dom] * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS}
    roof["traffic"], roof["traffic_note"] = measured_traffic(cfg["name"], dom)
    roof["step"] = dom
    roof["avg_ms"] = per_step[dom]
    return roof


def dense_baseline(cfg, steps, warmup, few_heads=False):
    """The same kernels in dense multi-head mode (no routers, E = 1), parameter-matched the way the
    paper matches its dense baselines (Sec. 3.1): H*E heads whose d_head gives the same number of
    parameters, rounded up to a multiple of 8.  few_heads: the paper's other dense baseline, which
    keeps SwitchHead's H heads and widens them instead (E times the matched width, capped at the
    256 the kernels take: 4 heads of 256 at c2, as in the paper's table of model sizes, App. A.5 "Hyperparameters")."""
    from paper_2312_07987_amd.inputs import make_inputs
    from paper_2312_07987_amd.runner import DeviceLayer
    H, E, dh = cfg["nheads"], cfg["E"], cfg["d_head"]
    heads = H * E
    qk_mats = 2 * H * E if cfg.get("qk_experts") else 2 * H   # query + key matrices of d_model x d_head
    dh_match = ((qk_mats + 2 * H * E) * dh + 2 * H * E) / (4.0 * H * E)
    dh2 = int(-(-dh_match // 8) * 8)
    if few_heads:
        heads, dh2 = H, min(256, int(-(-dh_match * E // 8) * 8))
    dc = dict(cfg, nheads=heads, d_head=dh2, E=1, k=1, bias0=0.0, name="dense", qk_experts=0)
    layer = DeviceLayer(dc, make_inputs(dc, seed=1), dense=True)

    def step():
        layer.forward()
        layer.backward()

    for _ in range(warmup):
        step()
    ms_step = time_loop(step, steps)
    ms_fwd = time_loop(layer.forward, steps)
    N = cfg["B"] * cfg["T"]
    return {"nheads": heads, "d_head": dh2, "d_head_param_matched": dh_match, "fwd_ms": ms_fwd, "fwd_bwd_ms": ms_step,
            "fwd_tokens_per_s": N / (ms_fwd * 1e-3), "fwd_bwd_tokens_per_s": N / (ms_step * 1e-3)}


def workload_string(cfg):
    return "%s: B=%d T=%d d_model=%d nheads=%d d_head=%d E=%d k=%d causal=%d bias0=%g%s" % (
        cfg["name"], cfg["B"], cfg["T"], cfg["d_model"], cfg["nheads"], cfg["d_head"], cfg["E"], cfg["k"],
        cfg["causal"], cfg["bias0"], (" qk_experts=1" if cfg.get("qk_experts") else "") + (" rope=1" if cfg.get("rope") else "") +
        (" T_q=%d" % cfg["T_q"] if cfg.get("T_q") else ""))


def other_workload(name, steps, warmup):
    """Forward+backward and forward time of another paper-shaped workload (same protocol), its per-step times and
    the roofline entry of its dominant step."""
    from paper_2312_07987_amd.flops import layer_flops
    from paper_2312_07987_amd.inputs import config, make_inputs
    from paper_2312_07987_amd.runner import DeviceLayer
    cfg = config(name)
    layer = DeviceLayer(cfg, make_inputs(cfg))

    def step():
        layer.forward()
        layer.backward()

    for _ in range(warmup):
        step()
    ms_step = time_loop(step, steps)
    ms_fwd = time_loop(layer.forward, steps)
    per_step = profile_steps(layer, steps)
    flops = step_work(cfg)[0]
    N = cfg["B"] * cfg["T"]
    lf = layer_flops(cfg["B"], cfg["T"], cfg["d_model"], cfg["nheads"], cfg["d_head"], cfg["E"], cfg["k"], bool(cfg["causal"]))
    out = {"workload": workload_string(cfg), "fwd_bwd_ms": ms_step, "fwd_ms": ms_fwd,
           "fwd_bwd_ms_median_events": event_median(step, steps),
           "fwd_bwd_tokens_per_s": N / (ms_step * 1e-3), "fwd_tokens_per_s": N / (ms_fwd * 1e-3),
           "fwd_bwd_tflops": lf["fwd_bwd"] / (ms_step * 1e-3) / 1e12,
           "fwd_bwd_frac_of_bf16_peak": lf["fwd_bwd"] / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
           "roofline": roofline_of(cfg, per_step),
           "step_ms": {n: round(v, 4) for n, v in sorted(per_step.items())},
           "step_tflops": {n: round(flops[n] / (per_step[n] * 1e-3) / 1e12, 1) for n in sorted(per_step) if n in flops}}
    if name == "c4":   # skewed routing: the per-expert token counts of every (side, head)
        counts = layer.routing()["offsets"]
        out["expert_counts_side_head_expert"] = (counts[..., 1:] - counts[..., :-1]).tolist()
    return out


def cpu_baseline(cfg, budget_tokens):
    """The float64 oracle, forward + backward, on the first sequences of the same workload."""
    import numpy as np
    from oracle import switchhead_oracle as orc
    from paper_2312_07987_amd.inputs import make_inputs
    sub = dict(cfg)
    sub["B"] = max(1, min(cfg["B"], budget_tokens // cfg["T"]))
    t = make_inputs(sub)
    t0 = time.perf_counter()
    f = orc.forward(t["x"], t["W_Q"], t["W_K"], t["W_V"], t["W_O"], t["W_S"], t["W_D"], t["b_S"], t["b_D"],
                    k=sub["k"], causal=bool(sub["causal"]), rope=bool(sub.get("rope")), T_q=sub.get("T_q"))
    t1 = time.perf_counter()
    orc.backward(t["x"], t["W_Q"], t["W_K"], t["W_V"], t["W_O"], t["W_S"], t["W_D"], f,
                 t["dy"][:, sub["T"] - (sub.get("T_q") or sub["T"]):])
    t2 = time.perf_counter()
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    ntok = sub["B"] * sub["T"]
    return {"value": ntok / (t2 - t0), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "float64 numpy oracle, forward+backward, first %d of %d sequences of %s (%d tokens, %.1f s; "
                      "forward alone %.0f tokens/s)" % (sub["B"], cfg["B"], cfg["name"], ntok, t2 - t0, ntok / (t1 - t0))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="c2", help="c1..c4 (c2 = the 262M-model-scale layer)")
    ap.add_argument("--qk-experts", action="store_true",
                    help="all four projections as expert mixtures (query and key banks like the value bank)")
    ap.add_argument("--rope", action="store_true", help="rotary position embedding of queries and keys")
    ap.add_argument("--context", type=int, default=1,
                    help="C >= 1: keys and values over C chunks of the config's T positions (C - 1 cached chunks in "
                         "front), queries for the last chunk only; tokens/s counts the current chunk's tokens")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-tokens", type=int, default=1 << 20, help="token budget of the oracle sample (whole sequences)")
    ap.add_argument("--no-dense", action="store_true",
                    help="skip the dense multi-head baselines and the short runs of the other workloads")
    ap.add_argument("--copy-only", action="store_true", help="run a plain 256 MiB device copy (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the layer would shard over the batch with one all-reduce of the "
              "weight gradients; that path is not built); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2312_07987_amd import binding
    from paper_2312_07987_amd.flops import layer_flops
    from paper_2312_07987_amd.inputs import config, make_inputs
    from paper_2312_07987_amd.runner import DeviceLayer

    if args.copy_only:
        # a plain copy of known size: 256 MiB read + 256 MiB written per launch, used to scale the
        # FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 256 << 20, "copy_bytes_written": 256 << 20, "launches": 5}))
        return

    cfg = config(args.config)
    if args.qk_experts:
        cfg["qk_experts"] = 1
    if args.rope:
        cfg["rope"] = 1
    if args.context > 1:
        cfg["T_q"] = cfg["T"]
        cfg["T"] = args.context * cfg["T"]
    host = make_inputs(cfg)
    layer = DeviceLayer(cfg, host)
    N = cfg["B"] * (cfg.get("T_q") or cfg["T"])   # tokens that get an output

    def step():
        layer.forward()
        layer.backward()

    for _ in range(args.warmup):
        step()
    ms_step = time_loop(step, args.steps)
    ms_fwd = time_loop(layer.forward, args.steps)

    ms_step_median = event_median(step, args.steps)
    ms_fwd_median = event_median(layer.forward, args.steps)
    per_step = profile_steps(layer, args.steps)
    flops = step_work(cfg)[0]
    roof = roofline_of(cfg, per_step)
    kept, scratch = binding.switchhead_workspace_parts(layer.shape)

    lf = layer_flops(cfg["B"], cfg["T"], cfg["d_model"], cfg["nheads"], cfg["d_head"], cfg["E"], cfg["k"],
                     bool(cfg["causal"]), qk_experts=bool(cfg.get("qk_experts")), T_q=cfg.get("T_q"))
    counts = layer.routing()["offsets"]
    out = {
        "metric": "switchhead_layer_fwd_bwd_tokens_per_s",
        "value": N / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": workload_string(cfg), "tokens_per_step": N},
        "roofline": roof,
        "extra": {
            "fwd_ms": ms_fwd, "fwd_tokens_per_s": N / (ms_fwd * 1e-3),
            # medians of per-call HIP-event times on the launch stream (ms_per_step and fwd_ms are wall-clock means
            # over exactly --steps calls between two device synchronisations)
            "fwd_bwd_ms_median_events": ms_step_median, "fwd_ms_median_events": ms_fwd_median,
            "workspace_bytes": {"kept_for_backward": kept, "scratch": scratch, "total": kept + scratch},
            "fwd_tflops": lf["fwd"] / (ms_fwd * 1e-3) / 1e12,
            "fwd_bwd_tflops": lf["fwd_bwd"] / (ms_step * 1e-3) / 1e12,
            "fwd_frac_of_bf16_peak": lf["fwd"] / (ms_fwd * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "fwd_bwd_frac_of_bf16_peak": lf["fwd_bwd"] / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "step_ms": {n: round(v, 4) for n, v in sorted(per_step.items())},
            # (the matrix-core family marks its two backward attention kernels, the fp32 family one
            # "bwd.attention" step; the routers' weight gradient, where it rides along the Q/K
            # weight-gradient launch, is not credited to that launch: "bwd.router_wsplit" only splits
            # its result)
            "step_tflops": {n: round(flops[n] / (per_step[n] * 1e-3) / 1e12, 1) for n in sorted(per_step) if n in flops},
            "expert_counts_side_head_expert": (counts[..., 1:] - counts[..., :-1]).tolist(),
        },
    }
    if not args.no_dense:
        out["extra"]["dense_mha"] = dense_baseline(cfg, args.steps, args.warmup)
        out["extra"]["dense_mha_few_heads"] = dense_baseline(cfg, args.steps, args.warmup, few_heads=True)
        if not (args.qk_experts or args.rope or args.context > 1):
            out["extra"]["other_workloads"] = {n: other_workload(n, args.steps, args.warmup)
                                               for n in ("c1", "c2", "c3", "c4") if n != cfg["name"]}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, args.cpu_tokens)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
