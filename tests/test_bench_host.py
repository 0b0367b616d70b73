"""Host logic of bench.py that needs no GPU: the refusal of more than one GPU and the
agreement of the per-step work table with the layer totals."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2312_07987_amd.flops import layer_flops  # noqa: E402
from paper_2312_07987_amd.inputs import config  # noqa: E402


def test_more_than_one_gpu_is_refused():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)


@pytest.mark.parametrize("name", ["c1", "c2", "c3"])
@pytest.mark.parametrize("variant", [{}, {"qk_experts": 1}, {"T_q": 0.5}])
def test_step_table_adds_up_to_the_layer_totals(name, variant):
    """The steps a forward + backward call launches, priced by bench.step_work, add up to
    flops.layer_flops (router logits are priced as ALU work, the routers' small backward GEMMs and the
    recomputation inside the dQ kernel are not algorithmic work of a step of their own)."""
    cfg = config(name)
    for key, v in variant.items():
        cfg[key] = int(cfg["T"] * v) if key == "T_q" else v
    flops, alu, _ = bench.step_work(cfg)
    lf = layer_flops(cfg["B"], cfg["T"], cfg["d_model"], cfg["nheads"], cfg["d_head"], cfg["E"], cfg["k"],
                     bool(cfg["causal"]), qk_experts=bool(cfg.get("qk_experts")), T_q=cfg.get("T_q"))
    if cfg.get("qk_experts"):
        qk_fwd = flops["fwd.q_experts"] + flops["fwd.k_experts"]
        qk_bwd = sum(flops[n] for n in ("bwd.q_wgrad_e", "bwd.k_wgrad_e", "bwd.q_dgrad_e", "bwd.k_dgrad_e"))
    else:
        qk_fwd = flops["fwd.q_proj"] + flops["fwd.k_proj"]
        qk_bwd = sum(flops[n] for n in ("bwd.q_wgrad", "bwd.k_wgrad", "bwd.q_dgrad", "bwd.k_dgrad"))
    fwd = alu["fwd.router"] + qk_fwd + flops["fwd.v_experts"] + flops["fwd.o_experts"] + flops["fwd.attention"]
    assert fwd == lf["fwd"]
    bwd = (flops["bwd.router_wgrad"] + flops["bwd.router_dgrad"] + qk_bwd + flops["bwd.v_wgrad"] + flops["bwd.v_dgrad"]
           + flops["bwd.o_wgrad"] + flops["bwd.o_dgrad"] + flops["bwd.attention"])
    assert abs(bwd - lf["bwd"]) <= 2   # integer halves of the attention count
    if not cfg.get("T_q"):
        assert flops["fwd.qk_proj"] == qk_fwd or cfg.get("qk_experts")
    if not cfg.get("qk_experts"):
        # the one GEMM that writes all of dx is priced as the three input gradients it replaces
        assert flops["bwd.dx_gemm"] == flops["bwd.v_dgrad"] + flops["bwd.q_dgrad"] + flops["bwd.k_dgrad"] + flops["bwd.router_dgrad"]


def test_counter_summaries_name_the_sources_they_were_taken_from():
    """bench.py quotes roofline.traffic from profiles/traffic_<cfg>.json only while the kernel sources hash to the value
    the summary names; both sides compute the hash the same way."""
    from paper_2312_07987_amd import prof_summary
    assert bench.source_hash() == prof_summary._source_hash()
    value, note = bench.measured_traffic("c2", "no.such.step")
    assert value is None and note
