"""Register budgets of the hot kernels, read from the compiler's own summary (hipcc -S, no GPU needed).
The expert-gathered row GEMMs run three work-groups per CU (at most 168 registers), the dense-row and
weight-gradient tiles, the ping-pong GEMM's waves and the forward / dQ attention kernels two per SIMD (at most 256), and none of them may
spill to scratch memory: a few registers more in a shared template silently cost a work-group per CU."""
import os
import re
import shutil
import subprocess

import pytest

pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc (the compiler's register summary)")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2312_07987_amd", "csrc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-S", "--cuda-device-only"]


def kernel_table(source, tmp_path):
    out = os.path.join(str(tmp_path), source + ".s")
    subprocess.run(["hipcc", *FLAGS, "-o", out, os.path.join(CSRC, source)], check=True, capture_output=True)
    text = open(out).read()
    names = re.findall(r"\.amdhsa_kernel (\S+)", text)
    demangled = subprocess.run(["c++filt"], input="\n".join(names), capture_output=True, text=True).stdout.splitlines()
    table = {}
    for name, dn in zip(names, demangled):
        body = text[text.index(".amdhsa_kernel " + name):]
        body = body[:body.index(".end_amdhsa_kernel")]
        table[dn] = (int(re.search(r"next_free_vgpr (\d+)", body).group(1)),
                     int(re.search(r"private_segment_fixed_size (\d+)", body).group(1)))
    return table


def test_row_gemm_and_weight_gradient_budgets(tmp_path):
    t = kernel_table("mfma_gemm.hip", tmp_path)
    small = [k for k in t if "mfma_row_gemm_kernel<sh::TileCfg<2, 2, 2, 2, 64, 1, 1>, 8," in k]
    assert len(small) >= 10
    for k in small:
        assert t[k][0] <= 168 and t[k][1] == 0, (k, t[k])
    two = [k for k in t if ("TileCfg<2, 2, 4, 2, 64, 1, 2>, 8," in k and ", 0>(" in k) or
           ("TileCfg<2, 2, 2, 4, 64, 1, 2>, 8," in k and ", 2>(" in k) or "mfma_wgrad_kernel<sh::WgCfg<" in k]
    assert len(two) >= 10
    for k in two:
        wide_loads = ">, 8," in k   # 16-byte loads: the paths of c2 and c3; the 8-byte forms (c1) spill a few dwords
        assert t[k][0] <= 256 and t[k][1] <= (0 if wide_loads else 128), (k, t[k])


def test_attention_budgets(tmp_path):
    t = kernel_table("mfma_attn.hip", tmp_path)
    seen = 0
    for k, (vgpr, scratch) in t.items():
        if "mfma_attn_fwd_kernel<128, 8, " in k or "mfma_attn_fwd_kernel<64, 8, " in k:   # one or two wave groups
            assert vgpr <= 256 and scratch == 0, (k, vgpr, scratch)
            seen += 1
        if "mfma_attn_dq_kernel<128, 8>" in k:
            assert vgpr <= 256 and scratch <= 32, (k, vgpr, scratch)   # five spilled dwords, outside the products
            seen += 1
        if "mfma_attn_dq_ds_kernel<128, 8, 128>" in k or "mfma_attn_dq_ds_kernel<64, 8, 128>" in k:
            assert vgpr <= 256 and scratch == 0, (k, vgpr, scratch)    # two work-groups per CU (trips of 128 keys)
            seen += 1
        if "mfma_attn_dq_ds_kernel<" in k and ", 256>" in k:
            assert vgpr <= 256 and scratch == 0, (k, vgpr, scratch)
            seen += 1
        if "mfma_attn_dkv_ws_kernel<" in k:   # eight waves, two per SIMD
            assert vgpr <= 256 and scratch == 0, (k, vgpr, scratch)
            seen += 1
        if "mfma_attn_dkv_kernel<128, 8" in k or "mfma_attn_dkv_kernel<96," in k:
            assert scratch == 0, (k, vgpr, scratch)
            seen += 1
    assert seen >= 16, seen


def test_ping_pong_gemm_budgets(tmp_path):
    # eight waves, one work-group per CU: two waves per SIMD leave 256 registers each
    t = kernel_table("mfma_pp.hip", tmp_path)
    kernels = [k for k in t if "pp_row_gemm_kernel<" in k]
    assert len(kernels) >= 6
    for k in kernels:
        assert t[k][0] <= 256 and t[k][1] == 0, (k, t[k])
