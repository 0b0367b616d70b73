"""The FLOP/MAC model against the numbers the paper prints (Tables 1 and 2, App. A.2)."""
import os
import re

import pytest

from paper_2312_07987_amd import flops

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_resource_tables.txt")


def _rows():
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        yield line.split()


def _matches(printed, value):
    """True if `value` rounds to the printed figure at the printed number of digits."""
    m = re.fullmatch(r"([0-9.]+)([MG])", printed)
    num, unit = m.group(1), {"M": 1e6, "G": 1e9}[m.group(2)]
    digits = len(num.split(".")[1]) if "." in num else 0
    return round(value / unit, digits) == float(num)


@pytest.mark.parametrize("row", list(_rows()), ids=lambda r: "-".join(r[:5]))
def test_paper_table_row(row):
    kind, H, dh, dm, T, k, E, macs, mem = row
    H, dh, dm, T = int(H), int(dh), int(dm), int(T)
    if kind == "dense":
        assert _matches(macs, flops.macs_dense_xl(H, dh, dm, T)), flops.macs_dense_xl(H, dh, dm, T)
        assert _matches(mem, flops.mem_dense_xl(H, dh, T))
    else:
        got = flops.macs_switchhead_tables(H, dh, dm, T, int(k), int(E))
        assert _matches(macs, got), got
        assert _matches(mem, flops.mem_switchhead_tables(H, dh, T))


def test_printed_formula_differs_from_tables():
    # The SwitchHead formula as printed in App. A.2 gives 200.3M where Table 1 prints 170.4M.
    assert round(flops.macs_switchhead_printed(2, 76, 412, 256, 2) / 1e6, 1) == 200.3


def test_layer_flops_closed_form():
    f = flops.layer_flops(32, 512, 1024, 4, 128, 5, 3)
    N = 32 * 512
    assert f["qk"] == 4 * N * 1024 * 4 * 128
    assert f["v"] == f["o"] == 2 * N * 3 * 1024 * 4 * 128
    assert f["attn"] == 4 * 32 * 4 * 128 * (512 * 513 // 2)
    assert f["fwd"] == f["router"] + f["qk"] + f["v"] + f["o"] + f["attn"]
    assert abs(f["fwd"] / 1e9 - 147.39) < 0.01
    g = flops.layer_flops(4, 4096, 1024, 4, 128, 8, 2)
    assert abs(g["fwd"] / 1e9 - 173.96) < 0.01
