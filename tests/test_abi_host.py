"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and turns bad arguments into error codes before anything touches a GPU."""
import ctypes
import os
import re

import pytest

from paper_2312_07987_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2312_07987_amd.build import build
        build()
    return binding.lib()


def test_exports_match_header(lib):
    text = open(os.path.join(ROOT, "include", "switchhead.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(switchhead_\w+)\s*\(", text))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_workspace_bytes_and_shape_errors(lib):
    ok = binding.make_shape(2, 64, 64, 2, 32, 4, 2, 1, "f32")
    n = binding.switchhead_workspace_bytes(ok)
    assert n > 0 and n % 256 == 0
    big = binding.make_shape(32, 512, 1024, 4, 128, 5, 3, 1, "bf16")
    assert binding.switchhead_workspace_bytes(big) > n
    for bad, word in ((binding.make_shape(2, 64, 64, 2, 32, 4, 5, 1, "f32"), "exceeds E"),
                      (binding.make_shape(0, 64, 64, 2, 32, 4, 2, 1, "f32"), "dimension"),
                      (binding.make_shape(2, 64, 64, 2, 32, 65, 2, 1, "f32"), "limit of 64"),
                      (binding.make_shape(2, 64, 64, 2, 32, 16, 9, 1, "f32"), "limit of 8"),
                      (binding.make_shape(2, 64, 64, 2, 512, 4, 2, 1, "f32"), "d_head"),
                      (binding.make_shape(2, 64, 64, 2, 32, 4, 2, 2, "f32"), "causal"),
                      (binding.make_shape(2, 64, 64, 2, 32, 4, 2, 1, "f32", qk_experts=2), "qk_experts"),
                      (binding.make_shape(2, 64, 64, 2, 32, 4, 2, 1, "f32", rope=3), "rope"),
                      (binding.make_shape(2, 64, 64, 2, 32, 4, 2, 1, "f32", T_q=65), "T_q"),
                      (binding.make_shape(2, 64, 64, 2, 32, 4, 2, 1, 7), "dtype")):
        assert binding.switchhead_workspace_bytes(bad) == 0
        assert word in binding.switchhead_last_error()


def test_workspace_split_and_score_gradient_scratch(lib):
    """The two parts add up; the kept part does not depend on what backward needs; the attention backward's score-gradient
    scratch (quadratic in T, head widths 64..128, bf16 only) hides in dead buffers at c2, is packed to the causal half at
    c3 and is dropped beyond 1 GiB."""
    c2 = binding.make_shape(32, 512, 1024, 4, 128, 5, 3, 1, "bf16")
    kept, scratch = binding.switchhead_workspace_parts(c2)
    assert kept + scratch == binding.switchhead_workspace_bytes(c2)
    assert kept < 130e6 and kept + scratch < 500e6
    c3 = binding.make_shape(4, 4096, 1024, 4, 128, 8, 2, 1, "bf16")
    c3_nomask = binding.make_shape(4, 4096, 1024, 4, 128, 8, 2, 0, "bf16")
    k3, s3 = binding.switchhead_workspace_parts(c3)
    k3n, s3n = binding.switchhead_workspace_parts(c3_nomask)
    assert k3 == k3n
    full = 4 * 4 * 4096 * 4096 * 2                      # the unpacked [B, H, T, T] bf16
    assert 0.45 * full < s3n - s3 < 0.5 * full          # the mask saves almost half of it
    # a head width outside 64..128 keeps no score gradient, so the mask changes nothing there
    narrow = [binding.switchhead_workspace_parts(binding.make_shape(4, 4096, 1024, 16, 32, 8, 2, c, "bf16")) for c in (0, 1)]
    assert narrow[0] == narrow[1]
    # beyond 1 GiB (here 2 GiB unpacked, a little over 1 GiB packed) it is recomputed instead: again no difference
    long_ = [binding.switchhead_workspace_parts(binding.make_shape(4, 8192, 1024, 4, 128, 8, 2, c, "bf16")) for c in (0, 1)]
    assert long_[0] == long_[1] and long_[0][1] < s3n
    # fp32 storage never keeps it
    f32 = [binding.switchhead_workspace_parts(binding.make_shape(4, 4096, 1024, 4, 128, 8, 2, c, "f32")) for c in (0, 1)]
    assert f32[0] == f32[1]


def test_forward_rejects_bad_arguments_without_launching(lib):
    s = binding.make_shape(2, 64, 64, 2, 32, 4, 2, 1, "f32")
    fake = ctypes.c_void_p(256)          # never dereferenced: every check below fails first
    sz = ctypes.c_size_t
    # NULL workspace
    rc = lib.switchhead_forward(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, None, None, fake,
                                None, sz(1 << 40), None)
    assert rc == binding.SH_ERR_INVALID_ARG and "workspace" in binding.switchhead_last_error()
    # workspace too small
    rc = lib.switchhead_forward(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, None, None, fake,
                                fake, sz(16), None)
    assert rc == binding.SH_ERR_WORKSPACE_TOO_SMALL
    # misaligned workspace
    rc = lib.switchhead_forward(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, None, None, fake,
                                ctypes.c_void_p(264), sz(1 << 40), None)
    assert rc == binding.SH_ERR_INVALID_ARG
    # NULL x
    rc = lib.switchhead_forward(ctypes.byref(s), None, fake, fake, fake, fake, fake, fake, None, None, fake,
                                fake, sz(1 << 40), None)
    assert rc == binding.SH_ERR_INVALID_ARG
    # dense mode needs E == 1
    rc = lib.switchhead_forward(ctypes.byref(s), fake, fake, fake, fake, fake, None, None, None, None, fake,
                                fake, sz(1 << 40), None)
    assert rc == binding.SH_ERR_INVALID_ARG and "dense" in binding.switchhead_last_error()
    # the allocation-free forward: a shape whose workspace exceeds the built-in one is refused before any GPU call
    big = binding.make_shape(32, 512, 1024, 4, 128, 5, 3, 1, "bf16")
    assert binding.switchhead_workspace_bytes(big) > binding.STATIC_WORKSPACE_BYTES
    rc = lib.switchhead_forward_static(ctypes.byref(big), fake, fake, fake, fake, fake, fake, fake, None, None, fake, None)
    assert rc == binding.SH_ERR_WORKSPACE_TOO_SMALL and "built-in" in binding.switchhead_last_error()
    bad = binding.make_shape(2, 64, 64, 2, 32, 4, 5, 1, "f32")
    rc = lib.switchhead_forward_static(ctypes.byref(bad), fake, fake, fake, fake, fake, fake, fake, None, None, fake, None)
    assert rc == binding.SH_ERR_INVALID_ARG
    # backward: NULL dy
    rc = lib.switchhead_backward(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, None,
                                 fake, sz(1 << 40), fake, fake, fake, fake, fake, None, None, None, None, None)
    assert rc == binding.SH_ERR_INVALID_ARG
    assert lib.switchhead_version().decode().count(".") == 1
    assert binding.switchhead_set_kernel_family(0) in (0, 1)
