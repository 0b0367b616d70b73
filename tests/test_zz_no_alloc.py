"""The allocation-free forward entry point (switchhead_forward_static: workspace in a device array built
into the library) against switchhead_forward on a caller's workspace, through the C ABI: several calls in
a row on the one shared array, each smaller than the one before, so that whatever an earlier call left in
the array would show."""
import numpy as np
import pytest

from paper_2312_07987_amd.inputs import config, make_inputs

pytestmark = pytest.mark.gpu


def test_static_workspace_forward_matches_the_caller_workspace_forward():
    from paper_2312_07987_amd import binding
    from paper_2312_07987_amd.runner import DeviceLayer
    cases = []
    c = config("c2"); c.update(B=1, T=128)                                  # matrix-core path, expert-set tables, ~15 MB
    cases.append((c, 7))
    c = config("c2"); c.update(B=2, T=96, d_model=256, nheads=2)            # smaller, same kernels
    cases.append((c, 8))
    cases.append((config("c0"), 9))                                         # fp32 storage, plain kernels
    for cfg, seed in cases:
        print("case", cfg, flush=True)
        t = make_inputs(cfg, seed=seed)
        layer = DeviceLayer(cfg, t)
        assert binding.switchhead_workspace_bytes(layer.shape) <= binding.STATIC_WORKSPACE_BYTES
        layer.forward()
        ref = layer.outputs().copy()
        layer.y.zero_()
        layer.forward_static()
        got = layer.outputs()
        if cfg["dtype"] == "bf16":
            assert np.array_equal(got, ref)      # this path adds its partial sums in a fixed order
        else:                                    # fp32 storage sums heads and slots with atomic adds
            assert np.max(np.abs(got - ref)) <= 1e-4 * np.max(np.abs(ref))
    # a shape that does not fit is refused, nothing is launched and y stays as it was
    big = config("c2")
    tb = make_inputs(dict(big, B=1, T=8), seed=1)
    small_layer = DeviceLayer(dict(big, B=1, T=8), tb)
    small_layer.shape = binding.make_shape(big["B"], big["T"], big["d_model"], big["nheads"], big["d_head"], big["E"], big["k"],
                                           1, "bf16")
    with pytest.raises(binding.SwitchHeadError) as e:
        small_layer.forward_static()
    assert e.value.code == binding.SH_ERR_WORKSPACE_TOO_SMALL
