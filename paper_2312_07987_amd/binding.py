"""ctypes binding of libswitchhead.so: the same entry points as include/switchhead.h, with
argument marshalling only.  Tensors are torch tensors on the GPU (device memory and streams
are all torch is used for); every step of the layer runs inside the library's kernels.

There is no fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libswitchhead.so")

SH_OK, SH_ERR_INVALID_ARG, SH_ERR_UNSUPPORTED, SH_ERR_WORKSPACE_TOO_SMALL, SH_ERR_HIP = range(5)
SH_F32, SH_BF16 = 0, 1

STATIC_WORKSPACE_BYTES = 16 << 20

EXPORTS = ("switchhead_workspace_bytes", "switchhead_workspace_parts", "switchhead_forward", "switchhead_forward_static", "switchhead_backward",
           "switchhead_get_routing", "switchhead_get_intermediates", "switchhead_last_error",
           "switchhead_set_kernel_family", "switchhead_version",
           "switchhead_profile_enable", "switchhead_profile_read")


class sh_shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("B", "T", "d_model", "nheads", "d_head", "E", "k", "causal", "dtype", "qk_experts", "rope", "T_q")]


class SwitchHeadError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("switchhead error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib():
    """Loads libswitchhead.so (once).  Raises if it is missing: build it first with
    `python -m paper_2312_07987_amd.build`."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            LIB_PATH + " is missing: build it with `python -m paper_2312_07987_amd.build` "
            "(there is no fallback implementation)")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    shp = ctypes.POINTER(sh_shape)
    L.switchhead_workspace_bytes.restype = sz
    L.switchhead_workspace_bytes.argtypes = [shp]
    L.switchhead_workspace_parts.restype = i32
    L.switchhead_workspace_parts.argtypes = [shp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.switchhead_forward.restype = i32
    L.switchhead_forward.argtypes = [shp] + [vp] * 10 + [vp, sz, vp]
    L.switchhead_forward_static.restype = i32
    L.switchhead_forward_static.argtypes = [shp] + [vp] * 10 + [vp]
    L.switchhead_backward.restype = i32
    L.switchhead_backward.argtypes = [shp] + [vp] * 8 + [vp, sz] + [vp] * 9 + [vp]
    L.switchhead_get_routing.restype = i32
    L.switchhead_get_routing.argtypes = [shp, vp, sz, vp, vp, vp, vp, vp]
    L.switchhead_get_intermediates.restype = i32
    L.switchhead_get_intermediates.argtypes = [shp, vp, sz, vp, vp, vp, vp, vp, vp]
    L.switchhead_last_error.restype = ctypes.c_char_p
    L.switchhead_last_error.argtypes = []
    L.switchhead_set_kernel_family.restype = i32
    L.switchhead_set_kernel_family.argtypes = [i32]
    L.switchhead_version.restype = ctypes.c_char_p
    L.switchhead_version.argtypes = []
    L.switchhead_profile_enable.restype = i32
    L.switchhead_profile_enable.argtypes = [i32]
    L.switchhead_profile_read.restype = i32
    L.switchhead_profile_read.argtypes = [ctypes.c_char_p, sz, ctypes.POINTER(ctypes.c_float),
                                          ctypes.POINTER(i32), i32]
    _lib = L
    return L


def make_shape(B, T, d_model, nheads, d_head, E, k, causal=1, dtype="bf16", qk_experts=0, rope=0, T_q=0):
    code = {"f32": SH_F32, "fp32": SH_F32, "bf16": SH_BF16}[dtype] if isinstance(dtype, str) else int(dtype)
    return sh_shape(B, T, d_model, nheads, d_head, E, k, int(causal), code, int(qk_experts), int(rope), int(T_q))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    return ctypes.c_void_p(int(stream))


def _check(code):
    if code != SH_OK:
        raise SwitchHeadError(code, lib().switchhead_last_error().decode())


def switchhead_workspace_bytes(shape):
    return int(lib().switchhead_workspace_bytes(ctypes.byref(shape)))


def switchhead_workspace_parts(shape):
    """(kept bytes, scratch bytes) of the workspace of this shape."""
    kept, scratch = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().switchhead_workspace_parts(ctypes.byref(shape), ctypes.byref(kept), ctypes.byref(scratch)))
    return int(kept.value), int(scratch.value)


def switchhead_last_error():
    return lib().switchhead_last_error().decode()


def switchhead_set_kernel_family(family):
    return int(lib().switchhead_set_kernel_family(int(family)))


def switchhead_version():
    return lib().switchhead_version().decode()


def switchhead_forward(shape, x, W_Q, W_K, W_V, W_O, W_S, W_D, b_S, b_D, y, workspace, stream=None):
    _check(lib().switchhead_forward(ctypes.byref(shape), _ptr(x), _ptr(W_Q), _ptr(W_K), _ptr(W_V), _ptr(W_O),
                                    _ptr(W_S), _ptr(W_D), _ptr(b_S), _ptr(b_D), _ptr(y),
                                    _ptr(workspace), workspace.numel() * workspace.element_size(),
                                    _stream(stream)))


def switchhead_forward_static(shape, x, W_Q, W_K, W_V, W_O, W_S, W_D, b_S, b_D, y, stream=None):
    _check(lib().switchhead_forward_static(ctypes.byref(shape), _ptr(x), _ptr(W_Q), _ptr(W_K), _ptr(W_V), _ptr(W_O),
                                           _ptr(W_S), _ptr(W_D), _ptr(b_S), _ptr(b_D), _ptr(y), _stream(stream)))


def switchhead_backward(shape, x, W_Q, W_K, W_V, W_O, W_S, W_D, dy, workspace,
                        dx, dW_Q, dW_K, dW_V, dW_O, dW_S, dW_D, db_S, db_D, stream=None):
    _check(lib().switchhead_backward(ctypes.byref(shape), _ptr(x), _ptr(W_Q), _ptr(W_K), _ptr(W_V), _ptr(W_O),
                                     _ptr(W_S), _ptr(W_D), _ptr(dy),
                                     _ptr(workspace), workspace.numel() * workspace.element_size(),
                                     _ptr(dx), _ptr(dW_Q), _ptr(dW_K), _ptr(dW_V), _ptr(dW_O),
                                     _ptr(dW_S), _ptr(dW_D), _ptr(db_S), _ptr(db_D), _stream(stream)))


def switchhead_get_routing(shape, workspace, topk_idx, gate, perm, expert_offsets, stream=None):
    _check(lib().switchhead_get_routing(ctypes.byref(shape), _ptr(workspace),
                                        workspace.numel() * workspace.element_size(),
                                        _ptr(topk_idx), _ptr(gate), _ptr(perm), _ptr(expert_offsets),
                                        _stream(stream)))


def switchhead_get_intermediates(shape, workspace, Q, K, V, ctx, lse, stream=None):
    _check(lib().switchhead_get_intermediates(ctypes.byref(shape), _ptr(workspace),
                                              workspace.numel() * workspace.element_size(),
                                              _ptr(Q), _ptr(K), _ptr(V), _ptr(ctx), _ptr(lse), _stream(stream)))


def switchhead_profile_enable(on):
    _check(lib().switchhead_profile_enable(int(bool(on))))


def switchhead_profile_read(max_entries=64):
    """Returns {step label: (total milliseconds, occurrences)} since the last read."""
    buf = ctypes.create_string_buffer(64 * max_entries)
    ms = (ctypes.c_float * max_entries)()
    cnt = (ctypes.c_int32 * max_entries)()
    n = lib().switchhead_profile_read(buf, len(buf), ms, cnt, max_entries)
    names = buf.value.decode().split("\n")[:n]
    return {names[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}
