"""Thin Python binding of the C ABI in include/lawcat.h (ctypes; argument marshalling only).

Function names match the C entry points.  Tensors are torch CUDA tensors used purely as
device buffers; every step of the path runs inside liblawcat.so.  There is no fallback:
if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblawcat.so")

DTYPE_F32, DTYPE_BF16 = 0, 1
PHI_IDENTITY, PHI_ELU1 = 0, 1
CARRY_AUTO, CARRY_SEQUENTIAL, CARRY_TWO_LEVEL = 0, 1, 2
CALL_CONV1D, CALL_GLA_PREFILL, CALL_GLA_STEP, CALL_LAYER_PREFILL, CALL_LAYER_PREFILL_FM, CALL_GLA_BACKWARD = 0, 1, 2, 3, 4, 5
CALL_CONV1D_BACKWARD = 6

EXPORTS = (
    "lawcat_workspace_bytes", "lawcat_conv1d_backward", "lawcat_conv1d_causal", "lawcat_gate_project", "lawcat_gla_backward", "lawcat_gla_prefill", "lawcat_gla_step", "lawcat_gla_steps",
    "lawcat_conv1d_feature", "lawcat_layer_prefill", "lawcat_layer_prefill_varlen", "lawcat_varlen_workspace_bytes", "lawcat_layer_prefill_fm", "lawcat_layer_prefill_static",
    "lawcat_layer_prefill_timed", "lawcat_status_string", "lawcat_version",
)


class Desc(ctypes.Structure):
    """Mirror of `lawcat_desc`."""

    _fields_ = [
        ("struct_size", ctypes.c_uint32),
        ("B", ctypes.c_int32), ("T", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("dk", ctypes.c_int32), ("dv", ctypes.c_int32),
        ("conv_width", ctypes.c_int32), ("dtype", ctypes.c_int32), ("feature_map", ctypes.c_int32),
        ("chunk", ctypes.c_int32), ("carry_mode", ctypes.c_int32), ("segment", ctypes.c_int32),
        ("gate_scale", ctypes.c_float), ("eps", ctypes.c_float),
    ]


class LawcatError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"lawcat status {status}: {status_string(status)}")


_lib = None


def lib() -> ctypes.CDLL:
    """Load liblawcat.so (built by paper_2509_18467_amd.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not built: run `python -m paper_2509_18467_amd.build` (or __graft_entry__.build())")
        L = ctypes.CDLL(LIB_PATH)
        vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
        dp = ctypes.POINTER(Desc)
        L.lawcat_workspace_bytes.argtypes = [dp, ci]
        L.lawcat_workspace_bytes.restype = sz
        L.lawcat_conv1d_causal.argtypes = [dp, ci] + [vp] * 6
        L.lawcat_conv1d_causal.restype = ci
        L.lawcat_gla_prefill.argtypes = [dp] + [vp] * 11 + [sz, vp]
        L.lawcat_gla_prefill.restype = ci
        L.lawcat_gla_step.argtypes = [dp] + [vp] * 8
        L.lawcat_gla_step.restype = ci
        L.lawcat_gla_steps.argtypes = [dp] + [vp] * 8
        L.lawcat_gla_steps.restype = ci
        L.lawcat_layer_prefill.argtypes = [dp] + [vp] * 17 + [sz, vp]
        L.lawcat_layer_prefill.restype = ci
        L.lawcat_status_string.argtypes = [ci]
        L.lawcat_status_string.restype = ctypes.c_char_p
        L.lawcat_version.restype = ci
        L.lawcat_gla_backward.argtypes = [dp] + [vp] * 15 + [sz, vp]
        L.lawcat_gla_backward.restype = ci
        L.lawcat_conv1d_backward.argtypes = [dp, ci] + [vp] * 8 + [sz, vp]
        L.lawcat_conv1d_backward.restype = ci
        L.lawcat_gate_project.argtypes = [dp, ci, ci] + [vp] * 6
        L.lawcat_gate_project.restype = ci
        L.lawcat_varlen_workspace_bytes.argtypes = [dp, ctypes.POINTER(ctypes.c_int32), ci]
        L.lawcat_varlen_workspace_bytes.restype = sz
        L.lawcat_layer_prefill_varlen.argtypes = [dp, ctypes.POINTER(ctypes.c_int32)] + [vp] * 18 + [sz, vp]
        L.lawcat_layer_prefill_varlen.restype = ci
        L.lawcat_conv1d_feature.argtypes = [dp, ci] + [vp] * 7
        L.lawcat_conv1d_feature.restype = ci
        L.lawcat_layer_prefill_fm.argtypes = [dp] + [vp] * 18 + [sz, vp]
        L.lawcat_layer_prefill_fm.restype = ci
        L.lawcat_layer_prefill_static.argtypes = [dp] + [vp] * 16 + [vp]
        L.lawcat_layer_prefill_static.restype = ci
        L.lawcat_layer_prefill_timed.argtypes = [dp] + [vp] * 17 + [sz, vp, vp, vp]
        L.lawcat_layer_prefill_timed.restype = ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().lawcat_status_string(int(status)).decode()


def version() -> int:
    return int(lib().lawcat_version())


def make_desc(B, T, Hq, Hkv, d, *, conv_width=4, dtype=DTYPE_BF16, feature_map=PHI_ELU1, chunk=0,
              carry_mode=CARRY_AUTO, segment=0, gate_scale=1.0, eps=0.0) -> Desc:
    return Desc(ctypes.sizeof(Desc), B, T, Hq, Hkv, d, d, conv_width, dtype, feature_map, chunk, carry_mode,
                segment, gate_scale, eps)


def workspace_bytes(desc: Desc, which_call: int) -> int:
    return int(lib().lawcat_workspace_bytes(ctypes.byref(desc), which_call))


def _p(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(st):
    if st != 0:
        raise LawcatError(st)


def conv1d_causal(desc, n_heads, x, w, halo, y, tail_out, stream=None):
    _check(lib().lawcat_conv1d_causal(ctypes.byref(desc), n_heads, _p(x), _p(w), _p(halo), _p(y), _p(tail_out),
                                      _stream(stream)))


def gla_prefill(desc, q, k, v, gate_logits, S0, z0, o, den_out, S_out, z_out, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lawcat_gla_prefill(ctypes.byref(desc), _p(q), _p(k), _p(v), _p(gate_logits), _p(S0), _p(z0),
                                    _p(o), _p(den_out), _p(S_out), _p(z_out), _p(workspace), nbytes,
                                    _stream(stream)))


def gla_step(desc, q, k, v, gate_logits, S, z, o, stream=None):
    _check(lib().lawcat_gla_step(ctypes.byref(desc), _p(q), _p(k), _p(v), _p(gate_logits), _p(S), _p(z), _p(o),
                                 _stream(stream)))


def gla_steps(desc, q, k, v, gate_logits, S, z, o, stream=None):
    _check(lib().lawcat_gla_steps(ctypes.byref(desc), _p(q), _p(k), _p(v), _p(gate_logits), _p(S), _p(z), _p(o),
                                  _stream(stream)))


def layer_prefill(desc, Q, K, V, gate_logits, wq, wk, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                  q_tail_out, k_tail_out, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lawcat_layer_prefill(ctypes.byref(desc), _p(Q), _p(K), _p(V), _p(gate_logits), _p(wq), _p(wk),
                                      _p(S0), _p(z0), _p(q_halo), _p(k_halo), _p(O), _p(den_out), _p(S_out),
                                      _p(z_out), _p(q_tail_out), _p(k_tail_out), _p(workspace), nbytes,
                                      _stream(stream)))


def gla_backward(desc, q, k, v, gate_logits, den, dO, S0, z0, dq, dk, dv, dg, dS0, dz0, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lawcat_gla_backward(ctypes.byref(desc), _p(q), _p(k), _p(v), _p(gate_logits), _p(den), _p(dO),
                                     _p(S0), _p(z0), _p(dq), _p(dk), _p(dv), _p(dg), _p(dS0), _p(dz0), _p(workspace),
                                     nbytes, _stream(stream)))


def conv1d_backward(desc, n_heads, x, w, halo, dy, dx, dw, dhalo, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lawcat_conv1d_backward(ctypes.byref(desc), n_heads, _p(x), _p(w), _p(halo), _p(dy), _p(dx), _p(dw),
                                        _p(dhalo), _p(workspace), nbytes, _stream(stream)))


def gate_project(desc, d_model, rank, x, w1, w2, bias, gate_logits, stream=None):
    _check(lib().lawcat_gate_project(ctypes.byref(desc), d_model, rank, _p(x), _p(w1), _p(w2), _p(bias), _p(gate_logits),
                                     _stream(stream)))


def varlen_workspace_bytes(desc, seq_start, one_launch=False):
    """Workspace bytes of a lawcat_layer_prefill_varlen call (one_launch: a device copy of the offsets is passed)."""
    starts = (ctypes.c_int32 * len(seq_start))(*[int(v) for v in seq_start])
    return int(lib().lawcat_varlen_workspace_bytes(ctypes.byref(desc), starts, 1 if one_launch else 0))


def layer_prefill_varlen(desc, seq_start, Q, K, V, gate_logits, wq, wk, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                         q_tail_out, k_tail_out, workspace, stream=None, seq_start_dev=None):
    """seq_start: host offsets (any int sequence); seq_start_dev: optional int32 device tensor holding the same."""
    starts = (ctypes.c_int32 * len(seq_start))(*[int(v) for v in seq_start])
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lawcat_layer_prefill_varlen(ctypes.byref(desc), starts, _p(seq_start_dev), _p(Q), _p(K), _p(V), _p(gate_logits), _p(wq),
                                             _p(wk), _p(S0), _p(z0), _p(q_halo), _p(k_halo), _p(O), _p(den_out), _p(S_out),
                                             _p(z_out), _p(q_tail_out), _p(k_tail_out), _p(workspace), nbytes,
                                             _stream(stream)))


def conv1d_feature(desc, n_heads, x, w, wf, halo, y, tail_out, stream=None):
    _check(lib().lawcat_conv1d_feature(ctypes.byref(desc), n_heads, _p(x), _p(w), _p(wf), _p(halo), _p(y),
                                       _p(tail_out), _stream(stream)))


def layer_prefill_fm(desc, Q, K, V, gate_logits, wq, wk, wf, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                     q_tail_out, k_tail_out, workspace, stream=None):
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lawcat_layer_prefill_fm(ctypes.byref(desc), _p(Q), _p(K), _p(V), _p(gate_logits), _p(wq), _p(wk),
                                         _p(wf), _p(S0), _p(z0), _p(q_halo), _p(k_halo), _p(O), _p(den_out),
                                         _p(S_out), _p(z_out), _p(q_tail_out), _p(k_tail_out), _p(workspace), nbytes,
                                         _stream(stream)))


STATIC_WORKSPACE_BYTES = 24 << 20


def layer_prefill_static(desc, Q, K, V, gate_logits, wq, wk, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                         q_tail_out, k_tail_out, stream=None):
    _check(lib().lawcat_layer_prefill_static(ctypes.byref(desc), _p(Q), _p(K), _p(V), _p(gate_logits), _p(wq),
                                             _p(wk), _p(S0), _p(z0), _p(q_halo), _p(k_halo), _p(O), _p(den_out),
                                             _p(S_out), _p(z_out), _p(q_tail_out), _p(k_tail_out),
                                             _stream(stream)))


def layer_prefill_timed(desc, Q, K, V, gate_logits, wq, wk, S0, z0, q_halo, k_halo, O, den_out, S_out, z_out,
                        q_tail_out, k_tail_out, workspace, ev_start, ev_stop, stream=None):
    """ev_start/ev_stop: raw hipEvent_t handles (ints)."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().lawcat_layer_prefill_timed(ctypes.byref(desc), _p(Q), _p(K), _p(V), _p(gate_logits), _p(wq),
                                            _p(wk), _p(S0), _p(z0), _p(q_halo), _p(k_halo), _p(O), _p(den_out),
                                            _p(S_out), _p(z_out), _p(q_tail_out), _p(k_tail_out), _p(workspace),
                                            nbytes, _stream(stream), ctypes.c_void_p(ev_start),
                                            ctypes.c_void_p(ev_stop)))


def alloc_workspace(desc, which_call, device="cuda"):
    n = workspace_bytes(desc, which_call)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)
