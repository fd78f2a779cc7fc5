"""ctypes front end of the fp64 C oracle (oracle/lawcat_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg.  It never imports the HIP package and the HIP package never imports it.

All functions take numpy arrays (any float dtype; converted to float64) laid out as in
the paper's layer: q [B,T,Hq,dk], k/g [B,T,Hkv,dk], v [B,T,Hkv,dv], conv weights [H,d,W].
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lawcat_oracle.c")
_LIB = os.path.join(_HERE, "liblawcat_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP over the independent recurrences)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O3", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        dp = ctypes.POINTER(ctypes.c_double)
        _lib.lawcat_oracle_conv1d_causal.argtypes = [ctypes.c_int] * 5 + [dp, dp, dp, ctypes.c_int, dp]
        _lib.lawcat_oracle_conv1d_causal.restype = None
        _lib.lawcat_oracle_gla_prefill.argtypes = (
            [ctypes.c_int] * 6 + [dp] * 4 + [ctypes.c_double] * 2 + [dp] * 7
        )
        _lib.lawcat_oracle_gla_prefill.restype = None
        _lib.lawcat_oracle_feature_linear.argtypes = [ctypes.c_int] * 5 + [dp, dp, ctypes.c_int, dp]
        _lib.lawcat_oracle_feature_linear.restype = None
        _lib.lawcat_oracle_gate_project.argtypes = [ctypes.c_int] * 5 + [dp, dp, dp, dp, dp]
        _lib.lawcat_oracle_gate_project.restype = None
        _lib.lawcat_oracle_gla_backward.argtypes = ([ctypes.c_int] * 6 + [dp] * 4 + [ctypes.c_double] * 2 + [dp] * 9)
        _lib.lawcat_oracle_gla_backward.restype = None
        _lib.lawcat_oracle_conv1d_backward.argtypes = [ctypes.c_int] * 5 + [dp, dp, dp, ctypes.c_int, dp, dp, dp, dp]
        _lib.lawcat_oracle_conv1d_backward.restype = None
        _lib.lawcat_oracle_max_threads.restype = ctypes.c_int
    return _lib


def _f64(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _ptr(a):
    dp = ctypes.POINTER(ctypes.c_double)
    return ctypes.cast(None, dp) if a is None else a.ctypes.data_as(dp)


def max_threads() -> int:
    return int(_load().lawcat_oracle_max_threads())


def conv1d_causal(x, w, halo=None, feature_map: int = 0):
    """Section 4.1: y[t] = phi(sum_delta w[..,delta] * x[t-delta]); x [B,T,H,d], w [H,d,W]."""
    lib = _load()
    x = _f64(x)
    w = _f64(w)
    halo = _f64(halo)
    B, T, H, d = x.shape
    W = w.shape[-1]
    assert w.shape == (H, d, W)
    if halo is not None:
        assert halo.shape == (B, W - 1, H, d)
    y = np.empty_like(x)
    lib.lawcat_oracle_conv1d_causal(B, T, H, d, W, _ptr(x), _ptr(w), _ptr(halo), int(feature_map), _ptr(y))
    return y


def feature_linear(x, wf, feature_map: int = 0):
    """Section 4.1: y = phi(x Wf) per head; x [B,T,H,d], wf [Hw,d,d] with H % Hw == 0: head h uses matrix
    h // (H // Hw), so a key head and the query heads of its group share one matrix."""
    lib = _load()
    x = _f64(x)
    wf = _f64(wf)
    B, T, H, d = x.shape
    Hw = wf.shape[0]
    assert wf.shape == (Hw, d, d) and H % Hw == 0
    y = np.empty_like(x)
    lib.lawcat_oracle_feature_linear(B, T, H, d, H // Hw, _ptr(x), _ptr(wf), int(feature_map), _ptr(y))
    return y


def gate_project(x, w1, w2, bias=None, Hkv: int = 1):
    """Section 4.2 / appendix (rank of the gate function): gate logits from the layer input through two
    consecutive low-rank linear layers.  x [B,T,dm], w1 [rank,dm], w2 [N,rank], bias None or [N]; returns
    [B,T,Hkv,N/Hkv]."""
    lib = _load()
    x, w1, w2 = _f64(x), _f64(w1), _f64(w2)
    B, T, dm = x.shape
    rank, N = w1.shape[0], w2.shape[0]
    assert w1.shape == (rank, dm) and w2.shape == (N, rank) and rank <= 1024 and N % Hkv == 0
    b = None if bias is None else _f64(bias)
    g = np.empty((B, T, N), dtype=np.float64)
    lib.lawcat_oracle_gate_project(B, T, dm, rank, N, _ptr(x), _ptr(w1), _ptr(w2), _ptr(b), _ptr(g))
    return g.reshape(B, T, Hkv, N // Hkv)


def gla_prefill(q, k, v, g, gate_scale: float = 1.0, eps: float = 0.0, S0=None, z0=None):
    """Section 4.2 recurrence + normalized output.  Returns dict(o, den, num, S, z)."""
    lib = _load()
    q, k, v, g, S0, z0 = map(_f64, (q, k, v, g, S0, z0))
    B, T, Hq, dk = q.shape
    Hkv = k.shape[2]
    dv = v.shape[3]
    assert k.shape == (B, T, Hkv, dk) and g.shape == (B, T, Hkv, dk) and v.shape == (B, T, Hkv, dv)
    assert Hq % Hkv == 0
    if S0 is not None:
        assert S0.shape == (B, Hkv, dk, dv)
    if z0 is not None:
        assert z0.shape == (B, Hkv, dk)
    o = np.empty((B, T, Hq, dv))
    num = np.empty((B, T, Hq, dv))
    den = np.empty((B, T, Hq))
    S = np.empty((B, Hkv, dk, dv))
    z = np.empty((B, Hkv, dk))
    lib.lawcat_oracle_gla_prefill(
        B, T, Hq, Hkv, dk, dv, _ptr(q), _ptr(k), _ptr(v), _ptr(g), float(gate_scale), float(eps),
        _ptr(S0), _ptr(z0), _ptr(o), _ptr(den), _ptr(num), _ptr(S), _ptr(z),
    )
    return {"o": o, "den": den, "num": num, "S": S, "z": z}


def gla_backward(q, k, v, g, dO, gate_scale: float = 1.0, eps: float = 0.0, S0=None, z0=None):
    """Adjoint of gla_prefill: gradients of a loss with dL/do = dO with respect to q, k, v, the gate logits and the
    start state.  Keeps every state of the forward recurrence: small cases only."""
    lib = _load()
    q, k, v, g, dO = (_f64(a) for a in (q, k, v, g, dO))
    B, T, Hq, dk = q.shape
    Hkv, dv = v.shape[2], v.shape[3]
    S0 = None if S0 is None else _f64(S0)
    z0 = None if z0 is None else _f64(z0)
    out = {"dq": np.empty_like(q), "dk": np.empty_like(k), "dv": np.empty_like(v), "dg": np.empty_like(g),
           "dS0": np.empty((B, Hkv, dk, dv)), "dz0": np.empty((B, Hkv, dk))}
    lib.lawcat_oracle_gla_backward(B, T, Hq, Hkv, dk, dv, _ptr(q), _ptr(k), _ptr(v), _ptr(g), float(gate_scale), float(eps),
                                   _ptr(S0), _ptr(z0), _ptr(dO), _ptr(out["dq"]), _ptr(out["dk"]), _ptr(out["dv"]),
                                   _ptr(out["dg"]), _ptr(out["dS0"]), _ptr(out["dz0"]))
    return out


def conv1d_backward(x, w, dy, halo=None, feature_map: int = 0):
    """Adjoint of conv1d_causal: returns dict(dx, dw, dhalo)."""
    lib = _load()
    x, w, dy = _f64(x), _f64(w), _f64(dy)
    B, T, H, d = x.shape
    W = w.shape[-1]
    halo = None if halo is None or W == 1 else _f64(halo)
    dx, dw = np.empty_like(x), np.empty_like(w)
    dhalo = None if halo is None else np.empty_like(halo)
    lib.lawcat_oracle_conv1d_backward(B, T, H, d, W, _ptr(x), _ptr(w), _ptr(halo), int(feature_map), _ptr(dy), _ptr(dx),
                                      _ptr(dw), _ptr(dhalo))
    return {"dx": dx, "dw": dw, "dhalo": dhalo}


def gla_step(q, k, v, g, S, z, gate_scale: float = 1.0, eps: float = 0.0):
    """One decode step: q [B,Hq,dk], k/g [B,Hkv,dk], v [B,Hkv,dv]; returns dict(o, den, S, z)."""
    r = gla_prefill(
        np.asarray(q)[:, None], np.asarray(k)[:, None], np.asarray(v)[:, None], np.asarray(g)[:, None],
        gate_scale, eps, S, z,
    )
    return {"o": r["o"][:, 0], "den": r["den"][:, 0], "num": r["num"][:, 0], "S": r["S"], "z": r["z"]}


def _tail(x, halo, W):
    """Last W-1 raw rows of [halo ; x] (the conv cache of section 4.1), oldest first."""
    x = _f64(x)
    B, T, H, d = x.shape
    prev = np.zeros((B, W - 1, H, d)) if halo is None else _f64(halo)
    full = np.concatenate([prev, x], axis=1)
    return full[:, full.shape[1] - (W - 1):]


def layer_prefill(Q, K, V, G, wq, wk, feature_map: int = 0, gate_scale: float = 1.0, eps: float = 0.0,
                  S0=None, z0=None, q_halo=None, k_halo=None, wf=None):
    """Conv1D on Q and on K (section 4.1), phi -- pointwise, or after the shared linear layer wf [Hkv,d,d] --
    then normalized GLA (section 4.2)."""
    W = np.asarray(wq).shape[-1]
    if wf is None:
        qd = conv1d_causal(Q, wq, q_halo, feature_map)
        kd = conv1d_causal(K, wk, k_halo, feature_map)
    else:
        qd = feature_linear(conv1d_causal(Q, wq, q_halo, 0), wf, feature_map)
        kd = feature_linear(conv1d_causal(K, wk, k_halo, 0), wf, feature_map)
    r = gla_prefill(qd, kd, V, G, gate_scale, eps, S0, z0)
    r["q_tail"] = _tail(Q, q_halo, W)
    r["k_tail"] = _tail(K, k_halo, W)
    r["q_dot"] = qd
    r["k_dot"] = kd
    return r
