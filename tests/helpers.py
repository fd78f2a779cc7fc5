"""Shared test plumbing: device upload, error metrics, one-call wrappers around the binding."""
from __future__ import annotations

import numpy as np
import torch

from paper_2509_18467_amd import lawcat
from paper_2509_18467_amd.inputs import Workload

# Parity bars (stated by the benchmark spec): fp32 storage max abs error <= 1e-4;
# bf16 storage max error <= 2e-2 of the reference RMS.
FP32_MAX_ABS = 1e-4
BF16_REL_RMS = 2e-2
BF16_HALF_ULP = 2.0 ** -8   # largest relative error of rounding a value to bf16 (8 significant bits)
FP32_REL = 2.0 ** -18       # 64 fp32 ulps: takes over from the absolute bar where |ref| > 26


def tdtype(wl: Workload):
    return torch.bfloat16 if wl.dtype == "bf16" else torch.float32


def dev(a, dtype=torch.float32):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda").to(dtype).contiguous()


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def rms(a):
    return float(np.sqrt(np.mean(np.asarray(a, dtype=np.float64) ** 2)))


def rel_rms_err(got, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - ref)) / max(rms(ref), 1e-300))


def max_abs_err(got, ref):
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - np.asarray(ref, dtype=np.float64))))


def bar(ref, wl: Workload, roundings: int = 0, terms=None):
    """Allowed error of every element.
    fp32 storage: 1e-4 absolute (the stated bar); where |ref| > 26 that is less than 64 fp32 ulps of the value
    itself, and 2^-18 |ref| takes over.
    bf16 storage: 2e-2 of RMS(ref) (the stated bar) + roundings * 2^-8 * terms.  `roundings` is 0 for every
    well-conditioned comparison.  Otherwise it is the number of bf16 roundings (each at most 2^-8 relative) on
    the factors of one product term, and `terms` the sum of the ABSOLUTE values of the terms that make up the
    element (default |ref|: no cancellation): the textbook forward error bound of a sum of products with rounded
    factors.  With signed features an element is a cancelling sum, and what it inherits from its terms'
    roundings is set by their size, not by its own or by the RMS."""
    ref = np.abs(np.asarray(ref, dtype=np.float64))
    if wl.dtype == "fp32":
        return np.maximum(FP32_MAX_ABS, FP32_REL * ref)
    terms = ref if terms is None else np.abs(np.asarray(terms, dtype=np.float64))
    return BF16_REL_RMS * rms(ref) + roundings * BF16_HALF_ULP * terms


def assert_close(got, ref, wl: Workload, what: str, roundings: int = 0, terms=None):
    """Every element within bar(); returns the largest error as a fraction of its bar."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    ratio = np.abs(got - ref) / bar(ref, wl, roundings, terms)
    worst = float(ratio.max()) if ratio.size else 0.0
    assert np.isfinite(got).all() or not np.isfinite(ref).all(), f"{what}: non-finite values"
    assert worst <= 1.0, (f"{what}: largest error is {worst:.3f} of its bar "
                          f"(max err / rms {rel_rms_err(got, ref):.3e}, max abs {max_abs_err(got, ref):.3e})")
    return worst


def quantile_err(got, ref, q=0.999, stride=7):
    """q-quantile of |got - ref| / RMS(ref) (on every `stride`-th element: the tensors are large)."""
    e = np.abs(np.asarray(got, dtype=np.float64) - np.asarray(ref, dtype=np.float64)).ravel()[::stride]
    return float(np.quantile(e, q) / max(rms(ref), 1e-300))


def desc_for(wl: Workload, **kw):
    return lawcat.make_desc(wl.B, wl.T, wl.Hq, wl.Hkv, wl.d, conv_width=wl.W,
                            dtype=lawcat.DTYPE_BF16 if wl.dtype == "bf16" else lawcat.DTYPE_F32, **kw)


def run_layer_prefill(wl: Workload, x: dict, feature_map=1, den=True, tails=True, wf=None, **desc_kw):
    """Upload x (numpy float32 dict from make_inputs), call lawcat_layer_prefill (lawcat_layer_prefill_fm if the
    shared feature matrix wf is given), return numpy float64 results."""
    dt = tdtype(wl)
    d = desc_for(wl, feature_map=feature_map, **desc_kw)
    Q, K, V, G, wq, wk = (dev(x[n], dt) for n in ("Q", "K", "V", "G", "wq", "wk"))
    S0, z0 = dev(x.get("S0")), dev(x.get("z0"))
    qh, kh = dev(x.get("q_halo"), dt), dev(x.get("k_halo"), dt)
    O = torch.empty_like(Q)
    den_out = torch.empty(wl.B, wl.T, wl.Hq, dtype=torch.float32, device="cuda") if den else None
    S = torch.empty(wl.B, wl.Hkv, wl.d, wl.d, dtype=torch.float32, device="cuda")
    z = torch.empty(wl.B, wl.Hkv, wl.d, dtype=torch.float32, device="cuda")
    qt = torch.empty(wl.B, wl.W - 1, wl.Hq, wl.d, dtype=dt, device="cuda") if tails and wl.W > 1 else None
    kt = torch.empty(wl.B, wl.W - 1, wl.Hkv, wl.d, dtype=dt, device="cuda") if tails and wl.W > 1 else None
    if wf is None:
        ws = lawcat.alloc_workspace(d, lawcat.CALL_LAYER_PREFILL)
        lawcat.layer_prefill(d, Q, K, V, G, wq, wk, S0, z0, qh, kh, O, den_out, S, z, qt, kt, ws)
    else:
        ws = lawcat.alloc_workspace(d, lawcat.CALL_LAYER_PREFILL_FM)
        lawcat.layer_prefill_fm(d, Q, K, V, G, wq, wk, dev(wf, dt), S0, z0, qh, kh, O, den_out, S, z, qt, kt, ws)
    torch.cuda.synchronize()
    r = {"o": host(O), "S": host(S), "z": host(z)}
    if den:
        r["den"] = host(den_out)
    if qt is not None:
        r["q_tail"], r["k_tail"] = host(qt), host(kt)
    if wf is not None:
        # q-dot and k-dot as the call staged them: the head of the workspace, k-dot at the next multiple of 256 bytes
        nq, nk = wl.B * wl.T * wl.Hq * wl.d, wl.B * wl.T * wl.Hkv * wl.d
        off = -(-nq * Q.element_size() // 256) * 256
        r["q_dot"] = host(ws[:nq * Q.element_size()].view(dt).reshape(wl.B, wl.T, wl.Hq, wl.d))
        r["k_dot"] = host(ws[off:off + nk * Q.element_size()].view(dt).reshape(wl.B, wl.T, wl.Hkv, wl.d))
    return r


def run_conv_feature(wl: Workload, x, w, wf, halo=None, feature_map=1):
    dt = tdtype(wl)
    H = x.shape[2]
    d = desc_for(wl, feature_map=feature_map)
    xd, wd, fd, hd = dev(x, dt), dev(w, dt), dev(wf, dt), dev(halo, dt)
    y = torch.empty_like(xd)
    tail = torch.empty(wl.B, wl.W - 1, H, wl.d, dtype=dt, device="cuda") if wl.W > 1 else None
    lawcat.conv1d_feature(d, H, xd, wd, fd, hd, y, tail)
    torch.cuda.synchronize()
    return host(y), (host(tail) if tail is not None else None)


def run_gate_project(wl: Workload, gi: dict, d_model: int, rank: int):
    dt = tdtype(wl)
    d = desc_for(wl)
    x, w1, w2, b = (dev(gi.get(k), dt) for k in ("x", "w1", "w2", "bias"))
    g = torch.empty(wl.B, wl.T, wl.Hkv, wl.d, dtype=dt, device="cuda")
    lawcat.gate_project(d, d_model, rank, x, w1, w2, b, g)
    torch.cuda.synchronize()
    return host(g)


def run_gla_prefill(wl: Workload, q, k, v, g, S0=None, z0=None, **desc_kw):
    dt = tdtype(wl)
    d = desc_for(wl, **desc_kw)
    q, k, v, g = (dev(a, dt) for a in (q, k, v, g))
    o = torch.empty_like(q)
    den_out = torch.empty(wl.B, wl.T, wl.Hq, dtype=torch.float32, device="cuda")
    S = torch.empty(wl.B, wl.Hkv, wl.d, wl.d, dtype=torch.float32, device="cuda")
    z = torch.empty(wl.B, wl.Hkv, wl.d, dtype=torch.float32, device="cuda")
    ws = lawcat.alloc_workspace(d, lawcat.CALL_GLA_PREFILL)
    lawcat.gla_prefill(d, q, k, v, g, dev(S0), dev(z0), o, den_out, S, z, ws)
    torch.cuda.synchronize()
    return {"o": host(o), "den": host(den_out), "S": host(S), "z": host(z)}


def run_conv(wl: Workload, x, w, halo=None, feature_map=0):
    dt = tdtype(wl)
    H = x.shape[2]
    d = desc_for(wl, feature_map=feature_map)
    xd, wd, hd = dev(x, dt), dev(w, dt), dev(halo, dt)
    y = torch.empty_like(xd)
    tail = torch.empty(wl.B, wl.W - 1, H, wl.d, dtype=dt, device="cuda") if wl.W > 1 else None
    lawcat.conv1d_causal(d, H, xd, wd, hd, y, tail)
    torch.cuda.synchronize()
    return host(y), (None if tail is None else host(tail))
