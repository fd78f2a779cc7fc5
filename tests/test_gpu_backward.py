"""GPU parity of lawcat_gla_backward against the oracle's adjoint (fp64, pinned by finite differences of the
forward oracle).  The call takes the forward's den; the test hands it the oracle's (as fp32), so that what is
compared is the backward arithmetic alone.  Gradients are signed: bf16 storage is held to 2e-2 of RMS
plus one half-ulp of the stored value, fp32 storage to the fp32 bar."""
import numpy as np
import pytest
import torch

from paper_2509_18467_amd import lawcat
from paper_2509_18467_amd.inputs import WORKLOADS, Workload, make_inputs, round_to_bf16

import helpers as H

pytestmark = pytest.mark.gpu


def _store(wl, a):
    a = np.asarray(a, dtype=np.float32)
    return round_to_bf16(a) if wl.dtype == "bf16" else a


@pytest.mark.parametrize("name,T,gate_scale,start,eps", [
    ("tiny", 256, 1.0, False, 0.0), ("tiny", 77, 0.5, True, 0.0),
    ("llama1b_8k", 700, 1.0, True, 0.0), ("llama1b_8k", 1500, 1.0, False, 0.0), ("mistral7b_16k", 300, 1.0, True, 0.0),
    ("mistral7b_16k", 1100, 0.7, False, 0.0), ("llama1b_8k", 900, 0.5, True, 0.3),
    # every instantiation of the sweeps: 1, 2, 4, 8 query heads per kv head and the generic one (3, 16), both head dims,
    # both storage types, more than one batch element
    ("B2 Hq4 Hkv2 d64 bf16", 400, 1.0, True, 0.0), ("B1 Hq16 Hkv2 d64 bf16", 300, 1.0, False, 0.0),
    ("B2 Hq6 Hkv2 d64 bf16", 200, 1.0, True, 0.0), ("B1 Hq16 Hkv1 d64 fp32", 150, 1.0, True, 0.0),
    ("B1 Hq2 Hkv2 d128 bf16", 300, 1.0, True, 0.0), ("B2 Hq4 Hkv2 d128 fp32", 200, 0.8, False, 0.0),
    ("B1 Hq8 Hkv1 d128 bf16", 260, 1.0, True, 0.0), ("B1 Hq3 Hkv1 d128 bf16", 100, 1.0, False, 0.0),
    ("B1 Hq4 Hkv1 d64 fp32", 2500, 1.0, True, 0.0),
])
def test_gla_backward(oracle, name, T, gate_scale, start, eps):
    if name in WORKLOADS:
        wl = WORKLOADS[name].with_T(T)
    else:
        f = dict((k.rstrip("0123456789"), k) for k in name.split())
        wl = Workload(name, B=int(f["B"][1:]), T=T, Hq=int(f["Hq"][2:]), Hkv=int(f["Hkv"][3:]), d=int(f["d"][1:]),
                      dtype=name.split()[-1])
    x = make_inputs(wl, seed=11, state=start)
    print("gla_backward", wl, "gate_scale", gate_scale, "start state", start, "eps", eps, flush=True)
    # positive features, as phi = 1 + ELU gives them
    q = _store(wl, oracle.conv1d_causal(x["Q"], x["wq"], None, 1))
    k = _store(wl, oracle.conv1d_causal(x["K"], x["wk"], None, 1))
    v, g = x["V"], x["G"]
    S0, z0 = x.get("S0"), x.get("z0")
    fwd = oracle.gla_prefill(q, k, v, g, gate_scale, eps, S0, z0)
    den = fwd["den"].astype(np.float32)
    dO = _store(wl, np.random.default_rng(5).standard_normal(fwd["o"].shape) * 0.5)
    ref = oracle.gla_backward(q, k, v, g, dO, gate_scale, eps, S0, z0)

    dt = H.tdtype(wl)
    desc = H.desc_for(wl, gate_scale=gate_scale, eps=eps)
    dq_, dk_, dv_, dg_ = (H.dev(a, dt) for a in (q, k, v, g))
    outs = {"dq": torch.empty_like(dq_), "dk": torch.empty_like(dk_), "dv": torch.empty_like(dv_), "dg": torch.empty_like(dg_)}
    dS0 = torch.empty(wl.B, wl.Hkv, wl.d, wl.d, device="cuda")
    dz0 = torch.empty(wl.B, wl.Hkv, wl.d, device="cuda")
    ws = lawcat.alloc_workspace(desc, lawcat.CALL_GLA_BACKWARD)
    lawcat.gla_backward(desc, dq_, dk_, dv_, dg_, H.dev(den), H.dev(dO, dt), H.dev(S0), H.dev(z0),
                        outs["dq"], outs["dk"], outs["dv"], outs["dg"], dS0, dz0, ws)
    torch.cuda.synchronize()
    got = {n: H.host(t) for n, t in outs.items()}
    got["dS0"], got["dz0"] = H.host(dS0), H.host(dz0)
    rnd = 1 if wl.dtype == "bf16" else 0
    for n in ("dq", "dk", "dv", "dg", "dS0", "dz0"):
        r = H.assert_close(got[n], ref[n], wl, f"gla_backward {n}", rnd if n in outs else 0)
        print(f"  {n}: error / bar {r:.3f}, max err / rms {H.rel_rms_err(got[n], ref[n]):.3e}", flush=True)


def _abs_term_sum_dw(oracle, x, w, halo, dy, phi):
    """sum over (b, t) of |du_t x_{t-delta}| per weight: the scale that the rounding error of an fp32 sum of
    signed terms is measured against (tolerance only; the expected dw is the oracle's)."""
    B, T, Hh, d = x.shape
    W = w.shape[-1]
    u = oracle.conv1d_causal(x, w, halo, 0)
    du = np.abs(dy * (np.where(u > 0, 1.0, np.exp(np.minimum(u, 0.0))) if phi == 1 else 1.0))
    prev = np.zeros((B, W - 1, Hh, d)) if halo is None else np.asarray(halo, dtype=np.float64)
    full = np.abs(np.concatenate([prev, x], axis=1))
    out = np.empty((Hh, d, W))
    for dl in range(W):
        out[:, :, dl] = (du * full[:, W - 1 - dl: W - 1 - dl + T]).sum(axis=(0, 1))
    return out


@pytest.mark.parametrize("name,B,T,W,phi,halo", [
    ("tiny", 1, 77, 4, 1, True), ("tiny", 2, 130, 4, 0, False), ("tiny", 1, 5, 3, 1, True), ("tiny", 3, 64, 2, 1, False),
    ("tiny", 1, 200, 1, 1, False), ("tiny", 1, 2, 4, 1, True),
    ("llama1b_8k", 1, 1500, 4, 1, True), ("llama1b_8k", 2, 333, 4, 1, False), ("mistral7b_16k", 1, 700, 4, 1, True),
    ("mistral7b_16k", 1, 129, 3, 0, True),
    # full size, the shape the benchmark's side op times
    ("llama1b_32k", 1, 32768, 4, 1, True), ("mistral7b_16k", 1, 16384, 4, 1, True),
])
def test_conv1d_backward(oracle, name, B, T, W, phi, halo):
    import dataclasses
    wl = dataclasses.replace(WORKLOADS[name].with_T(T), B=B, W=W)
    xin = make_inputs(wl, seed=21, halo=halo)
    print("conv1d_backward", wl, "phi", phi, "halo", halo, flush=True)
    x, w = xin["Q"], xin["wq"]
    hl = xin.get("q_halo") if (halo and W > 1) else None
    dy = _store(wl, np.random.default_rng(6).standard_normal(x.shape) * 0.5)
    ref = oracle.conv1d_backward(x, w, dy, hl, phi)

    dt = H.tdtype(wl)
    desc = H.desc_for(wl, feature_map=phi)
    dx = torch.empty(x.shape, dtype=dt, device="cuda")
    dw = torch.empty(w.shape, dtype=torch.float32, device="cuda")
    dh = torch.empty(B, W - 1, wl.Hq, wl.d, dtype=dt, device="cuda") if W > 1 else None
    ws = lawcat.alloc_workspace(desc, lawcat.CALL_CONV1D_BACKWARD)
    lawcat.conv1d_backward(desc, wl.Hq, H.dev(x, dt), H.dev(w, dt), H.dev(hl, dt), H.dev(dy, dt), dx, dw, dh, ws)
    torch.cuda.synchronize()
    rnd = 1 if wl.dtype == "bf16" else 0
    r = H.assert_close(H.host(dx), ref["dx"], wl, "conv1d_backward dx", rnd)
    print(f"  dx: error / bar {r:.3f}", flush=True)
    if hl is not None:
        r = H.assert_close(H.host(dh), ref["dhalo"], wl, "conv1d_backward dhalo", rnd)
        print(f"  dhalo: error / bar {r:.3f}", flush=True)
    # dw is an fp32 sum over all tokens of signed products: 64 fp32 ulps of the sum of their absolute values
    scale = _abs_term_sum_dw(oracle, x, w, hl, dy, phi)
    ratio = np.abs(H.host(dw) - ref["dw"]) / (2.0 ** -18 * scale + 1e-6)
    print(f"  dw: error / bar {ratio.max():.3f}", flush=True)
    assert ratio.max() <= 1.0, f"conv1d_backward dw: largest error is {ratio.max():.3f} of its bar"


@pytest.mark.parametrize("name,T", [("llama1b_8k", 1300), ("mistral7b_16k", 500)])
def test_layer_backward_as_a_chain_of_calls(oracle, name, T):
    """lawcat_gla_backward, then lawcat_conv1d_backward on (Q, wq, dq) and (K, wk, dk), against the same chain of
    the oracle's adjoints (pinned on the CPU against finite differences of the oracle's whole layer).  Each GPU
    stage is fed the oracle's result of the stage before it, rounded to storage, as everywhere in this file."""
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=23, halo=True, state=True)
    print("layer backward", wl, flush=True)
    dt = H.tdtype(wl)
    desc = H.desc_for(wl, feature_map=1)
    q = _store(wl, oracle.conv1d_causal(x["Q"], x["wq"], x["q_halo"], 1))
    k = _store(wl, oracle.conv1d_causal(x["K"], x["wk"], x["k_halo"], 1))
    fwd = oracle.gla_prefill(q, k, x["V"], x["G"], 1.0, 0.0, x["S0"], x["z0"])
    dO = _store(wl, np.random.default_rng(8).standard_normal(fwd["o"].shape) * 0.5)
    ga = oracle.gla_backward(q, k, x["V"], x["G"], dO, 1.0, 0.0, x["S0"], x["z0"])
    got = {}
    for nm, src, wt, hl, dy, heads in (("q", "Q", "wq", "q_halo", ga["dq"], wl.Hq), ("k", "K", "wk", "k_halo", ga["dk"], wl.Hkv)):
        dyr = _store(wl, dy)
        ref = oracle.conv1d_backward(x[src], x[wt], dyr, x[hl], 1)
        dx = torch.empty(x[src].shape, dtype=dt, device="cuda")
        dw = torch.empty(x[wt].shape, dtype=torch.float32, device="cuda")
        ws = lawcat.alloc_workspace(desc, lawcat.CALL_CONV1D_BACKWARD)
        lawcat.conv1d_backward(desc, heads, H.dev(x[src], dt), H.dev(x[wt], dt), H.dev(x[hl], dt), H.dev(dyr, dt), dx, dw,
                               None, ws)
        torch.cuda.synchronize()
        r = H.assert_close(H.host(dx), ref["dx"], wl, f"layer backward d{src}", 1)
        scale = _abs_term_sum_dw(oracle, x[src], x[wt], x[hl], dyr, 1)
        rw = (np.abs(H.host(dw) - ref["dw"]) / (2.0 ** -18 * scale + 1e-6)).max()
        print(f"  d{src}: error / bar {r:.3f}; d{wt}: {rw:.3f}", flush=True)
        assert rw <= 1.0, f"layer backward d{wt}: largest error is {rw:.3f} of its bar"


@pytest.mark.parametrize("T", [1, 7, 8, 9, 65])
@pytest.mark.parametrize("gates", ["closed", "open", "mixed"])
def test_gla_backward_short_sequences_and_saturated_gates(oracle, T, gates):
    """Sequences shorter than, equal to and just longer than a staged block of 8 tokens and a 64-token segment,
    with gate logits at -30 (nothing is carried: alpha ~ 1e-13), +30 (nothing decays) or a mix of both with
    ordinary ones.  fp32 storage: the backward has no floor on the decay, so the fp32 bar holds throughout."""
    wl = Workload(f"edge T{T} {gates}", B=2, T=T, Hq=4, Hkv=2, d=64, dtype="fp32")
    x = make_inputs(wl, seed=31, state=True)
    rng = np.random.default_rng(32)
    g = x["G"].copy()
    if gates == "closed":
        g[:] = -30.0
    elif gates == "open":
        g[:] = 30.0
    else:
        pick = rng.random(g.shape)
        g[pick < 0.1] = -30.0
        g[pick > 0.9] = 30.0
    q = np.abs(x["Q"]).astype(np.float32) + 0.1
    k = np.abs(x["K"]).astype(np.float32) + 0.1
    v, S0, z0 = x["V"], x["S0"], np.abs(x["z0"]) + 0.5
    fwd = oracle.gla_prefill(q, k, v, g, 1.0, 0.0, S0, z0)
    dO = (rng.standard_normal(fwd["o"].shape) * 0.5).astype(np.float32)
    ref = oracle.gla_backward(q, k, v, g, dO, 1.0, 0.0, S0, z0)
    desc = H.desc_for(wl)
    tq, tk, tv, tg = (H.dev(a) for a in (q, k, v, g))
    outs = {"dq": torch.empty_like(tq), "dk": torch.empty_like(tk), "dv": torch.empty_like(tv), "dg": torch.empty_like(tg),
            "dS0": torch.empty(wl.B, wl.Hkv, wl.d, wl.d, device="cuda"), "dz0": torch.empty(wl.B, wl.Hkv, wl.d, device="cuda")}
    ws = lawcat.alloc_workspace(desc, lawcat.CALL_GLA_BACKWARD)
    lawcat.gla_backward(desc, tq, tk, tv, tg, H.dev(fwd["den"].astype(np.float32)), H.dev(dO), H.dev(S0), H.dev(z0),
                        outs["dq"], outs["dk"], outs["dv"], outs["dg"], outs["dS0"], outs["dz0"], ws)
    torch.cuda.synchronize()
    for n, t in outs.items():
        H.assert_close(H.host(t), ref[n], wl, f"gla_backward {n} (T={T}, gates {gates})")


@pytest.mark.parametrize("name,T", [("llama1b_8k", 1300), ("mistral7b_16k", 600)])
def test_backward_after_the_forward_call(oracle, name, T):
    """As a caller uses the pair: lawcat_gla_prefill's own den_out (matrix-core path, about 1e-3 off the oracle's)
    goes into lawcat_gla_backward.  A relative error of den scales dnum and dden of that token and head alike, so it
    arrives in the gradients as the same relative error: the bars of the backward alone still hold."""
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=11, state=True)
    print("forward + backward", wl, flush=True)
    q = _store(wl, oracle.conv1d_causal(x["Q"], x["wq"], None, 1))
    k = _store(wl, oracle.conv1d_causal(x["K"], x["wk"], None, 1))
    v, g, S0, z0 = x["V"], x["G"], x["S0"], x["z0"]
    dt = H.tdtype(wl)
    desc = H.desc_for(wl)
    tq, tk, tv, tg = (H.dev(a, dt) for a in (q, k, v, g))
    o, den = torch.empty_like(tq), torch.empty(wl.B, wl.T, wl.Hq, device="cuda")
    lawcat.gla_prefill(desc, tq, tk, tv, tg, H.dev(S0), H.dev(z0), o, den, torch.empty(wl.B, wl.Hkv, wl.d, wl.d, device="cuda"),
                       torch.empty(wl.B, wl.Hkv, wl.d, device="cuda"), lawcat.alloc_workspace(desc, lawcat.CALL_GLA_PREFILL))
    dO = _store(wl, np.random.default_rng(5).standard_normal(tuple(o.shape)) * 0.5)
    ref = oracle.gla_backward(q, k, v, g, dO, 1.0, 0.0, S0, z0)
    outs = {"dq": torch.empty_like(tq), "dk": torch.empty_like(tk), "dv": torch.empty_like(tv), "dg": torch.empty_like(tg)}
    lawcat.gla_backward(desc, tq, tk, tv, tg, den, H.dev(dO, dt), H.dev(S0), H.dev(z0), outs["dq"], outs["dk"], outs["dv"],
                        outs["dg"], None, None, lawcat.alloc_workspace(desc, lawcat.CALL_GLA_BACKWARD))
    torch.cuda.synchronize()
    for n, t in outs.items():
        r = H.assert_close(H.host(t), ref[n], wl, f"forward + backward {n}", 1)
        print(f"  {n}: error / bar {r:.3f}", flush=True)


@pytest.mark.parametrize("name", ["llama1b_32k", "mistral7b_16k"])
def test_gla_backward_full_size(oracle, name):
    """The two headline shapes at full length, in the launch plan the benchmark's side op times (128 / 64
    segments per kv head), every element of every gradient against the oracle (10-20 s of host time each)."""
    wl = WORKLOADS[name]
    x = make_inputs(wl, seed=13, state=True)
    print("gla_backward full size", wl, flush=True)
    q = _store(wl, oracle.conv1d_causal(x["Q"], x["wq"], None, 1))
    k = _store(wl, oracle.conv1d_causal(x["K"], x["wk"], None, 1))
    v, g, S0, z0 = x["V"], x["G"], x["S0"], x["z0"]
    fwd = oracle.gla_prefill(q, k, v, g, 1.0, 0.0, S0, z0)
    den = fwd["den"].astype(np.float32)
    dO = _store(wl, np.random.default_rng(5).standard_normal(fwd["o"].shape) * 0.5)
    del fwd
    ref = oracle.gla_backward(q, k, v, g, dO, 1.0, 0.0, S0, z0)
    dt = H.tdtype(wl)
    desc = H.desc_for(wl)
    tq, tk, tv, tg = (H.dev(a, dt) for a in (q, k, v, g))
    outs = {"dq": torch.empty_like(tq), "dk": torch.empty_like(tk), "dv": torch.empty_like(tv), "dg": torch.empty_like(tg),
            "dS0": torch.empty(wl.B, wl.Hkv, wl.d, wl.d, device="cuda"), "dz0": torch.empty(wl.B, wl.Hkv, wl.d, device="cuda")}
    lawcat.gla_backward(desc, tq, tk, tv, tg, H.dev(den), H.dev(dO, dt), H.dev(S0), H.dev(z0), outs["dq"], outs["dk"],
                        outs["dv"], outs["dg"], outs["dS0"], outs["dz0"], lawcat.alloc_workspace(desc, lawcat.CALL_GLA_BACKWARD))
    torch.cuda.synchronize()
    for n, t in outs.items():
        r = H.assert_close(H.host(t), ref[n], wl, f"gla_backward full size {n}", 1 if n in ("dq", "dk", "dv", "dg") else 0)
        print(f"  {n}: error / bar {r:.3f}", flush=True)
