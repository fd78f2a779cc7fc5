"""Repeated-run stability of the bf16 matrix-core prefill.

The path has no atomics and a fixed reduction order, so two calls on the same inputs must agree bit for
bit.  The check exists because kernel shapes that were parity-correct on most runs still produced, now and
then, a few wrong output tiles on gfx950 (an MFMA operand register reused too early by the compiler's
schedule); a fault of that kind shows up here as a run that differs from the first.  Every template
instantiation of the chunk kernels is covered: head dim x group size x (plain | fused conv, both feature
maps), at a size with fewer workgroups than compute units and at one with several per unit.
"""
import numpy as np
import pytest
import torch

import helpers as H
from paper_2509_18467_amd import lawcat
from paper_2509_18467_amd.inputs import Workload, make_inputs

pytestmark = pytest.mark.gpu

RUNS = 12


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t.view(torch.int32)


@pytest.mark.parametrize("mode", ["plain", "conv_identity", "conv_elu1"])
@pytest.mark.parametrize("group", [1, 2, 4])
@pytest.mark.parametrize("d", [64, 128])
def test_repeated_calls_are_bit_identical(d, group, mode):
    for B, Hkv, T in ((1, 8, 700), (2, 16, 1500)):
        wl = Workload("det", B=B, T=T, Hq=Hkv * group, Hkv=Hkv, d=d)
        x = make_inputs(wl, seed=3, state=True, halo=True)
        dt = torch.bfloat16
        Q, K, V, G, wq, wk = (H.dev(x[n], dt) for n in ("Q", "K", "V", "G", "wq", "wk"))
        S0, z0 = H.dev(x["S0"]), H.dev(x["z0"])
        qh, kh = H.dev(x["q_halo"], dt), H.dev(x["k_halo"], dt)
        if mode == "plain":  # already transformed, positive q-dot and k-dot
            Q, K = Q.abs(), K.abs()
        desc = H.desc_for(wl, feature_map=0 if mode == "conv_identity" else 1)
        call = lawcat.CALL_GLA_PREFILL if mode == "plain" else lawcat.CALL_LAYER_PREFILL
        ws = lawcat.alloc_workspace(desc, call)
        first = None
        for it in range(RUNS):
            O = torch.empty_like(Q)
            den = torch.empty(B, T, wl.Hq, dtype=torch.float32, device="cuda")
            S = torch.empty(B, Hkv, d, d, dtype=torch.float32, device="cuda")
            z = torch.empty(B, Hkv, d, dtype=torch.float32, device="cuda")
            if mode == "plain":
                lawcat.gla_prefill(desc, Q, K, V, G, S0, z0, O, den, S, z, ws)
            else:
                lawcat.layer_prefill(desc, Q, K, V, G, wq, wk, S0, z0, qh, kh, O, den, S, z, None, None, ws)
            torch.cuda.synchronize()
            cur = {"o": O, "den": den, "S": S, "z": z}
            if first is None:
                first = cur
                continue
            for name in cur:
                same = torch.equal(_bits(cur[name]), _bits(first[name]))
                assert same, (f"d={d} group={group} {mode} B={B} T={T}: {name} of call {it} differs from call 0 in "
                              f"{int((_bits(cur[name]) != _bits(first[name])).sum())} elements")


@pytest.mark.parametrize("d", [64, 128])
def test_matrix_core_side_kernels_are_bit_identical(d):
    """The conv + feature-matrix kernel and the gate projection reduce in a fixed order too (the gate projection
    adds its four partial sums in wave order): repeated calls agree bit for bit, at a size with several
    workgroups per compute unit and the 32-token workgroups of the gate kernel."""
    from paper_2509_18467_amd.inputs import make_feature_weights, make_gate_inputs

    wl = Workload("det_side", B=1, T=16400, Hq=32, Hkv=8, d=d)
    dt = torch.bfloat16
    x = make_inputs(wl, seed=5, halo=True)
    dm = 2048 if d == 64 else 4096
    gi = make_gate_inputs(wl, dm, 32, seed=5)
    desc = H.desc_for(wl, feature_map=1)
    Q, wq, qh = H.dev(x["Q"], dt), H.dev(x["wq"], dt), H.dev(x["q_halo"], dt)
    wf = H.dev(make_feature_weights(wl, seed=5), dt)
    gx, gw1, gw2, gb = (H.dev(gi[k], dt) for k in ("x", "w1", "w2", "bias"))
    first = None
    for it in range(RUNS):
        y = torch.empty_like(Q)
        g = torch.empty(wl.B, wl.T, wl.Hkv, d, dtype=dt, device="cuda")
        lawcat.conv1d_feature(desc, wl.Hq, Q, wq, wf, qh, y, None)
        lawcat.gate_project(desc, dm, 32, gx, gw1, gw2, gb, g)
        torch.cuda.synchronize()
        cur = {"feature": y, "gate": g}
        if first is None:
            first = cur
            continue
        for name in cur:
            assert torch.equal(_bits(cur[name]), _bits(first[name])), f"d={d}: {name} of call {it} differs from call 0"


@pytest.mark.parametrize("d", [64, 128])
def test_backward_is_bit_identical(d):
    """The backward adds the rows of dv through shuffles and LDS in a fixed order and carries segment states
    through an ordered scan: no atomics, so repeated calls agree bit for bit (several segments per head)."""
    wl = Workload("det_bwd", B=2, T=3000, Hq=8, Hkv=2, d=d)
    dt = torch.bfloat16
    x = make_inputs(wl, seed=9, state=True)
    desc = H.desc_for(wl)
    q, k = (torch.nn.functional.elu(H.dev(x[n], dt).float()).add(1).to(dt) for n in ("Q", "K"))
    v, g, S0, z0 = H.dev(x["V"], dt), H.dev(x["G"], dt), H.dev(x["S0"]), H.dev(x["z0"])
    o = torch.empty_like(q)
    den = torch.empty(wl.B, wl.T, wl.Hq, device="cuda")
    ws = lawcat.alloc_workspace(desc, lawcat.CALL_GLA_PREFILL)
    lawcat.gla_prefill(desc, q, k, v, g, S0, z0, o, den, torch.empty_like(S0), torch.empty_like(z0), ws)
    dO = torch.randn(o.shape, device="cuda", generator=torch.Generator("cuda").manual_seed(3)).to(dt)
    wb = lawcat.alloc_workspace(desc, lawcat.CALL_GLA_BACKWARD)
    dconv = H.desc_for(wl, feature_map=1)
    Qraw, wq = H.dev(x["Q"], dt), H.dev(x["wq"], dt)
    wc = lawcat.alloc_workspace(dconv, lawcat.CALL_CONV1D_BACKWARD)
    first = None
    for it in range(RUNS):
        cur = {"dq": torch.empty_like(q), "dk": torch.empty_like(k), "dv": torch.empty_like(v), "dg": torch.empty_like(g),
               "dS0": torch.empty_like(S0), "dz0": torch.empty_like(z0)}
        wb.fill_(0xFF)     # NaN patterns: nothing is read before it is written
        lawcat.gla_backward(desc, q, k, v, g, den, dO, S0, z0, cur["dq"], cur["dk"], cur["dv"], cur["dg"], cur["dS0"],
                            cur["dz0"], wb)
        # and the conv's adjoint on the query side (dw: per-strip partial sums added in strip order)
        cur["dQ"], cur["dwq"] = torch.empty_like(q), torch.empty(wl.Hq, d, wl.W, device="cuda")
        wc.fill_(0xFF)
        lawcat.conv1d_backward(dconv, wl.Hq, Qraw, wq, None, cur["dq"], cur["dQ"], cur["dwq"], None, wc)
        torch.cuda.synchronize()
        for name, t in cur.items():
            assert torch.isfinite(t.float()).all(), f"d={d}: {name} of call {it} is not finite"
        if first is None:
            first = cur
            continue
        for name in cur:
            assert torch.equal(_bits(cur[name]), _bits(first[name])), f"d={d}: {name} of call {it} differs from call 0"
