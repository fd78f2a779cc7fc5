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


@pytest.mark.parametrize("name,T,gate_scale,start", [
    ("tiny", 256, 1.0, False), ("tiny", 77, 0.5, True),
    ("llama1b_8k", 700, 1.0, True), ("llama1b_8k", 1500, 1.0, False), ("mistral7b_16k", 300, 1.0, True),
    ("mistral7b_16k", 1100, 0.7, False),
])
def test_gla_backward(oracle, name, T, gate_scale, start):
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=11, state=start)
    print("gla_backward", wl, "gate_scale", gate_scale, "start state", start, flush=True)
    # positive features, as phi = 1 + ELU gives them
    q = _store(wl, oracle.conv1d_causal(x["Q"], x["wq"], None, 1))
    k = _store(wl, oracle.conv1d_causal(x["K"], x["wk"], None, 1))
    v, g = x["V"], x["G"]
    S0, z0 = x.get("S0"), x.get("z0")
    fwd = oracle.gla_prefill(q, k, v, g, gate_scale, 0.0, S0, z0)
    den = fwd["den"].astype(np.float32)
    dO = _store(wl, np.random.default_rng(5).standard_normal(fwd["o"].shape) * 0.5)
    ref = oracle.gla_backward(q, k, v, g, dO, gate_scale, 0.0, S0, z0)

    dt = H.tdtype(wl)
    desc = H.desc_for(wl, gate_scale=gate_scale)
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
