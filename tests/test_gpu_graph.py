"""The prefill call only enqueues kernels on the caller's stream (no allocation, no memset, no
synchronization), so it can be captured into a HIP graph.  The graph is replayed several times with
the inputs changed in place and eager work and synchronizations in between; every replay must
reproduce the eager call bit for bit."""
import pytest
import torch

from paper_2509_18467_amd import lawcat
from paper_2509_18467_amd.inputs import WORKLOADS, make_inputs

import helpers as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,T", [("llama1b_8k", 2000), ("mistral7b_16k", 1100)])
def test_layer_prefill_in_a_captured_graph(name, T):
    wl = WORKLOADS[name].with_T(T)
    dt = torch.bfloat16
    desc = H.desc_for(wl, feature_map=1)
    xs = [make_inputs(wl, seed=40 + i, state=True) for i in range(3)]
    names = ("Q", "K", "V", "G", "wq", "wk")
    st = {n: H.dev(xs[0][n], dt) for n in names}           # static input buffers of the graph
    S0, z0 = H.dev(xs[0]["S0"]), H.dev(xs[0]["z0"])

    def outputs():
        return (torch.empty_like(st["Q"]), torch.empty(wl.B, wl.T, wl.Hq, device="cuda"),
                torch.empty(wl.B, wl.Hkv, wl.d, wl.d, device="cuda"), torch.empty(wl.B, wl.Hkv, wl.d, device="cuda"))

    ws = lawcat.alloc_workspace(desc, lawcat.CALL_LAYER_PREFILL)
    gO, gden, gS, gz = outputs()

    def call(O, den, S, z):
        lawcat.layer_prefill(desc, st["Q"], st["K"], st["V"], st["G"], st["wq"], st["wk"], S0, z0, None, None,
                             O, den, S, z, None, None, ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(gO, gden, gS, gz)                              # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(gO, gden, gS, gz)
    for rep in range(4):
        x = xs[rep % 3]
        for n in names:
            st[n].copy_(H.dev(x[n], dt))
        S0.copy_(H.dev(x["S0"])); z0.copy_(H.dev(x["z0"]))
        for t in (gO, gden, gS, gz):
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eO, eden, eS, ez = outputs()
        call(eO, eden, eS, ez)                              # eager, same inputs
        torch.cuda.synchronize()
        for got, ref, what in ((gO, eO, "o"), (gden, eden, "den"), (gS, eS, "S"), (gz, ez, "z")):
            assert torch.equal(got.view(torch.int16 if got.dtype == dt else torch.int32),
                               ref.view(torch.int16 if ref.dtype == dt else torch.int32)), f"replay {rep}: {what} differs"
