"""Seeded random shapes through the fused layer call against the oracle (bf16 storage, 1+ELU).

The hand-picked cases of test_gpu_parity.py sit at tile boundaries chosen by the author; this list
is drawn blindly: batch, length (from one token to a few segments), group size, head dim, conv
width, with or without conv halos and a start state, every carry mode.  Same bars as everywhere."""
import numpy as np
import pytest

from paper_2509_18467_amd.inputs import Workload, make_inputs

import helpers as H

pytestmark = pytest.mark.gpu


def _cases(n=36):
    rng = np.random.default_rng(20240917)
    out = []
    for i in range(n):
        d = int(rng.choice([64, 128]))
        group = int(rng.choice([1, 1, 2, 3, 4, 4, 6, 8]))
        Hkv = int(rng.integers(1, 4))
        B = int(rng.integers(1, 4))
        T = int(rng.choice([1, 2, 3, 15, 16, 17, 63, 64, 65, 127, 200, 511, 513, 777, 1025, 1531, 2300]))
        W = int(rng.choice([4, 4, 4, 3, 2, 1]))
        extras = bool(rng.integers(0, 2))
        carry = int(rng.choice([0, 0, 1, 2]))
        segment = int(rng.choice([0, 0, 64, 128, 192])) if carry != 1 else 0
        out.append((i, B, T, Hkv * group, Hkv, d, W, extras, carry, segment))
    return out


@pytest.mark.parametrize("i,B,T,Hq,Hkv,d,W,extras,carry,segment", _cases())
def test_random_shape(oracle, i, B, T, Hq, Hkv, d, W, extras, carry, segment):
    wl = Workload(f"rnd{i}", B, T, Hq, Hkv, d, W, "bf16")
    x = make_inputs(wl, seed=1000 + i, halo=extras and W > 1, state=extras)
    print("random shape", wl, "extras", extras, "carry", carry, "segment", segment, flush=True)
    got = H.run_layer_prefill(wl, x, feature_map=1, carry_mode=carry, segment=segment)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1, 1.0, 0.0,
                               x.get("S0"), x.get("z0"), x.get("q_halo"), x.get("k_halo"))
    tag = f"random[{wl.name}]"
    H.assert_close(got["o"], ref["o"], wl, tag + " o")
    H.assert_close(got["den"], ref["den"], wl, tag + " den")
    H.assert_close(got["S"], ref["S"], wl, tag + " S")
    H.assert_close(got["z"], ref["z"], wl, tag + " z")
    if W > 1:
        assert np.array_equal(got["q_tail"], ref["q_tail"]) and np.array_equal(got["k_tail"], ref["k_tail"])
