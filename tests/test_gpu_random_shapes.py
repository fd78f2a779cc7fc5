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


def _packed_cases(n=12):
    rng = np.random.default_rng(20250301)
    out = []
    for i in range(n):
        d = int(rng.choice([64, 128]))
        group = int(rng.choice([1, 2, 4, 4, 3]))
        Hkv = int(rng.integers(1, 4))
        nseq = int(rng.integers(1, 9))
        lengths = tuple(int(v) for v in rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 130, 200, 511, 700, 1100, 2050], size=nseq))
        W = int(rng.choice([4, 4, 3, 2, 1]))
        segment = int(rng.choice([0, 0, 0, 64, 128]))
        out.append((i, lengths, Hkv * group, Hkv, d, W, segment))
    return out


@pytest.mark.parametrize("i,lengths,Hq,Hkv,d,W,segment", _packed_cases())
def test_random_packed_batch(oracle, i, lengths, Hq, Hkv, d, W, segment):
    """Blindly drawn packed batches (1 .. 8 sequences of 1 .. 2050 tokens) through the one-launch form of
    lawcat_layer_prefill_varlen: every sequence against the oracle on that sequence alone."""
    import torch

    from paper_2509_18467_amd import lawcat

    n, total = len(lengths), sum(lengths)
    starts = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    wl = Workload(f"packed{i}", 1, total, Hq, Hkv, d, W, "bf16")
    x = make_inputs(wl, seed=2000 + i)
    per = Workload("per_seq", n, 1, Hq, Hkv, d, max(W, 2), "bf16")
    ext = make_inputs(per, seed=3000 + i, halo=True, state=True)
    if W > 1:
        ext["q_halo"], ext["k_halo"] = ext["q_halo"][:, :W - 1], ext["k_halo"][:, :W - 1]
    print("random packed batch", wl, lengths, "segment", segment, flush=True)
    dt = torch.bfloat16
    desc = H.desc_for(Workload("v", n, max(lengths), Hq, Hkv, d, W, "bf16"), feature_map=1, segment=segment)
    Q, K, V, G = (H.dev(x[k][0], dt) for k in ("Q", "K", "V", "G"))
    wq, wk = H.dev(x["wq"], dt), H.dev(x["wk"], dt)
    S0, z0 = H.dev(ext["S0"]), H.dev(ext["z0"])
    qh = H.dev(ext["q_halo"], dt) if W > 1 else None
    kh = H.dev(ext["k_halo"], dt) if W > 1 else None
    O = torch.empty_like(Q)
    den = torch.empty(total, Hq, dtype=torch.float32, device="cuda")
    S = torch.empty(n, Hkv, d, d, dtype=torch.float32, device="cuda")
    z = torch.empty(n, Hkv, d, dtype=torch.float32, device="cuda")
    qt = torch.empty(n, W - 1, Hq, d, dtype=dt, device="cuda") if W > 1 else None
    kt = torch.empty(n, W - 1, Hkv, d, dtype=dt, device="cuda") if W > 1 else None
    ws = torch.empty(max(lawcat.varlen_workspace_bytes(desc, starts, True), 16), dtype=torch.uint8, device="cuda")
    lawcat.layer_prefill_varlen(desc, starts, Q, K, V, G, wq, wk, S0, z0, qh, kh, O, den, S, z, qt, kt, ws,
                                seq_start_dev=torch.tensor(starts, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    o_h, den_h, S_h, z_h = (H.host(t) for t in (O, den, S, z))
    for j in range(n):
        a, b = int(starts[j]), int(starts[j + 1])
        one = Workload(f"packed{i}_seq{j}", 1, b - a, Hq, Hkv, d, W, "bf16")
        ref = oracle.layer_prefill(x["Q"][:, a:b], x["K"][:, a:b], x["V"][:, a:b], x["G"][:, a:b], x["wq"], x["wk"], 1,
                                   1.0, 0.0, ext["S0"][j:j + 1], ext["z0"][j:j + 1],
                                   ext["q_halo"][j:j + 1] if W > 1 else None, ext["k_halo"][j:j + 1] if W > 1 else None)
        tag = f"packed[{i}] sequence {j} (T={b - a})"
        H.assert_close(o_h[None, a:b], ref["o"], one, tag + " o")
        H.assert_close(den_h[None, a:b], ref["den"], one, tag + " den")
        H.assert_close(S_h[j:j + 1], ref["S"], one, tag + " S")
        H.assert_close(z_h[j:j + 1], ref["z"], one, tag + " z")
        if W > 1:
            assert np.array_equal(H.host(qt)[j:j + 1], ref["q_tail"]) and np.array_equal(H.host(kt)[j:j + 1], ref["k_tail"])
