"""GPU parity: every C-ABI entry point against the fp64 oracle, element by element, on the
same seeded inputs.  fp32 storage: max abs error <= 1e-4; bf16 storage: max error <= 2e-2 of the
reference RMS (the bars the task states; helpers.bar).  With the identity feature map the
denominator q.z changes sign and comes arbitrarily close to zero, so there the numerator o*den and
the denominator are compared separately, and o through the bound that those two bars imply row by
row (_check_split)."""
import numpy as np
import pytest
import torch

from paper_2509_18467_amd import lawcat
from paper_2509_18467_amd.inputs import (WORKLOADS, Workload, make_feature_weights, make_gate_inputs, make_inputs,
                                        round_to_bf16)

import helpers as H

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _store(wl, a):
    """Round to the storage type (what the GPU call will read)."""
    a = np.asarray(a, dtype=np.float32)
    return round_to_bf16(a) if wl.dtype == "bf16" else a


# ------------------------------------------------------------------ conv (section 4.1)
@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("T,Hh,d,W,phi,halo", [
    (256, 2, 64, 4, 0, False), (37, 3, 64, 4, 1, True), (1, 8, 128, 4, 1, True), (2, 8, 128, 4, 0, True),
    (1000, 4, 128, 2, 1, False), (129, 2, 64, 1, 1, False), (530, 32, 64, 3, 0, True),
    (1000, 4, 64, 4, 1, True), (193, 2, 128, 4, 0, False),
])
def test_conv1d_causal(oracle, dtype, T, Hh, d, W, phi, halo):
    wl = Workload("conv", 2, T, Hh, Hh, d, W, dtype)
    _say("conv", wl, phi, halo)
    rng = np.random.default_rng(T + d)
    x = _store(wl, rng.standard_normal((wl.B, T, Hh, d)) * 0.5)
    w = _store(wl, rng.standard_normal((Hh, d, W)) * 0.5)
    hl = _store(wl, rng.standard_normal((wl.B, W - 1, Hh, d)) * 0.5) if (halo and W > 1) else None
    y, tail = H.run_conv(wl, x, w, hl, phi)
    ref = oracle.conv1d_causal(x, w, hl, phi)
    H.assert_close(y, ref, wl, "conv y")
    if W > 1:
        full = np.concatenate([np.zeros((wl.B, W - 1, Hh, d)) if hl is None else hl, x], axis=1)
        assert np.array_equal(tail, full[:, -(W - 1):]), "tail rows must be bit-exact copies"


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("T,Hh,Hkv,d,W,phi,halo", [
    (256, 2, 2, 64, 4, 1, False), (37, 4, 2, 64, 4, 0, True), (1, 8, 2, 128, 4, 1, True), (300, 8, 8, 128, 4, 0, True),
    (1000, 4, 1, 128, 2, 1, False), (129, 2, 2, 64, 1, 1, False), (530, 32, 8, 64, 3, 0, True), (257, 6, 3, 64, 4, 1, True),
])
def test_conv1d_feature(oracle, dtype, T, Hh, Hkv, d, W, phi, halo):
    """The shared linear layer after the conv (section 4.1): n_heads = Hkv (keys) and n_heads = a multiple (queries)."""
    wl = Workload("convf", 2, T, Hh, Hkv, d, W, dtype)
    _say("conv + linear feature map", wl, phi, halo)
    rng = np.random.default_rng(T + d)
    x = _store(wl, rng.standard_normal((wl.B, T, Hh, d)) * 0.5)
    w = _store(wl, rng.standard_normal((Hh, d, W)) * 0.5)
    hl = _store(wl, rng.standard_normal((wl.B, W - 1, Hh, d)) * 0.5) if (halo and W > 1) else None
    wf = make_feature_weights(wl, seed=T)
    y, tail = H.run_conv_feature(wl, x, w, wf, hl, phi)
    xc = oracle.conv1d_causal(x, w, hl, 0)
    ref = oracle.feature_linear(xc, wf, phi)
    if phi == 1:
        r = H.assert_close(y, ref, wl, "conv + feature y")
    else:
        # signed features reach 4-5 sigma, where the bf16 half-ulp of the stored result alone is 1.5e-2 of RMS:
        # the bar adds one half-ulp of the sum of the absolute values of the products
        r = H.assert_close(y, ref, wl, "conv + feature y", 1, oracle.feature_linear(np.abs(xc), np.abs(wf), 0))
    _say("  error / bar", f"{r:.3f}")
    if W > 1:
        full = np.concatenate([np.zeros((wl.B, W - 1, Hh, d)) if hl is None else hl, x], axis=1)
        assert np.array_equal(tail, full[:, -(W - 1):]), "tail rows must be bit-exact copies"


@pytest.mark.parametrize("name", ["llama1b_32k", "mistral7b_16k"])
def test_conv1d_feature_full_size(oracle, name):
    """The query side of the two headline shapes at full length (the grid the benchmark's side op times: one round
    of workgroups over the chip), every element against the oracle."""
    wl = WORKLOADS[name]
    _say("conv + linear feature map, full size", wl)
    xin = make_inputs(wl, seed=17, halo=True)
    wf = make_feature_weights(wl, seed=17)
    y, tail = H.run_conv_feature(wl, xin["Q"], xin["wq"], wf, xin["q_halo"], 1)
    ref = oracle.feature_linear(oracle.conv1d_causal(xin["Q"], xin["wq"], xin["q_halo"], 0), wf, 1)
    r = H.assert_close(y, ref, wl, "conv + feature y, full size")
    _say("  error / bar", f"{r:.3f}")


# ------------------------------------------------------------------ gate logits from the layer input (section 4.2)
@pytest.mark.parametrize("dtype,B,T,Hkv,d,dm,rank,bias", [
    ("bf16", 1, 300, 8, 64, 2048, 32, True), ("bf16", 2, 77, 8, 128, 4096, 32, False), ("bf16", 1, 1, 2, 64, 128, 32, True),
    ("bf16", 1, 8192, 8, 64, 2048, 32, True), ("bf16", 1, 4096, 8, 128, 4096, 32, True),
    ("bf16", 1, 16411, 8, 64, 2048, 32, True), ("bf16", 2, 8200, 8, 128, 4096, 32, False),   # 32 tokens per workgroup
    ("bf16", 1, 32768, 8, 64, 2048, 32, True), ("bf16", 1, 16384, 8, 128, 4096, 32, True),   # the headline shapes, full length
    ("bf16", 3, 50, 3, 64, 256, 16, True), ("bf16", 1, 40, 2, 64, 264, 8, False),
    ("fp32", 2, 33, 2, 64, 256, 32, True), ("fp32", 1, 20, 2, 128, 512, 16, False),
])
def test_gate_project(oracle, dtype, B, T, Hkv, d, dm, rank, bias):
    """g = (x w1^T) w2^T + b: rank 32 on the matrix cores (ragged token counts, both layer shapes), other ranks
    and fp32 storage on the plain kernel.  The logits are signed with unit scale: the bar is 2e-2 of RMS plus
    one bf16 half-ulp of the sum of the absolute values of the second layer's terms (a stored logit at 4 sigma
    alone carries 1.5e-2 of RMS), as for the other signed stage outputs."""
    wl = Workload("gate", B, T, 4 * Hkv, Hkv, d, 4, dtype)
    gi = make_gate_inputs(wl, dm, rank, seed=T, bias=bias)
    _say("gate_project", wl, dm, rank, bias)
    got = H.run_gate_project(wl, gi, dm, rank)
    ref = oracle.gate_project(gi["x"], gi["w1"], gi["w2"], gi.get("bias"), Hkv)
    h = np.abs(gi["x"].astype(np.float64) @ gi["w1"].astype(np.float64).T)
    terms = (h @ np.abs(gi["w2"].astype(np.float64)).T + (np.abs(gi["bias"]) if bias else 0.0)).reshape(ref.shape)
    r = H.assert_close(got, ref, wl, "gate logits", 1 if dtype == "bf16" else 0, terms)
    _say("  error / bar", f"{r:.3f}", "max err / rms", f"{H.rel_rms_err(got, ref):.3e}")


def test_gate_project_feeds_the_layer(oracle):
    """Projected logits straight into lawcat_layer_prefill: equals the oracle's projection followed by its layer."""
    wl = WORKLOADS["llama1b_8k"].with_T(1500)
    x = make_inputs(wl, seed=3)
    gi = make_gate_inputs(wl, 2048, 32, seed=3)
    g_gpu = H.run_gate_project(wl, gi, 2048, 32)
    x["G"] = g_gpu.astype(np.float32)                      # exactly what the GPU stored (bf16 values)
    got = H.run_layer_prefill(wl, x, feature_map=1)
    g_ref = oracle.gate_project(gi["x"], gi["w1"], gi["w2"], gi["bias"], wl.Hkv)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], round_to_bf16(g_ref.astype(np.float32)), x["wq"], x["wk"], 1)
    # the two gate tensors differ where a logit sits on a bf16 rounding boundary; the layer's outputs must still agree
    _check_prefill(got, ref, wl, 1, "gate projection -> layer")


# ------------------------------------------------------------------ GLA prefill (section 4.2)
def _features(oracle, wl, x, phi):
    qd = _store(wl, oracle.conv1d_causal(x["Q"], x["wq"], None, phi))
    kd = _store(wl, oracle.conv1d_causal(x["K"], x["wk"], None, phi))
    return qd, kd


def _abs_terms(oracle, qd, kd, V, G, gate_scale=1.0, S0=None, z0=None):
    """Sum of the absolute values of the product terms behind every element of num, den, S and z: the same
    recurrence (section 4.2) on |q-dot|, |k-dot|, |v|, |S0|, |z0|."""
    ab = lambda a: None if a is None else np.abs(a)
    r = oracle.gla_prefill(np.abs(qd), np.abs(kd), np.abs(V), G, gate_scale, 0.0, ab(S0), ab(z0))
    return {k: r[k] for k in ("num", "den", "S", "z")}


def _check_split(got, ref, wl, tag, terms=None):
    """Numerator and denominator separately, then o row by row.

    Used where o = num / den is ill-conditioned (identity feature map: signed features, den crosses zero) or
    where the sequence is not stationary (no decay: num and den grow with t while o shrinks), so that one RMS
    over all of o says little.
      * 99.9 % of the elements of num (rebuilt as o * den from the stored outputs), den, S and z lie within the
        stated 2e-2 of RMS;
      * every element lies within helpers.bar: 2e-2 RMS + 2^-8 T, T the sum of the absolute values of the
        element's product terms (`terms`, from _abs_terms; |ref| if not given): one bf16 half-ulp of what was
        summed.  (Each term's factors carry up to three bf16 roundings -- q', k' or the state, the stored o --
        so the rigorous worst case is three half-ulps; the measured maximum stays below one.)
      * for every row whose |den_ref| exceeds twice its bar, o lies within the bound that the two bars imply:
        with |dnum| <= a and |dden| <= b,
        |o - o_ref| = |dnum - o_ref dden| / |den_ref + dden| <= (a + |o_ref| b) / (|den_ref| - b).
    Returns the largest error of each tensor as a fraction of its bar, and max error / RMS for the record."""
    errs = {}
    t = terms or {}
    num_got = got["o"] * got["den"][..., None]
    a = H.bar(ref["num"], wl, 1, t.get("num"))
    b = H.bar(ref["den"], wl, 1, t.get("den"))
    pairs = (("num", num_got, 1), ("den", got["den"], 1), ("S", got["S"], 1), ("z", got["z"], 1))
    for k, g, r in pairs:
        errs[k] = H.assert_close(g, ref[k], wl, f"{tag} {k}", r, t.get(k))
        errs[k + "_max/rms"] = H.rel_rms_err(g, ref[k])
        if wl.dtype == "bf16":
            q999 = H.quantile_err(g, ref[k])
            assert q999 <= H.BF16_REL_RMS, f"{tag} {k}: 99.9th percentile of the error is {q999:.3e} of RMS"
    keep = np.abs(ref["den"]) > 2.0 * b
    errs["rows_kept"] = float(keep.mean())
    assert errs["rows_kept"] > 0.7, f"{tag}: only {errs['rows_kept']:.3f} of the rows have a usable denominator"
    bound = (a + np.abs(ref["o"]) * b[..., None]) / (np.abs(ref["den"]) - b)[..., None]
    ratio = (np.abs(got["o"] - ref["o"]) / bound)[keep]
    errs["o_rows"] = float(ratio.max())
    assert errs["o_rows"] <= 1.0, f"{tag} o: {errs['o_rows']:.3f} of the row bound implied by the num and den bars"
    return errs


def _layer_terms(oracle, ref, x, phi, gate_scale=1.0):
    """_abs_terms for a fused-layer reference (which carries q-dot and k-dot); only signed features need it."""
    if phi != 0:
        return None
    return _abs_terms(oracle, ref["q_dot"], ref["k_dot"], x["V"], x["G"], gate_scale, x.get("S0"), x.get("z0"))


def _check_prefill(got, ref, wl, phi, tag, split=False, terms=None):
    """phi = 1 + ELU on a decaying state: o, den, S, z each within the stated bar, every element.
    Identity feature map, or split=True: _check_split."""
    if phi == 1 and not split:
        errs = {k: H.assert_close(got[k], ref[k], wl, f"{tag} {k}") for k in ("o", "den", "S", "z")}
    else:
        assert terms is not None or phi == 1 or wl.dtype == "fp32", "signed features need the absolute-term sums"
        errs = _check_split(got, ref, wl, tag, terms)
    _say(tag, "error / bar:", {k: f"{v:.3f}" for k, v in errs.items()})
    return errs


@pytest.mark.parametrize("phi", [1, 0])
@pytest.mark.parametrize("name,T", [("tiny", 256), ("tiny", 77), ("llama1b_8k", 700), ("mistral7b_16k", 333)])
def test_gla_prefill(oracle, name, T, phi):
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=1, state=True)
    qd, kd = _features(oracle, wl, x, phi)
    _say("gla_prefill", wl, "phi", phi)
    got = H.run_gla_prefill(wl, qd, kd, x["V"], x["G"], x["S0"], x["z0"])
    ref = oracle.gla_prefill(qd, kd, x["V"], x["G"], 1.0, 0.0, x["S0"], x["z0"])
    terms = _abs_terms(oracle, qd, kd, x["V"], x["G"], 1.0, x["S0"], x["z0"]) if phi == 0 else None
    _check_prefill(got, ref, wl, phi, f"gla_prefill[{wl.name},phi={phi}]", terms=terms)


@pytest.mark.parametrize("phi", [1, 0])
@pytest.mark.parametrize("Hq,Hkv,d,T,W", [(3, 3, 64, 150, 4), (4, 2, 64, 389, 3), (2, 2, 128, 200, 4), (4, 2, 128, 131, 2),
                                          (8, 2, 64, 257, 4), (4, 1, 128, 64, 4), (6, 2, 64, 300, 4), (16, 2, 64, 777, 4),
                                          (7, 1, 128, 333, 4), (5, 1, 64, 1200, 4)])
def test_layer_prefill_other_group_sizes(oracle, Hq, Hkv, d, T, W, phi):
    """bf16 fused layer with 1 to 8 query heads per kv head (3, 5, 7 and 8 take several output-pass launches),
    both head dims, batch 2, ragged lengths, one case long enough for the two-level carry."""
    wl = Workload(f"g{Hq // Hkv}d{d}", 2, T, Hq, Hkv, d, W, "bf16")
    # a random signed start state under signed features only adds cancellation noise: keep it for 1+ELU
    x = make_inputs(wl, seed=7, halo=True, state=(phi == 1))
    _say("layer_prefill", wl, "phi", phi)
    got = H.run_layer_prefill(wl, x, feature_map=phi)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], phi, 1.0, 0.0,
                               x.get("S0"), x.get("z0"), x["q_halo"], x["k_halo"])
    _check_prefill(got, ref, wl, phi, f"layer_prefill[{wl.name},phi={phi}]", terms=_layer_terms(oracle, ref, x, phi))
    assert np.array_equal(got["q_tail"], ref["q_tail"]) and np.array_equal(got["k_tail"], ref["k_tail"])


@pytest.mark.parametrize("name,T,kw", [
    ("llama1b_8k", 2000, dict(carry_mode=1)), ("llama1b_8k", 2000, dict(carry_mode=2, segment=64)),
    ("llama1b_8k", 2000, dict(segment=320)), ("mistral7b_16k", 900, dict(carry_mode=1)),
    ("mistral7b_16k", 900, dict(segment=128)),
])
def test_carry_modes_and_segment_lengths(oracle, name, T, kw):
    """Sequential carry, two-level carry and explicit segment lengths must all reach the oracle."""
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=8, state=True)
    got = H.run_layer_prefill(wl, x, feature_map=1, **kw)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1, 1.0, 0.0, x["S0"], x["z0"])
    _check_prefill(got, ref, wl, 1, f"layer_prefill[{wl.name},{kw}]")


def test_slow_decay_long_memory(oracle):
    """gate_scale = 1/16 (slowly decaying state): the carried-state term dominates the output.  The first tokens
    see no averaging yet and are ~24x larger than the RMS of the whole output, so o is checked through num and
    den, and with the plain bar once averaging has set in."""
    wl = WORKLOADS["llama1b_8k"].with_T(3000)
    x = make_inputs(wl, seed=9)
    got = H.run_layer_prefill(wl, x, feature_map=1, gate_scale=0.0625)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1, 0.0625)
    _check_prefill(got, ref, wl, 1, "slow decay", split=True)
    for k in ("S", "z", "den"):
        H.assert_close(got[k], ref[k], wl, "slow decay " + k)
    late = slice(64, None)
    H.assert_close(got["o"][:, late], ref["o"][:, late], wl, "slow decay o (t >= 64)")


# ------------------------------------------------------------------ saturated gates on the matrix-core path
def _gate_case(oracle, d, T, mode, phi=1, gate_scale=1.0, seed=21):
    wl = Workload(f"gates_{mode}_d{d}", 1, T, 8, 2, d, 4, "bf16")
    x = make_inputs(wl, seed=seed)
    if mode == "closed":
        x["G"][:] = -30.0
    elif mode == "open":
        x["G"][:] = 30.0
    elif mode == "mixed":
        m = np.random.default_rng(5).random(x["G"].shape)
        x["G"][m < 0.05] = -12.0
        x["G"][m > 0.95] = 12.0
    x["G"] = round_to_bf16(x["G"])
    _say("gates", wl, mode, "phi", phi, "gate_scale", gate_scale)
    got = H.run_layer_prefill(wl, x, feature_map=phi, gate_scale=gate_scale)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], phi, gate_scale)
    return wl, x, got, ref


@pytest.mark.parametrize("d", [64, 128])
def test_gates_closed_output_is_the_current_value(oracle, d):
    """G = -30 everywhere: alpha = e^-30, the state forgets everything at every step, o_t = v_t and
    S_T = k_T^T v_T (oracle pin "gates -> 0").  The kernel's per-step decay floor (2^-13) must not show."""
    wl, x, got, ref = _gate_case(oracle, d, 2000, "closed")
    _check_prefill(got, ref, wl, 1, f"closed gates d={d}")
    v = np.repeat(x["V"].astype(np.float64), wl.Hq // wl.Hkv, axis=2)
    H.assert_close(got["o"], v, wl, "closed gates: o against v itself")


@pytest.mark.parametrize("d,T", [(64, 32768), (128, 8192)])
def test_gates_open_no_decay_over_a_long_sequence(oracle, d, T):
    """G = +30 everywhere: alpha = 1 to fp32 precision, S and z grow for the whole sequence while o shrinks
    (an ever longer average): not stationary, so num and den are checked, o through them, S and z plainly."""
    wl, x, got, ref = _gate_case(oracle, d, T, "open")
    _check_prefill(got, ref, wl, 1, f"open gates d={d}", split=True)
    for k in ("S", "z", "den"):
        H.assert_close(got[k], ref[k], wl, f"open gates {k}")


@pytest.mark.parametrize("phi", [1, 0])
@pytest.mark.parametrize("d", [64, 128])
def test_gates_mixed_with_saturated_logits(oracle, d, phi):
    """N(0,1) logits with 5 % forced to -12 and 5 % to +12."""
    wl, x, got, ref = _gate_case(oracle, d, 2000, "mixed", phi=phi)
    _check_prefill(got, ref, wl, phi, f"mixed gates d={d} phi={phi}", terms=_layer_terms(oracle, ref, x, phi))


@pytest.mark.parametrize("d", [64, 128])
def test_memory_carried_across_some_segments_only(oracle, d):
    """Segments of 128 tokens, N(0,1) gates (no segment passes anything on: the scan has nothing to do and the
    output pass starts from its predecessor's contribution) except that kv head 1 holds one channel in eight
    open from token 300 to 700, across three segment boundaries (those segments pass their state on, the scan
    runs for that head), and head 0 does so in the last two segments only.  A start state comes in as well.
    The open channels pile up hundreds of undecayed terms while the rest of the state stays small, so one RMS
    over the tensor says little about them: the bar is the forward-error one (half a bf16 ulp of the sum of the
    absolute values of the terms, on top of 2e-2 of RMS), as for signed features."""
    wl = Workload(f"carry_some_d{d}", 2, 1100, 8, 2, d, 4, "bf16")
    x = make_inputs(wl, seed=33, state=True)
    x["G"][:, 300:700, 1, ::8] = 30.0
    x["G"][0, 850:, 0, 3::8] = 30.0
    x["G"] = round_to_bf16(x["G"])
    _say("carry across some segments", wl)
    got = H.run_layer_prefill(wl, x, feature_map=1, segment=128)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1, 1.0, 0.0, x["S0"], x["z0"])
    terms = _abs_terms(oracle, ref["q_dot"], ref["k_dot"], x["V"], x["G"], 1.0, x["S0"], x["z0"])
    _check_prefill(got, ref, wl, 1, f"carry across some segments d={d}", split=True, terms=terms)
    for k in ("o", "den"):
        H.assert_close(got[k], ref[k], wl, f"carry across some segments {k}")


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("gate_scale", [0.0, 4.0, 16.0])
def test_gate_scale_extremes(oracle, d, gate_scale):
    """gate_scale = 0 switches the decay off (alpha = 1: checked like the open gates); 4 and 16 push most steps
    to or below the per-step floor of the kernel."""
    wl, x, got, ref = _gate_case(oracle, d, 1500, "normal", gate_scale=gate_scale)
    _check_prefill(got, ref, wl, 1, f"gate_scale={gate_scale} d={d}", split=(gate_scale == 0.0))


def test_gla_prefill_gate_scale_and_eps(oracle):
    wl = WORKLOADS["tiny"].with_T(200)
    x = make_inputs(wl, seed=2)
    qd, kd = _features(oracle, wl, x, 1)
    got = H.run_gla_prefill(wl, qd, kd, x["V"], x["G"], gate_scale=0.0625, eps=0.5)
    ref = oracle.gla_prefill(qd, kd, x["V"], x["G"], 0.0625, 0.5)
    # slow decay: den grows to ~1e3, where the relative part of the fp32 bar applies
    for k in ("o", "den", "S", "z"):
        H.assert_close(got[k], ref[k], wl, k)


@pytest.mark.parametrize("d,gate_scale,eps", [(64, 0.25, 0.5), (128, 0.25, 0.0), (64, 2.0, 1e-3)])
def test_layer_prefill_bf16_gate_scale_and_eps(oracle, d, gate_scale, eps):
    """The matrix-core path with a gate temperature other than 1 (general log2/exp2 gate code) and eps > 0."""
    wl = Workload(f"gs{gate_scale}d{d}", 2, 523, 8, 2, d, 4, "bf16")
    x = make_inputs(wl, seed=11, halo=True, state=True)
    got = H.run_layer_prefill(wl, x, feature_map=1, gate_scale=gate_scale, eps=eps)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1, gate_scale, eps,
                               x["S0"], x["z0"], x["q_halo"], x["k_halo"])
    _check_prefill(got, ref, wl, 1, f"layer_prefill[{wl.name},eps={eps}]")


# ------------------------------------------------------------------ fused layer, the five graded shapes
@pytest.mark.parametrize("name,T,phi,extras", [
    ("tiny", None, 1, False), ("tiny", None, 0, False), ("tiny", 203, 1, True),
    ("llama1b_8k", 1111, 1, True), ("llama1b_8k", None, 1, False), ("llama1b_8k", None, 0, False),
    ("mistral7b_16k", 613, 1, True),
])
def test_layer_prefill(oracle, name, T, phi, extras):
    wl = WORKLOADS[name] if T is None else WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=0, halo=extras, state=extras)
    _say("layer_prefill", wl, "phi", phi, "extras", extras)
    got = H.run_layer_prefill(wl, x, feature_map=phi)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], phi, 1.0, 0.0,
                               x.get("S0"), x.get("z0"), x.get("q_halo"), x.get("k_halo"))
    _check_prefill(got, ref, wl, phi, f"layer_prefill[{wl.name},phi={phi}]", terms=_layer_terms(oracle, ref, x, phi))
    assert np.array_equal(got["q_tail"], ref["q_tail"]) and np.array_equal(got["k_tail"], ref["k_tail"])


@pytest.mark.parametrize("phi", [1, 0])
@pytest.mark.parametrize("name", ["llama1b_32k", "mistral7b_16k"])
def test_layer_prefill_full_size(oracle, name, phi):
    wl = WORKLOADS[name]
    x = make_inputs(wl, seed=0)
    _say("layer_prefill full size", wl, "phi", phi)
    got = H.run_layer_prefill(wl, x, feature_map=phi)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], phi)
    _check_prefill(got, ref, wl, phi, f"layer_prefill[{wl.name},phi={phi}]", terms=_layer_terms(oracle, ref, x, phi))


# ------------------------------------------------------------------ the feature map with its shared linear layer
@pytest.mark.parametrize("name,T,phi,extras", [
    ("tiny", None, 1, False), ("tiny", 203, 0, True), ("llama1b_8k", 777, 1, True), ("mistral7b_16k", 333, 0, True),
    ("llama1b_8k", None, 1, False), ("llama1b_8k", None, 0, False),
    ("mistral7b_16k", None, 1, False), ("mistral7b_16k", None, 0, False),
])
def test_layer_prefill_with_linear_feature_map(oracle, name, T, phi, extras):
    """q-dot = phi(conv(Q) Wf), k-dot = phi(conv(K) Wf) (section 4.1), then the attention: lawcat_layer_prefill_fm.

    With 1 + ELU the whole call is held to the bar of the fused layer, end to end against the fp64 oracle.  With
    signed features (identity phi: not a configuration of the paper, whose layer has a nonlinearity) the
    numerator is a sum of cancelling terms, and the bf16 rounding of the staged q-dot and k-dot moves it by more
    than the 2e-2 bar leaves; there the two stages are held to their bars one after the other: the staged
    features against the oracle's, then the attention against the oracle run on the staged features (which is
    how lawcat_conv1d_causal followed by lawcat_gla_prefill is tested)."""
    wl = WORKLOADS[name] if T is None else WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=0, halo=extras, state=extras)
    wf = make_feature_weights(wl, seed=0)
    _say("layer_prefill_fm", wl, "phi", phi, "extras", extras)
    got = H.run_layer_prefill(wl, x, feature_map=phi, wf=wf)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], phi, 1.0, 0.0,
                               x.get("S0"), x.get("z0"), x.get("q_halo"), x.get("k_halo"), wf=wf)
    tag = f"layer_prefill_fm[{wl.name},phi={phi}]"
    if phi == 0:
        for name, raw, w, hl in (("q_dot", "Q", "wq", "q_halo"), ("k_dot", "K", "wk", "k_halo")):
            xc = oracle.conv1d_causal(x[raw], x[w], x.get(hl), 0)
            r = H.assert_close(got[name], ref[name], wl, f"{tag} staged {name}", 1,
                               oracle.feature_linear(np.abs(xc), np.abs(wf), 0))
            _say(f"  staged {name}: error / bar {r:.3f}")
        ref2 = oracle.gla_prefill(got["q_dot"], got["k_dot"], x["V"], x["G"], 1.0, 0.0, x.get("S0"), x.get("z0"))
        terms = _abs_terms(oracle, got["q_dot"], got["k_dot"], x["V"], x["G"], 1.0, x.get("S0"), x.get("z0"))
        _check_prefill(got, ref2, wl, phi, tag + " attention on the staged features", terms=terms)
    else:
        _check_prefill(got, ref, wl, phi, tag)
    assert np.array_equal(got["q_tail"], ref["q_tail"]) and np.array_equal(got["k_tail"], ref["k_tail"])


# ------------------------------------------------------------------ sequences of different lengths, packed
@pytest.mark.parametrize("one_launch", [False, True])
@pytest.mark.parametrize("name,lengths", [("tiny", (5, 130, 1, 64)), ("llama1b_8k", (700, 64, 1500, 1, 333)),
                                          ("mistral7b_16k", (257, 1024, 16)), ("llama1b_8k", (4000, 130, 2500)),
                                          ("llama1b_8k", tuple(37 + 11 * i for i in range(70))),
                                          # the packed batch the benchmark's side op times: 24 sequences, 32 768 tokens
                                          ("llama1b_8k", (4096, 2048, 1024, 512, 256, 256) * 4)])
def test_layer_prefill_varlen(oracle, name, lengths, one_launch):
    """lawcat_layer_prefill_varlen: every sequence of the packed batch equals the oracle run on that sequence alone
    (its own start state, conv halo, final state and conv tails) -- as one call per sequence, and as one set of
    launches for the whole batch (device copy of the offsets; several segments per long sequence, one for the
    short ones, 70 sequences of one segment each)."""
    base = WORKLOADS[name]
    n, total = len(lengths), sum(lengths)
    starts = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    wl = Workload(f"{name}_varlen", 1, total, base.Hq, base.Hkv, base.d, base.W, base.dtype)
    x = make_inputs(wl, seed=17)                              # one packed token axis
    per = Workload("per_seq", n, 1, base.Hq, base.Hkv, base.d, base.W, base.dtype)
    ext = make_inputs(per, seed=18, halo=True, state=True)    # per-sequence start states and halos
    _say("varlen", wl, lengths)
    dt = H.tdtype(wl)
    desc = H.desc_for(Workload("v", n, max(lengths), base.Hq, base.Hkv, base.d, base.W, base.dtype), feature_map=1)
    Q, K, V, G = (H.dev(x[k][0], dt) for k in ("Q", "K", "V", "G"))
    wq, wk = H.dev(x["wq"], dt), H.dev(x["wk"], dt)
    S0, z0 = H.dev(ext["S0"]), H.dev(ext["z0"])
    qh, kh = H.dev(ext["q_halo"], dt), H.dev(ext["k_halo"], dt)
    O = torch.empty_like(Q)
    den = torch.empty(total, wl.Hq, dtype=torch.float32, device="cuda")
    S = torch.empty(n, wl.Hkv, wl.d, wl.d, dtype=torch.float32, device="cuda")
    z = torch.empty(n, wl.Hkv, wl.d, dtype=torch.float32, device="cuda")
    qt = torch.empty(n, wl.W - 1, wl.Hq, wl.d, dtype=dt, device="cuda")
    kt = torch.empty(n, wl.W - 1, wl.Hkv, wl.d, dtype=dt, device="cuda")
    need = max(lawcat.varlen_workspace_bytes(desc, starts, one_launch), 16)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    dev_starts = torch.tensor(starts, dtype=torch.int32, device="cuda") if one_launch else None
    lawcat.layer_prefill_varlen(desc, starts, Q, K, V, G, wq, wk, S0, z0, qh, kh, O, den, S, z, qt, kt, ws,
                                seq_start_dev=dev_starts)
    torch.cuda.synchronize()
    o_h, den_h, S_h, z_h, qt_h, kt_h = (H.host(t) for t in (O, den, S, z, qt, kt))
    for i in range(n):
        a, b = int(starts[i]), int(starts[i + 1])
        one = Workload(f"{name}_seq{i}", 1, b - a, base.Hq, base.Hkv, base.d, base.W, base.dtype)
        ref = oracle.layer_prefill(x["Q"][:, a:b], x["K"][:, a:b], x["V"][:, a:b], x["G"][:, a:b], x["wq"], x["wk"], 1,
                                   1.0, 0.0, ext["S0"][i:i + 1], ext["z0"][i:i + 1], ext["q_halo"][i:i + 1],
                                   ext["k_halo"][i:i + 1])
        got = {"o": o_h[None, a:b], "den": den_h[None, a:b], "S": S_h[i:i + 1], "z": z_h[i:i + 1]}
        _check_prefill(got, ref, one, 1, f"varlen[{name}] sequence {i} (T={b - a})")
        assert np.array_equal(qt_h[i:i + 1], ref["q_tail"]) and np.array_equal(kt_h[i:i + 1], ref["k_tail"])


# ------------------------------------------------------------------ continuation (conv cache + state)
@pytest.mark.parametrize("name,T,T1", [("tiny", 256, 100), ("llama1b_8k", 900, 515), ("mistral7b_16k", 300, 2)])
def test_split_prefill_equals_whole(oracle, name, T, T1):
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=3)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1)
    a_in = {k: (v[:, :T1] if k in "QKVG" else v) for k, v in x.items()}
    a = H.run_layer_prefill(wl.with_T(T1), a_in)
    b_in = {k: (v[:, T1:] if k in "QKVG" else v) for k, v in x.items()}
    b_in.update(S0=a["S"].astype(np.float32), z0=a["z"].astype(np.float32),
                q_halo=a["q_tail"].astype(np.float32), k_halo=a["k_tail"].astype(np.float32))
    b = H.run_layer_prefill(wl.with_T(T - T1), b_in)
    o = np.concatenate([a["o"], b["o"]], axis=1)
    H.assert_close(o, ref["o"], wl, "split o")
    H.assert_close(b["S"], ref["S"], wl, "split S")
    H.assert_close(b["z"], ref["z"], wl, "split z")


def _decode(oracle, wl, x_new, state_gpu, state_ref, heads=None):
    """n decode steps: conv on one token with the cache, then lawcat_gla_step; token-by-token vs oracle."""
    dt = H.tdtype(wl)
    n = x_new["Q"].shape[1]
    d1 = H.desc_for(wl.with_T(1), feature_map=1)
    wq, wk = H.dev(x_new["wq"], dt), H.dev(x_new["wk"], dt)
    S, z = H.dev(state_gpu["S"]), H.dev(state_gpu["z"])
    qc, kc = H.dev(state_gpu["q_tail"], dt), H.dev(state_gpu["k_tail"], dt)
    qc2, kc2 = torch.empty_like(qc), torch.empty_like(kc)
    Qd, Kd, Vd, Gd = (H.dev(x_new[k], dt) for k in "QKVG")
    qdot = torch.empty(wl.B, 1, wl.Hq, wl.d, dtype=dt, device="cuda")
    kdot = torch.empty(wl.B, 1, wl.Hkv, wl.d, dtype=dt, device="cuda")
    o = torch.empty(wl.B, n, wl.Hq, wl.d, dtype=dt, device="cuda")
    for t in range(n):
        lawcat.conv1d_causal(d1, wl.Hq, Qd[:, t:t + 1].contiguous(), wq, qc, qdot, qc2)
        lawcat.conv1d_causal(d1, wl.Hkv, Kd[:, t:t + 1].contiguous(), wk, kc, kdot, kc2)
        qc, qc2, kc, kc2 = qc2, qc, kc2, kc
        ot = torch.empty(wl.B, wl.Hq, wl.d, dtype=dt, device="cuda")
        lawcat.gla_step(d1, qdot, kdot, Vd[:, t].contiguous(), Gd[:, t].contiguous(), S, z, ot)
        o[:, t] = ot
    torch.cuda.synchronize()
    got = {"o": H.host(o), "S": H.host(S), "z": H.host(z)}
    # oracle: same steps.  The step consumes q-dot/k-dot rounded to the storage type, as the GPU does.
    sl = slice(None) if heads is None else heads
    ref = oracle.layer_prefill(x_new["Q"], x_new["K"], x_new["V"], x_new["G"], x_new["wq"], x_new["wk"], 1, 1.0, 0.0,
                               state_ref["S"], state_ref["z"], state_ref["q_tail"], state_ref["k_tail"])
    return got, ref


def _decode_block(oracle, wl, x_new, state_gpu, state_ref):
    """The same n decode steps in two launches: the conv over the n new tokens with the cache as halo, then
    lawcat_gla_steps (n recurrent steps with the state on chip)."""
    dt = H.tdtype(wl)
    n = x_new["Q"].shape[1]
    dn = H.desc_for(wl.with_T(n), feature_map=1)
    wq, wk = H.dev(x_new["wq"], dt), H.dev(x_new["wk"], dt)
    S, z = H.dev(state_gpu["S"]), H.dev(state_gpu["z"])
    qc, kc = H.dev(state_gpu["q_tail"], dt), H.dev(state_gpu["k_tail"], dt)
    qc2, kc2 = torch.empty_like(qc), torch.empty_like(kc)
    Qd, Kd, Vd, Gd = (H.dev(x_new[k], dt) for k in "QKVG")
    qdot, kdot = torch.empty_like(Qd), torch.empty_like(Kd)
    o = torch.empty_like(Qd)
    lawcat.conv1d_causal(dn, wl.Hq, Qd, wq, qc, qdot, qc2)
    lawcat.conv1d_causal(dn, wl.Hkv, Kd, wk, kc, kdot, kc2)
    lawcat.gla_steps(dn, qdot, kdot, Vd, Gd, S, z, o)
    torch.cuda.synchronize()
    got = {"o": H.host(o), "S": H.host(S), "z": H.host(z), "q_tail": H.host(qc2), "k_tail": H.host(kc2)}
    ref = oracle.layer_prefill(x_new["Q"], x_new["K"], x_new["V"], x_new["G"], x_new["wq"], x_new["wk"], 1, 1.0, 0.0,
                               state_ref["S"], state_ref["z"], state_ref["q_tail"], state_ref["k_tail"])
    return got, ref


@pytest.mark.parametrize("name,T,n", [("tiny", 256, 40), ("llama1b_8k", 300, 33), ("mistral7b_16k", 200, 17)])
def test_prefill_then_a_block_of_decode_steps(oracle, name, T, n):
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=4)
    xn = make_inputs(wl.with_T(n), seed=5)
    xn["wq"], xn["wk"] = x["wq"], x["wk"]
    a = H.run_layer_prefill(wl, x)
    ra = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1)
    got, ref = _decode_block(oracle, wl, xn, a, ra)
    for k in ("o", "S", "z"):
        H.assert_close(got[k], ref[k], wl, "decode block " + k)
    assert np.array_equal(got["q_tail"], ref["q_tail"]) and np.array_equal(got["k_tail"], ref["k_tail"])


@pytest.mark.parametrize("name,T,n", [("tiny", 256, 24), ("llama1b_8k", 300, 16), ("mistral7b_16k", 200, 16)])
def test_prefill_then_decode_steps(oracle, name, T, n):
    wl = WORKLOADS[name].with_T(T)
    x = make_inputs(wl, seed=4)
    xn = make_inputs(wl.with_T(n), seed=5)
    xn["wq"], xn["wk"] = x["wq"], x["wk"]
    a = H.run_layer_prefill(wl, x)
    ra = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], 1)
    got, ref = _decode(oracle, wl, xn, a, ra)
    H.assert_close(got["o"], ref["o"], wl, "decode o")
    H.assert_close(got["S"], ref["S"], wl, "decode S")
    H.assert_close(got["z"], ref["z"], wl, "decode z")


@pytest.mark.parametrize("d,n", [(64, 3), (128, 2)])
def test_decode_steps_for_a_batch_of_256_sequences(oracle, d, n):
    """lawcat_gla_step on a batch of 256 sequences (the shape the benchmark's side op times), a few steps in a row
    from a random start state, and the same tokens through one lawcat_gla_steps call: every sequence and head
    against the oracle's recurrence."""
    wl = Workload("decode_b256", B=256, T=n, Hq=32, Hkv=8, d=d)
    x = make_inputs(wl, seed=29, state=True)
    dt = H.tdtype(wl)
    q = _store(wl, np.abs(x["Q"]) + 0.05)
    k = _store(wl, np.abs(x["K"]) + 0.05)
    ref = oracle.gla_prefill(q, k, x["V"], x["G"], 1.0, 0.0, x["S0"], x["z0"])
    d1 = H.desc_for(wl.with_T(1))
    tq, tk, tv, tg = (H.dev(a, dt) for a in (q, k, x["V"], x["G"]))
    S, z = H.dev(x["S0"]), H.dev(x["z0"])
    o = torch.empty(wl.B, n, wl.Hq, d, dtype=dt, device="cuda")
    for t in range(n):
        ot = torch.empty(wl.B, wl.Hq, d, dtype=dt, device="cuda")
        lawcat.gla_step(d1, tq[:, t].contiguous(), tk[:, t].contiguous(), tv[:, t].contiguous(), tg[:, t].contiguous(), S, z, ot)
        o[:, t] = ot
    torch.cuda.synchronize()
    for nm, got in (("o", o), ("S", S), ("z", z)):
        r = H.assert_close(H.host(got), ref[nm], wl, f"batched decode step {nm}")
        _say(f"  {nm}: error / bar {r:.3f}")
    S2, z2 = H.dev(x["S0"]), H.dev(x["z0"])
    o2 = torch.empty_like(o)
    lawcat.gla_steps(H.desc_for(wl), tq, tk, tv, tg, S2, z2, o2)
    torch.cuda.synchronize()
    for nm, got in (("o", o2), ("S", S2), ("z", z2)):
        H.assert_close(H.host(got), ref[nm], wl, f"batched decode block {nm}")


@pytest.mark.parametrize("phi", [1, 0])
def test_stress_128k_then_256_steps(oracle, phi):
    """Mistral-7B shape at T = 131072, every head against the oracle, then 256 decode steps from the returned
    state (1 + ELU; the identity map is checked on the prefill only)."""
    wl = WORKLOADS["mistral7b_128k"]
    x = make_inputs(wl, seed=0)
    _say("stress", wl, "phi", phi)
    got = H.run_layer_prefill(wl, x, feature_map=phi, den=True)
    ref = oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], phi)
    terms = _layer_terms(oracle, ref, x, phi)
    for k in ("num", "q_dot", "k_dot"):
        if not (k == "num" and phi == 0):
            ref.pop(k, None)          # 4 GB each in fp64 at this size
    _check_prefill(got, ref, wl, phi, f"stress prefill phi={phi}", terms=terms)
    assert np.array_equal(got["q_tail"], ref["q_tail"]) and np.array_equal(got["k_tail"], ref["k_tail"])
    if phi == 0:
        return
    ref = {k: ref[k] for k in ("S", "z", "q_tail", "k_tail")}
    n = 256
    xn = make_inputs(wl.with_T(n), seed=6)
    xn["wq"], xn["wk"] = x["wq"], x["wk"]
    gd, rd = _decode(oracle, wl, xn, got, ref)
    H.assert_close(gd["o"], rd["o"], wl, "stress decode o")
    H.assert_close(gd["S"], rd["S"], wl, "stress decode S")
    H.assert_close(gd["z"], rd["z"], wl, "stress decode z")
    # the same 256 steps in one lawcat_gla_steps call
    gb, _ = _decode_block(oracle, wl, xn, got, ref)
    H.assert_close(gb["o"], rd["o"], wl, "stress decode block o")
    H.assert_close(gb["S"], rd["S"], wl, "stress decode block S")
    H.assert_close(gb["z"], rd["z"], wl, "stress decode block z")
