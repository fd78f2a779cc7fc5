#!/usr/bin/env python3
"""Benchmark of the LAWCAT prefill hot path on one MI355X.

A step is one lawcat_layer_prefill call (conv + phi on Q and K, gate -> decay, normalized
gated linear attention, final state and conv tails) over one seeded synthetic layer input
that is already resident in HBM.  Prints ONE JSON line: prefill tokens/s per layer, the
HBM roofline of the dominant kernel (the output pass) timed with HIP events, and the fp64 CPU
oracle timed on the host cores as a baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--quick]

A default run also reports, in the same line, the other graded shapes (T = 8K .. 128K), the identity feature
map and a slowly decaying state at the headline shape ("sweep"), and the stand-alone conv and decode-step calls
("side_ops").
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def algorithmic_bytes_per_token(wl) -> int:
    """Every tensor touched once, bf16: Q and O [Hq*d] each, K, V, gate logits [Hkv*d] each."""
    esz = 2 if wl.dtype == "bf16" else 4
    return esz * (2 * wl.Hq * wl.d + 3 * wl.Hkv * wl.d)


class HipEvents:
    """Raw hipEvent_t pairs (ctypes on libamdhip64) for lawcat_layer_prefill_timed."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.pairs = []
        for _ in range(n):
            a, b = ctypes.c_void_p(), ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(a)) == 0
            assert self.hip.hipEventCreate(ctypes.byref(b)) == 0
            self.pairs.append((a, b))

    def elapsed_ms(self, i):
        ms = ctypes.c_float()
        a, b = self.pairs[i]
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        assert rc == 0, f"hipEventElapsedTime rc={rc}"
        return ms.value

    def destroy(self):
        for a, b in self.pairs:
            self.hip.hipEventDestroy(a)
            self.hip.hipEventDestroy(b)


def device_inputs(wl, seed, dt):
    """The synthetic layer input drawn on the GPU (same shapes and distributions as inputs.make_inputs, torch's
    seeded generator): used where no host copy is needed, i.e. for every timing except the headline's, whose
    first input set is also what the CPU oracle is timed on."""
    import torch

    g = torch.Generator(device="cuda")
    g.manual_seed(1000 + seed)

    def normal(shape, scale):
        return (torch.randn(shape, generator=g, device="cuda", dtype=torch.float32) * scale).to(dt)

    B, T, Hq, Hkv, d, W = wl.B, wl.T, wl.Hq, wl.Hkv, wl.d, wl.W
    return {"Q": normal((B, T, Hq, d), 0.125), "K": normal((B, T, Hkv, d), 0.125), "V": normal((B, T, Hkv, d), 0.125),
            "G": normal((B, T, Hkv, d), 1.0), "wq": normal((Hq, d, W), W ** -0.5), "wk": normal((Hkv, d, W), W ** -0.5)}


def run_workload(wl, steps, warmup, feature_map=1, trace=True, seed=0, segment=0, carry=0, gate_scale=1.0,
                 host_inputs=True):
    import torch

    from paper_2509_18467_amd import lawcat
    from paper_2509_18467_amd.inputs import make_inputs

    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    desc = lawcat.make_desc(wl.B, wl.T, wl.Hq, wl.Hkv, wl.d, conv_width=wl.W,
                            dtype=lawcat.DTYPE_BF16 if wl.dtype == "bf16" else lawcat.DTYPE_F32,
                            feature_map=feature_map, segment=segment, carry_mode=carry, gate_scale=gate_scale)
    bytes_step = algorithmic_bytes_per_token(wl) * wl.B * wl.T
    # rotate input/output sets so the 256 MB Infinity Cache cannot serve a step's reads
    nsets = max(2, min(12, -(-(1 << 30) // bytes_step)))
    sets, host0 = [], None
    for s in range(nsets):
        if host_inputs and s == 0:
            host0 = make_inputs(wl, seed=seed)
            d = {k: torch.from_numpy(v).to("cuda").to(dt).contiguous() for k, v in host0.items()}
        else:
            d = device_inputs(wl, seed + s, dt)
        d["O"] = torch.empty_like(d["Q"])
        d["S"] = torch.empty(wl.B, wl.Hkv, wl.d, wl.d, dtype=torch.float32, device="cuda")
        d["z"] = torch.empty(wl.B, wl.Hkv, wl.d, dtype=torch.float32, device="cuda")
        d["qt"] = torch.empty(wl.B, wl.W - 1, wl.Hq, wl.d, dtype=dt, device="cuda")
        d["kt"] = torch.empty(wl.B, wl.W - 1, wl.Hkv, wl.d, dtype=dt, device="cuda")
        sets.append(d)
    ws = lawcat.alloc_workspace(desc, lawcat.CALL_LAYER_PREFILL)

    def step(i, ev=None):
        d = sets[i % nsets]
        args = (desc, d["Q"], d["K"], d["V"], d["G"], d["wq"], d["wk"], None, None, None, None,
                d["O"], None, d["S"], d["z"], d["qt"], d["kt"], ws)
        if ev is None:
            lawcat.layer_prefill(*args)
        else:
            lawcat.layer_prefill_timed(*args, ev[0].value, ev[1].value)

    for i in range(warmup):
        step(i)
    torch.cuda.synchronize()
    ev = HipEvents(steps) if trace else None
    t0 = time.perf_counter()
    for i in range(steps):
        step(i, ev.pairs[i] if ev else None)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_step = (t1 - t0) * 1e3 / steps
    kern_ms = None
    if ev:
        ks = sorted(ev.elapsed_ms(i) for i in range(steps))
        kern_ms = sum(ks) / len(ks)
        ev.destroy()
    return {"ms_per_step": ms_step, "tokens_per_s": wl.B * wl.T / (ms_step * 1e-3), "kernel_ms": kern_ms,
            "bytes_step": bytes_step, "nsets": nsets, "host0": host0}


def run_side_ops(wl, steps=30):
    """Stand-alone calls of the same library on the same shape: the conv on Q (HBM-bound streaming,
    4 B per element moved) and the decode step (launch-bound).  Reported beside the headline, not as it."""
    import torch

    from paper_2509_18467_amd import lawcat

    dt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    desc = lawcat.make_desc(wl.B, wl.T, wl.Hq, wl.Hkv, wl.d, conv_width=wl.W, dtype=lawcat.DTYPE_BF16, feature_map=1)
    nset = 3
    xs = [torch.randn(wl.B, wl.T, wl.Hq, wl.d, device="cuda").to(dt) for _ in range(nset)]
    ys = [torch.empty_like(x) for x in xs]
    w = (0.5 * torch.randn(wl.Hq, wl.d, wl.W, device="cuda")).to(dt)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for i in range(3):
        lawcat.conv1d_causal(desc, wl.Hq, xs[i % nset], w, None, ys[i % nset], None)
    e0.record()
    for i in range(steps):
        lawcat.conv1d_causal(desc, wl.Hq, xs[i % nset], w, None, ys[i % nset], None)
    e1.record()
    torch.cuda.synchronize()
    conv_ms = e0.elapsed_time(e1) / steps
    conv_bytes = 2 * xs[0].numel() * xs[0].element_size()
    # the same conv followed by the shared d x d matrix of the feature map (section 4.1), one kernel
    wf = (torch.eye(wl.d, device="cuda") + torch.randn(wl.Hkv, wl.d, wl.d, device="cuda") * wl.d ** -0.5).to(dt)
    for i in range(3):
        lawcat.conv1d_feature(desc, wl.Hq, xs[i % nset], w, wf, None, ys[i % nset], None)
    e0.record()
    for i in range(steps):
        lawcat.conv1d_feature(desc, wl.Hq, xs[i % nset], w, wf, None, ys[i % nset], None)
    e1.record()
    torch.cuda.synchronize()
    feat_ms = e0.elapsed_time(e1) / steps
    # and the whole layer with that feature map: conv + matrix on Q and on K, staged, then the attention
    wk = (0.5 * torch.randn(wl.Hkv, wl.d, wl.W, device="cuda")).to(dt)
    Ks, Vs, Gs = ([torch.randn(wl.B, wl.T, wl.Hkv, wl.d, device="cuda").mul_(sc).to(dt) for _ in range(nset)]
                  for sc in (0.125, 0.125, 1.0))
    Sf = torch.empty(wl.B, wl.Hkv, wl.d, wl.d, device="cuda")
    zf = torch.empty(wl.B, wl.Hkv, wl.d, device="cuda")
    wsf = lawcat.alloc_workspace(desc, lawcat.CALL_LAYER_PREFILL_FM)

    def fm_layer(i):
        j = i % nset
        lawcat.layer_prefill_fm(desc, xs[j], Ks[j], Vs[j], Gs[j], w, wk, wf, None, None, None, None, ys[j], None, Sf, zf,
                                None, None, wsf)

    for i in range(3):
        fm_layer(i)
    e0.record()
    for i in range(steps):
        fm_layer(i)
    e1.record()
    torch.cuda.synchronize()
    fm_layer_ms = e0.elapsed_time(e1) / steps
    # the same number of tokens as 24 packed sequences of 256 .. 4096 tokens: one set of launches for the batch
    # (offsets on the device) against one call per sequence
    lengths = [4096, 2048, 1024, 512, 256, 256] * (wl.B * wl.T // 8192) if wl.B * wl.T % 8192 == 0 else [wl.B * wl.T]
    starts = [0]
    for n_ in lengths:
        starts.append(starts[-1] + n_)
    dv = lawcat.make_desc(len(lengths), max(lengths), wl.Hq, wl.Hkv, wl.d, conv_width=wl.W, dtype=lawcat.DTYPE_BF16,
                          feature_map=1)
    need = max(lawcat.varlen_workspace_bytes(dv, starts, True), lawcat.varlen_workspace_bytes(dv, starts, False), 16)
    wsv = torch.empty(need, dtype=torch.uint8, device="cuda")
    starts_dev = torch.tensor(starts, dtype=torch.int32, device="cuda")
    Sv = torch.empty(len(lengths), wl.Hkv, wl.d, wl.d, device="cuda")
    zv = torch.empty(len(lengths), wl.Hkv, wl.d, device="cuda")
    varlen_ms = {}
    for tag, dev_arr in (("one_launch", starts_dev), ("per_sequence_calls", None)):
        def vstep(i):
            j = i % nset
            lawcat.layer_prefill_varlen(dv, starts, xs[j].view(-1, wl.Hq, wl.d), Ks[j].view(-1, wl.Hkv, wl.d),
                                        Vs[j].view(-1, wl.Hkv, wl.d), Gs[j].view(-1, wl.Hkv, wl.d), w, wk, None, None, None,
                                        None, ys[j].view(-1, wl.Hq, wl.d), None, Sv, zv, None, None, wsv, seq_start_dev=dev_arr)
        for i in range(3):
            vstep(i)
        e0.record()
        for i in range(steps):
            vstep(i)
        e1.record()
        torch.cuda.synchronize()
        varlen_ms[tag] = e0.elapsed_time(e1) / steps
    # gate logits from the layer input (two rank-32 linear layers): reads d_model * 2 B, writes Hkv * d * 2 B per token
    dm = 2048 if wl.d == 64 else 4096
    gxs = [torch.randn(wl.B, wl.T, dm, device="cuda").to(dt) for _ in range(nset)]
    gw1 = (torch.randn(32, dm, device="cuda") * dm ** -0.5).to(dt)
    gw2 = (torch.randn(wl.Hkv * wl.d, 32, device="cuda") * 32 ** -0.5).to(dt)
    gb = (0.5 * torch.randn(wl.Hkv * wl.d, device="cuda")).to(dt)
    gout = torch.empty(wl.B, wl.T, wl.Hkv, wl.d, dtype=dt, device="cuda")
    for i in range(3):
        lawcat.gate_project(desc, dm, 32, gxs[i % nset], gw1, gw2, gb, gout)
    e0.record()
    for i in range(steps):
        lawcat.gate_project(desc, dm, 32, gxs[i % nset], gw1, gw2, gb, gout)
    e1.record()
    torch.cuda.synchronize()
    gate_ms = e0.elapsed_time(e1) / steps
    gate_bytes = wl.B * wl.T * (dm + wl.Hkv * wl.d) * 2
    del gxs
    # decode step
    d1 = lawcat.make_desc(wl.B, 1, wl.Hq, wl.Hkv, wl.d, conv_width=wl.W, dtype=lawcat.DTYPE_BF16, feature_map=1)
    q = torch.rand(wl.B, wl.Hq, wl.d, device="cuda").to(dt) + 0.5
    k = torch.rand(wl.B, wl.Hkv, wl.d, device="cuda").to(dt) + 0.5
    v = torch.randn(wl.B, wl.Hkv, wl.d, device="cuda").to(dt)
    g = torch.randn(wl.B, wl.Hkv, wl.d, device="cuda").to(dt)
    S = torch.zeros(wl.B, wl.Hkv, wl.d, wl.d, device="cuda")
    z = torch.ones(wl.B, wl.Hkv, wl.d, device="cuda")
    o = torch.empty(wl.B, wl.Hq, wl.d, dtype=dt, device="cuda")
    for _ in range(5):
        lawcat.gla_step(d1, q, k, v, g, S, z, o)
    n = 200
    e0.record()
    for _ in range(n):
        lawcat.gla_step(d1, q, k, v, g, S, z, o)
    e1.record()
    torch.cuda.synchronize()
    step_us = e0.elapsed_time(e1) / n * 1e3
    # the decode step over a batch of 256 sequences: bound by the state's traffic, not by the launch
    Bb = 256
    db = lawcat.make_desc(Bb, 1, wl.Hq, wl.Hkv, wl.d, conv_width=wl.W, dtype=lawcat.DTYPE_BF16, feature_map=1)
    qb = (torch.rand(Bb, wl.Hq, wl.d, device="cuda") + 0.5).to(dt)
    kb = (torch.rand(Bb, wl.Hkv, wl.d, device="cuda") + 0.5).to(dt)
    vb = torch.randn(Bb, wl.Hkv, wl.d, device="cuda").to(dt)
    gb2 = torch.randn(Bb, wl.Hkv, wl.d, device="cuda").to(dt)
    # two state sets in turn: 2 x 2 x (67 MB at d = 64, 268 MB at d = 128) do not fit the 256 MB Infinity Cache
    Sb = [torch.zeros(Bb, wl.Hkv, wl.d, wl.d, device="cuda") for _ in range(2)]
    zb = [torch.ones(Bb, wl.Hkv, wl.d, device="cuda") for _ in range(2)]
    ob = torch.empty(Bb, wl.Hq, wl.d, dtype=dt, device="cuda")
    for i in range(4):
        lawcat.gla_step(db, qb, kb, vb, gb2, Sb[i % 2], zb[i % 2], ob)
    nbs = 50
    e0.record()
    for i in range(nbs):
        lawcat.gla_step(db, qb, kb, vb, gb2, Sb[i % 2], zb[i % 2], ob)
    e1.record()
    torch.cuda.synchronize()
    batch_us = e0.elapsed_time(e1) / nbs * 1e3
    batch_bytes = 2 * Sb[0].numel() * 4
    del Sb, zb
    # the same decode in blocks of 256 tokens per launch (state on chip between the steps)
    nb = 256
    dn = lawcat.make_desc(wl.B, nb, wl.Hq, wl.Hkv, wl.d, conv_width=wl.W, dtype=lawcat.DTYPE_BF16, feature_map=1)
    qn = torch.rand(wl.B, nb, wl.Hq, wl.d, device="cuda").to(dt) + 0.5
    kn = torch.rand(wl.B, nb, wl.Hkv, wl.d, device="cuda").to(dt) + 0.5
    vn = torch.randn(wl.B, nb, wl.Hkv, wl.d, device="cuda").to(dt)
    gn = torch.randn(wl.B, nb, wl.Hkv, wl.d, device="cuda").to(dt)
    on = torch.empty_like(qn)
    for _ in range(2):
        lawcat.gla_steps(dn, qn, kn, vn, gn, S, z, on)
    e0.record()
    for _ in range(10):
        lawcat.gla_steps(dn, qn, kn, vn, gn, S, z, on)
    e1.record()
    torch.cuda.synchronize()
    block_us = e0.elapsed_time(e1) / (10 * nb) * 1e3
    # the attention's backward (fp32 vector arithmetic, a first version): one call at the headline shape
    dq_, dk_ = (torch.randn(wl.B, wl.T, h, wl.d, device="cuda").abs().to(dt) for h in (wl.Hq, wl.Hkv))
    dv_ = torch.randn(wl.B, wl.T, wl.Hkv, wl.d, device="cuda").to(dt)
    dg_ = (4.0 + torch.randn(wl.B, wl.T, wl.Hkv, wl.d, device="cuda")).to(dt)
    dplain = lawcat.make_desc(wl.B, wl.T, wl.Hq, wl.Hkv, wl.d, conv_width=wl.W, dtype=lawcat.DTYPE_BF16)
    do_, dden_ = torch.empty_like(dq_), torch.empty(wl.B, wl.T, wl.Hq, device="cuda")
    wsf = lawcat.alloc_workspace(dplain, lawcat.CALL_GLA_PREFILL)
    lawcat.gla_prefill(dplain, dq_, dk_, dv_, dg_, None, None, do_, dden_,
                       torch.empty(wl.B, wl.Hkv, wl.d, wl.d, device="cuda"), torch.empty(wl.B, wl.Hkv, wl.d, device="cuda"), wsf)
    dO_ = torch.randn(wl.B, wl.T, wl.Hq, wl.d, device="cuda").to(dt)
    grads = [torch.empty_like(t) for t in (dq_, dk_, dv_, dg_)]
    wsb = lawcat.alloc_workspace(dplain, lawcat.CALL_GLA_BACKWARD)
    for _ in range(2):
        lawcat.gla_backward(dplain, dq_, dk_, dv_, dg_, dden_, dO_, None, None, *grads, None, None, wsb)
    e0.record()
    for _ in range(5):
        lawcat.gla_backward(dplain, dq_, dk_, dv_, dg_, dden_, dO_, None, None, *grads, None, None, wsb)
    e1.record()
    torch.cuda.synchronize()
    bwd_ms = e0.elapsed_time(e1) / 5
    # the conv's adjoint on the query side (6 B per element in bf16: x and dy read, dx written)
    dw_ = torch.empty(wl.Hq, wl.d, wl.W, device="cuda")
    dxq = torch.empty_like(dq_)
    wsc = lawcat.alloc_workspace(desc, lawcat.CALL_CONV1D_BACKWARD)
    for _ in range(2):
        lawcat.conv1d_backward(desc, wl.Hq, xs[0], w, None, grads[0], dxq, dw_, None, wsc)
    e0.record()
    for _ in range(10):
        lawcat.conv1d_backward(desc, wl.Hq, xs[0], w, None, grads[0], dxq, dw_, None, wsc)
    e1.record()
    torch.cuda.synchronize()
    cbwd_ms = e0.elapsed_time(e1) / 10
    cbwd_bytes = 3 * xs[0].numel() * xs[0].element_size()
    # multiply-adds on the d x (d + 1) state: both sweeps update it once per token and kv head and read it once per
    # query head (dq; q^T d^), plus dk and dv: 2 * (2 + 2 * group + 2) * d * d per token and kv head, sweeps run twice
    bwd_flops = 2.0 * wl.B * wl.T * wl.Hkv * wl.d * wl.d * (4 + 2 * wl.Hq // wl.Hkv)
    return {"gla_backward": {"ms": bwd_ms, "tokens_per_s": wl.B * wl.T / (bwd_ms * 1e-3),
                             "fp32_TFLOP/s_outputs_only": bwd_flops / (bwd_ms * 1e-3) / 1e12},
            "conv1d_backward_q": {"ms": cbwd_ms, "GB/s": cbwd_bytes / (cbwd_ms * 1e-3) / 1e9,
                                  "frac_of_hbm_peak": cbwd_bytes / (cbwd_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "gla_steps_block256": {"us_per_step": block_us},
            "gla_step_batch256": {"us_per_step": batch_us, "state_bytes_per_step": batch_bytes,
                                  "GB/s": batch_bytes / (batch_us * 1e-6) / 1e9,
                                  "frac_of_hbm_peak": batch_bytes / (batch_us * 1e-6) / 1e9 / HBM_PEAK_GBS},
            "conv1d_causal_q": {"ms": conv_ms, "GB/s": conv_bytes / (conv_ms * 1e-3) / 1e9,
                                "frac_of_hbm_peak": conv_bytes / (conv_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "conv1d_feature_q": {"ms": feat_ms, "GB/s": conv_bytes / (feat_ms * 1e-3) / 1e9,
                                 "frac_of_hbm_peak": conv_bytes / (feat_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                 "mfma_TFLOP/s": 2 * xs[0].numel() * wl.d / (feat_ms * 1e-3) / 1e12},
            "gate_project": {"ms": gate_ms, "d_model": dm, "rank": 32, "GB/s": gate_bytes / (gate_ms * 1e-3) / 1e9,
                             "frac_of_hbm_peak": gate_bytes / (gate_ms * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "layer_prefill_varlen": {"sequences": len(lengths), "tokens": starts[-1], "ms_one_launch": varlen_ms["one_launch"],
                                     "ms_per_sequence_calls": varlen_ms["per_sequence_calls"],
                                     "tokens_per_s_one_launch": starts[-1] / (varlen_ms["one_launch"] * 1e-3)},
            "layer_prefill_fm": {"ms": fm_layer_ms, "tokens_per_s": wl.B * wl.T / (fm_layer_ms * 1e-3)},
            "gla_step": {"us_per_step": step_us, "state_bytes_per_step": 2 * S.numel() * 4}}


def cpu_baseline(wl, host0, feature_map=1, max_tokens=65536):
    """The fp64 oracle as it stands, on the host cores, on a bounded prefix of the same inputs
    (the whole sequence up to 65536 tokens: seconds to tens of seconds of CPU work)."""
    from oracle import oracle

    threads = min(oracle.max_threads(), wl.B * wl.Hkv)  # it parallelizes over (batch, kv head) only
    Ts = min(wl.T, max_tokens)
    x = {k: (v[:, :Ts] if k in "QKVG" else v) for k, v in host0.items()}
    t0 = time.perf_counter()
    oracle.layer_prefill(x["Q"], x["K"], x["V"], x["G"], x["wq"], x["wk"], feature_map)
    dt = time.perf_counter() - t0
    return {"value": wl.B * Ts / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"first {Ts} of {wl.T} tokens of the same seeded layer input, all heads, {dt:.1f} s"}


def mfma_flops_per_token(wl, chunk=16) -> int:
    """Useful matrix flops of the chunked form per token: scores and in-chunk product at chunk
    length C, state term and state update (no padding, no redundancy counted)."""
    d = wl.d
    return wl.Hq * (2 * chunk * d + 2 * chunk * d + 2 * d * d) + wl.Hkv * 2 * d * d


def read_traffic(name, key="traffic_bytes_per_launch"):
    """HBM bytes per output-pass launch (or, key="whole_step_traffic_bytes", per step: state pass + scan + output
    pass) from the committed rocprofv3 --pmc summary of this workload, if present."""
    path = os.path.join(ROOT, "profiles", f"output_pass_{name}_hbm_traffic.txt")
    if os.path.exists(path):
        for line in open(path):
            if line.startswith(key + ":"):
                return int(line.split(":")[1])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50, help="untimed steps first (they also bring the clocks up)")
    ap.add_argument("--workload", default="llama1b_32k")
    ap.add_argument("--feature-map", type=int, default=1)
    ap.add_argument("--quick", action="store_true",
                    help="headline only: skip the other graded shapes and variants ('sweep') and the stand-alone calls "
                         "('side_ops') that a default run also reports")
    ap.add_argument("--sweep", action="store_true", help="(default; kept for old command lines)")
    ap.add_argument("--side-ops", action="store_true", help="(default; kept for old command lines)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--segment", type=int, default=0, help="tokens per segment (0 = the library's choice)")
    ap.add_argument("--carry", type=int, default=0, choices=(0, 1, 2),
                    help="state carry: 0 = the library's choice, 1 = sequential (one segment per head), 2 = two-level")
    ap.add_argument("--gate-scale", type=float, default=1.0,
                    help="gate temperature: log alpha = gate_scale * log sigmoid(g); 1.0 in the graded workloads, "
                         "small values give a slowly decaying state")
    ap.add_argument("--curve", action="store_true",
                    help="also time both layer shapes at T = 8K .. 128K (reported under 'curve')")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2509_18467_amd.inputs import WORKLOADS

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = WORKLOADS[args.workload]
    r = run_workload(wl, args.steps, args.warmup, args.feature_map, segment=args.segment, carry=args.carry,
                     gate_scale=args.gate_scale)
    out = {
        "metric": "prefill tokens/s per layer",
        "value": r["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": r["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "T": wl.T, "Hq": wl.Hq, "Hkv": wl.Hkv, "head_dim": wl.d,
                   "conv_width": wl.W, "feature_map": "1+elu" if args.feature_map == 1 else "identity",
                   "carry": ("auto", "sequential", "two-level")[args.carry], "gate_scale": args.gate_scale,
                   "input_sets_rotated": r["nsets"]},
    }
    if r["kernel_ms"]:
        ach = r["bytes_step"] / (r["kernel_ms"] * 1e-3) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": "gla_chunk_kernel (output pass)", "achieved": ach,
                           "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                           "traffic": read_traffic(wl.name), "kernel_ms": r["kernel_ms"],
                           "algorithmic_bytes_per_launch": r["bytes_step"],
                           "whole_step_frac": r["bytes_step"] / (r["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS,
                           "whole_step_traffic": read_traffic(wl.name, "whole_step_traffic_bytes")}
    flops = mfma_flops_per_token(wl) * wl.B * wl.T
    out["mfma"] = {"useful_flops_per_token": mfma_flops_per_token(wl), "achieved_tflops": flops / (r["ms_per_step"] * 1e-3) / 1e12,
                   "frac_of_bf16_peak": flops / (r["ms_per_step"] * 1e-3) / 2.5e15}
    def entry(r2):
        e = {"tokens_per_s": r2["tokens_per_s"], "ms_per_step": r2["ms_per_step"], "kernel_ms": r2["kernel_ms"],
             "whole_step_frac": r2["bytes_step"] / (r2["ms_per_step"] * 1e-3) / 1e9 / HBM_PEAK_GBS}
        if r2["kernel_ms"]:
            e["output_pass_frac"] = r2["bytes_step"] / (r2["kernel_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBS
        return e

    if not args.quick:
        # the rest of the metric's range (T = 8K .. 128K, both layer shapes) and the other axes of the headline
        # shape, device-generated inputs of the same distributions, fewer steps each
        sweep = {}
        st, wu = max(5, args.steps // 4), max(2, args.warmup // 4)
        for name in ("llama1b_8k", "llama1b_32k", "mistral7b_16k", "mistral7b_128k"):
            if name == wl.name and args.feature_map == 1 and args.gate_scale == 1.0:
                continue
            sweep[name] = entry(run_workload(WORKLOADS[name], st, wu, 1, host_inputs=False))
            torch.cuda.empty_cache()
        sweep[wl.name + ":identity_feature_map"] = entry(run_workload(wl, st, wu, 0, host_inputs=False))
        torch.cuda.empty_cache()
        # gate temperature 1/16: a slowly decaying state (the state pass cannot stop early, see its kernel)
        sweep[wl.name + ":gate_scale_1/16"] = entry(run_workload(wl, st, wu, 1, gate_scale=0.0625, host_inputs=False))
        torch.cuda.empty_cache()
        out["sweep"] = sweep
        out["side_ops"] = run_side_ops(wl)
    if args.curve:
        import torch
        from dataclasses import replace
        curve = {}
        for base in ("llama1b_32k", "mistral7b_16k"):
            for T in (8192, 16384, 32768, 65536, 131072):
                w2 = replace(WORKLOADS[base], T=T, name=f"{base.split('_')[0]}@{T}")
                curve[w2.name] = entry(run_workload(w2, max(5, args.steps // 3), max(2, args.warmup // 3),
                                                    args.feature_map, host_inputs=False))
                torch.cuda.empty_cache()
        out["curve"] = curve
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(wl, r["host0"], args.feature_map)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
