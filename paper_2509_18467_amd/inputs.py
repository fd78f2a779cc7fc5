"""Seeded synthetic inputs for the LAWCAT prefill path.

This module is the only code shared by the HIP path and the CPU oracle.  It holds
none of the method's arithmetic: it draws random tensors of the workload shapes,
rounds them to the storage type once, and returns them as float32 numpy arrays
(bf16 values are exactly representable in float32, so both sides see the same
numbers).

Shapes follow the layer of the paper's Fig. 1 / section 4 with grouped-query
heads: Q [B,T,Hq,d], K/V/gate logits [B,T,Hkv,d], conv weights [H,d,W] with
w[..., 0] multiplying the current token (section 4.1, sum over delta).
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    T: int
    Hq: int
    Hkv: int
    d: int
    W: int = 4
    dtype: str = "bf16"  # storage type of Q, K, V, gate logits, conv weights, O: "bf16" | "fp32"

    def with_T(self, T: int) -> "Workload":
        return replace(self, T=T, name=f"{self.name}@T{T}")


# The five graded shapes: a tiny fp32 case and Llama-3.2-1B / Mistral-7B shaped layers.
WORKLOADS = {
    "tiny": Workload("tiny", B=1, T=256, Hq=2, Hkv=2, d=64, dtype="fp32"),
    "llama1b_8k": Workload("llama1b_8k", B=1, T=8192, Hq=32, Hkv=8, d=64),
    "llama1b_32k": Workload("llama1b_32k", B=1, T=32768, Hq=32, Hkv=8, d=64),
    "mistral7b_16k": Workload("mistral7b_16k", B=1, T=16384, Hq=32, Hkv=8, d=128),
    "mistral7b_128k": Workload("mistral7b_128k", B=1, T=131072, Hq=32, Hkv=8, d=128),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bf16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def make_inputs(wl: Workload, seed: int = 0, halo: bool = False, state: bool = False) -> dict:
    """Draw Q, K, V, G, wq, wk (in that fixed order) from numpy's default_rng(seed).

    Q, K, V ~ N(0,1)/8; gate logits G ~ N(0,1); conv weights ~ N(0, variance 1/W).
    Optional extras, drawn afterwards: conv halos (W-1 raw rows before the first token)
    and a start state S0, z0.
    """
    rng = np.random.default_rng(seed)
    f32 = np.float32

    def normal(shape, scale):
        a = rng.standard_normal(shape, dtype=f32)
        a *= f32(scale)
        return a

    B, T, Hq, Hkv, d, W = wl.B, wl.T, wl.Hq, wl.Hkv, wl.d, wl.W
    out = {
        "Q": normal((B, T, Hq, d), 0.125),
        "K": normal((B, T, Hkv, d), 0.125),
        "V": normal((B, T, Hkv, d), 0.125),
        "G": normal((B, T, Hkv, d), 1.0),
        "wq": normal((Hq, d, W), 1.0 / np.sqrt(W)),
        "wk": normal((Hkv, d, W), 1.0 / np.sqrt(W)),
    }
    if halo:
        out["q_halo"] = normal((B, W - 1, Hq, d), 0.125)
        out["k_halo"] = normal((B, W - 1, Hkv, d), 0.125)
    if wl.dtype == "bf16":
        for key in list(out):
            out[key] = round_to_bf16(out[key])
    if state:  # states are always fp32
        out["S0"] = normal((B, Hkv, d, d), 0.25)
        out["z0"] = np.abs(normal((B, Hkv, d), 2.0)) + f32(1.0)
    return out


def make_feature_weights(wl: Workload, seed: int = 0) -> np.ndarray:
    """wf [Hkv,d,d] for the shared linear layer of the feature map: the identity (where a converted model
    starts) plus a dense N(0, 1/d) perturbation of the same energy, from a generator of its own so that the
    tensors of make_inputs do not depend on it."""
    rng = np.random.default_rng([seed, 0x5746])
    wf = rng.standard_normal((wl.Hkv, wl.d, wl.d), dtype=np.float32)
    wf *= np.float32(1.0 / np.sqrt(wl.d))
    wf += np.eye(wl.d, dtype=np.float32)
    return round_to_bf16(wf) if wl.dtype == "bf16" else wf


def make_gate_inputs(wl: Workload, d_model: int, rank: int = 32, seed: int = 0, bias: bool = True) -> dict:
    """Layer input and the two low-rank gate matrices: x ~ N(0,1) (a normalized hidden state), w1 [rank,d_model]
    ~ N(0, 1/d_model), w2 [Hkv*d, rank] ~ N(0, 1/rank), bias ~ N(0, 1/4): gate logits of unit scale, as the G of
    make_inputs.  A generator of its own."""
    rng = np.random.default_rng([seed, 0x4750])
    f32 = np.float32
    N = wl.Hkv * wl.d
    out = {"x": rng.standard_normal((wl.B, wl.T, d_model), dtype=f32),
           "w1": rng.standard_normal((rank, d_model), dtype=f32) * f32(d_model ** -0.5),
           "w2": rng.standard_normal((N, rank), dtype=f32) * f32(rank ** -0.5)}
    if bias:
        out["bias"] = rng.standard_normal((N,), dtype=f32) * f32(0.5)
    if wl.dtype == "bf16":
        for k in list(out):
            out[k] = round_to_bf16(out[k])
    return out
