"""Helpers shared by the tests: error metrics and adapters between the seeded inputs, the oracle
and the HIP path.  (The oracle and the HIP path never import each other; only tests see both.)"""
from __future__ import annotations

from typing import Dict, List, Sequence

import torch

from oracle import prefill_oracle as O

# Tolerances of the parity gate: max |gpu - ref| / max |ref| per compared tensor.
TOL = {"bf16": 2e-2, "fp32": 1e-4}


def max_rel_err(got: torch.Tensor, ref: torch.Tensor) -> float:
    """E = max_i |g_i - r_i| / max_i |r_i|  (the gate)."""
    got = got.detach().to("cpu", torch.float64)
    ref = ref.detach().to("cpu", torch.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.numel() == 0:
        return 0.0
    denom = ref.abs().max().item()
    return (got - ref).abs().max().item() / (denom if denom > 0 else 1.0)


def floor_rel_err(got: torch.Tensor, ref: torch.Tensor) -> float:
    """E_floor = max_i |g_i - r_i| / max(|r_i|, rms(r))  (reported, stricter)."""
    got = got.detach().to("cpu", torch.float64)
    ref = ref.detach().to("cpu", torch.float64)
    if ref.numel() == 0:
        return 0.0
    rms = ref.pow(2).mean().sqrt().item()
    return ((got - ref).abs() / torch.clamp(ref.abs(), min=max(rms, 1e-30))).max().item()


def fro_rel_err(got: torch.Tensor, ref: torch.Tensor) -> float:
    got = got.detach().to("cpu", torch.float64)
    ref = ref.detach().to("cpu", torch.float64)
    n = ref.norm().item()
    return (got - ref).norm().item() / (n if n > 0 else 1.0)


def oracle_shape(spec) -> O.Shape:
    return O.Shape(spec.n_layers, spec.hidden, spec.n_q_heads, spec.n_kv_heads, spec.head_dim,
                   spec.ffn, spec.rms_eps, spec.rope_theta, getattr(spec, "n_experts", 0),
                   getattr(spec, "top_k", 0))


def oracle_layers(weights: Sequence[Dict[str, torch.Tensor]]) -> List[O.LayerWeights]:
    """The same bits the GPU received (already rounded to the storage dtype), on the CPU."""
    return [O.LayerWeights(**{k: v.detach().to("cpu") for k, v in w.items()}) for w in weights]
