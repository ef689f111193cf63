"""Seeded synthetic inputs for the prefill path: shapes, weights, hidden states, prompt-length
mixes, arrival processes and block-table permutations.

This module holds NO arithmetic of the method.  It only draws numbers and rounds them to the
storage dtype; both the HIP path's tests/benchmark and the CPU oracle's tests are fed from here,
so both sides always see the same bits.

Workloads (stand-ins for the paper's QwenTrace length mix, Table 1, and ShareGPT prompts,
Section 6.5, neither of which ships with the paper; the paper itself replaces prompt contents by
random tokens of the traced lengths, Section 6.1 "Workloads"):
  cfg1  tiny 2-layer stack, one 256-token prompt, fp32 and bf16
  cfg2  Llama-3-8B-shaped, 4 layers, one 8192-token prompt (the benchmark workload)
  cfg3  Llama-3-8B-shaped, 32 layers, 16 prompts with log-normal lengths, paged KV
  cfg4  32768-token prompt preempted by Poisson arrivals of 128..1024-token prompts
  cfg5  Qwen2.5-32B-shaped, 64 layers, prompts of 65536/32768/16384/8192 tokens
Values: hidden states ~ N(0,1), weights ~ N(0,0.02), norm gains = 1.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class ShapeSpec:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float
    rope_theta: float
    n_experts: int = 0          # > 0: mixture-of-experts FFN, `ffn` is one expert's width
    top_k: int = 0

    @property
    def qkv_width(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def params_per_layer(self) -> int:
        d = self.hidden
        ffn = 3 * d * self.ffn * max(1, self.n_experts) + d * self.n_experts
        return d * self.qkv_width + self.n_q_heads * self.head_dim * d + ffn

    def with_layers(self, n_layers: int) -> "ShapeSpec":
        return replace(self, n_layers=n_layers)


TINY = ShapeSpec(2, 256, 4, 2, 64, 704, 1e-5, 10000.0)
LLAMA3_8B = ShapeSpec(32, 4096, 32, 8, 128, 14336, 1e-5, 500000.0)
QWEN25_32B = ShapeSpec(64, 5120, 40, 8, 128, 27648, 1e-5, 1000000.0)
# Mixture-of-experts shapes (Section 7): a tiny one for element-by-element parity and the shape of
# the 30B-A3B model the paper evaluates (128 experts of width 768, 8 per token).
TINY_MOE = ShapeSpec(2, 256, 4, 2, 64, 128, 1e-5, 10000.0, n_experts=8, top_k=2)
QWEN3_30B_A3B = ShapeSpec(48, 2048, 32, 4, 128, 768, 1e-6, 1000000.0, n_experts=128, top_k=8)

CONFIGS: Dict[str, dict] = {
    "cfg1": dict(shape=TINY, seed=1, lengths=[256]),
    "cfg2": dict(shape=LLAMA3_8B.with_layers(4), seed=2, lengths=[8192]),
    "cfg3": dict(shape=LLAMA3_8B, seed=3, lengths=None),          # lengths from lognormal_lengths
    "cfg4": dict(shape=LLAMA3_8B, seed=4, lengths=[32768]),
    "cfg5": dict(shape=QWEN25_32B, seed=5, lengths=[65536, 32768, 16384, 8192]),
    # One short request of the kind cfg4's arrivals are (128..1024 tokens), through the full stack.
    "short": dict(shape=LLAMA3_8B, seed=9, lengths=[256]),
    # Mixture-of-experts widening (not one of the baseline configurations): four layers of the
    # 30B-A3B shape, one 8192-token prompt.
    "moe": dict(shape=QWEN3_30B_A3B.with_layers(4), seed=7, lengths=[8192]),
}

STORAGE_DTYPES = {"fp32": torch.float32, "bf16": torch.bfloat16}


def _generator(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def normal_tensor(size: Sequence[int], std: float, seed: int, dtype: torch.dtype,
                  device="cpu") -> torch.Tensor:
    """N(0, std) drawn in fp32 from a generator seeded with `seed`, then rounded once to `dtype`
    (round-to-nearest-even).  The rounded tensor is the single source of truth for both sides."""
    g = _generator(seed, device)
    t = torch.randn(tuple(size), generator=g, dtype=torch.float32, device=device)
    if std != 1.0:
        t.mul_(std)
    return t.to(dtype)


def make_layer_weights(shape: ShapeSpec, layer: int, seed: int, dtype: torch.dtype,
                       device="cpu") -> Dict[str, torch.Tensor]:
    """One layer's parameters, row-major [out, in]:
    attn_norm [d] (ones), w_qkv [(Hq+2Hkv)D, d], w_o [d, Hq D], mlp_norm [d] (ones),
    w_gate_up [2F, d], w_down [d, F]."""
    d, f = shape.hidden, shape.ffn
    base = seed * 1000003 + layer * 101
    out = {
        "attn_norm": torch.ones(d, dtype=dtype, device=device),
        "w_qkv": normal_tensor((shape.qkv_width, d), 0.02, base + 1, dtype, device),
        "w_o": normal_tensor((d, shape.n_q_heads * shape.head_dim), 0.02, base + 2, dtype, device),
        "mlp_norm": torch.ones(d, dtype=dtype, device=device),
    }
    if shape.n_experts:
        # Mixture of experts: w_router [E, d] (wider spread, so that the selection is not a
        # near-tie everywhere), w_gate_up [E, 2F, d], w_down [E, d, F].
        e = shape.n_experts
        out["w_router"] = normal_tensor((e, d), 0.2, base + 5, dtype, device)
        out["w_gate_up"] = normal_tensor((e, 2 * f, d), 0.02, base + 3, dtype, device)
        out["w_down"] = normal_tensor((e, d, f), 0.02, base + 4, dtype, device)
    else:
        out["w_gate_up"] = normal_tensor((2 * f, d), 0.02, base + 3, dtype, device)
        out["w_down"] = normal_tensor((d, f), 0.02, base + 4, dtype, device)
    return out


def make_weights(shape: ShapeSpec, seed: int, dtype: torch.dtype, device="cpu"
                 ) -> List[Dict[str, torch.Tensor]]:
    return [make_layer_weights(shape, l, seed, dtype, device) for l in range(shape.n_layers)]


def make_hidden(n_tokens: int, hidden: int, seed: int, dtype: torch.dtype, device="cpu"
                ) -> torch.Tensor:
    """Input hidden states [T, d] ~ N(0,1) (the configs have no embedding table)."""
    return normal_tensor((n_tokens, hidden), 1.0, seed * 7919 + 17, dtype, device)


def randomize_gains(weights: List[Dict[str, torch.Tensor]], seed: int) -> None:
    """Tests only: replace the all-ones norm gains by 1 + N(0, 0.1) so that a kernel that drops
    the gain cannot pass.  (The benchmark configs keep gains at 1.)"""
    for l, w in enumerate(weights):
        for i, name in enumerate(("attn_norm", "mlp_norm")):
            g = w[name]
            noise = normal_tensor(g.shape, 0.1, seed * 31 + l * 2 + i, torch.float32, g.device)
            w[name] = (1.0 + noise).to(g.dtype)


def cu_seqlens_of(lengths: Sequence[int]) -> List[int]:
    cu = [0]
    for n in lengths:
        cu.append(cu[-1] + int(n))
    return cu


def lognormal_lengths(n_prompts: int, seed: int, median: float = 1024.0, sigma: float = 1.0,
                      lo: int = 64, hi: int = 32768) -> List[int]:
    """cfg3's prompt lengths: round(median * exp(sigma * z)), z ~ N(0,1), clipped to [lo, hi]."""
    rng = np.random.Generator(np.random.PCG64(seed))
    z = rng.standard_normal(n_prompts)
    n = np.rint(median * np.exp(sigma * z)).astype(np.int64)
    return [int(v) for v in np.clip(n, lo, hi)]


def poisson_arrivals(rate_per_s: float, duration_s: float, seed: int, lo: int = 128,
                     hi: int = 1024) -> List[Tuple[float, int]]:
    """cfg4's short requests: (arrival time in s, prompt length) with exponential inter-arrival
    times of mean 1/rate over `duration_s`, lengths uniform on {lo..hi}."""
    rng = np.random.Generator(np.random.PCG64(seed))
    t, out = 0.0, []
    while True:
        t += float(rng.exponential(1.0 / rate_per_s))
        if t >= duration_s:
            return out
        out.append((t, int(rng.integers(lo, hi + 1))))


# Request classes of the paper's evaluation trace: (name, mean, std of the prompt length in tokens,
# share of requests) from Table 1 and the Llama3-8B TTFT SLO in seconds from Table 2.
TRACE_CLASSES = (("text", 590.0, 652.0, 0.68, 0.25), ("image", 532.0, 510.0, 0.08, 0.5),
                 ("search", 5976.0, 3456.0, 0.20, 4.0), ("file", 6833.0, 5186.0, 0.04, 6.0))


def multi_slo_trace(rate_per_s: float, duration_s: float, seed: int, slo_scale: float = 1.0,
                    max_tokens: int = 32768) -> List[Tuple[int, int, float, float, str]]:
    """Stand-in for the production trace of Section 6.1 (which does not ship): Poisson arrivals at
    `rate_per_s` over `duration_s`; each request draws one of the four classes by Table 1's
    shares, a log-normal prompt length matched to that class's mean and standard deviation
    (clipped to [16, max_tokens]) and the class's SLO times `slo_scale`.
    Returns (id, n_tokens, arrival_s, ttft_slo_s, class name), ids in arrival order."""
    rng = np.random.Generator(np.random.PCG64(seed))
    shares = np.cumsum([c[3] for c in TRACE_CLASSES])
    t, out = 0.0, []
    while True:
        t += float(rng.exponential(1.0 / rate_per_s))
        if t >= duration_s:
            return out
        k = int(np.searchsorted(shares, rng.random() * shares[-1]))
        name, mean, std, _, slo = TRACE_CLASSES[min(k, len(TRACE_CLASSES) - 1)]
        sigma2 = float(np.log(1.0 + (std / mean) ** 2))
        n = float(rng.lognormal(np.log(mean) - sigma2 / 2.0, np.sqrt(sigma2)))
        out.append((len(out), int(min(max_tokens, max(16, round(n)))), round(t, 6), slo * slo_scale, name))


def permuted_block_tables(lengths: Sequence[int], cached: Optional[Sequence[int]],
                          block_tokens: int, pool_blocks: int, seed: int
                          ) -> Tuple[np.ndarray, int]:
    """A block table [n_seqs, max_blocks] (int32, -1 padded) whose physical block ids are a
    seeded random permutation of the pool, as in cfg3.  Returns (table, max_blocks)."""
    cached = [0] * len(lengths) if cached is None else list(cached)
    need = [-(-(int(c) + int(n)) // block_tokens) for n, c in zip(lengths, cached)]
    total = sum(need)
    if total > pool_blocks:
        raise ValueError(f"pool of {pool_blocks} blocks cannot hold {total}")
    rng = np.random.Generator(np.random.PCG64(seed))
    perm = rng.permutation(pool_blocks)[:total].astype(np.int32)
    max_blocks = max(need) if need else 0
    table = np.full((len(lengths), max(max_blocks, 1)), -1, dtype=np.int32)
    at = 0
    for s, nb in enumerate(need):
        table[s, :nb] = perm[at:at + nb]
        at += nb
    return table, max(max_blocks, 1)


def sample_rows(cu_seqlens: Sequence[int], n_rows: int, seed: int) -> List[int]:
    """Token rows for sampled-output checks: first and last row of every sequence plus seeded
    uniform picks, sorted, unique."""
    rng = np.random.Generator(np.random.PCG64(seed))
    total = int(cu_seqlens[-1])
    rows = set()
    for s in range(len(cu_seqlens) - 1):
        if cu_seqlens[s + 1] > cu_seqlens[s]:
            rows.add(int(cu_seqlens[s]))
            rows.add(int(cu_seqlens[s + 1]) - 1)
    while len(rows) < min(n_rows, total):
        rows.add(int(rng.integers(0, total)))
    return sorted(rows)
