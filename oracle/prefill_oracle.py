"""CPU oracle for the op-preemptible prefill forward pass.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain, fp64 statement of what the prefill hot path computes.  It exists so
that the HIP kernels can be checked against something that is obviously the definition.  Only
tests, the smoke check and the benchmark's `cpu_baseline` leg may import it; the product path
(the C-ABI library and its Python binding) never does, and this file imports nothing from the
product package.

What it follows
---------------
FlowPrefill (arxiv 2602.16603), Section 2.1 "Transformer-based Generative Inference":
  * Eq. (1): Q, K, V are linear projections of the hidden states.
  * Eq. (2): Attention(Q, K, V) = softmax(Q K^T / sqrt(d_k)) V.
  * the sentence after Eq. (2): attention is followed by a position-wise FFN and residual
    connections, repeated over all L layers.
Section 3.1 (small-chunk paragraph): attention is causal, and a later chunk of a prompt attends
to the keys/values that earlier chunks left in the KV cache.
Section 5.1 lists the operators of a dense layer (qkv_proj, attn, o_proj, gate_up_proj,
down_proj); the layer evaluated is the Llama/Qwen pre-norm block, so between those operators sit
RMSNorm, rotary position embedding and SiLU(gate)*up.

The paper's equations are the textbook MHA; the evaluated models add the following, which the
paper does not spell out and which are fixed here (and identically, but independently, in the
HIP path):
  * weights are stored row-major [out, in] and applied as y = x W^T; the fused QKV weight has
    rows [all Q heads | all K heads | all V heads]; the fused gate/up weight has rows [gate | up];
  * RMSNorm: x * g / sqrt(mean(x^2) + eps), eps inside the square root;
  * rotary embedding pairs element j with element j + D/2 of a head ("half split"), angle
    p * theta^(-2j/D), no scaling, p = absolute position of the token in its own sequence;
  * grouped-query attention: query head h reads KV head h // (Hq / Hkv);
  * the KV cache holds K after rotation and V unrotated;
  * softmax scale 1/sqrt(head_dim); no biases; no final norm or LM head: the output is the
    residual stream after the last layer.

Everything is fp64: inputs arrive as whatever the harness rounded them to (fp32, or bf16 values
widened), are widened to fp64 once, and nothing is rounded afterwards.  There is no tiling, no
online softmax and no paging: each step is the formula written out.  `torch.matmul` on CPU
tensors is the one library primitive used (a dense matrix product); `einsum` is not used so the
index order can be read off every line.

Pins (tests/test_oracle_pins.py): brute-force Python-loop attention on tiny inputs, softmax rows
summing to one, single-token and equal-key closed forms, GQA == MHA with repeated KV heads,
causality under suffix extension, chunked-with-cache == one-shot, packed == separate sequences,
RoPE as a textbook 2-D rotation / identity at position 0 / norm preservation / relative-position
property, RMSNorm scale invariance and unit RMS, SiLU closed-form values, zero-weight residual
wiring, GEMM against a Python triple loop, a whole-stack cross-check against a scalar
per-token pure-Python transcription on a tiny shape, and for the mixture-of-experts FFN: identical
experts == the dense FFN, top_k == E == the softmax-weighted sum of all experts, a one-hot router
== that expert alone, a pure-Python loop on tiny inputs, weights summing to one.  The paper prints no tensor values, so no
number here comes from the paper.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

F64 = torch.float64


@dataclass(frozen=True)
class Shape:
    """Static description of the decoder stack (the fields of the C ABI's fp_shape that matter
    to the arithmetic)."""
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    n_experts: int = 0            # > 0: mixture-of-experts FFN (Section 7), `ffn` is one expert's width
    top_k: int = 0

    @property
    def q_width(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_width(self) -> int:
        return self.n_kv_heads * self.head_dim


@dataclass
class LayerWeights:
    """One layer's parameters, any float dtype, CPU.  Shapes:
    attn_norm [d], w_qkv [(Hq+2Hkv)D, d], w_o [d, Hq D], mlp_norm [d], w_gate_up [2F, d],
    w_down [d, F]."""
    attn_norm: torch.Tensor
    w_qkv: torch.Tensor
    w_o: torch.Tensor
    mlp_norm: torch.Tensor
    w_gate_up: torch.Tensor
    w_down: torch.Tensor
    # Mixture-of-experts layers: w_router [E, d]; w_gate_up [E, 2F, d]; w_down [E, d, F].
    w_router: Optional[torch.Tensor] = None


def _f64(t: torch.Tensor) -> torch.Tensor:
    return t.detach().to(device="cpu", dtype=F64)


# --------------------------------------------------------------------------------------------
# Elementary operators
# --------------------------------------------------------------------------------------------

def rmsnorm(x: torch.Tensor, gain: torch.Tensor, eps: float) -> torch.Tensor:
    """Row-wise RMS normalisation: x_j * g_j / sqrt(mean_j(x_j^2) + eps).

    The norm that precedes qkv_proj and gate_up_proj in the evaluated (Llama/Qwen) layers of
    Section 6.1; the paper itself only says "FFN and residual connections" (Section 2.1)."""
    x = _f64(x)
    gain = _f64(gain)
    mean_sq = (x * x).sum(dim=-1, keepdim=True) / x.shape[-1]
    return x / torch.sqrt(mean_sq + eps) * gain


def linear(x: torch.Tensor, w: torch.Tensor) -> torch.Tensor:
    """y = x W^T with W stored [out, in] -- Eq. (1) in row-vector form (the paper writes the
    column-vector form W X)."""
    return torch.matmul(_f64(x), _f64(w).transpose(0, 1))


def rope_rotate(u: torch.Tensor, positions: torch.Tensor, theta: float) -> torch.Tensor:
    """Rotary position embedding of u [n, H, D] at integer positions [n].

    For j in [0, D/2): angle = p * theta^(-2j/D); the pair (u_j, u_{j+D/2}) is rotated by that
    angle:  u_j' = u_j cos - u_{j+D/2} sin,  u_{j+D/2}' = u_{j+D/2} cos + u_j sin."""
    u = _f64(u)
    n, _, dim = u.shape
    half = dim // 2
    j = torch.arange(half, dtype=F64)
    inv_freq = torch.pow(torch.tensor(float(theta), dtype=F64), -2.0 * j / dim)   # [D/2]
    angle = positions.to(F64).reshape(n, 1) * inv_freq.reshape(1, half)          # [n, D/2]
    cos = torch.cos(angle).reshape(n, 1, half)
    sin = torch.sin(angle).reshape(n, 1, half)
    a = u[:, :, :half]
    b = u[:, :, half:]
    return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1)


def causal_attention(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                     q_positions: torch.Tensor) -> torch.Tensor:
    """Eq. (2) with a causal mask and grouped KV heads, for ONE sequence.

    q [n, Hq, D] are the new tokens' (rotated) queries at absolute positions q_positions [n];
    k, v [m, Hkv, D] hold every key/value of the sequence from position 0 to m-1 (cache prefix
    followed by the new tokens).  Query i sees keys j <= q_positions[i].  Returns [n, Hq, D]."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    n, hq, dim = q.shape
    m, hkv, _ = k.shape
    group = hq // hkv
    scale = 1.0 / math.sqrt(dim)
    key_pos = torch.arange(m).reshape(1, m)
    visible = key_pos <= q_positions.reshape(n, 1)                                # [n, m]
    out = torch.empty((n, hq, dim), dtype=F64)
    if n == 0:                       # an empty sequence in a packed batch has no rows to fill
        return out
    for h in range(hq):
        g = h // group
        scores = torch.matmul(q[:, h, :], k[:, g, :].transpose(0, 1)) * scale    # [n, m]
        scores = scores.masked_fill(~visible, float("-inf"))
        scores = scores - scores.max(dim=-1, keepdim=True).values
        weights = torch.exp(scores)
        weights = weights / weights.sum(dim=-1, keepdim=True)
        out[:, h, :] = torch.matmul(weights, v[:, g, :])
    return out


def attention_probabilities(q: torch.Tensor, k: torch.Tensor, q_positions: torch.Tensor,
                            q_head: int, kv_head: int) -> torch.Tensor:
    """The softmax matrix of one head, exposed so a test can check that rows sum to one."""
    q, k = _f64(q), _f64(k)
    n, _, dim = q.shape
    m = k.shape[0]
    scores = torch.matmul(q[:, q_head, :], k[:, kv_head, :].transpose(0, 1)) / math.sqrt(dim)
    visible = torch.arange(m).reshape(1, m) <= q_positions.reshape(n, 1)
    scores = scores.masked_fill(~visible, float("-inf"))
    scores = scores - scores.max(dim=-1, keepdim=True).values
    weights = torch.exp(scores)
    return weights / weights.sum(dim=-1, keepdim=True)


def silu_mul(gate_up: torch.Tensor) -> torch.Tensor:
    """[.., 2F] -> [.., F]:  gate / (1 + exp(-gate)) * up, gate = first F columns."""
    gate_up = _f64(gate_up)
    f = gate_up.shape[-1] // 2
    gate = gate_up[..., :f]
    up = gate_up[..., f:]
    return gate / (1.0 + torch.exp(-gate)) * up


# --------------------------------------------------------------------------------------------
# Mixture-of-experts FFN (Section 7, "Mixture-of-Experts (MoE) models": a gated router -- the
# `gate` operator -- and several expert FFNs -- the `experts` operator).  The paper names the two
# operators and nothing else; fixed here, as in the MoE family it evaluates: router logits
# h W_r^T, softmax over ALL experts, the top_k most probable experts per token (ties: lower expert
# index), their probabilities renormalised to sum to one, every expert a SwiGLU FFN, the layer's
# output the weighted sum of the selected experts' outputs; no shared expert, no bias.
# --------------------------------------------------------------------------------------------
def moe_route(h: torch.Tensor, w_router: torch.Tensor, top_k: int) -> Tuple[torch.Tensor, torch.Tensor]:
    """-> expert ids [T, top_k] (int64, most probable first) and their weights [T, top_k]."""
    logits = linear(h, w_router)
    prob = torch.exp(logits - logits.max(dim=-1, keepdim=True).values)
    prob = prob / prob.sum(dim=-1, keepdim=True)
    n_tokens, n_experts = prob.shape
    ids = torch.empty((n_tokens, top_k), dtype=torch.int64)
    wts = torch.empty((n_tokens, top_k), dtype=F64)
    for t in range(n_tokens):
        order = sorted(range(n_experts), key=lambda e: (-float(prob[t, e]), e))[:top_k]
        chosen = prob[t, order]
        ids[t] = torch.tensor(order)
        wts[t] = chosen / chosen.sum()
    return ids, wts


def moe_weights_for(h: torch.Tensor, w_router: torch.Tensor, ids: torch.Tensor) -> torch.Tensor:
    """The renormalised router probabilities of GIVEN expert ids [T, k] (any order)."""
    prob = torch.softmax(linear(h, w_router), dim=-1)
    chosen = torch.gather(prob, 1, ids.to(torch.int64))
    return chosen / chosen.sum(dim=-1, keepdim=True)


def moe_selection_shortfall(h: torch.Tensor, w_router: torch.Tensor, ids: torch.Tensor,
                            top_k: int, relative: bool = False) -> torch.Tensor:
    """Per token: (the oracle's k-th largest router probability) - (the smallest probability among
    the given experts), clipped at 0; with `relative`, divided by that k-th largest probability.
    Zero when `ids` is a top-k set of the oracle's probabilities; a value of the order of the
    implementation's rounding error means the implementation resolved a near-tie the other way."""
    prob = torch.softmax(linear(h, w_router), dim=-1)
    kth = torch.sort(prob, dim=-1, descending=True).values[:, top_k - 1]
    weakest = torch.gather(prob, 1, ids.to(torch.int64).cpu()).min(dim=-1).values
    gap = torch.clamp(kth - weakest, min=0.0)
    return gap / kth if relative else gap


def moe_mlp(h: torch.Tensor, w_router: torch.Tensor, w_gate_up: torch.Tensor, w_down: torch.Tensor,
            top_k: int, forced_ids: Optional[torch.Tensor] = None,
            weights_out: Optional[List[torch.Tensor]] = None) -> torch.Tensor:
    """sum_j weight_j * down_e(j)( silu_mul( gate_up_e(j)( h ) ) ) per token.  `forced_ids` [T, k]
    replaces the router's own SELECTION (the weights stay the oracle's own probabilities of those
    experts, renormalised): for checking an implementation whose decision between two experts a
    rounding error apart may legitimately differ -- the test then also checks that the forced
    selection is a valid top-k of the oracle's probabilities to within that rounding error."""
    h = _f64(h)
    if forced_ids is not None:
        ids = forced_ids.to(torch.int64).cpu()
        wts = moe_weights_for(h, w_router, ids)
    else:
        ids, wts = moe_route(h, w_router, top_k)
    if weights_out is not None:          # read-out for tests: the weights this layer applied, [T, k]
        weights_out.append(_f64(wts).clone())
    out = torch.zeros_like(h)
    for e in range(w_gate_up.shape[0]):
        rows, slots = torch.nonzero(ids == e, as_tuple=True)
        if rows.numel() == 0:
            continue
        y = linear(silu_mul(linear(h[rows], w_gate_up[e])), w_down[e])
        out.index_add_(0, rows, y * _f64(wts)[rows, slots].unsqueeze(-1))
    return out


# --------------------------------------------------------------------------------------------
# One layer / whole stack
# --------------------------------------------------------------------------------------------

@dataclass
class KVState:
    """Contiguous (un-paged) per-layer, per-sequence cache: k[layer][seq], v[layer][seq] are
    [len, Hkv, D] fp64 tensors (K rotated, V raw)."""
    k: List[List[torch.Tensor]]
    v: List[List[torch.Tensor]]

    @staticmethod
    def empty(shape: Shape, n_seqs: int) -> "KVState":
        z = lambda: torch.zeros((0, shape.n_kv_heads, shape.head_dim), dtype=F64)
        return KVState(k=[[z() for _ in range(n_seqs)] for _ in range(shape.n_layers)],
                       v=[[z() for _ in range(n_seqs)] for _ in range(shape.n_layers)])

    def lengths(self) -> List[int]:
        return [int(t.shape[0]) for t in self.k[0]] if self.k else []


def layer_forward(shape: Shape, w: LayerWeights, x: torch.Tensor, cu_seqlens: Sequence[int],
                  k_prev: List[torch.Tensor], v_prev: List[torch.Tensor],
                  forced_ids: Optional[torch.Tensor] = None,
                  shortfall_out: Optional[List[torch.Tensor]] = None,
                  weights_out: Optional[List[torch.Tensor]] = None
                  ) -> Tuple[torch.Tensor, List[torch.Tensor], List[torch.Tensor]]:
    """One decoder layer over a packed batch.

    x [T, d]; sequence s owns rows cu_seqlens[s]:cu_seqlens[s+1]; k_prev[s], v_prev[s] are the
    cached keys/values of that sequence from earlier chunks (possibly empty).  Returns the new
    residual stream and the extended caches."""
    x = _f64(x)
    hq, hkv, dim = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    h = rmsnorm(x, w.attn_norm, shape.rms_eps)
    qkv = linear(h, w.w_qkv)                                                      # Eq. (1)
    q_all = qkv[:, :shape.q_width]
    k_all = qkv[:, shape.q_width:shape.q_width + shape.kv_width]
    v_all = qkv[:, shape.q_width + shape.kv_width:]
    attn_out = torch.empty((x.shape[0], shape.q_width), dtype=F64)
    k_next, v_next = [], []
    for s in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        n = hi - lo
        cached = int(k_prev[s].shape[0])
        pos = torch.arange(cached, cached + n)
        q = rope_rotate(q_all[lo:hi].reshape(n, hq, dim), pos, shape.rope_theta)
        k_new = rope_rotate(k_all[lo:hi].reshape(n, hkv, dim), pos, shape.rope_theta)
        v_new = v_all[lo:hi].reshape(n, hkv, dim)
        k_full = torch.cat([k_prev[s], k_new], dim=0)
        v_full = torch.cat([v_prev[s], v_new], dim=0)
        o = causal_attention(q, k_full, v_full, pos)                              # Eq. (2)
        attn_out[lo:hi] = o.reshape(n, hq * dim)
        k_next.append(k_full)
        v_next.append(v_full)
    x = x + linear(attn_out, w.w_o)
    h2 = rmsnorm(x, w.mlp_norm, shape.rms_eps)
    if w.w_router is not None:
        if forced_ids is not None and shortfall_out is not None:
            shortfall_out.append(moe_selection_shortfall(h2, w.w_router, forced_ids, shape.top_k))
            shortfall_out.append(moe_selection_shortfall(h2, w.w_router, forced_ids, shape.top_k, relative=True))
        x = x + moe_mlp(h2, w.w_router, w.w_gate_up, w.w_down, shape.top_k, forced_ids, weights_out)
    else:
        act = silu_mul(linear(h2, w.w_gate_up))
        x = x + linear(act, w.w_down)
    return x, k_next, v_next


def prefill(shape: Shape, layers: Sequence[LayerWeights], x: torch.Tensor,
            cu_seqlens: Sequence[int], cache: Optional[KVState] = None,
            forced_ids: Optional[Sequence[torch.Tensor]] = None,
            shortfall_out: Optional[List[torch.Tensor]] = None,
            weights_out: Optional[List[torch.Tensor]] = None) -> Tuple[torch.Tensor, KVState]:
    """The whole stack over a packed batch of (chunks of) prompts.  `cache` carries what earlier
    chunks of the same sequences left behind (None = empty).  Returns the final residual stream
    [T, d] and the extended cache."""
    n_seqs = len(cu_seqlens) - 1
    if cache is None:
        cache = KVState.empty(shape, n_seqs)
    x = _f64(x)
    new_k, new_v = [], []
    for layer in range(shape.n_layers):
        x, k_l, v_l = layer_forward(shape, layers[layer], x, cu_seqlens,
                                    cache.k[layer], cache.v[layer],
                                    None if forced_ids is None else forced_ids[layer], shortfall_out,
                                    weights_out)
        new_k.append(k_l)
        new_v.append(v_l)
    return x, KVState(k=new_k, v=new_v)


def prefill_chunked(shape: Shape, layers: Sequence[LayerWeights], x: torch.Tensor,
                    chunk: int) -> Tuple[torch.Tensor, KVState]:
    """One prompt [n, d] processed `chunk` tokens at a time through the WHOLE stack, each chunk
    reading the cache left by the previous ones (Section 3.1's chunked prefill)."""
    n = x.shape[0]
    cache = None
    outs = []
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        y, cache = prefill(shape, layers, x[lo:hi], [0, hi - lo], cache)
        outs.append(y)
    return torch.cat(outs, dim=0), cache


def layer_sampled_rows(shape: Shape, w: LayerWeights, x: torch.Tensor,
                       cu_seqlens: Sequence[int], rows: Sequence[int]
                       ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Teacher-forced check of one layer at full size: given the layer's input x [T, d] (no
    cached prefix), return K (rotated) and V for ALL tokens ([T, Hkv, D] each) and the layer's
    output residual for the token rows listed in `rows` only ([len(rows), d]).

    Same formulas as layer_forward; the only saving is that queries, the output projection and
    the MLP are evaluated for the sampled rows instead of all rows."""
    x = _f64(x)
    hq, hkv, dim = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    qw, kvw = shape.q_width, shape.kv_width
    h = rmsnorm(x, w.attn_norm, shape.rms_eps)
    wqkv = _f64(w.w_qkv)
    kv = torch.matmul(h, wqkv[qw:].transpose(0, 1))                               # [T, 2 Hkv D]
    t_total = x.shape[0]
    k_rot = torch.empty((t_total, hkv, dim), dtype=F64)
    v_raw = kv[:, kvw:].reshape(t_total, hkv, dim).clone()
    seq_of_row, pos_of_row = {}, {}
    for s in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        pos = torch.arange(0, hi - lo)
        k_rot[lo:hi] = rope_rotate(kv[lo:hi, :kvw].reshape(hi - lo, hkv, dim), pos,
                                   shape.rope_theta)
        for r in rows:
            if lo <= r < hi:
                seq_of_row[r] = (lo, hi)
                pos_of_row[r] = r - lo
    # Queries, output projection and MLP for the sampled rows only, all rows at once per matmul;
    # attention row by row (each row has its own causal extent).
    rows = [int(r) for r in rows]
    h_rows = h[rows]                                                             # [R, d]
    q_rows = torch.matmul(h_rows, wqkv[:qw].transpose(0, 1)).reshape(len(rows), hq, dim)
    attn_rows = torch.empty((len(rows), hq * dim), dtype=F64)
    for idx, r in enumerate(rows):
        lo, hi = seq_of_row[r]
        p = pos_of_row[r]
        pos = torch.tensor([p])
        q = rope_rotate(q_rows[idx:idx + 1], pos, shape.rope_theta)
        o = causal_attention(q, k_rot[lo:lo + p + 1], v_raw[lo:lo + p + 1], pos)
        attn_rows[idx] = o.reshape(hq * dim)
    xr = x[rows] + linear(attn_rows, w.w_o)
    h2 = rmsnorm(xr, w.mlp_norm, shape.rms_eps)
    act = silu_mul(linear(h2, w.w_gate_up))
    out = xr + linear(act, w.w_down)
    return k_rot, v_raw, out
