"""Pins for the CPU oracle: every check here compares the oracle with something that is NOT the
oracle -- a pure-Python scalar loop, a closed form, or an invariant the mathematics fixes.

The paper (FlowPrefill, Section 2.1, Eq. 1-2; Section 3.1 for causal attention with a KV cache)
prints no tensor values, so no expected number comes from it; each pin is chosen so that a
plausible slip in the oracle (dropped term, wrong sign, wrong index, transposed operand, wrong
head mapping) fails at least one test.
"""
import math
import random

import pytest
import torch

from oracle import prefill_oracle as O

F64 = torch.float64


def rnd(*size, seed=0, std=1.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(*size, generator=g, dtype=F64) * std


# ---------------------------------------------------------------------------------------------
# scalar pure-Python reference pieces (lists and math only)
# ---------------------------------------------------------------------------------------------

def py_attention(q, k, v, q_pos, hq, hkv, dim):
    """q[n][hq][dim], k/v[m][hkv][dim] as nested lists."""
    n, m = len(q), len(k)
    out = [[[0.0] * dim for _ in range(hq)] for _ in range(n)]
    for i in range(n):
        for h in range(hq):
            g = h // (hq // hkv)
            s = []
            for j in range(m):
                if j <= q_pos[i]:
                    s.append(sum(q[i][h][c] * k[j][g][c] for c in range(dim)) / math.sqrt(dim))
            mx = max(s)
            e = [math.exp(t - mx) for t in s]
            z = sum(e)
            for c in range(dim):
                out[i][h][c] = sum(e[j] / z * v[j][g][c] for j in range(len(s)))
    return out


def py_rope(vec, pos, theta):
    dim = len(vec)
    half = dim // 2
    out = [0.0] * dim
    for j in range(half):
        ang = pos * theta ** (-2.0 * j / dim)
        out[j] = vec[j] * math.cos(ang) - vec[j + half] * math.sin(ang)
        out[j + half] = vec[j + half] * math.cos(ang) + vec[j] * math.sin(ang)
    return out


def py_rmsnorm(row, gain, eps):
    ms = sum(t * t for t in row) / len(row)
    return [t / math.sqrt(ms + eps) * g for t, g in zip(row, gain)]


def py_matvec(w, x):
    """w[out][in] applied to x[in]."""
    return [sum(wr[c] * x[c] for c in range(len(x))) for wr in w]


def py_prefill(shape, layers, x, cached_k=None, cached_v=None):
    """Whole stack for ONE sequence in scalar Python.  x[n][d].  cached_k/v[layer] = list of
    [hkv][dim] rows from an earlier chunk.  Returns final x and per-layer K, V rows."""
    hq, hkv, dim, d, f = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.hidden, shape.ffn
    n = len(x)
    ks, vs = [], []
    for l, w in enumerate(layers):
        kc = list(cached_k[l]) if cached_k else []
        vc = list(cached_v[l]) if cached_v else []
        base = len(kc)
        qs = []
        for i in range(n):
            h = py_rmsnorm(x[i], w["attn_norm"], shape.rms_eps)
            qkv = py_matvec(w["w_qkv"], h)
            q = [py_rope(qkv[a * dim:(a + 1) * dim], base + i, shape.rope_theta) for a in range(hq)]
            off = hq * dim
            k = [py_rope(qkv[off + a * dim: off + (a + 1) * dim], base + i, shape.rope_theta)
                 for a in range(hkv)]
            off += hkv * dim
            v = [qkv[off + a * dim: off + (a + 1) * dim] for a in range(hkv)]
            qs.append(q)
            kc.append(k)
            vc.append(v)
        o = py_attention(qs, kc, vc, [base + i for i in range(n)], hq, hkv, dim)
        nx = []
        for i in range(n):
            flat = [t for head in o[i] for t in head]
            r = [a + b for a, b in zip(x[i], py_matvec(w["w_o"], flat))]
            h2 = py_rmsnorm(r, w["mlp_norm"], shape.rms_eps)
            gu = py_matvec(w["w_gate_up"], h2)
            act = [gu[c] / (1.0 + math.exp(-gu[c])) * gu[f + c] for c in range(f)]
            nx.append([a + b for a, b in zip(r, py_matvec(w["w_down"], act))])
        x = nx
        ks.append(kc)
        vs.append(vc)
    return x, ks, vs


def tiny_model(seed=0, n_layers=2, d=8, hq=2, hkv=1, dim=4, f=6, theta=100.0):
    shape = O.Shape(n_layers, d, hq, hkv, dim, f, 1e-5, theta)
    layers, plain = [], []
    for l in range(n_layers):
        w = dict(attn_norm=1.0 + rnd(d, seed=seed + 10 * l + 1, std=0.2),
                 w_qkv=rnd((hq + 2 * hkv) * dim, d, seed=seed + 10 * l + 2, std=0.4),
                 w_o=rnd(d, hq * dim, seed=seed + 10 * l + 3, std=0.4),
                 mlp_norm=1.0 + rnd(d, seed=seed + 10 * l + 4, std=0.2),
                 w_gate_up=rnd(2 * f, d, seed=seed + 10 * l + 5, std=0.4),
                 w_down=rnd(d, f, seed=seed + 10 * l + 6, std=0.4))
        layers.append(O.LayerWeights(**w))
        plain.append({k: v.tolist() for k, v in w.items()})
    return shape, layers, plain


# ---------------------------------------------------------------------------------------------
# attention
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n,cached,hq,hkv,dim", [(7, 0, 4, 2, 8), (5, 6, 2, 2, 4), (1, 0, 4, 1, 2),
                                                 (12, 3, 6, 2, 6)])
def test_attention_matches_bruteforce_loops(n, cached, hq, hkv, dim):
    m = cached + n
    q, k, v = rnd(n, hq, dim, seed=1), rnd(m, hkv, dim, seed=2), rnd(m, hkv, dim, seed=3)
    pos = torch.arange(cached, m)
    got = O.causal_attention(q, k, v, pos)
    want = torch.tensor(py_attention(q.tolist(), k.tolist(), v.tolist(), pos.tolist(), hq, hkv, dim),
                        dtype=F64)
    assert torch.allclose(got, want, rtol=0, atol=1e-13)


def test_softmax_rows_sum_to_one_and_are_causal():
    n, cached = 9, 4
    q, k = rnd(n, 2, 8, seed=4), rnd(n + cached, 1, 8, seed=5)
    pos = torch.arange(cached, cached + n)
    p = O.attention_probabilities(q, k, pos, q_head=1, kv_head=0)
    assert torch.allclose(p.sum(dim=-1), torch.ones(n, dtype=F64), atol=1e-14)
    for i in range(n):
        assert torch.all(p[i, cached + i + 1:] == 0)
        assert torch.all(p[i, :cached + i + 1] > 0)


def test_single_token_returns_its_value():
    q, k, v = rnd(1, 4, 8, seed=6), rnd(1, 2, 8, seed=7), rnd(1, 2, 8, seed=8)
    o = O.causal_attention(q, k, v, torch.tensor([0]))
    for h in range(4):
        assert torch.equal(o[0, h], v[0, h // 2])


def test_equal_keys_give_running_mean_of_values():
    n, dim = 10, 4
    q = rnd(n, 2, dim, seed=9)
    k = rnd(1, 1, dim, seed=10).expand(n, 1, dim).clone()
    v = rnd(n, 1, dim, seed=11)
    o = O.causal_attention(q, k, v, torch.arange(n))
    for i in range(n):
        mean = v[: i + 1, 0].mean(dim=0)
        assert torch.allclose(o[i, 0], mean, atol=1e-14)
        assert torch.allclose(o[i, 1], mean, atol=1e-14)


def test_gqa_equals_mha_with_repeated_kv_heads():
    n, hq, hkv, dim = 8, 6, 2, 4
    q, k, v = rnd(n, hq, dim, seed=12), rnd(n, hkv, dim, seed=13), rnd(n, hkv, dim, seed=14)
    pos = torch.arange(n)
    got = O.causal_attention(q, k, v, pos)
    k_rep = k.repeat_interleave(hq // hkv, dim=1)
    v_rep = v.repeat_interleave(hq // hkv, dim=1)
    want = O.causal_attention(q, k_rep, v_rep, pos)
    assert torch.allclose(got, want, atol=1e-14)
    # consecutive grouping, not strided: head 1 must use kv head 0, head 3 kv head 1
    alt = O.causal_attention(q, k.repeat(1, hq // hkv, 1), v.repeat(1, hq // hkv, 1), pos)
    assert not torch.allclose(got, alt, atol=1e-6)


def test_scale_is_inverse_sqrt_head_dim():
    # two keys, one query, D = 4: weights are softmax([q.k0, q.k1] / 2)
    q = torch.tensor([[[1.0, 2.0, 0.0, -1.0]]], dtype=F64)
    k = torch.tensor([[[1.0, 0.0, 0.0, 0.0]], [[0.0, 1.0, 0.0, 1.0]]], dtype=F64)
    v = torch.tensor([[[1.0, 0.0, 0.0, 0.0]], [[0.0, 1.0, 0.0, 0.0]]], dtype=F64)
    o = O.causal_attention(q, k, v, torch.tensor([1]))
    s0, s1 = 1.0 / 2.0, (2.0 - 1.0) / 2.0
    w0 = math.exp(s0) / (math.exp(s0) + math.exp(s1))
    assert abs(o[0, 0, 0].item() - w0) < 1e-15 and abs(o[0, 0, 1].item() - (1 - w0)) < 1e-15


# ---------------------------------------------------------------------------------------------
# RoPE, RMSNorm, SiLU, linear
# ---------------------------------------------------------------------------------------------

def test_rope_is_a_plane_rotation_for_two_dims():
    u = torch.tensor([[[3.0, 4.0]]], dtype=F64)
    out = O.rope_rotate(u, torch.tensor([5]), theta=10000.0)   # j = 0 -> angle = p
    c, s = math.cos(5.0), math.sin(5.0)
    assert abs(out[0, 0, 0].item() - (3 * c - 4 * s)) < 1e-14
    assert abs(out[0, 0, 1].item() - (4 * c + 3 * s)) < 1e-14


def test_rope_pairs_half_split_and_uses_theta_power():
    dim, theta, p = 8, 50.0, 11
    u = rnd(3, 2, dim, seed=15)
    out = O.rope_rotate(u, torch.tensor([p, p + 1, 0]), theta)
    for t, pos in enumerate([p, p + 1, 0]):
        for h in range(2):
            want = py_rope(u[t, h].tolist(), pos, theta)
            assert torch.allclose(out[t, h], torch.tensor(want, dtype=F64), atol=1e-14)
    assert torch.equal(out[2], u[2])                            # position 0 is the identity


def test_rope_preserves_norm_and_depends_on_relative_position():
    dim, theta = 16, 1000.0
    q, k = rnd(1, 1, dim, seed=16), rnd(1, 1, dim, seed=17)
    def dot(m, n):
        a = O.rope_rotate(q, torch.tensor([m]), theta)
        b = O.rope_rotate(k, torch.tensor([n]), theta)
        return (a * b).sum().item()
    assert abs(dot(7, 3) - dot(104, 100)) < 1e-12
    assert abs(dot(7, 3) - dot(3, 7)) > 1e-6
    r = O.rope_rotate(q, torch.tensor([12345]), theta)
    assert abs(r.norm().item() - q.norm().item()) < 1e-12


def test_rmsnorm_closed_form_and_invariances():
    out = O.rmsnorm(torch.tensor([[3.0, 4.0]], dtype=F64), torch.tensor([2.0, 0.5], dtype=F64), 0.5)
    denom = math.sqrt(12.5 + 0.5)
    assert torch.allclose(out, torch.tensor([[3.0 * 2.0 / denom, 4.0 * 0.5 / denom]], dtype=F64),
                          atol=1e-15)
    x = rnd(5, 32, seed=18)
    ones = torch.ones(32, dtype=F64)
    y = O.rmsnorm(x, ones, 0.0)
    assert torch.allclose((y * y).mean(dim=-1), torch.ones(5, dtype=F64), atol=1e-14)
    assert torch.allclose(O.rmsnorm(3.7 * x, ones, 0.0), y, atol=1e-14)
    for r in range(5):
        want = py_rmsnorm(x[r].tolist(), [1.0] * 32, 1e-5)
        assert torch.allclose(O.rmsnorm(x, ones, 1e-5)[r], torch.tensor(want, dtype=F64), atol=1e-14)


def test_silu_mul_values_and_column_order():
    gu = torch.tensor([[0.0, 1.0, 40.0, -40.0, 5.0, 2.0, 3.0, 7.0]], dtype=F64)   # gate | up
    out = O.silu_mul(gu)
    assert out[0, 0].item() == 0.0
    assert abs(out[0, 1].item() - 2.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(out[0, 2].item() - 40.0 * 3.0) < 1e-12
    assert abs(out[0, 3].item()) < 1e-14


def test_linear_is_x_times_w_transposed():
    x, w = rnd(3, 5, seed=19), rnd(4, 5, seed=20)
    got = O.linear(x, w)
    assert got.shape == (3, 4)
    for i in range(3):
        want = py_matvec(w.tolist(), x[i].tolist())
        assert torch.allclose(got[i], torch.tensor(want, dtype=F64), atol=1e-14)


# ---------------------------------------------------------------------------------------------
# whole stack
# ---------------------------------------------------------------------------------------------

def test_whole_stack_matches_scalar_python_transcription():
    shape, layers, plain = tiny_model(seed=100)
    x = rnd(5, shape.hidden, seed=21)
    got, cache = O.prefill(shape, layers, x, [0, 5])
    want, ks, vs = py_prefill(shape, plain, x.tolist())
    assert torch.allclose(got, torch.tensor(want, dtype=F64), atol=1e-12)
    for l in range(shape.n_layers):
        assert torch.allclose(cache.k[l][0], torch.tensor(ks[l], dtype=F64), atol=1e-12)
        assert torch.allclose(cache.v[l][0], torch.tensor(vs[l], dtype=F64), atol=1e-12)


def test_whole_stack_with_cached_prefix_matches_scalar_python():
    shape, layers, plain = tiny_model(seed=200, hq=4, hkv=2, dim=2, d=6, f=5)
    x = rnd(7, shape.hidden, seed=22)
    _, ks, vs = py_prefill(shape, plain, x[:3].tolist())
    want, _, _ = py_prefill(shape, plain, x[3:].tolist(), ks, vs)
    _, cache = O.prefill(shape, layers, x[:3], [0, 3])
    got, _ = O.prefill(shape, layers, x[3:], [0, 4], cache)
    assert torch.allclose(got, torch.tensor(want, dtype=F64), atol=1e-12)


def test_zero_output_weights_leave_residual_untouched():
    shape, layers, _ = tiny_model(seed=300)
    for w in layers:
        w.w_o = torch.zeros_like(w.w_o)
        w.w_down = torch.zeros_like(w.w_down)
    x = rnd(6, shape.hidden, seed=23)
    got, _ = O.prefill(shape, layers, x, [0, 6])
    assert torch.equal(got, x)


def test_zero_gate_weights_remove_mlp_contribution():
    shape, layers, _ = tiny_model(seed=400, n_layers=1)
    x = rnd(4, shape.hidden, seed=24)
    w = layers[0]
    full, _ = O.prefill(shape, layers, x, [0, 4])
    f = shape.ffn
    w.w_gate_up = torch.cat([torch.zeros(f, shape.hidden, dtype=F64), w.w_gate_up[f:]], dim=0)
    no_gate, _ = O.prefill(shape, layers, x, [0, 4])
    w.w_down = torch.zeros_like(w.w_down)
    attn_only, _ = O.prefill(shape, layers, x, [0, 4])
    assert torch.allclose(no_gate, attn_only, atol=1e-15)
    assert not torch.allclose(full, attn_only, atol=1e-6)


def test_causality_prefix_unchanged_when_suffix_appended():
    shape, layers, _ = tiny_model(seed=500)
    x = rnd(12, shape.hidden, seed=25)
    short, c_short = O.prefill(shape, layers, x[:7], [0, 7])
    full, c_full = O.prefill(shape, layers, x, [0, 12])
    # library matmuls of different heights may reassociate: allow rounding-level slack only
    assert torch.allclose(full[:7], short, rtol=0, atol=1e-13)
    for l in range(shape.n_layers):
        assert torch.allclose(c_full.k[l][0][:7], c_short.k[l][0], rtol=0, atol=1e-13)
        assert torch.allclose(c_full.v[l][0][:7], c_short.v[l][0], rtol=0, atol=1e-13)


@pytest.mark.parametrize("chunk", [1, 3, 7, 11, 64])
def test_chunked_prefill_with_cache_equals_one_shot(chunk):
    shape, layers, _ = tiny_model(seed=600, hq=4, hkv=2, dim=4, d=16, f=12)
    x = rnd(11, shape.hidden, seed=26)
    one, c_one = O.prefill(shape, layers, x, [0, 11])
    chk, c_chk = O.prefill_chunked(shape, layers, x, chunk)
    assert torch.allclose(one, chk, rtol=0, atol=1e-12)
    for l in range(shape.n_layers):
        assert torch.allclose(c_one.k[l][0], c_chk.k[l][0], rtol=0, atol=1e-12)
        assert torch.allclose(c_one.v[l][0], c_chk.v[l][0], rtol=0, atol=1e-12)


def test_packed_batch_equals_sequences_alone_and_permutes():
    shape, layers, _ = tiny_model(seed=700)
    lens = [3, 6, 1, 5]
    xs = [rnd(n, shape.hidden, seed=30 + i) for i, n in enumerate(lens)]
    cu = [0, 3, 9, 10, 15]
    packed, cache = O.prefill(shape, layers, torch.cat(xs), cu)
    for s, xseq in enumerate(xs):
        alone, c_alone = O.prefill(shape, layers, xseq, [0, lens[s]])
        assert torch.allclose(packed[cu[s]:cu[s + 1]], alone, rtol=0, atol=1e-13)
        assert torch.allclose(cache.k[1][s], c_alone.k[1][0], rtol=0, atol=1e-13)
    order = [2, 0, 3, 1]
    cu2 = [0]
    for s in order:
        cu2.append(cu2[-1] + lens[s])
    permuted, _ = O.prefill(shape, layers, torch.cat([xs[s] for s in order]), cu2)
    for i, s in enumerate(order):
        assert torch.allclose(permuted[cu2[i]:cu2[i + 1]], packed[cu[s]:cu[s + 1]], rtol=0, atol=1e-13)


def test_sampled_rows_equal_full_layer():
    shape, layers, _ = tiny_model(seed=800, n_layers=1, hq=4, hkv=2, dim=4, d=16, f=10)
    cu = [0, 5, 6, 14]
    x = rnd(14, shape.hidden, seed=40)
    full, k_l, v_l = O.layer_forward(shape, layers[0], x, cu,
                                     *[[torch.zeros((0, 2, 4), dtype=F64)] * 3] * 2)
    rows = [0, 4, 5, 9, 13]
    k_rot, v_raw, out = O.layer_sampled_rows(shape, layers[0], x, cu, rows)
    assert torch.allclose(out, full[rows], rtol=0, atol=1e-13)
    assert torch.allclose(k_rot, torch.cat(k_l), rtol=0, atol=1e-13)
    assert torch.allclose(v_raw, torch.cat(v_l), rtol=0, atol=1e-13)


# ---------------------------------------------------------------------------------------------
# Mixture-of-experts FFN (Section 7): pins of the oracle's router + experts.
# ---------------------------------------------------------------------------------------------
def _moe_inputs(n=9, d=8, f=6, e=4, seed=70):
    g = torch.Generator().manual_seed(seed)
    h = torch.randn((n, d), generator=g, dtype=torch.float64)
    wr = torch.randn((e, d), generator=g, dtype=torch.float64)
    wgu = torch.randn((e, 2 * f, d), generator=g, dtype=torch.float64) * 0.5
    wd = torch.randn((e, d, f), generator=g, dtype=torch.float64) * 0.5
    return h, wr, wgu, wd


def test_moe_identical_experts_equal_the_dense_ffn():
    h, wr, wgu, wd = _moe_inputs()
    wgu[:] = wgu[0]
    wd[:] = wd[0]
    dense = O.linear(O.silu_mul(O.linear(h, wgu[0])), wd[0])
    for k in (1, 2, 4):
        assert torch.allclose(O.moe_mlp(h, wr, wgu, wd, k), dense, rtol=1e-12, atol=1e-12)


def test_moe_top_k_equal_to_all_experts_is_the_softmax_weighted_sum():
    h, wr, wgu, wd = _moe_inputs()
    prob = torch.softmax(h @ wr.T, dim=-1)
    want = sum(prob[:, e:e + 1] * O.linear(O.silu_mul(O.linear(h, wgu[e])), wd[e]) for e in range(4))
    assert torch.allclose(O.moe_mlp(h, wr, wgu, wd, 4), want, rtol=1e-12, atol=1e-12)


def test_moe_one_hot_router_selects_that_expert_alone():
    h, wr, wgu, wd = _moe_inputs()
    h = h.abs() + 0.1                               # positive features so one row of W_r dominates
    wr = torch.zeros_like(wr)
    wr[2] = 50.0
    want = O.linear(O.silu_mul(O.linear(h, wgu[2])), wd[2])
    assert torch.allclose(O.moe_mlp(h, wr, wgu, wd, 1), want, rtol=1e-12, atol=1e-12)
    ids, wts = O.moe_route(h, wr, 1)
    assert (ids == 2).all() and torch.allclose(wts, torch.ones_like(wts))


def test_moe_matches_python_loops_on_tiny_inputs():
    h, wr, wgu, wd = _moe_inputs(n=5, d=4, f=3, e=4, seed=71)
    k = 2
    got = O.moe_mlp(h, wr, wgu, wd, k)
    ids, wts = O.moe_route(h, wr, k)
    for t in range(h.shape[0]):
        logits = [sum(float(h[t, c]) * float(wr[e, c]) for c in range(4)) for e in range(4)]
        mx = max(logits)
        ex = [math.exp(v - mx) for v in logits]
        prob = [v / sum(ex) for v in ex]
        order = sorted(range(4), key=lambda e: (-prob[e], e))[:k]
        assert [int(i) for i in ids[t]] == order
        norm = sum(prob[e] for e in order)
        want = [0.0] * 4
        for e in order:
            gu = [sum(float(h[t, c]) * float(wgu[e, r, c]) for c in range(4)) for r in range(6)]
            act = [gu[r] / (1.0 + math.exp(-gu[r])) * gu[3 + r] for r in range(3)]
            y = [sum(act[r] * float(wd[e, c, r]) for r in range(3)) for c in range(4)]
            want = [want[c] + prob[e] / norm * y[c] for c in range(4)]
        assert torch.allclose(got[t], torch.tensor(want, dtype=torch.float64), rtol=1e-10, atol=1e-12)
        assert abs(float(wts[t].sum()) - 1.0) < 1e-12 and len(set(order)) == k


def test_moe_forcing_the_oracles_own_selection_changes_nothing():
    h, wr, wgu, wd = _moe_inputs()
    ids, wts = O.moe_route(h, wr, 2)
    assert torch.allclose(O.moe_mlp(h, wr, wgu, wd, 2, forced_ids=ids), O.moe_mlp(h, wr, wgu, wd, 2), rtol=1e-13, atol=1e-13)
    assert torch.allclose(O.moe_weights_for(h, wr, ids), wts, rtol=1e-13, atol=1e-13)
    assert float(O.moe_selection_shortfall(h, wr, ids, 2).max()) == 0.0
    worse = ids.clone()
    worse[:, 1] = torch.tensor([[e for e in range(4) if e not in row.tolist()][0] for row in ids])   # swap in an unselected expert
    assert float(O.moe_selection_shortfall(h, wr, worse, 2).min()) > 0.0


def test_moe_shortfall_and_weights_closed_form():
    """A one-hot activation makes the router logits a column of W_r, so the probabilities, the
    renormalised weights of any expert set and the shortfall of a set that misses the k-th
    expert are all hand-computable: p = softmax(l); weights = p[ids] / sum p[ids]; shortfall =
    p_(k) - min p[ids] (Section 7: the `gate` operator; reading: softmax over all experts, then
    top-k, then renormalise)."""
    import math
    logits = [0.3, 2.0, -1.0, 1.5, 0.9, -0.2]                # experts sorted by p: 1, 3, 4, 0, 5, 2
    h = torch.zeros((1, 4), dtype=torch.float64)
    h[0, 2] = 1.0
    wr = torch.zeros((6, 4), dtype=torch.float64)
    wr[:, 2] = torch.tensor(logits, dtype=torch.float64)
    z = sum(math.exp(v) for v in logits)
    p = [math.exp(v) / z for v in logits]
    ids, wts = O.moe_route(h, wr, 3)
    assert ids.tolist() == [[1, 3, 4]]
    s3 = p[1] + p[3] + p[4]
    assert wts[0].tolist() == pytest.approx([p[1] / s3, p[3] / s3, p[4] / s3], rel=1e-14)
    # expert 0 (4th) instead of expert 4 (3rd): not a top-3 set; the shortfall is p_(3) - p[0]
    other = torch.tensor([[3, 0, 1]])
    assert float(O.moe_selection_shortfall(h, wr, other, 3)[0]) == pytest.approx(p[4] - p[0], rel=1e-13)
    assert float(O.moe_selection_shortfall(h, wr, other, 3, relative=True)[0]) == pytest.approx(1.0 - p[0] / p[4], rel=1e-12)
    so = p[3] + p[0] + p[1]
    assert O.moe_weights_for(h, wr, other)[0].tolist() == pytest.approx([p[3] / so, p[0] / so, p[1] / so], rel=1e-14)
    # any ordering of a true top-3 set has no shortfall
    assert float(O.moe_selection_shortfall(h, wr, torch.tensor([[4, 1, 3]]), 3)[0]) == 0.0
