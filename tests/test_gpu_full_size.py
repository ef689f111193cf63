"""Parity at the benchmark's full size and on shrunken twins of the large configurations.

cfg2 (Llama-3-8B-shaped, 4 layers, one 8192-token prompt) is checked two ways in the launch
configuration bench.py times: (a) teacher-forced, one layer at a time -- the oracle is fed the
GPU's own input to layer l and must reproduce the layer's K and V for ALL tokens and the layer's
output for sampled token rows; (b) end to end against a full oracle run.  cfg3 and cfg5 are far
beyond what a CPU oracle finishes (hours to days), so they are covered by twins with the same
head / hidden / FFN shapes, fewer layers and shorter prompts, plus the teacher-forced check.
"""
import numpy as np
import pytest
import torch

from oracle import prefill_oracle as O
from paper_2602_16603_amd import inputs as I
from tests.util import TOL, floor_rel_err, fro_rel_err, max_rel_err, oracle_layers, oracle_shape

pytestmark = pytest.mark.gpu


def _mods():
    from paper_2602_16603_amd import binding, runner
    return binding, runner


# Bounds on the two stricter metrics that were only printed before (S12 of the readings: E is the
# gate; E_floor = max |g-r| / max(|r|, rms r) and the Frobenius ratio are asserted with about 2x
# head-room over what one layer / four layers of bf16-stored operators measure, so that a
# regression shows).  One teacher-forced layer: observed E_floor 0.8-2.5e-2, Frobenius 1.9-4.4e-3.
LAYER_E_FLOOR, LAYER_FRO = 5e-2, 8e-3
STACK4_E_FLOOR, STACK4_FRO = 1.2e-1, 1.5e-2      # four layers end to end: observed 5.5e-2, 7.9e-3


def _teacher_forced(spec, seed, lengths, layers_to_check, n_rows, block_tables=None, pool_blocks=None):
    B, R = _mods()
    total = sum(lengths)
    cu = I.cu_seqlens_of(lengths)
    weights = I.make_weights(spec, seed, torch.bfloat16, "cuda")
    pool = pool_blocks or (total // 16 + len(lengths) + 8)
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, pool, max(lengths))
    hidden = I.make_hidden(total, spec.hidden, seed, torch.bfloat16, "cuda")
    if block_tables is None:
        task = model.begin(hidden, lengths)
    else:
        task = model.begin(hidden, lengths, cached=[0] * len(lengths), block_tables=block_tables)
    rows = I.sample_rows(cu, n_rows, seed)
    shape1 = oracle_shape(spec.with_layers(1))
    for layer in range(spec.n_layers):
        x_in = task.hidden().cpu() if layer in layers_to_check else None
        st, done = task.advance(B.FP_OPS_PER_LAYER)
        assert done == B.FP_OPS_PER_LAYER
        if layer not in layers_to_check:
            continue
        print(f"  layer {layer}: oracle on {len(rows)} rows + all K/V", flush=True)
        w = oracle_layers([weights[layer]])[0]
        k_ref, v_ref, out_ref = O.layer_sampled_rows(shape1, w, x_in, cu, rows)
        x_out = task.hidden().cpu()
        e = max_rel_err(x_out[rows], out_ref)
        e_floor, fro = floor_rel_err(x_out[rows], out_ref), fro_rel_err(x_out[rows], out_ref)
        print(f"    rows: E={e:.3e} E_floor={e_floor:.3e} fro={fro:.3e}", flush=True)
        assert e <= TOL["bf16"]
        assert e_floor <= LAYER_E_FLOOR and fro <= LAYER_FRO
        for s in range(len(lengths)):
            k, v = task.kv(layer, s)
            assert max_rel_err(k, k_ref[cu[s]:cu[s + 1]]) <= TOL["bf16"]
            assert max_rel_err(v, v_ref[cu[s]:cu[s + 1]]) <= TOL["bf16"]
    assert task.cursor() == (spec.n_layers, 0)
    task.end()
    model.close()


def test_cfg2_full_size_teacher_forced_layers():
    cfg = I.CONFIGS["cfg2"]
    _teacher_forced(cfg["shape"], cfg["seed"], cfg["lengths"], layers_to_check={0, 2, 3}, n_rows=48)


def test_cfg2_full_size_end_to_end():
    """Whole cfg2 against a whole oracle run (about 20 TFLOP of fp64 on the host: ~1-2 minutes)."""
    B, R = _mods()
    cfg = I.CONFIGS["cfg2"]
    spec, seed, lengths = cfg["shape"], cfg["seed"], cfg["lengths"]
    n = lengths[0]
    weights = I.make_weights(spec, seed, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, n // 16 + 8, n)
    hidden = I.make_hidden(n, spec.hidden, seed, torch.bfloat16, "cuda")
    task = model.begin(hidden, lengths)
    task.run_to_completion()
    got = task.hidden().cpu()
    kv = [task.kv(layer, 0) for layer in range(spec.n_layers)]
    kv = [(k.cpu(), v.cpu()) for k, v in kv]
    task.end()
    model.close()
    print("  running the fp64 oracle on the full cfg2 ...", flush=True)
    x_ref, cache = O.prefill(oracle_shape(spec), oracle_layers(weights), hidden.cpu(), [0, n])
    e = max_rel_err(got, x_ref)
    e_floor, fro = floor_rel_err(got, x_ref), fro_rel_err(got, x_ref)
    print(f"  hidden: E={e:.3e} E_floor={e_floor:.3e} fro={fro:.3e}", flush=True)
    assert e <= TOL["bf16"]
    assert e_floor <= STACK4_E_FLOOR and fro <= STACK4_FRO
    for layer in range(spec.n_layers):
        assert max_rel_err(kv[layer][0], cache.k[layer][0]) <= TOL["bf16"]
        assert max_rel_err(kv[layer][1], cache.v[layer][0]) <= TOL["bf16"]


def test_cfg3_twin_lognormal_batch_paged():
    """cfg3's structure at 1/8 of its lengths and 2 of its 32 layers: 16 prompts with log-normal
    lengths packed with cu_seqlens, 16-token blocks drawn as a seeded permutation of the pool."""
    B, R = _mods()
    cfg = I.CONFIGS["cfg3"]
    spec = cfg["shape"].with_layers(2)
    lengths = [max(8, n // 8) for n in I.lognormal_lengths(16, cfg["seed"])]
    total = sum(lengths)
    pool = total // 16 + 64
    table, _ = I.permuted_block_tables(lengths, None, 16, pool, seed=cfg["seed"])
    weights = I.make_weights(spec, cfg["seed"], torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, pool, max(lengths))
    hidden = I.make_hidden(total, spec.hidden, cfg["seed"], torch.bfloat16, "cuda")
    task = model.begin(hidden, lengths, cached=[0] * 16, block_tables=table)
    task.run_to_completion()
    print(f"  lengths {lengths}", flush=True)
    x_ref, cache = O.prefill(oracle_shape(spec), oracle_layers(weights), hidden.cpu(),
                             I.cu_seqlens_of(lengths))
    got = task.hidden()
    e = max_rel_err(got, x_ref)
    print(f"  hidden: E={e:.3e} fro={fro_rel_err(got, x_ref):.3e}", flush=True)
    assert e <= TOL["bf16"]
    for layer in range(spec.n_layers):
        for s in range(16):
            k, v = task.kv(layer, s)
            assert max_rel_err(k, cache.k[layer][s]) <= TOL["bf16"]
            assert max_rel_err(v, cache.v[layer][s]) <= TOL["bf16"]
    task.end()
    model.close()


def test_cfg3_full_lengths_teacher_forced_one_layer():
    """cfg3's real prompt lengths (about 27k tokens in 16 prompts, longest up to 32768), one
    layer of the 8B shape, teacher-forced: K/V of all tokens and sampled output rows."""
    cfg = I.CONFIGS["cfg3"]
    lengths = I.lognormal_lengths(16, cfg["seed"])
    total = sum(lengths)
    pool = total // 16 + 64
    table, _ = I.permuted_block_tables(lengths, None, 16, pool, seed=cfg["seed"])
    _teacher_forced(cfg["shape"].with_layers(1), cfg["seed"], lengths, {0}, n_rows=64,
                    block_tables=table, pool_blocks=pool)


def test_cfg5_twin_qwen32b_shape():
    """cfg5's shape (hidden 5120, 40 query / 8 KV heads, FFN 27648, theta 1e6: five query heads
    per KV head) with one layer and its four prompt lengths divided by 32."""
    B, R = _mods()
    cfg = I.CONFIGS["cfg5"]
    spec = cfg["shape"].with_layers(1)
    lengths = [n // 32 for n in cfg["lengths"]]
    total = sum(lengths)
    weights = I.make_weights(spec, cfg["seed"], torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, total // 16 + 16, max(lengths))
    hidden = I.make_hidden(total, spec.hidden, cfg["seed"], torch.bfloat16, "cuda")
    task = model.begin(hidden, lengths)
    task.run_to_completion()
    x_ref, cache = O.prefill(oracle_shape(spec), oracle_layers(weights), hidden.cpu(),
                             I.cu_seqlens_of(lengths))
    got = task.hidden()
    e = max_rel_err(got, x_ref)
    print(f"  hidden: E={e:.3e} fro={fro_rel_err(got, x_ref):.3e}", flush=True)
    assert e <= TOL["bf16"]
    for s in range(len(lengths)):
        k, v = task.kv(0, s)
        assert max_rel_err(k, cache.k[0][s]) <= TOL["bf16"]
        assert max_rel_err(v, cache.v[0][s]) <= TOL["bf16"]
    task.end()
    model.close()


def test_cfg5_long_prompt_teacher_forced_one_layer():
    """One layer of the 32B shape on a single 65536-token prompt (cfg5's longest): K/V of all
    tokens and sampled output rows, including the last row, which attends to all 65536 keys."""
    cfg = I.CONFIGS["cfg5"]
    _teacher_forced(cfg["shape"].with_layers(1), cfg["seed"], [65536], {0}, n_rows=24)


# ---- parity at depth: the real 32- and 64-layer stacks, teacher-forced at layers 0, L/2, L-1 ----
# The oracle cannot run these stacks end to end (hours to days), so each checked layer is fed the
# GPU's own input to that layer -- whatever 16, 31, 32 or 63 layers of bf16-stored operators have
# made of the residual stream by then (its rms grows from 1 to about 10) -- and must reproduce the
# layer's K and V for all tokens and its output on sampled rows.

def test_cfg3_real_32_layer_batch_teacher_forced_at_depth():
    """cfg3 as BASELINE states it: the full 32-layer 8B stack on the 16 log-normal prompts (45712
    tokens), paged KV with a seeded permutation of the pool; layers 0, 16 and 31."""
    cfg = I.CONFIGS["cfg3"]
    lengths = I.lognormal_lengths(16, cfg["seed"])
    total = sum(lengths)
    pool = total // 16 + 64
    table, _ = I.permuted_block_tables(lengths, None, 16, pool, seed=cfg["seed"])
    _teacher_forced(cfg["shape"], cfg["seed"], lengths, {0, 16, 31}, n_rows=48,
                    block_tables=table, pool_blocks=pool)


def test_8b_32_layer_single_8192_token_prompt_teacher_forced_at_depth():
    """The benchmark's prompt (8192 tokens) through all 32 layers of the 8B shape; layers 0, 16, 31."""
    cfg = I.CONFIGS["cfg3"]
    _teacher_forced(cfg["shape"], 2, [8192], {0, 16, 31}, n_rows=48)


def test_cfg5_real_64_layer_stack_teacher_forced_at_depth():
    """The full 64-layer 32B-shaped stack (62 GB of weights in HBM) on cfg5's four prompts at one
    eighth of their lengths (8192 + 4096 + 2048 + 1024 tokens); layers 0, 32 and 63."""
    cfg = I.CONFIGS["cfg5"]
    lengths = [n // 8 for n in cfg["lengths"]]
    _teacher_forced(cfg["shape"], cfg["seed"], lengths, {0, 32, 63}, n_rows=48)
