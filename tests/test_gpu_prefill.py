"""End-to-end parity of the HIP prefill path (through the C ABI) against the CPU oracle on the
same seeded inputs: final residual stream and every layer's K (rotated) and V, element by
element; plus the GPU-side invariants (chunked == one-shot, packed == alone, any block-table
permutation)."""
import numpy as np
import pytest
import torch

from oracle import prefill_oracle as O
from paper_2602_16603_amd import inputs as I
from tests.util import TOL, fro_rel_err, max_rel_err, oracle_layers, oracle_shape

pytestmark = pytest.mark.gpu

DT = {"fp32": (0, torch.float32), "bf16": (1, torch.bfloat16)}


def _runner():
    from paper_2602_16603_amd import runner
    return runner


def build(spec, seed, name, pool_blocks=None, max_position=None, total_tokens=0, random_gains=False):
    R = _runner()
    code, td = DT[name]
    weights = I.make_weights(spec, seed, td, "cpu")
    if random_gains:
        I.randomize_gains(weights, seed)
    pool_blocks = pool_blocks or (total_tokens // 16 + 64)
    model = R.PrefillModel(spec, weights, code, pool_blocks, max_position or max(total_tokens, 16))
    return model, weights


def check_against_oracle(spec, weights, hidden_cpu, lengths, task, name, cache=None):
    x_ref, cache_ref = O.prefill(oracle_shape(spec), oracle_layers(weights), hidden_cpu,
                                 I.cu_seqlens_of(lengths), cache)
    tol = TOL[name]
    got = task.hidden()
    e = max_rel_err(got, x_ref)
    print(f"  hidden: E={e:.3e} fro={fro_rel_err(got, x_ref):.3e}", flush=True)
    assert e <= tol, f"hidden states off by {e}"
    for layer in range(spec.n_layers):
        for s in range(len(lengths)):
            k, v = task.kv(layer, s)
            ek = max_rel_err(k, cache_ref.k[layer][s])
            ev = max_rel_err(v, cache_ref.v[layer][s])
            assert ek <= tol and ev <= tol, f"layer {layer} seq {s}: K {ek} V {ev}"
    return cache_ref


@pytest.mark.parametrize("name", ["fp32", "bf16"])
def test_cfg1_tiny_prompt(name):
    """cfg1: 2 layers, hidden 256, 4/2 heads of 64, FFN 704, one 256-token prompt."""
    cfg = I.CONFIGS["cfg1"]
    spec, n = cfg["shape"], cfg["lengths"][0]
    model, weights = build(spec, cfg["seed"], name, total_tokens=n)
    hidden = I.make_hidden(n, spec.hidden, cfg["seed"], DT[name][1], "cpu")
    task = model.begin(hidden.cuda(), [n])
    task.run_to_completion()
    assert task.cursor() == (spec.n_layers, 0)
    check_against_oracle(spec, weights, hidden, [n], task, name)
    task.end()
    model.close()


@pytest.mark.parametrize("name", ["fp32", "bf16"])
def test_ragged_packed_batch_with_permuted_blocks_and_random_gains(name):
    """Packed varlen batch (lengths straddle the 16-token block, the 64-key tile and the
    256-row query tile), block table = seeded permutation of the pool, norm gains != 1."""
    spec = I.TINY
    lengths = [1, 300, 17, 64, 0, 255, 513, 16]
    total = sum(lengths)
    model, weights = build(spec, 21, name, pool_blocks=256, max_position=1024, random_gains=True)
    hidden = I.make_hidden(total, spec.hidden, 21, DT[name][1], "cpu")
    table, _ = I.permuted_block_tables(lengths, None, 16, 256, seed=5)
    task = model.begin(hidden.cuda(), lengths, cached=[0] * len(lengths), block_tables=table)
    task.run_to_completion()
    check_against_oracle(spec, weights, hidden, lengths, task, name)
    # Same batch with library-allocated (identity-ordered) blocks must give the same bits.
    task2 = model.begin(hidden.cuda(), lengths)
    task2.run_to_completion()
    assert torch.equal(task.hidden(), task2.hidden())
    task.end()
    task2.end()
    model.close()


@pytest.mark.parametrize("name", ["fp32", "bf16"])
@pytest.mark.parametrize("chunk", [16, 100, 257])
def test_chunked_prefill_reads_cached_prefix(name, chunk):
    """A prompt run chunk by chunk, every chunk attending to the KV its predecessors left in the
    paged cache (Section 3.1), equals the oracle's one-shot prefill."""
    spec = I.TINY
    n = 600
    model, weights = build(spec, 22, name, pool_blocks=64, max_position=n, random_gains=True)
    hidden = I.make_hidden(n, spec.hidden, 22, DT[name][1], "cpu")
    x_ref, cache_ref = O.prefill(oracle_shape(spec), oracle_layers(weights), hidden, [0, n])
    from paper_2602_16603_amd import binding as B
    blocks = B.fp_kv_alloc(model.handle, (n + 15) // 16)
    table = np.asarray(blocks, dtype=np.int32).reshape(1, -1)
    outs, last = [], None
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        task = model.begin(hidden[lo:hi].contiguous().cuda(), [hi - lo], cached=[lo],
                           block_tables=table, boundary_mask=B.FP_BOUNDARY_NONE)
        task.run_to_completion()
        outs.append(task.hidden())
        if last is not None:
            last.end()
        last = task
    got = torch.cat(outs)
    assert max_rel_err(got, x_ref) <= TOL[name]
    for layer in range(spec.n_layers):
        k, v = last.kv(layer, 0)
        assert max_rel_err(k, cache_ref.k[layer][0]) <= TOL[name]
        assert max_rel_err(v, cache_ref.v[layer][0]) <= TOL[name]
    last.end()
    B.fp_kv_free(model.handle, blocks)
    model.close()


def test_8b_head_shapes_small_twin_bf16():
    """Llama-3-8B head/hidden/FFN shapes, 2 layers, ragged lengths (shrunken twin of cfg2/cfg3):
    exercises head_dim 128, GQA 32/8, K = 14336 and the 256x256 GEMM tiles."""
    spec = I.LLAMA3_8B.with_layers(2)
    lengths = [700, 130, 333]
    total = sum(lengths)
    model, weights = build(spec, 23, "bf16", total_tokens=total, max_position=1024)
    hidden = I.make_hidden(total, spec.hidden, 23, torch.bfloat16, "cpu")
    task = model.begin(hidden.cuda(), lengths)
    task.run_to_completion()
    check_against_oracle(spec, weights, hidden, lengths, task, "bf16")
    task.end()
    model.close()


@pytest.mark.parametrize("lengths", [[128], [512, 40], [1024]])
def test_short_requests_8b_shape_use_split_k(lengths):
    """The 128..1024-token requests of the preemption workload: too few output tiles to fill the
    chip, so the projections run on the 128-column tile (up to 512 tokens), are split over K and
    reduced in a fixed order by kernels that also carry the small operator that follows."""
    spec = I.LLAMA3_8B.with_layers(1)
    total = sum(lengths)
    model, weights = build(spec, 26, "bf16", total_tokens=total, max_position=1024)
    hidden = I.make_hidden(total, spec.hidden, 26, torch.bfloat16, "cpu")
    task = model.begin(hidden.cuda(), lengths)
    task.run_to_completion()
    check_against_oracle(spec, weights, hidden, lengths, task, "bf16")
    again = model.begin(hidden.cuda(), lengths)          # fixed reduction order: same bits every run
    again.run_to_completion()
    assert torch.equal(task.hidden(), again.hidden())
    task.end()
    again.end()
    model.close()


def test_packed_equals_alone_on_gpu_bf16():
    spec = I.TINY
    lengths = [90, 270, 33]
    model, _ = build(spec, 24, "bf16", pool_blocks=128, max_position=512)
    hidden = I.make_hidden(sum(lengths), spec.hidden, 24, torch.bfloat16, "cuda")
    packed = model.begin(hidden, lengths)
    packed.run_to_completion()
    out = packed.hidden()
    cu = I.cu_seqlens_of(lengths)
    for s, n in enumerate(lengths):
        alone = model.begin(hidden[cu[s]:cu[s + 1]].contiguous(), [n])
        alone.run_to_completion()
        # different M changes no per-row arithmetic order in these kernels: bit-equal
        assert torch.equal(alone.hidden(), out[cu[s]:cu[s + 1]])
        alone.end()
    packed.end()
    model.close()


def test_empty_batch_and_invalid_arguments():
    from paper_2602_16603_amd import binding as B
    spec = I.TINY
    model, _ = build(spec, 25, "bf16", pool_blocks=8, max_position=64)
    hidden = I.make_hidden(16, spec.hidden, 25, torch.bfloat16, "cuda")
    empty = model.begin(hidden[:0].contiguous(), [0])
    st, _ = empty.advance()
    assert st == B.FP_DONE
    empty.end()
    with pytest.raises(B.FlowPrefillError):          # beyond max_position
        model.begin(I.make_hidden(80, spec.hidden, 1, torch.bfloat16, "cuda"), [80])
    with pytest.raises(B.FlowPrefillError):          # pool exhausted (8 blocks = 128 tokens)
        a = model.begin(I.make_hidden(64, spec.hidden, 1, torch.bfloat16, "cuda"), [64])
        b = model.begin(I.make_hidden(64, spec.hidden, 1, torch.bfloat16, "cuda"), [64])
        try:
            model.begin(I.make_hidden(16, spec.hidden, 1, torch.bfloat16, "cuda"), [16])
        finally:
            a.end()
            b.end()
    with pytest.raises(B.FlowPrefillError):          # block id outside the pool
        model.begin(hidden, [16], cached=[0], block_tables=np.array([[99]], dtype=np.int32))
    model.close()
