"""Operator-boundary preemption on the GPU (FlowPrefill Section 5.1): a task parked at any
boundary, with another request run in between, resumes to a result that is bit-identical to an
uninterrupted run; a signal raised from another thread is acknowledged at a boundary."""
import threading
import time

import pytest
import torch

from paper_2602_16603_amd import inputs as I

pytestmark = pytest.mark.gpu


def _mods():
    from paper_2602_16603_amd import binding, runner
    return binding, runner


def _snapshot(task, spec):
    out = [task.hidden()]
    for layer in range(spec.n_layers):
        for s in range(len(task.lengths)):
            out.extend(task.kv(layer, s))
    return out


def _same(a, b):
    return len(a) == len(b) and all(torch.equal(x, y) for x, y in zip(a, b))


def _sweep(spec, lengths, short_len, seed, pool_blocks, device_weights=False):
    B, R = _mods()
    where = "cuda" if device_weights else "cpu"
    weights = I.make_weights(spec, seed, torch.bfloat16, where)
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, pool_blocks, max(max(lengths), short_len))
    hidden = I.make_hidden(sum(lengths), spec.hidden, seed, torch.bfloat16, "cuda")
    short = I.make_hidden(short_len, spec.hidden, seed + 1, torch.bfloat16, "cuda")

    base = model.begin(hidden, lengths)
    base.run_to_completion()
    want = _snapshot(base, spec)
    base.end()
    again = model.begin(hidden, lengths)            # determinism of the uninterrupted run itself
    again.run_to_completion()
    assert _same(_snapshot(again, spec), want)
    again.end()

    total_ops = spec.n_layers * B.FP_OPS_PER_LAYER
    for boundary in range(total_ops):
        print(f"  preempt before op {boundary}", flush=True)
        task = model.begin(hidden, lengths)
        if boundary:
            st, done = task.advance(boundary)
            assert st == B.FP_OK and done == boundary
        assert task.cursor() == (boundary // 9, boundary % 9)
        assert task.preempt() == B.FP_PREEMPTED
        with pytest.raises(B.FlowPrefillError):      # a parked task does not advance
            task.advance()
        other = model.begin(short, [short_len])      # the higher-priority request runs meanwhile
        other.run_to_completion()
        other.end()
        task.resume()
        task.run_to_completion()
        assert _same(_snapshot(task, spec), want), f"resume after boundary {boundary} differs"
        task.end()
    model.close()


def test_resume_is_bit_identical_at_every_boundary_tiny():
    _sweep(I.TINY, [300, 77], 50, seed=31, pool_blocks=64)


def test_resume_is_bit_identical_at_every_boundary_cfg2():
    """cfg2: Llama-3-8B-shaped 4-layer stack, one 8192-token prompt, a preempt injected at each
    of the 36 operator boundaries in turn, a 512-token request served in between."""
    cfg = I.CONFIGS["cfg2"]
    _sweep(cfg["shape"], cfg["lengths"], 512, seed=cfg["seed"], pool_blocks=8192 // 16 + 64,
           device_weights=True)


def test_signal_from_another_thread_parks_at_a_boundary():
    B, R = _mods()
    spec = I.LLAMA3_8B.with_layers(2)
    n = 2048
    weights = I.make_weights(spec, 33, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, n // 16 + 8, n)
    hidden = I.make_hidden(n, spec.hidden, 33, torch.bfloat16, "cuda")
    base = model.begin(hidden, [n])
    base.run_to_completion()
    want = _snapshot(base, spec)
    base.end()
    parked = 0
    for delay_ms in (0.0, 0.3, 1.0, 2.0, 4.0, 8.0):
        for mask in (B.FP_BOUNDARY_EVERY_OP, B.FP_BOUNDARY_PAPER_OPS, B.FP_BOUNDARY_LAYER):
            task = model.begin(hidden, [n], boundary_mask=mask)
            result = {}
            def work(task=task, result=result):
                try:
                    result["st"] = task.advance()[0]
                except B.FlowPrefillError as exc:       # parked before advance began
                    result["st"] = exc.status
            th = threading.Thread(target=work)
            th.start()
            time.sleep(delay_ms / 1e3)
            try:
                st = task.preempt()
            except B.FlowPrefillError:
                st = None                  # advance had not started yet or raced: not an error path we test
            th.join(30)
            assert not th.is_alive()
            if st == B.FP_PREEMPTED:
                parked += 1
                layer, op = task.cursor()
                if result.get("st") == B.FP_PREEMPTED and (layer, op) != (0, 0):
                    prev = (op - 1) % 9
                    assert (mask >> prev) & 1, f"parked after op {prev} not in mask {mask:#x}"
                task.resume()
                task.run_to_completion()
            elif st == B.FP_DONE:
                assert result.get("st") == B.FP_DONE
            else:
                task.run_to_completion() if task.cursor() != (spec.n_layers, 0) else None
            assert _same(_snapshot(task, spec), want)
            task.end()
    assert parked > 0
    model.close()


def test_state_errors():
    B, R = _mods()
    spec = I.TINY
    weights = I.make_weights(spec, 34, torch.bfloat16, "cpu")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, 16, 64)
    hidden = I.make_hidden(32, spec.hidden, 34, torch.bfloat16, "cuda")
    task = model.begin(hidden, [32])
    with pytest.raises(B.FlowPrefillError) as e:
        task.resume()                                   # not parked
    assert e.value.status == B.FP_ERR_STATE
    assert task.preempt() == B.FP_PREEMPTED             # idle task parks at once
    with pytest.raises(B.FlowPrefillError):
        task.preempt()                                  # already parked
    task.resume()
    task.run_to_completion()
    assert task.preempt() == B.FP_DONE                  # preempt racing with completion
    with pytest.raises(B.FlowPrefillError):
        task.advance()                                  # done
    task.end()
    model.close()


@pytest.mark.parametrize("ahead", [1, 2])
def test_blocking_time_is_bounded_by_launch_ahead_operators(ahead):
    """Section 5.1: with a check after every operator the wait for an acknowledgement is bounded by
    the operators already handed to the device -- launch_ahead of them (the host enqueues operator
    i only once operator i - launch_ahead has completed).  Signals raised at 16 different moments
    of a 2-layer 8B-shaped prefill of 8192 tokens; signal -> acknowledgement (device drained) must
    stay below launch_ahead x the slowest operator + 1 ms of host slack (thread wake-up, drain)."""
    B, R = _mods()
    spec = I.LLAMA3_8B.with_layers(2)
    n = 8192
    weights = I.make_weights(spec, 35, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, n // 16 + 8, n)
    hidden = I.make_hidden(n, spec.hidden, 35, torch.bfloat16, "cuda")
    for _ in range(2):                                   # warm-up, then a timed run for the operator times
        task = model.begin(hidden, [n])
        B.fp_prefill_set_timing(task.handle, True)
        task.run_to_completion()
        op_ms = B.fp_prefill_op_times(task.handle, spec.n_layers * 9)
        task.end()
    slowest_ms, total_ms = max(op_ms), sum(op_ms)
    bound_ms = ahead * slowest_ms + 1.0
    worst, parked = 0.0, 0
    for i in range(16):
        delay_ms = total_ms * (i + 0.5) / 18.0           # spread over the run, always before its end
        task = model.begin(hidden, [n])
        B.fp_prefill_set_launch_ahead(task.handle, ahead)
        th = threading.Thread(target=lambda t=task: t.advance())
        th.start()
        time.sleep(delay_ms / 1e3)
        t0 = time.perf_counter()
        st = B.fp_preempt_signal(task.handle)
        if st == B.FP_OK:
            st = B.fp_preempt_wait(task.handle)
        blocked_ms = (time.perf_counter() - t0) * 1e3
        th.join(30)
        assert not th.is_alive()
        if st == B.FP_PREEMPTED and task.cursor() != (0, 0):
            parked += 1
            worst = max(worst, blocked_ms)
            assert blocked_ms <= bound_ms, (f"signal {delay_ms:.2f} ms into the run: blocked {blocked_ms:.3f} ms "
                                            f"> {ahead} x {slowest_ms:.3f} ms + 1 ms")
        task.end()
    print(f"  launch_ahead {ahead}: {parked} preemptions, worst blocking {worst:.3f} ms, "
          f"slowest operator {slowest_ms:.3f} ms, bound {bound_ms:.3f} ms", flush=True)
    assert parked >= 8
    model.close()


def test_preserved_kv_state_is_addressable_through_the_block_tables():
    """fp_prefill_kv hands out what a preempted task preserves of its KV cache (Section 4): the
    layer's slice of the paged pools and the task's block tables.  Reading the pools through the
    tables reproduces fp_prefill_kv_gather for every position, key head and channel (keys
    [block][Hkv][16][D], values transposed inside the block [block][Hkv][D][16])."""
    B, R = _mods()
    spec = I.TINY
    lengths = [70, 0, 33]
    blocks = 24
    weights = I.make_weights(spec, 36, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, blocks, 128)
    hidden = I.make_hidden(sum(lengths), spec.hidden, 36, torch.bfloat16, "cuda")
    table, _ = I.permuted_block_tables(lengths, None, 16, blocks, seed=36)
    task = model.begin(hidden, lengths, cached=[0, 0, 0], block_tables=table)
    st, done = task.advance(9 + 3)                       # layer 0 complete, layer 1 through rope_kvwrite
    assert st == B.FP_OK and done == 12
    assert task.preempt() == B.FP_PREEMPTED
    per_layer = blocks * spec.n_kv_heads * 16 * spec.head_dim
    k_all, v_all = B.fp_model_kv_pools(model.handle)
    for layer in range(spec.n_layers):
        k_ptr, v_ptr, tables = task.kv_pools(layer)
        assert k_ptr == k_all + layer * per_layer * 2 and v_ptr == v_all + layer * per_layer * 2
        assert (tables == table).all()
        kp = R.copy_from_device_ptr(k_ptr, (blocks, spec.n_kv_heads, 16, spec.head_dim), torch.bfloat16)
        vp = R.copy_from_device_ptr(v_ptr, (blocks, spec.n_kv_heads, spec.head_dim, 16), torch.bfloat16)
        for s, n in enumerate(lengths):
            if n == 0:
                continue
            k_ref, v_ref = task.kv(layer, s)
            pos = torch.arange(n)
            blk = torch.as_tensor(tables[s], device="cuda").long()[pos // 16]
            k_got = kp[blk, :, pos % 16, :]                        # [n, Hkv, D]
            v_got = vp[blk, :, :, pos % 16]                        # [n, Hkv, D]
            assert torch.equal(k_got, k_ref) and torch.equal(v_got, v_ref)
    with pytest.raises(B.FlowPrefillError):
        task.kv_pools(spec.n_layers)
    task.resume()
    task.run_to_completion()
    task.end()
    model.close()


def test_model_destroy_is_refused_while_a_task_is_alive():
    B, R = _mods()
    spec = I.TINY
    weights = I.make_weights(spec, 37, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, 16, 64)
    hidden = I.make_hidden(32, spec.hidden, 37, torch.bfloat16, "cuda")
    task = model.begin(hidden, [32])
    B.fp_model_destroy(model.handle)                      # refused: the task's buffers live in the model
    assert "not ended" in B.fp_last_error()
    task.run_to_completion()                              # the model is still whole
    first = task.hidden()
    task.end()
    again = model.begin(hidden, [32])
    again.run_to_completion()
    assert torch.equal(again.hidden(), first)
    again.end()
    model.close()
