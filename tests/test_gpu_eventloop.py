"""The event-driven driver on the real library (FlowPrefill Section 5.2 skeleton over Section
5.1's mechanism): short requests arriving while a long prompt runs preempt it at an operator
boundary, run, and the long prompt resumes -- to bit-identical results, both for one
operator-preemptible task and for operator-level checks inside chunks (Section 6.5)."""
import threading
import time

import pytest
import torch

from paper_2602_16603_amd import inputs as I
from tests.util import TOL, max_rel_err
from paper_2602_16603_amd.eventloop import EventLoop, MixedPool, Request, feed_arrivals

pytestmark = pytest.mark.gpu


def _mods():
    from paper_2602_16603_amd import binding, runner
    return binding, runner


class RecordingPool(MixedPool):
    """Keeps every finished task alive so the test can read its KV cache, and counts how many
    tasks are inside `run` at once."""

    def __init__(self, *a, **k):
        super().__init__(*a, **k)
        self.kept = {}
        self.active = 0
        self.max_active = 0
        self.lock = threading.Lock()

    def submit(self, req):
        task = super().submit(req)
        self.kept[req.name] = task
        return task

    def run(self, task):
        with self.lock:
            self.active += 1
            self.max_active = max(self.max_active, self.active)
        try:
            return super().run(task)
        finally:
            with self.lock:
                self.active -= 1

    def finish(self, task):
        pass                      # ended by the test after inspection


def _kv_of_blocks(model, spec, blocks, n):
    """K/V of every layer for a sequence living in `blocks` (read through a throw-away 0-token view)."""
    B, R = _mods()
    out = []
    probe = model.begin(torch.empty((0, spec.hidden), dtype=torch.bfloat16, device="cuda"), [0], cached=[n],
                        block_tables=blocks.reshape(1, -1), boundary_mask=0)
    for layer in range(spec.n_layers):
        out.extend(probe.kv(layer, 0))
    probe.end()
    return out


@pytest.mark.parametrize("chunk", [0, 1024])
def test_short_arrivals_preempt_long_prompt_and_results_are_identical(chunk):
    B, R = _mods()
    spec = I.LLAMA3_8B.with_layers(2)
    long_n, short_n = 8192, 128
    weights = I.make_weights(spec, 41, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, 2 * (long_n // 16) + 64, long_n)
    long_h = I.make_hidden(long_n, spec.hidden, 41, torch.bfloat16, "cuda")
    short_h = I.make_hidden(short_n, spec.hidden, 42, torch.bfloat16, "cuda")

    def run(arrival_times):
        pool = RecordingPool(model, B.FP_BOUNDARY_EVERY_OP, launch_ahead=1,
                             chunk_op_mask=B.FP_BOUNDARY_EVERY_OP if chunk else 0)
        loop = EventLoop(pool, priority=lambda r: (r.name == "L", r.order))
        shorts = [Request(f"s{i}", short_n, (short_h, 0), arrival=t) for i, t in enumerate(arrival_times)]
        loop.post_arrival(Request("L", long_n, (long_h, chunk)))
        loop.step(5.0)
        feed_arrivals(loop, shorts)
        loop.run(1 + len(shorts), timeout_s=60)
        loop.close()
        long_task = pool.kept["L"]
        if chunk:
            kv = _kv_of_blocks(model, spec, long_task.blocks, long_n)
        else:
            kv = [t for layer in range(spec.n_layers) for t in long_task.kv(layer, 0)] + [long_task.hidden()]
        short_out = [pool.kept[f"s{i}"].hidden() for i in range(len(shorts))]
        for task in pool.kept.values():
            task.end()
        return loop, pool, kv, short_out

    quiet_loop, _, want_kv, _ = run([])
    assert quiet_loop.commands == ["submit L"]
    loop, pool, got_kv, short_out = run([0.0005, 0.002, 0.0022, 0.004])
    assert pool.max_active == 1                                   # at most one task executes
    assert sorted(r.name for r in loop.finished) == ["L", "s0", "s1", "s2", "s3"]
    assert loop.commands[0] == "submit L" and "preempt L" in loop.commands and "resume L" in loop.commands
    assert loop.rounds <= 2 * 5                                   # one arrival + one completion per request
    assert len(got_kv) == len(want_kv) and all(torch.equal(a, b) for a, b in zip(got_kv, want_kv))
    for out in short_out[1:]:
        assert torch.equal(out, short_out[0])                     # identical shorts, identical results
    model.close()


def test_scheduler_driven_loop_batches_shorts_and_resumes_long_bit_identically():
    """The native scheduler (S-EDF + SLO-aware batching) driving the real library: a loose-SLO long
    prompt is preempted by tight-SLO shorts that arrive together, the shorts run as ONE packed
    variable-length task (Algorithm 1), the long prompt resumes; the long prompt's result equals
    an uninterrupted run bit for bit and every batched short agrees with the same prompt run alone
    (to rounding: the split-K factor of the projections depends on the batch's token count)."""
    from paper_2602_16603_amd.eventloop import BatchPool, SloEventLoop, SloRequest, feed_slo_arrivals
    B, R = _mods()
    spec = I.LLAMA3_8B.with_layers(2)
    long_n = 8192
    short_ns = [128, 300, 77]
    weights = I.make_weights(spec, 43, torch.bfloat16, "cuda")
    model = R.PrefillModel(spec, weights, B.FP_DTYPE_BF16, 4 * (long_n // 16) + 256, long_n)
    long_h = I.make_hidden(long_n, spec.hidden, 43, torch.bfloat16, "cuda")
    short_h = [I.make_hidden(n, spec.hidden, 44 + i, torch.bfloat16, "cuda") for i, n in enumerate(short_ns)]

    class KeepPool(BatchPool):
        def __init__(self, *a, **k):
            super().__init__(*a, **k)
            self.kept = []

        def submit(self, reqs):
            task = super().submit(reqs)
            self.kept.append(([r.id for r in reqs], task))
            return task

        def finish(self, task):
            pass

    def alone(h, n):
        t = model.begin(h, [n])
        t.run_to_completion()
        out = t.hidden()
        t.end()
        return out

    want_long = alone(long_h, long_n)
    want_short = [alone(h, n) for h, n in zip(short_h, short_ns)]

    pool = KeepPool(model, B.FP_BOUNDARY_EVERY_OP)
    # 1 ms + 10 us per token: the long prompt is predicted at ~83 ms, well inside its 6 s SLO.
    loop = SloEventLoop(pool, token_budget=4096, ttft_coef=[1e-3, 1e-5], policy=B.FP_SCHED_SEDF, batching=True)
    reqs = [SloRequest(0, long_n, 6.0, 0.0, long_h, "file")]
    reqs += [SloRequest(1 + i, n, 0.25, 0.003, h, "text") for i, (h, n) in enumerate(zip(short_h, short_ns))]
    feed_slo_arrivals(loop, reqs)
    t0 = time.perf_counter()
    while len(loop.finished) < len(reqs) and time.perf_counter() - t0 < 60:
        loop.step(0.05)
    assert sorted(r.id for r in loop.finished) == [0, 1, 2, 3]
    assert loop.commands["preempt"] >= 1 and loop.commands["resume"] >= 1
    batches = {tuple(ids): task for ids, task in pool.kept}
    assert any(len(ids) > 1 for ids in batches), "the simultaneous shorts were not batched"
    for ids, task in batches.items():
        got = task.hidden()
        if ids == (0,):
            assert torch.equal(got, want_long)                    # preempted + resumed == uninterrupted
        else:
            cu = I.cu_seqlens_of([short_ns[i - 1] for i in ids])
            for k, i in enumerate(ids):
                assert max_rel_err(got[cu[k]:cu[k + 1]], want_short[i - 1]) <= TOL["bf16"]   # packed ~ alone
    loop.close()
    for _, task in pool.kept:
        task.end()
    model.close()
