"""SloEventLoop (event loop under the native scheduler) on the CPU with a timed fake pool: every
request finishes exactly once, at most one execution runs at a time (Section 4), a tight-SLO
arrival overtakes a running loose-SLO prefill (preempt -> submit -> resume, Section 5.2), short
requests that arrive together are batched under one execution (Algorithm 1), and FCFS issues no
preempt."""
import threading
import time

from paper_2602_16603_amd import binding as B
from paper_2602_16603_amd.eventloop import DONE, PREEMPTED, SloEventLoop, SloRequest, feed_slo_arrivals

SEC_PER_TOKEN = 2e-5


class TimedTask:
    def __init__(self, reqs):
        self.reqs = reqs
        self.left = sum(r.n_tokens for r in reqs) * SEC_PER_TOKEN
        self.signal = threading.Event()
        self.done = False


class TimedPool:
    """An execution takes SEC_PER_TOKEN per token; it checks its signal every millisecond."""

    def __init__(self):
        self.active = 0
        self.max_active = 0
        self.lock = threading.Lock()
        self.submitted = []

    def submit(self, reqs):
        self.submitted.append([r.id for r in reqs])
        return TimedTask(reqs)

    def run(self, t):
        with self.lock:
            self.active += 1
            self.max_active = max(self.max_active, self.active)
        try:
            while t.left > 0:
                if t.signal.is_set():
                    t.signal.clear()
                    return PREEMPTED
                dt = min(1e-3, t.left)
                time.sleep(dt)
                t.left -= dt
            t.done = True
            return DONE
        finally:
            with self.lock:
                self.active -= 1

    def preempt(self, t):
        t.signal.set()
        while t.signal.is_set() and not t.done:
            time.sleep(2e-4)
        if t.done:
            t.signal.clear()
        return DONE if t.done else PREEMPTED

    def resume(self, t):
        pass

    def finish(self, t):
        pass


def drive(loop, reqs, timeout=20.0):
    feed_slo_arrivals(loop, reqs)
    t0 = time.perf_counter()
    while len(loop.finished) < len(reqs) and time.perf_counter() - t0 < timeout:
        loop.step(0.02)
    loop.close()


def test_tight_slo_overtakes_and_short_requests_batch():
    pool = TimedPool()
    loop = SloEventLoop(pool, token_budget=4096, ttft_coef=[0.0, SEC_PER_TOKEN], policy=B.FP_SCHED_SEDF, batching=True)
    reqs = [SloRequest(0, 20000, 6.0, 0.00, kind="file"),        # 0.4 s of work, loose SLO
            SloRequest(1, 500, 0.25, 0.05, kind="text"),          # arrive together while 0 runs
            SloRequest(2, 400, 0.25, 0.05, kind="text"),
            SloRequest(3, 300, 0.25, 0.05, kind="text")]
    drive(loop, reqs)
    assert sorted(r.id for r in loop.finished) == [0, 1, 2, 3]
    assert pool.max_active == 1
    assert loop.commands["preempt"] >= 1 and loop.commands["resume"] >= 1
    assert any(len(b) > 1 for b in pool.submitted)                # Algorithm 1 merged some shorts
    by_id = {r.id: r for r in loop.finished}
    assert all(by_id[i].t_finished - by_id[i].t_arrived <= 0.25 for i in (1, 2, 3))
    assert by_id[0].t_finished > max(by_id[i].t_finished for i in (1, 2, 3))
    assert loop.rounds <= 2 * len(reqs)


def test_fcfs_never_preempts():
    pool = TimedPool()
    loop = SloEventLoop(pool, token_budget=4096, ttft_coef=[0.0, SEC_PER_TOKEN], policy=B.FP_SCHED_FCFS, batching=False)
    reqs = [SloRequest(0, 10000, 6.0, 0.00), SloRequest(1, 500, 0.25, 0.03), SloRequest(2, 500, 0.25, 0.06)]
    drive(loop, reqs)
    assert [r.id for r in loop.finished] == [0, 1, 2]
    assert loop.commands["preempt"] == 0 and loop.commands["resume"] == 0
