"""Host logic of the event-driven driver, on the CPU with a fake execution pool: the command
sequence of the paper's worked two-request example (Section 5.2, Fig. 7), the at-most-one-running
invariant (Section 4) and the two-rounds-per-request count (Section 6.4, scheduling cost)."""
import os
import threading

from paper_2602_16603_amd.eventloop import DONE, PREEMPTED, EventLoop, Request

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "two_request_trace.txt")


class FakeTask:
    def __init__(self, name, steps):
        self.name, self.steps, self.cursor = name, steps, 0
        self.signal = threading.Event()
        self.acked = threading.Event()
        self.step_gate = threading.Semaphore(0)     # the test releases one "operator" at a time
        self.done = False
        self.at_gate = threading.Event()            # set while blocked inside an "operator"


class FakePool:
    """Tasks advance one fake operator per released permit and check the signal in between."""

    def __init__(self):
        self.tasks = {}
        self.active = 0
        self.max_active = 0
        self.lock = threading.Lock()

    def submit(self, req):
        t = FakeTask(req.name, req.n_tokens)
        self.tasks[req.name] = t
        return t

    def run(self, t):
        with self.lock:
            self.active += 1
            self.max_active = max(self.max_active, self.active)
        try:
            while t.cursor < t.steps:
                if t.signal.is_set():
                    t.signal.clear()
                    t.acked.set()
                    return PREEMPTED
                t.at_gate.set()
                t.step_gate.acquire()
                t.at_gate.clear()
                t.cursor += 1
            t.done = True
            t.acked.set()
            return DONE
        finally:
            with self.lock:
                self.active -= 1

    def preempt(self, t):
        t.acked.clear()
        t.signal.set()
        t.step_gate.release()            # let the operator in flight finish
        t.acked.wait(5)
        return DONE if t.done else PREEMPTED

    def resume(self, t):
        pass

    def finish(self, t):
        pass


def test_two_request_example_issues_the_papers_commands():
    want = [l.strip() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    pool = FakePool()
    loop = EventLoop(pool)
    a = Request("A", n_tokens=6)            # long, low priority
    b = Request("B", n_tokens=2)            # short, high priority
    loop.post_arrival(a)
    loop._round(*loop.events.get(timeout=5))
    pool.tasks["A"].step_gate.release()     # A makes some progress
    loop.post_arrival(b)
    loop._round(*loop.events.get(timeout=5))
    assert pool.tasks["A"].cursor < 6
    for _ in range(2):
        pool.tasks["B"].step_gate.release()
    loop._round(*loop.events.get(timeout=5))          # completion of B
    for _ in range(6):
        pool.tasks["A"].step_gate.release()
    loop._round(*loop.events.get(timeout=5))          # completion of A
    assert loop.commands == want
    assert [r.name for r in loop.finished] == ["B", "A"]
    assert pool.max_active == 1                       # at most one task executes at any time
    assert loop.rounds == 4 == 2 * 2                  # one arrival + one completion per request
    assert len(loop.preempt_latency_s) == 1
    loop.close()


def test_lower_priority_arrival_does_not_preempt():
    pool = FakePool()
    loop = EventLoop(pool)
    loop.post_arrival(Request("S", n_tokens=2))
    loop._round(*loop.events.get(timeout=5))
    loop.post_arrival(Request("L", n_tokens=9))
    loop._round(*loop.events.get(timeout=5))
    assert loop.commands == ["submit S"]
    for _ in range(2):
        pool.tasks["S"].step_gate.release()
    loop._round(*loop.events.get(timeout=5))
    assert loop.commands == ["submit S", "submit L"]
    for _ in range(9):
        pool.tasks["L"].step_gate.release()
    loop.run(2, timeout_s=5)
    assert [r.name for r in loop.finished] == ["S", "L"]
    loop.close()


def test_preempt_racing_with_completion_is_treated_as_completion():
    pool = FakePool()
    loop = EventLoop(pool)
    loop.post_arrival(Request("A", n_tokens=1))
    loop._round(*loop.events.get(timeout=5))
    assert pool.tasks["A"].at_gate.wait(5)         # A's only operator is in flight
    # A needs exactly one more operator; the preempt's "let the op in flight finish" completes it.
    loop.post_arrival(Request("B", n_tokens=0))
    loop._round(*loop.events.get(timeout=5))
    assert "preempt A" not in loop.commands
    assert loop.commands == ["submit A", "submit B"]
    loop.run(2, timeout_s=5)
    assert sorted(r.name for r in loop.finished) == ["A", "B"]
    loop.close()
