"""Minimal event-driven driver of the execution pool (FlowPrefill Section 5.2, Algorithm 2, the
command skeleton only): scheduling rounds are triggered by exactly two kinds of events, request
arrival and task completion; each round picks the highest-priority request H and, if it is not
the running one, issues preempt (for the running task) followed by submit or resume (for H).

There is no scheduler policy here: priority is a caller-supplied key (default: fewer prompt
tokens first, then earlier arrival), and batching (Algorithm 1), slack (Eq. 3) and TTFT
prediction are left out.  The pool object does the work; this module only sequences commands
and records what it issued and how long each preempt blocked (signal -> acknowledgement,
Section 6.4).
"""
from __future__ import annotations

import queue
import threading
import time
from dataclasses import dataclass, field
from typing import Any, Callable, List, Optional, Tuple

DONE, PREEMPTED = 1, 2     # status codes shared with the C ABI (FP_DONE, FP_PREEMPTED)


@dataclass
class Request:
    name: str
    n_tokens: int
    payload: Any = None                 # whatever the pool needs to build the task
    arrival: float = 0.0                # seconds, relative to the start of the run
    order: int = 0
    handle: Any = None
    t_arrived: float = 0.0              # wall clock stamps (perf_counter)
    t_finished: float = 0.0


def default_priority(r: Request) -> Tuple[int, int]:
    """Smaller is more urgent: short prompts first, ties by arrival order."""
    return (r.n_tokens, r.order)


class EventLoop:
    """pool must provide: submit(request) -> handle, run(handle) -> status (blocking, DONE or
    PREEMPTED), preempt(handle) -> status (blocking until acknowledged; DONE if the task finished
    first), resume(handle), finish(handle)."""

    def __init__(self, pool, priority: Callable[[Request], Any] = default_priority):
        self.pool = pool
        self.priority = priority
        self.events: "queue.Queue[Tuple[str, Optional[Request]]]" = queue.Queue()
        self.jobs: "queue.Queue[Optional[Request]]" = queue.Queue()
        self.waiting: List[Request] = []         # Q_w
        self.preempted: List[Request] = []       # Q_p
        self.running: Optional[Request] = None   # E
        self.finished: List[Request] = []
        self.commands: List[str] = []
        self.rounds = 0
        self.preempt_latency_s: List[float] = []
        self._early_done = set()
        self._arrivals = 0
        self._worker = threading.Thread(target=self._work, daemon=True)
        self._worker.start()

    # ---- executor thread: runs whatever task the scheduler made current ----
    def _work(self) -> None:
        while True:
            req = self.jobs.get()
            if req is None:
                return
            status = self.pool.run(req.handle)
            if status == DONE:
                self.events.put(("completion", req))
            # PREEMPTED: the scheduler already holds the acknowledgement; nothing to post.

    # ---- event sources ----
    def post_arrival(self, req: Request) -> None:
        req.t_arrived = time.perf_counter()
        self.events.put(("arrival", req))

    # ---- one scheduling round (Algorithm 2, one iteration of its loop) ----
    def _round(self, kind: str, req: Optional[Request]) -> None:
        self.rounds += 1
        if kind == "arrival":
            req.order = self._arrivals
            self._arrivals += 1
            self.waiting.append(req)
        elif kind == "completion":
            if req.name in self._early_done:
                self._early_done.discard(req.name)
            else:
                self._complete(req)
        candidates = self.waiting + self.preempted + ([self.running] if self.running else [])
        if not candidates:
            return
        best = min(candidates, key=self.priority)
        if best is self.running:
            return
        if self.running is not None:
            victim = self.running
            t0 = time.perf_counter()
            status = self.pool.preempt(victim.handle)
            self.preempt_latency_s.append(time.perf_counter() - t0)
            if status == PREEMPTED:
                self.commands.append(f"preempt {victim.name}")
                self.preempted.append(victim)
                self.running = None
            else:       # it finished before the next boundary: its completion event is on its way
                self._early_done.add(victim.name)
                self._complete(victim)
        if best in self.waiting:
            best.handle = self.pool.submit(best)
            self.commands.append(f"submit {best.name}")
            self.waiting.remove(best)
        else:
            self.pool.resume(best.handle)
            self.commands.append(f"resume {best.name}")
            self.preempted.remove(best)
        self.running = best
        self.jobs.put(best)

    def _complete(self, req: Request) -> None:
        req.t_finished = time.perf_counter()
        self.pool.finish(req.handle)
        self.finished.append(req)
        if self.running is req:
            self.running = None

    # ---- main loop ----
    def run(self, n_requests: int, timeout_s: float = 600.0) -> None:
        """Consumes events sequentially until n_requests have finished."""
        deadline = time.perf_counter() + timeout_s
        while len(self.finished) < n_requests:
            left = deadline - time.perf_counter()
            if left <= 0:
                raise TimeoutError("event loop timed out")
            try:
                kind, req = self.events.get(timeout=min(left, 1.0))
            except queue.Empty:
                continue
            self._round(kind, req)

    def close(self) -> None:
        self.jobs.put(None)
        self._worker.join(timeout=10)


def feed_arrivals(loop: EventLoop, requests: List[Request]) -> threading.Thread:
    """Posts each request's arrival event at its `arrival` time (seconds from now)."""
    t0 = time.perf_counter()

    def feeder():
        for r in sorted(requests, key=lambda r: r.arrival):
            delay = t0 + r.arrival - time.perf_counter()
            if delay > 0:
                time.sleep(delay)
            loop.post_arrival(r)

    th = threading.Thread(target=feeder, daemon=True)
    th.start()
    return th


class PrefillPool:
    """The execution pool over the HIP library: at most one task runs; parked tasks keep their
    workspace and KV blocks (Section 4)."""

    def __init__(self, model, boundary_mask: int):
        self.model = model
        self.boundary_mask = boundary_mask

    def submit(self, req: Request):
        return self.model.begin(req.payload, [req.n_tokens], boundary_mask=self.boundary_mask)

    def run(self, task) -> int:
        status, _ = task.advance()
        return status

    def preempt(self, task) -> int:
        return task.preempt()

    def resume(self, task) -> None:
        task.resume()

    def finish(self, task) -> None:
        task.end()
