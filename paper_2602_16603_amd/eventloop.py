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

    def __init__(self, pool, priority: Callable[[Request], Any] = default_priority,
                 on_complete: Optional[Callable[[Request], None]] = None):
        self.pool = pool
        self.priority = priority
        self.on_complete = on_complete           # e.g. re-issue a background request
        self.events: "queue.Queue[Tuple[str, Optional[Request]]]" = queue.Queue()
        self.jobs: "queue.Queue[Optional[Request]]" = queue.Queue()
        self.waiting: List[Request] = []         # Q_w
        self.preempted: List[Request] = []       # Q_p
        self.running: Optional[Request] = None   # E
        self.finished: List[Request] = []
        self.commands: List[str] = []
        self.rounds = 0
        self.preempt_latency_s: List[float] = []
        self.preempt_victims: List[str] = []     # name of the task each latency sample belongs to
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
            self.preempt_victims.append(victim.name)
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
        if self.on_complete is not None:
            self.on_complete(req)

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

    def step(self, timeout_s: float) -> bool:
        """Handles at most one event; False if none arrived within the timeout."""
        try:
            kind, req = self.events.get(timeout=timeout_s)
        except queue.Empty:
            return False
        self._round(kind, req)
        return True

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


def _advance_or_parked(task) -> int:
    """Runs the task to its next stop.  The scheduler may have parked the task between making it
    current and this thread reaching advance (fp_preempt on an idle task parks it at once); the
    library then refuses the advance with FP_ERR_STATE, which here simply means PREEMPTED."""
    from . import binding as B
    try:
        status, _ = task.advance()
        return status
    except B.FlowPrefillError as exc:
        if exc.status == B.FP_ERR_STATE:
            return PREEMPTED
        raise


class PrefillPool:
    """The execution pool over the HIP library: at most one task runs; parked tasks keep their
    workspace and KV blocks (Section 4)."""

    def __init__(self, model, boundary_mask: int):
        self.model = model
        self.boundary_mask = boundary_mask

    def submit(self, req: Request):
        return self.model.begin(req.payload, [req.n_tokens], boundary_mask=self.boundary_mask)

    def run(self, task) -> int:
        return _advance_or_parked(task)

    def preempt(self, task) -> int:
        return task.preempt()

    def resume(self, task) -> None:
        task.resume()

    def finish(self, task) -> None:
        task.end()


class ChunkedPrefillTask:
    """Chunked prefill of one prompt: the prompt is run `chunk` tokens at a time through the
    whole stack, every chunk attending to the KV its predecessors left in the paged cache.

    op_mask == 0: the fixed-chunk baseline of Section 3.1 / Fig. 2 -- the scheduler can take the
    GPU only between chunks.  op_mask != 0: operator-level preemption combined with chunking
    (Section 6.5, "FlowPrefill with chunked prefill"): every chunk is an operator-preemptible
    task, so a request is honoured at the next operator boundary inside the running chunk, and
    chunking only caps how long the longest operator can be.  Host logic only."""

    def __init__(self, model, hidden, n_tokens: int, chunk: int, op_mask: int = 0, launch_ahead: int = 2):
        from . import binding as B
        self._B = B
        self.model, self.hidden, self.n, self.chunk = model, hidden, n_tokens, chunk
        self.op_mask, self.launch_ahead = op_mask, launch_ahead
        self.blocks = B.fp_kv_alloc(model.handle, (n_tokens + 15) // 16)
        self.table = self.blocks.reshape(1, -1)
        self.done_tokens = 0
        self.cond = threading.Condition()
        self.signal = False
        self.parked = False
        self.parked_inside = False          # parked at an operator boundary inside self.current
        self.finished = False
        self.current = None                 # the chunk's task while it exists

    def run(self) -> int:
        B = self._B
        while self.done_tokens < self.n:
            if self.current is None:
                lo, hi = self.done_tokens, min(self.n, self.done_tokens + self.chunk)
                with self.cond:                    # chunk boundary
                    if self.signal:
                        self.signal = False
                        self.parked = True
                        self.cond.notify_all()
                        return PREEMPTED
                    task = self.model.begin(self.hidden[lo:hi], [hi - lo], cached=[lo],
                                            block_tables=self.table, boundary_mask=self.op_mask)
                    if self.op_mask:
                        B.fp_prefill_set_launch_ahead(task.handle, self.launch_ahead)
                    self.current = task
            status = _advance_or_parked(self.current)
            with self.cond:
                if status == PREEMPTED:            # parked at an operator boundary inside the chunk
                    self.signal = False
                    self.parked = True
                    self.parked_inside = True
                    self.cond.notify_all()
                    return PREEMPTED
                self.done_tokens += self.current.lengths[0]
                self.current.end()
                self.current = None
        with self.cond:
            self.finished = True
            self.signal = False
            self.cond.notify_all()
        return DONE

    def preempt(self) -> int:
        B = self._B
        with self.cond:
            if not self.finished and not self.parked:
                self.signal = True
                if self.op_mask and self.current is not None:
                    # Non-blocking: sets the running chunk's signal (or parks it if its advance
                    # has not begun).  Under the lock, so the chunk's task cannot be ended meanwhile.
                    B.fp_preempt_signal(self.current.handle)
                self.cond.wait_for(lambda: self.parked or self.finished)
            return DONE if self.finished else PREEMPTED

    def resume(self) -> None:
        with self.cond:
            self.parked = False
            if self.parked_inside:
                self.parked_inside = False
                self.current.resume()

    def end(self) -> None:
        if self.current is not None:
            self.current.end()
            self.current = None
        if self.blocks is not None:
            self._B.fp_kv_free(self.model.handle, self.blocks)
            self.blocks = None


class MixedPool:
    """Execution pool for the preemption workload: requests whose payload is a
    (hidden, chunk) pair with chunk > 0 run as fixed chunked prefill, all others as one
    operator-preemptible task.  chunk_op_mask != 0 makes the chunks themselves operator-preemptible."""

    def __init__(self, model, boundary_mask: int, launch_ahead: int = 2, short_tokens: int = 2048,
                 chunk_op_mask: int = 0):
        self.model, self.boundary_mask, self.launch_ahead = model, boundary_mask, launch_ahead
        self.chunk_op_mask = chunk_op_mask
        self.short_tokens = short_tokens     # requests up to this size run with unbounded launch-ahead

    def submit(self, req: Request):
        hidden, chunk = req.payload
        if chunk:
            return ChunkedPrefillTask(self.model, hidden, req.n_tokens, chunk, self.chunk_op_mask, self.launch_ahead)
        task = self.model.begin(hidden, [req.n_tokens], boundary_mask=self.boundary_mask)
        from . import binding as B
        B.fp_prefill_set_launch_ahead(task.handle, 0 if req.n_tokens <= self.short_tokens else self.launch_ahead)
        return task

    def run(self, task) -> int:
        if isinstance(task, ChunkedPrefillTask):
            return task.run()
        return _advance_or_parked(task)

    def preempt(self, task) -> int:
        return task.preempt()

    def resume(self, task) -> None:
        task.resume()

    def finish(self, task) -> None:
        task.end()


# ---------------------------------------------------------------------------------------------
# Event loop under the native scheduler (fp_sched_*): S-EDF priority, SLO-aware batching,
# Algorithm 2's round after every arrival and completion event.
# ---------------------------------------------------------------------------------------------
@dataclass
class SloRequest:
    id: int
    n_tokens: int
    slo: float                          # TTFT SLO in seconds
    arrival: float                      # seconds from the start of the run
    hidden: Any = None                  # [n_tokens, d] device tensor (or a view of a shared one)
    kind: str = ""
    t_arrived: float = 0.0
    t_finished: float = 0.0


class SloEventLoop:
    """Drives `pool` with the decisions of the native scheduler.  pool must provide
    submit(list of SloRequest) -> handle, run(handle) -> DONE | PREEMPTED (blocking),
    preempt(handle) -> PREEMPTED | DONE (blocking until acknowledged), resume(handle),
    finish(handle).  One execution = one batch head and the requests batched under it."""

    def __init__(self, pool, token_budget: int, ttft_coef, policy: int, batching: bool):
        from . import binding as B
        self._B = B
        self.pool = pool
        self.sched = B.fp_sched_create(token_budget, ttft_coef, policy, batching)
        self.events: "queue.Queue[Tuple[str, Any]]" = queue.Queue()
        self.jobs: "queue.Queue[Optional[int]]" = queue.Queue()
        self.requests = {}                   # id -> SloRequest, everything seen so far
        self.handles = {}                    # head id -> execution handle
        self.members = {}                    # head id -> [SloRequest]
        self.running: Optional[int] = None
        self.finished: List[SloRequest] = []
        self.rounds = 0
        self.commands = {"submit": 0, "preempt": 0, "resume": 0}
        self.batch_sizes: List[int] = []
        self.preempt_latency_s: List[float] = []
        self._retired = set()
        self.t0 = time.perf_counter()
        self._worker = threading.Thread(target=self._work, daemon=True)
        self._worker.start()

    def now(self) -> float:
        return time.perf_counter() - self.t0

    def _work(self) -> None:
        while True:
            head = self.jobs.get()
            if head is None:
                return
            if self.pool.run(self.handles[head]) == DONE:
                self.events.put(("completion", head))

    def post_arrival(self, req: SloRequest) -> None:
        req.t_arrived = self.now()
        self.events.put(("arrival", req))

    def _finish_execution(self, head: int) -> None:
        t = self.now()
        self.pool.finish(self.handles.pop(head))
        for r in self.members.pop(head):
            r.t_finished = t
            self.finished.append(r)

    def _round(self, kind: str, what) -> None:
        B = self._B
        if kind == "arrival":
            self.requests[what.id] = what
            B.fp_sched_arrive(self.sched, what.id, what.n_tokens, what.t_arrived, what.slo)
        else:
            if what in self._retired:           # finished while being preempted; already retired
                self._retired.discard(what)
                return
            B.fp_sched_complete(self.sched, what)
            self._finish_execution(what)
            self.running = None
        self.rounds += 1
        pre, action, head, batch = B.fp_sched_round(self.sched, self.now())
        if pre is not None:
            t0 = time.perf_counter()
            status = self.pool.preempt(self.handles[pre])
            self.preempt_latency_s.append(time.perf_counter() - t0)
            self.commands["preempt"] += 1
            if status == DONE:                  # it finished before the next boundary
                B.fp_sched_retire(self.sched, pre)
                self._retired.add(pre)
                self._finish_execution(pre)
        if action == B.FP_SCHED_SUBMIT:
            reqs = [self.requests[i] for i in batch]
            self.handles[head] = self.pool.submit(reqs)
            self.members[head] = reqs
            self.commands["submit"] += 1
            self.batch_sizes.append(len(reqs))
        elif action == B.FP_SCHED_RESUME:
            self.pool.resume(self.handles[head])
            self.commands["resume"] += 1
        if action != B.FP_SCHED_NONE:
            self.running = head
            self.jobs.put(head)

    def step(self, timeout_s: float) -> bool:
        try:
            kind, what = self.events.get(timeout=timeout_s)
        except queue.Empty:
            return False
        self._round(kind, what)
        return True

    def close(self) -> None:
        """Stops the executor thread; parks and ends whatever is still queued or running."""
        if self.running is not None:
            self.pool.preempt(self.handles[self.running])
        self.jobs.put(None)
        self._worker.join(timeout=30)
        for head in list(self.handles):
            self.pool.finish(self.handles.pop(head))
        self._B.fp_sched_destroy(self.sched)
        self.sched = 0


def feed_slo_arrivals(loop: SloEventLoop, requests: List[SloRequest]) -> threading.Thread:
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


class BatchPool:
    """Execution pool for SloEventLoop: a batch of requests becomes one packed variable-length
    prefill task (operator-preemptible with `boundary_mask`), or -- chunk > 0, single requests
    only -- fixed chunked prefill whose only boundaries are chunk ends (the CP baselines)."""

    def __init__(self, model, boundary_mask: int, chunk: int = 0, launch_ahead: int = 2,
                 short_tokens: int = 2048):
        self.model, self.boundary_mask, self.chunk = model, boundary_mask, chunk
        self.launch_ahead, self.short_tokens = launch_ahead, short_tokens

    def submit(self, reqs: List[SloRequest]):
        import torch
        from . import binding as B
        total = sum(r.n_tokens for r in reqs)
        if self.chunk and len(reqs) == 1 and total > self.chunk:
            return ChunkedPrefillTask(self.model, reqs[0].hidden, total, self.chunk, 0, self.launch_ahead)
        hidden = reqs[0].hidden if len(reqs) == 1 else torch.cat([r.hidden for r in reqs])
        task = self.model.begin(hidden, [r.n_tokens for r in reqs],
                                boundary_mask=self.boundary_mask if not self.chunk else B.FP_BOUNDARY_NONE)
        B.fp_prefill_set_launch_ahead(task.handle, 0 if total <= self.short_tokens else self.launch_ahead)
        return task

    def run(self, task) -> int:
        if isinstance(task, ChunkedPrefillTask):
            return task.run()
        return _advance_or_parked(task)

    def preempt(self, task) -> int:
        return task.preempt()

    def resume(self, task) -> None:
        task.resume()

    def finish(self, task) -> None:
        task.end()

