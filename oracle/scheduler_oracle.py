"""CPU oracle of FlowPrefill's event-driven scheduler: the S-EDF priority (Eq. (3)), SLO-aware
batching (Algorithm 1) and one scheduling round (Algorithm 2), plus a small discrete-event
simulator that drives a scheduler over a request trace on an idealised single executor.

TEST INFRASTRUCTURE ONLY.  Nothing in the product imports this module; the product's scheduler
is the native one behind fp_sched_* and shares no code with this file.

Plain Python on purpose: lists, sorts and the paper's steps in the paper's order and notation
(Q_w waiting, Q_p preempted, E running, H highest priority, B batch, C candidates, G token
budget).  Readings where the paper is silent or inconsistent:
  * sgn(0) = +1 (the text calls non-negative slack good; Eq. (3) leaves zero open);
  * ties in priority are broken by earlier arrival, then smaller id, so a round is deterministic;
  * "while True then" in Algorithm 2 is "while True do";
  * C = Q_all \\ Q_p \\ {H} as printed would contain the running execution E; a running task
    cannot be merged into a new batch, so E is left out: C = Q_w \\ {H}, visited in priority order;
  * Algorithm 1 keeps scanning after a request that does not fit, with the strict comparisons
    T_remain > L and n < G as printed;
  * the TTFT estimate of a request is predict(its token count) -- for a batch head the aggregate
    count Algorithm 1 stored in H.num_tokens -- also when the request was partly executed before
    being preempted (the paper does not say how progress enters the estimate).

Pinned (tests/test_scheduler_oracle.py) by: the paper's two-request walk-through (Section 5.2,
"An illustrated example"), the ordering Eq. (3) is described to give (earliest deadline among
non-negative slack first; every negative-slack request behind every non-negative one), the closed
form Algorithm 1 has for equal-sized candidates under a linear latency model, its behaviour on a
misfit and at equality of both comparisons, the textbook property
that preemptive EDF meets every deadline of a feasible single-machine instance (S-EDF equals
EDF while all slacks are non-negative), and the bound "at most two scheduling rounds per request"
of Section 6.3.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence, Tuple

WAITING, PREEMPTED, RUNNING, FINISHED = 0, 1, 2, 3

POLICY_SEDF, POLICY_EDF, POLICY_FCFS = 0, 1, 2


@dataclass
class Req:
    id: int
    num_tokens: int            # Algorithm 1 overwrites this on the batch head with the aggregate
    arrival: float
    deadline: float            # arrival + TTFT SLO
    state: int = WAITING
    members: List[int] = field(default_factory=list)   # ids batched under this head (head included)


def sgn(x: float) -> float:
    return 1.0 if x >= 0.0 else -1.0


def priority(r: Req, now: float, predict: Callable[[int], float]) -> float:
    """Eq. (3): sgn(slack) / deadline with slack = deadline - now - predicted TTFT."""
    slack = r.deadline - now - predict(r.num_tokens)
    return sgn(slack) / r.deadline


def slo_aware_batching(H: Req, C: Sequence[Req], G: int, now: float,
                       predict: Callable[[int], float]) -> Tuple[Req, List[Req]]:
    """Algorithm 1.  Returns (H, B); H.num_tokens is updated to the batch's token count."""
    B = [H]
    T_remain = H.deadline - now
    N = H.num_tokens
    for r in C:
        n = N + r.num_tokens
        L = predict(n)
        if T_remain > L and n < G:
            B.append(r)
            H.num_tokens = n
            N = n
    return H, B


@dataclass
class Decision:
    preempt: Optional[int] = None      # id of the execution to preempt first
    action: str = "none"               # "submit" | "resume" | "none"
    head: Optional[int] = None
    batch: List[int] = field(default_factory=list)   # ids submitted together (head first)


class Scheduler:
    """State of Algorithm 2 (Q_w, Q_p, E) and one iteration of its loop per call to round()."""

    def __init__(self, G: int, predict: Callable[[int], float], policy: int = POLICY_SEDF,
                 batching: bool = True):
        self.G, self.predict, self.policy, self.batching = G, predict, policy, batching
        self.reqs: Dict[int, Req] = {}
        self.Q_w: List[Req] = []
        self.Q_p: List[Req] = []
        self.E: Optional[Req] = None

    # -- events -------------------------------------------------------------------------------
    def arrive(self, id: int, num_tokens: int, arrival: float, slo: float) -> None:
        r = Req(id, num_tokens, arrival, arrival + slo)
        r.members = [id]
        self.reqs[id] = r
        self.Q_w.append(r)

    def complete(self, head_id: int) -> List[int]:
        """The running execution (head and everything batched under it) has finished."""
        r = self.reqs[head_id]
        assert self.E is r
        r.state = FINISHED
        self.E = None
        return list(r.members)

    def retire(self, id: int) -> List[int]:
        """A preempted execution turned out to have finished before it reached a boundary (the
        preempt command raced with its completion): it leaves Q_p for good."""
        r = self.reqs[id]
        assert r.state == PREEMPTED
        self.Q_p.remove(r)
        r.state = FINISHED
        return list(r.members)

    # -- one scheduling round -----------------------------------------------------------------
    def _key(self, r: Req, now: float):
        if self.policy == POLICY_SEDF:
            p = priority(r, now, self.predict)
        elif self.policy == POLICY_EDF:
            p = 1.0 / r.deadline
        else:                                     # first come first served
            p = -r.arrival
        return (-p, r.arrival, r.id)              # ascending sort = descending priority

    def round(self, now: float) -> Decision:
        d = Decision()
        Q_all = self.Q_w + self.Q_p + ([self.E] if self.E is not None else [])
        if not Q_all:
            return d
        ranked = sorted(Q_all, key=lambda r: self._key(r, now))
        H = ranked[0]
        if self.policy == POLICY_FCFS and self.E is not None:
            return d                              # the baseline never preempts
        B: List[Req] = []
        if H.state == WAITING:
            C = [r for r in ranked if r.state == WAITING and r is not H] if self.batching else []
            H, B = slo_aware_batching(H, C, self.G, now, self.predict)
        if H is not self.E:
            if self.E is not None:
                d.preempt = self.E.id
                self.E.state = PREEMPTED
                self.Q_p.append(self.E)
            if B:
                d.action = "submit"
                d.batch = [r.id for r in B]
                H.members = list(d.batch)
                for r in B:
                    self.Q_w.remove(r)
            else:
                d.action = "resume"
                self.Q_p.remove(H)
            d.head = H.id
            H.state = RUNNING
            self.E = H
        return d


# ---------------------------------------------------------------------------------------------
# Discrete-event simulation on an ideal executor: an execution of n tokens needs service(n)
# seconds of executor time in total, can be preempted at any instant at no cost and resumed
# later where it stopped.  Used to pin the scheduler and to compare two implementations of it.
# ---------------------------------------------------------------------------------------------
def simulate(trace: Sequence[Tuple[int, int, float, float]], make_scheduler, service: Callable[[int], float],
             log: Optional[List] = None):
    """trace: (id, num_tokens, arrival, slo) sorted by arrival.  make_scheduler() returns an object
    with arrive / complete / round as above.  Returns {id: finish_time}, number of rounds."""
    sched = make_scheduler()
    finish: Dict[int, float] = {}
    remaining: Dict[int, float] = {}        # head id -> seconds of service left
    running: Optional[int] = None
    started_at = 0.0
    now = 0.0
    i = 0
    rounds = 0
    n = len(trace)
    while len(finish) < n:
        t_arr = trace[i][2] if i < n else float("inf")
        t_done = started_at + remaining[running] if running is not None else float("inf")
        if t_arr == float("inf") and t_done == float("inf"):
            raise RuntimeError("scheduler left requests queued with nothing running")
        if t_arr <= t_done:
            now = t_arr
            if running is not None:
                remaining[running] -= now - started_at
                started_at = now
            while i < n and trace[i][2] == now:
                sched.arrive(trace[i][0], trace[i][1], trace[i][2], trace[i][3])
                i += 1
        else:
            now = t_done
            for m in sched.complete(running):
                finish[m] = now
            del remaining[running]
            running = None
        d = sched.round(now)
        rounds += 1
        if log is not None:
            log.append((now, d.preempt, d.action, d.head, tuple(d.batch)))
        if d.action != "none":
            if d.preempt is not None:
                assert d.preempt == running
                # remaining[running] is already up to date
            if d.action == "submit":
                tokens = sum(t[1] for t in trace if t[0] in set(d.batch))
                remaining[d.head] = service(tokens)
            running = d.head
            started_at = now
    return finish, rounds
