"""Pins of the scheduler oracle (Eq. (3), Algorithms 1 and 2 of FlowPrefill Section 5.2) against
things the paper and the mathematics fix, and parity of the native fp_sched_* implementation with
the oracle over seeded random traces (integer decisions: compared exactly).  CPU only."""
import itertools
import os
import random

import pytest

from oracle import scheduler_oracle as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "scheduler_two_request_example.txt")


def poly(coef):
    def predict(n):
        y = 0.0
        for c in reversed(coef):
            y = y * float(n) + c
        return y
    return predict


def commands(d: S.Decision, names):
    out = []
    if d.preempt is not None:
        out.append(f"preempt {names[d.preempt]}")
    if d.action != "none":
        out.append(f"{d.action} {names[d.head]}")
    return ", ".join(out) if out else "none"


def test_two_request_walk_through_of_the_paper():
    want = [l.strip() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    names = {0: "A", 1: "B"}
    s = S.Scheduler(G=8192, predict=poly([0.0, 1e-4]))
    got = []
    s.arrive(0, 6000, 0.0, 6.0)                    # A: long prompt, loose SLO
    got.append("arrival A -> " + commands(s.round(0.0), names))
    s.arrive(1, 500, 0.1, 0.25)                    # B: short prompt, tight SLO
    got.append("arrival B -> " + commands(s.round(0.1), names))
    s.complete(1)
    got.append("completion B -> " + commands(s.round(0.15), names))
    s.complete(0)
    got.append("completion A -> " + commands(s.round(0.8), names))
    assert got == want


def test_priority_orders_as_eq3_is_described():
    """Earliest deadline first among requests with non-negative slack; every request that can no
    longer make its deadline ranks behind every request that still can; sgn(0) counts as +."""
    predict = poly([0.0, 1e-3])                    # 1 ms per token
    now = 10.0
    ok_early = S.Req(0, 100, 9.0, 10.5)            # slack 0.4
    ok_late = S.Req(1, 100, 9.0, 12.0)             # slack 1.9
    lost_early = S.Req(2, 2000, 9.0, 10.2)         # slack -1.8
    lost_late = S.Req(3, 5000, 9.0, 13.0)          # slack -2.0
    edge = S.Req(4, 1000, 9.0, 11.0)               # slack exactly 0
    p = {r.id: S.priority(r, now, predict) for r in (ok_early, ok_late, lost_early, lost_late, edge)}
    assert p[0] > p[4] > p[1] > 0 > p[3] > p[2]
    assert p[0] == 1.0 / 10.5 and p[2] == -1.0 / 10.2


def test_batching_closed_form_for_equal_candidates():
    """Linear latency a*n and k equal candidates of s tokens: the number admitted is the largest k
    with a*(N0 + k*s) < T_remain and N0 + k*s < G (strict, as printed)."""
    a, s_tok, n0 = 1e-3, 100, 250
    predict = poly([0.0, a])
    for t_remain, G in [(1.0, 10 ** 9), (10 ** 9, 1000), (0.5, 700), (0.3, 10 ** 9), (0.351, 10 ** 9), (0.35, 10 ** 9)]:
        H = S.Req(0, n0, 0.0, t_remain)            # now = 0, so T_remain = deadline
        C = [S.Req(i + 1, s_tok, 0.0, 99.0) for i in range(20)]
        _, B = S.slo_aware_batching(H, C, G, 0.0, predict)
        k = 0
        while k < 20 and a * (n0 + (k + 1) * s_tok) < t_remain and n0 + (k + 1) * s_tok < G:
            k += 1
        assert len(B) - 1 == k
        assert H.num_tokens == n0 + k * s_tok
        assert [r.id for r in B] == list(range(k + 1))          # admitted in candidate order


def test_batching_keeps_scanning_after_a_misfit_and_respects_strictness():
    predict = poly([0.0, 1e-3])
    H = S.Req(0, 100, 0.0, 1.0)
    big, small = S.Req(1, 5000, 0.0, 9.0), S.Req(2, 50, 0.0, 9.0)
    _, B = S.slo_aware_batching(H, [big, small], 10 ** 6, 0.0, predict)
    assert [r.id for r in B] == [0, 2]
    H = S.Req(0, 100, 0.0, 1.0)
    exact = S.Req(3, 900, 0.0, 9.0)                # predicted latency == T_remain: not admitted
    _, B = S.slo_aware_batching(H, [exact], 10 ** 6, 0.0, predict)
    assert [r.id for r in B] == [0]
    H = S.Req(0, 100, 0.0, 1.0)
    at_budget = S.Req(4, 100, 0.0, 9.0)            # n == G: not admitted
    _, B = S.slo_aware_batching(H, [at_budget], 200, 0.0, predict)
    assert [r.id for r in B] == [0]


def demand_feasible(jobs, service):
    """Textbook test for preemptive single-machine feasibility: for every window [a, d] the work
    of the jobs released at or after a with deadline at or before d fits into d - a."""
    for a in {j[2] for j in jobs}:
        for d in {j[2] + j[3] for j in jobs}:
            if d > a:
                work = sum(service(j[1]) for j in jobs if j[2] >= a and j[2] + j[3] <= d)
                if work > d - a + 1e-12:
                    return False
    return True


@pytest.mark.parametrize("seed", range(40))
def test_edf_rounds_meet_every_deadline_of_a_feasible_instance(seed):
    """Preemptive EDF is optimal on one machine: if the instance is feasible every deadline is
    met.  Pins the round's queue bookkeeping and command sequencing (submit / preempt / resume).
    S-EDF with a zero TTFT estimate never sees negative slack before a deadline has passed, so it
    must take the same decisions."""
    rng = random.Random(seed)
    service = lambda n: n * 1e-3
    jobs = []
    for i in range(rng.randint(2, 6)):
        n = rng.randint(50, 900)
        arr = round(rng.uniform(0, 2.0), 3)
        jobs.append((i, n, arr, round(service(n) + rng.uniform(0.0, 2.5), 3)))
    jobs.sort(key=lambda j: j[2])
    if not demand_feasible(jobs, service):
        pytest.skip("drawn instance is not feasible")
    deadline = {j[0]: j[2] + j[3] for j in jobs}
    log_edf, log_sedf = [], []
    fin, rounds = S.simulate(jobs, lambda: S.Scheduler(10 ** 9, poly([0.0]), S.POLICY_EDF, batching=False), service, log_edf)
    assert all(fin[i] <= deadline[i] + 1e-9 for i in fin)
    assert rounds <= 2 * len(jobs)                              # Section 6.3: at most two events per request
    fin2, _ = S.simulate(jobs, lambda: S.Scheduler(10 ** 9, poly([0.0]), S.POLICY_SEDF, batching=False), service, log_sedf)
    assert log_sedf == log_edf and fin2 == fin


def test_sedf_serves_a_lost_request_after_the_ones_that_can_still_make_it():
    """Overload: X cannot meet its deadline any more (negative slack) although its deadline is
    the earliest; plain EDF runs it first and makes Y late too, S-EDF runs Y first."""
    predict = service = lambda n: n * 1e-3
    trace = [(0, 2000, 0.0, 1.0), (1, 500, 0.0, 1.2)]          # X needs 2.0 s, deadline 1.0
    fin_edf, _ = S.simulate(trace, lambda: S.Scheduler(10 ** 9, predict, S.POLICY_EDF, batching=False), service)
    fin_sedf, _ = S.simulate(trace, lambda: S.Scheduler(10 ** 9, predict, S.POLICY_SEDF, batching=False), service)
    assert fin_edf[1] > 1.2 and fin_sedf[1] <= 1.2
    assert fin_sedf[0] == pytest.approx(2.5)


def test_fcfs_never_preempts_and_serves_in_arrival_order():
    service = lambda n: n * 1e-3
    trace = [(0, 3000, 0.0, 10.0), (1, 100, 0.5, 0.2), (2, 100, 0.6, 0.1)]
    log = []
    fin, _ = S.simulate(trace, lambda: S.Scheduler(10 ** 9, service, S.POLICY_FCFS, batching=False), service, log)
    assert all(entry[1] is None for entry in log)               # no preempt command ever
    assert fin[0] < fin[1] < fin[2]


# ---------------------------------------------------------------------------------------------
# Native implementation (fp_sched_*) against the oracle: same events in, same decisions out.
# ---------------------------------------------------------------------------------------------
class NativeScheduler:
    def __init__(self, G, coef, policy, batching):
        from paper_2602_16603_amd import binding as B
        self.B = B
        self.h = B.fp_sched_create(G, coef, policy, batching)
        self.members = {}

    def arrive(self, id, n, arrival, slo):
        self.B.fp_sched_arrive(self.h, id, n, arrival, slo)

    def complete(self, head):
        self.B.fp_sched_complete(self.h, head)
        return self.members.pop(head)

    def round(self, now):
        pre, action, head, batch = self.B.fp_sched_round(self.h, now)
        d = S.Decision(preempt=pre, action={0: "none", 1: "submit", 2: "resume"}[action], head=head, batch=batch)
        if action == 1:
            self.members[head] = list(batch)
        return d

    def __del__(self):
        self.B.fp_sched_destroy(self.h)


def table1_like_trace(rng, n, rate):
    """Four request classes with the length statistics and mix of Table 1 and the Llama3-8B TTFT
    SLOs of Table 2 (log-normal lengths matched to each class's mean and standard deviation)."""
    import math
    classes = [(590, 652, 0.68, 0.25), (532, 510, 0.08, 0.5), (5976, 3456, 0.20, 4.0), (6833, 5186, 0.04, 6.0)]
    t, out = 0.0, []
    for i in range(n):
        t += rng.expovariate(rate)
        u, acc = rng.random(), 0.0
        for mean, std, ratio, slo in classes:
            acc += ratio
            if u <= acc:
                break
        sigma2 = math.log(1.0 + (std / mean) ** 2)
        tokens = int(max(16, min(32768, round(rng.lognormvariate(math.log(mean) - sigma2 / 2, math.sqrt(sigma2))))))
        out.append((i, tokens, round(t, 6), slo))
    return out


@pytest.mark.parametrize("policy,batching", [(0, True), (0, False), (1, False), (2, False)])
@pytest.mark.parametrize("seed", range(6))
def test_native_scheduler_takes_the_oracles_decisions(policy, batching, seed):
    rng = random.Random(1000 + seed)
    coef = [2e-3, 2.0e-5, 1.0e-10]                 # ~20 us per token plus a small quadratic term
    predict = poly(coef)
    trace = table1_like_trace(rng, 300, rate=rng.choice([5.0, 20.0, 60.0]))
    G = 8192
    log_o, log_n = [], []
    fin_o, rounds_o = S.simulate(trace, lambda: S.Scheduler(G, predict, policy, batching), predict, log_o)
    fin_n, rounds_n = S.simulate(trace, lambda: NativeScheduler(G, coef, policy, batching), predict, log_n)
    assert max(len(e[4]) for e in log_o) < 64      # stays below the ABI's batch limit
    assert log_n == log_o
    assert fin_n == fin_o and rounds_n == rounds_o
    if batching:
        assert any(len(e[4]) > 1 for e in log_o)   # the trace does exercise Algorithm 1


def test_retire_after_a_preempt_that_raced_with_completion():
    """B preempts A, but A had already finished: A is retired from Q_p and never resumed; the
    oracle and the native scheduler agree on what follows."""
    from paper_2602_16603_amd import binding as B
    o = S.Scheduler(8192, poly([0.0, 1e-4]), S.POLICY_SEDF, batching=False)
    n = B.fp_sched_create(8192, [0.0, 1e-4], B.FP_SCHED_SEDF, False)
    for sch_arrive in (lambda *a: o.arrive(*a), lambda *a: B.fp_sched_arrive(n, *a)):
        sch_arrive(0, 6000, 0.0, 6.0)
    assert o.round(0.0).action == "submit" and B.fp_sched_round(n, 0.0)[1] == B.FP_SCHED_SUBMIT
    o.arrive(1, 500, 0.1, 0.25); B.fp_sched_arrive(n, 1, 500, 0.1, 0.25)
    d = o.round(0.1); pre, action, head, batch = B.fp_sched_round(n, 0.1)
    assert d.preempt == 0 == pre and d.head == 1 == head
    assert o.retire(0) == [0]; B.fp_sched_retire(n, 0)
    o.complete(1); B.fp_sched_complete(n, 1)
    assert o.round(0.2).action == "none" and B.fp_sched_round(n, 0.2)[1] == B.FP_SCHED_NONE
    B.fp_sched_destroy(n)


def test_native_scheduler_rejects_bad_calls():
    from paper_2602_16603_amd import binding as B
    with pytest.raises(B.FlowPrefillError):
        B.fp_sched_create(0, [1.0])
    s = B.fp_sched_create(100, [0.0, 1e-3])
    B.fp_sched_arrive(s, 7, 10, 0.0, 1.0)
    with pytest.raises(B.FlowPrefillError):
        B.fp_sched_arrive(s, 7, 10, 0.0, 1.0)      # duplicate id
    with pytest.raises(B.FlowPrefillError):
        B.fp_sched_complete(s, 7)                  # not running yet
    assert B.fp_sched_round(s, 0.0)[1] == B.FP_SCHED_SUBMIT
    with pytest.raises(B.FlowPrefillError):
        B.fp_sched_retire(s, 7)                    # running, not preempted
    B.fp_sched_complete(s, 7)
    assert B.fp_sched_predict(s, 1000) == pytest.approx(1.0)
    B.fp_sched_destroy(s)
