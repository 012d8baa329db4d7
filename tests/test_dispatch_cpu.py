"""The dispatcher loops (dispatch.py) on a virtual clock, without a GPU: a request "runs" by moving
the clock, so the loops' decisions can be compared with the library's replay of the same trace
(calvo_sched_simulate), which in turn is pinned to the scheduling oracle."""
import math

import numpy as np
import pytest

from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import dispatch

MODEL = (2.0e-6, 1.0e-3, 3.0e-5, 2.0e-3)
POLICIES = [cb.CALVO_POLICY_FIFO, cb.CALVO_POLICY_SJF, cb.CALVO_POLICY_SJF_PT, cb.CALVO_POLICY_LSTF, cb.CALVO_POLICY_EDF]


class Clock:
    def __init__(self):
        self.t = 0.0

    def __call__(self):
        return self.t

    def sleep(self, dt):
        self.t += max(dt, 0.0)


def trace(seed, n=40, rate=12.0):
    rng = np.random.default_rng(seed)
    t, jobs = 0.0, []
    for _ in range(n):
        t += rng.exponential(1.0 / rate)
        ctx, qry = int(rng.integers(1000, 40000)), int(rng.integers(10, 2000))
        solo = sum(cb.calvo_cost_estimate(MODEL, (0.0, 0.0, ctx, qry)))
        jobs.append((t, t + solo * float(rng.choice([2.0, 4.0, 8.0])), ctx, qry))
    return jobs


@pytest.mark.parametrize("policy", POLICIES)
@pytest.mark.parametrize("seed", [1, 2])
def test_serial_loop_reproduces_the_replay(policy, seed):
    jobs = trace(seed)
    clk = Clock()

    def run(i):
        clk.sleep(sum(cb.calvo_cost_estimate(MODEL, jobs[i])))

    start, fin = dispatch.serve_trace(policy, MODEL, jobs, run, clock=clk, sleep=clk.sleep)
    s0, f0 = cb.calvo_sched_simulate(policy, MODEL, jobs, pipelined=0)
    assert np.allclose(start, s0, atol=1e-9) and np.allclose(fin, f0, atol=1e-9)


@pytest.mark.parametrize("policy", POLICIES)
def test_two_stage_loop_follows_the_two_stage_replay(policy):
    """A two-stage server on the virtual clock: loading one request at a time, computation in loading
    order as soon as the request is loaded.  The loop only notices events when it polls, so its times
    trail the replay by at most one poll interval per decision."""
    jobs = trace(3, n=24)
    n = len(jobs)
    clk = Clock()
    poll = 1e-4
    load_end, comp_end = [math.inf] * n, [math.inf] * n
    comp_free = [0.0]

    def try_issue(i):
        t_load, t_comp = cb.calvo_cost_estimate(MODEL, jobs[i])
        load_end[i] = clk.t + t_load
        comp_end[i] = max(load_end[i], comp_free[0]) + t_comp
        comp_free[0] = comp_end[i]
        return True

    start, fin = dispatch.serve_trace_two_stage(policy, MODEL, jobs, try_issue, lambda i: clk.t >= load_end[i],
                                                lambda i: clk.t >= comp_end[i], clock=clk, sleep=clk.sleep, poll_s=poll)
    s1, f1 = cb.calvo_sched_simulate(policy, MODEL, jobs, pipelined=1)
    order_loop, order_replay = np.argsort(start, kind="stable"), np.argsort(s1, kind="stable")
    if list(order_loop) == list(order_replay):             # same decisions: times agree up to the polling lag
        assert np.all(np.array(fin) >= f1 - 1e-9) and np.all(np.array(fin) - f1 <= 3 * n * poll)
    else:                                                   # a poll-sized lag flipped a near-tie: totals still agree
        assert abs(max(fin) - f1.max()) <= 3 * n * poll + max(sum(cb.calvo_cost_estimate(MODEL, j)) for j in jobs)
    assert sorted(order_loop) == list(range(n))


def test_two_stage_loop_retries_a_request_that_cannot_be_issued_yet():
    jobs = [(0.0, math.inf, 1000, 10), (0.0, math.inf, 2000, 10)]
    clk = Clock()
    refused = [3]                                           # the first three attempts find no room
    ends = {}

    def try_issue(i):
        if refused[0] > 0:
            refused[0] -= 1
            return False
        ends[i] = clk.t + 0.01
        return True

    start, fin = dispatch.serve_trace_two_stage(cb.CALVO_POLICY_FIFO, MODEL, jobs, try_issue, lambda i: clk.t >= ends[i],
                                                lambda i: clk.t >= ends[i] + 0.005, clock=clk, sleep=clk.sleep, poll_s=1e-4)
    assert refused[0] == 0 and start[0] >= 3e-4 - 1e-12 and start[1] >= start[0] + 0.01 - 1e-9
    assert fin[0] >= 0.015 and fin[1] >= fin[0]


def test_pooled_loop_grants_waits_and_releases():
    """Three requests of 6 slots on a pool of 10: the second has to wait until the first lets go."""
    pool = cb.calvo_pool_create(10)
    try:
        jobs = [(0.0, math.inf, 100, 1), (0.0, math.inf, 100, 1), (0.0, math.inf, 100, 1)]
        clk = Clock()
        seen = []

        def run(i, table):
            assert len(table) == 6 and len(set(table.tolist())) == 6
            seen.append(set(table.tolist()))
            clk.sleep(0.01)

        start, fin, reactive, waited = dispatch.serve_trace_pooled(cb.CALVO_POLICY_FIFO, None, jobs, pool, [6, 6, 6], run,
                                                                  hold_s=[0.05, 0.05, 0.05], clock=clk, sleep=clk.sleep)
        assert reactive == [False, True, True]
        assert waited[1] >= 0.05 - 1e-9 and waited[2] >= 0.05 - 1e-9
        assert cb.calvo_pool_counts(pool)["used"] == 0
    finally:
        cb.calvo_pool_destroy(pool)
