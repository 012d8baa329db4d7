"""Pins for the scheduling oracle (none re-uses its code path): the paper's worked example,
brute force over service orders, closed forms, conservation properties."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import sched_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sched_worked_example.txt")


def read_golden():
    reqs, printed = {}, {}
    for line in open(GOLDEN):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        if len(f) == 3:
            reqs[f[0]] = (float(f[1]), float(f[2]))
        else:
            printed[f[0]] = float(f[1])
    return reqs, printed


def test_worked_example_of_the_paper():
    """Section 2.3: 0.49 s when R1 is served first (FIFO, compute-only SJF), 0.41 s when the
    loading time is part of the cost (R2 first)."""
    reqs, printed = read_golden()
    load = [reqs["R1"][0], reqs["R2"][0]]
    comp = [reqs["R1"][1], reqs["R2"][1]]
    # a model that reproduces the profiled times exactly: 1 s per "token", tokens = seconds * 1000
    model = (1e-3, 0.0, 1e-3, 0.0)
    jobs = [(0.0, math.inf, round(load[0] * 1000), round(comp[0] * 1000)),      # R1 arrives first
            (1e-9, math.inf, round(load[1] * 1000), round(comp[1] * 1000))]
    now = 1e-9                                                                   # both are queued

    def avg_ttft(policy):
        first = so.pick(policy, model, jobs, None, now)
        order = [first, 1 - first]
        t, ttft = now, []
        for i in order:
            t += load[i] + comp[i]
            ttft.append(t - jobs[i][0])
        return first, sum(ttft) / 2

    first, avg = avg_ttft(so.FIFO)
    assert first == 0 and round(avg, 2) == printed["FIFO"]
    first, avg = avg_ttft(so.SJF_PT)                  # compute-only: 19 < 25 "tokens" -> R1 first
    assert first == 0 and round(avg, 2) == printed["SJF_COMPUTE_ONLY"]
    first, avg = avg_ttft(so.SJF)                     # 0.224 s < 0.380 s -> R2 first
    assert first == 1 and round(avg, 2) == printed["SJF_LOADING_AWARE"]
    # the replay gives the same numbers when both requests are there from the start
    jobs0 = [(0.0, math.inf, j[2], j[3]) for j in jobs]
    _, fin = so.simulate(so.SJF, model, jobs0, load, comp)
    assert round(sum(fin) / 2, 2) == printed["SJF_LOADING_AWARE"]
    _, fin = so.simulate(so.FIFO, model, jobs0, load, comp)
    assert round(sum(fin) / 2, 2) == printed["FIFO"]


def random_jobs(rng, n, all_at_zero=True):
    jobs = []
    for _ in range(n):
        ctx = int(rng.integers(0, 40000))
        query = int(rng.integers(1, 2000))
        arrival = 0.0 if all_at_zero else float(rng.uniform(0, 2.0))
        jobs.append((arrival, arrival + float(rng.uniform(0.05, 3.0)), ctx, query))
    return jobs


MODEL = (1.2e-5, 0.004, 2.5e-5, 0.002)


@pytest.mark.parametrize("seed", range(6))
def test_sjf_is_the_best_order_for_the_mean_when_all_are_present(seed):
    rng = np.random.default_rng(seed)
    jobs = random_jobs(rng, 6)
    cost = [sum(so.estimate(MODEL, j)) for j in jobs]
    _, fin = so.simulate(so.SJF, MODEL, jobs)
    best = min(sum(itertools.accumulate(cost[i] for i in perm)) for perm in itertools.permutations(range(6)))
    assert abs(sum(fin) - best) < 1e-9


@pytest.mark.parametrize("seed", range(6))
def test_edf_meets_all_deadlines_whenever_some_order_does(seed):
    rng = np.random.default_rng(100 + seed)
    jobs = random_jobs(rng, 6)
    cost = [sum(so.estimate(MODEL, j)) for j in jobs]
    feasible = any(all(t <= jobs[i][1] for i, t in zip(perm, itertools.accumulate(cost[i] for i in perm)))
                   for perm in itertools.permutations(range(6)))
    _, fin = so.simulate(so.EDF, MODEL, jobs)
    assert all(f <= j[1] for f, j in zip(fin, jobs)) == feasible


def test_lstf_priority_is_the_slack_and_equals_edf_for_equal_costs():
    job = (0.3, 2.0, 10000, 100)
    t_load, t_comp = 1.2e-5 * 10000 + 0.004, 2.5e-5 * 100 + 0.002
    assert so.estimate(MODEL, job) == (t_load, t_comp)
    assert so.priority(so.LSTF, MODEL, job) == 2.0 - t_load - t_comp
    rng = np.random.default_rng(7)
    jobs = [(0.0, float(d), 5000, 64) for d in rng.uniform(0.1, 2.0, 8)]
    assert so.simulate(so.LSTF, MODEL, jobs)[0] == so.simulate(so.EDF, MODEL, jobs)[0]
    # a long job with a late deadline can be more urgent than a short job with an earlier one
    jobs = [(0.0, 1.0, 0, 100), (0.0, 1.2, 90000, 100)]
    assert so.pick(so.EDF, MODEL, jobs, None, 0.0) == 0 and so.pick(so.LSTF, MODEL, jobs, None, 0.0) == 1


def test_zero_token_components_cost_nothing_and_ties_go_to_the_earlier_arrival():
    assert so.estimate(MODEL, (0, 0, 0, 10)) == (0.0, 2.5e-5 * 10 + 0.002)
    assert so.estimate(MODEL, (0, 0, 10, 0)) == (1.2e-5 * 10 + 0.004, 0.0)
    jobs = [(0.5, 9.0, 100, 10), (0.2, 9.0, 100, 10), (0.2, 9.0, 100, 10)]
    for policy in (so.SJF, so.SJF_PT, so.LSTF, so.EDF, so.FIFO):
        assert so.pick(policy, MODEL, jobs, None, 1.0) == 1
        assert so.pick(policy, MODEL, jobs, [False, True, False], 1.0) == 2
        assert so.pick(policy, MODEL, jobs, None, 0.1) == -1


@pytest.mark.parametrize("policy", [so.FIFO, so.SJF, so.SJF_PT, so.LSTF, so.EDF])
@pytest.mark.parametrize("pipelined", [False, True])
def test_replay_is_work_conserving_and_never_starts_before_arrival(policy, pipelined):
    rng = np.random.default_rng(policy * 2 + pipelined)
    jobs = random_jobs(rng, 12, all_at_zero=False)
    load = [float(x) for x in rng.uniform(0.01, 0.3, 12)]
    comp = [float(x) for x in rng.uniform(0.005, 0.1, 12)]
    start, fin = so.simulate(policy, MODEL, jobs, load, comp, pipelined)
    order = sorted(range(12), key=lambda i: start[i])
    for i in range(12):
        assert start[i] >= jobs[i][0]
        assert fin[i] >= start[i] + load[i] + comp[i] - 1e-12
    for a, b in zip(order, order[1:]):
        busy_until = start[a] + load[a] + (0 if pipelined else comp[a])
        assert start[b] >= busy_until - 1e-12                       # non-preemptive, one at a time per stage
        if start[b] > busy_until + 1e-12:                           # the stage idled: nobody had arrived
            assert all(jobs[i][0] >= start[b] - 1e-12 for i in order[order.index(b):])
    if not pipelined:
        assert all(abs(fin[i] - (start[i] + load[i] + comp[i])) < 1e-12 for i in range(12))
    # pipelining the two stages never finishes the FIFO trace later
    if policy == so.FIFO and pipelined:
        _, fin_serial = so.simulate(policy, MODEL, jobs, load, comp, False)
        assert max(fin) <= max(fin_serial) + 1e-12


def test_staged_replay_by_hand():
    """Both stages serve their highest-priority ready request (Section 3.1).  Worked by hand, times given
    directly: A (load 1, compute 10) and B (load 1, compute 5) arrive at 0, D (load 1, compute 1) at 1.5,
    SJF.  Loading: B at 0 (6 < 11), A at 1, D at 2.  Compute: B 1-6; at 6 both A (loaded at 2) and D
    (loaded at 3) wait and D is the shorter job: D 6-7, A 7-17.  In loading order (the plain pipelined
    replay) A would compute 6-16 and D 16-17."""
    model = (1.0, 0.0, 1.0, 0.0)                       # cost = tokens, so priorities are the times themselves
    jobs = [(0.0, math.inf, 1, 10), (0.0, math.inf, 1, 5), (1.5, math.inf, 1, 1)]
    start, fin = so.simulate(so.SJF, model, jobs, pipelined=2)
    assert start == [1.0, 0.0, 2.0] and fin == [17.0, 6.0, 7.0]
    start, fin = so.simulate(so.SJF, model, jobs, pipelined=True)
    assert start == [1.0, 0.0, 2.0] and fin == [16.0, 6.0, 17.0]
    # FIFO keeps arrival order in both stages: A loads first and B, D wait behind its computation
    start, fin = so.simulate(so.FIFO, model, jobs, pipelined=2)
    assert start == [0.0, 1.0, 2.0] and fin == [11.0, 16.0, 17.0]


@pytest.mark.parametrize("policy", [so.FIFO, so.SJF, so.SJF_PT, so.LSTF, so.EDF])
def test_staged_replay_conserves_work_and_respects_both_stages(policy):
    rng = np.random.default_rng(70 + policy)
    n = 14
    jobs = random_jobs(rng, n, all_at_zero=False)
    load = [float(x) for x in rng.uniform(0.01, 0.3, n)]
    comp = [float(x) for x in rng.uniform(0.005, 0.4, n)]
    start, fin = so.simulate(policy, MODEL, jobs, load, comp, 2)
    for i in range(n):
        assert start[i] >= jobs[i][0] and fin[i] >= start[i] + load[i] + comp[i] - 1e-12
    by_load = sorted(range(n), key=lambda i: start[i])
    for a, b in zip(by_load, by_load[1:]):                      # the loading stage holds one job at a time
        assert start[b] >= start[a] + load[a] - 1e-12
    by_comp = sorted(range(n), key=lambda i: fin[i])
    for a, b in zip(by_comp, by_comp[1:]):                      # and so does the compute stage
        assert fin[b] - comp[b] >= fin[a] - 1e-12
    # the compute stage never idles while a loaded job waits: every compute start is either the end of the
    # previous computation or the moment the job's own loading finished
    for k, i in enumerate(by_comp):
        cs = fin[i] - comp[i]
        prev_end = fin[by_comp[k - 1]] if k else -math.inf
        assert abs(cs - prev_end) < 1e-9 or abs(cs - (start[i] + load[i])) < 1e-9 or \
            any(abs(cs - (start[j] + load[j])) < 1e-9 for j in range(n))
    # with nothing to load and everybody present, the staged replay is the single-server one
    zero = [0.0] * n
    present = [(0.0, j[1], j[2], j[3]) for j in jobs]
    assert so.simulate(policy, MODEL, present, zero, comp, 2)[1] == so.simulate(policy, MODEL, present, zero, comp, False)[1]


@pytest.mark.parametrize("seed", range(6))
def test_staged_sjf_beats_loading_order_on_average_when_compute_queues(seed):
    """Brute force over all compute orders of a small loaded backlog: when every job is loaded before the
    compute stage frees up, the staged SJF replay computes them in the order that minimises the mean."""
    rng = np.random.default_rng(300 + seed)
    n = 6
    comp = [float(x) for x in rng.uniform(0.1, 2.0, n)]
    load = [1e-3] * n                                           # everything is loaded by t = 6 ms
    model = (0.0, 0.0, 1.0, 0.0)
    jobs = [(0.0, math.inf, 1, int(c * 1000)) for c in comp]    # SJF priority = compute tokens
    blocker = [(0.0, math.inf, 1, 1)]                           # a first job that occupies the compute stage
    all_jobs = blocker + jobs
    times_l = [1e-3] + load
    times_c = [1.0] + comp
    _, fin = so.simulate(so.SJF, model, all_jobs, times_l, times_c, 2)
    best = min(sum(itertools.accumulate(comp[i] for i in perm)) for perm in itertools.permutations(range(n)))
    # the blocker (fewest tokens) loads and computes first, ending at 1.001; the rest follow back to back
    got = sum(f - fin[0] for f in fin[1:])
    assert abs(got - best) < 1e-9


def test_line_fit_closed_forms():
    a, b = so.fit_line([1000, 3000], [0.1, 0.5])
    assert abs(a - 2e-4) < 1e-15 and abs(b + 0.1) < 1e-12
    rng = np.random.default_rng(3)
    x = rng.uniform(100, 50000, 40)
    y = 1.3e-5 * x + 0.02
    a, b = so.fit_line(list(x), list(y))
    assert abs(a - 1.3e-5) < 1e-15 and abs(b - 0.02) < 1e-10
    y_noisy = y + rng.normal(0, 1e-3, 40)
    a, b = so.fit_line(list(x), list(y_noisy))
    pa, pb = np.polyfit(x, y_noisy, 1)
    assert abs(a - pa) < 1e-12 and abs(b - pb) < 1e-9
