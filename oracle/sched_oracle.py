"""CPU oracle for the inter-request scheduling part.  TEST INFRASTRUCTURE ONLY.

Only tests/ may import this file.  Plain Python floats (fp64), one decision at a time, no
shared code with the library.

What it follows (paper Section 3.2): the service cost of a request is modelled as two
independent linear components - T_load in the number of context tokens to load, T_comp in
the number of query tokens; shortest-job-first on T_load + T_comp optimises the average
TTFT; least-slack-time-first with LST = DDL - T_load - T_comp optimises SLO attainment.
Compared policies (Section 4.3): FIFO, SJF on the prefill token count only (SJF-PT), and
earliest deadline first.

Readings taken where the paper is silent: service is non-preemptive; the scheduler decides
whenever the server (its loading stage, when loading and computation are pipelined as in
Section 3.1) becomes free, among the requests that have arrived by then; if none has, it
idles until the next arrival; ties go to the earlier arrival, then to the lower index; the
token count that SJF-PT orders by is the number of tokens that are computed (the query
tokens); a component with zero tokens costs nothing (no fixed term).

Pins (tests/test_oracle_sched.py): the two-request example the paper works out in Section
2.3 (0.49 s vs 0.41 s average TTFT), brute force over all service orders (SJF is the best
order for the mean when all requests are present; EDF meets every deadline whenever some
order does), closed forms of the line fit, conservation properties of the replay.
"""
from __future__ import annotations

import math

FIFO, SJF, SJF_PT, LSTF, EDF = range(5)


def fit_line(tokens, seconds):
    """Ordinary least squares line through the samples: returns (per_token_s, fixed_s)."""
    n = len(tokens)
    assert n >= 2 and n == len(seconds)
    mx = math.fsum(tokens) / n
    my = math.fsum(seconds) / n
    sxx = math.fsum((x - mx) ** 2 for x in tokens)
    sxy = math.fsum((x - mx) * (y - my) for x, y in zip(tokens, seconds))
    assert sxx > 0
    a = sxy / sxx
    return a, my - a * mx


def estimate(model, job):
    """(T_load, T_comp) of a job (arrival, deadline, ctx_tokens, query_tokens) under
    model = (load_per_token, load_fixed, comp_per_token, comp_fixed)."""
    la, lb, ca, cb = model
    _, _, ctx, query = job
    t_load = la * ctx + lb if ctx > 0 else 0.0
    t_comp = ca * query + cb if query > 0 else 0.0
    return t_load, t_comp


def priority(policy, model, job):
    arrival, deadline, ctx, query = job
    if policy == FIFO:
        return arrival
    if policy == SJF_PT:
        return float(query)
    if policy == EDF:
        return deadline
    t_load, t_comp = estimate(model, job)
    if policy == SJF:
        return t_load + t_comp
    if policy == LSTF:
        return deadline - t_load - t_comp
    raise ValueError(policy)


def pick(policy, model, jobs, done, now):
    """Index of the job served next at time now, or -1 if no unserved job has arrived."""
    best = None
    for i, job in enumerate(jobs):
        if (done is not None and done[i]) or not (job[0] <= now):
            continue
        key = (priority(policy, model, job), job[0], i)
        if best is None or key < best:
            best = key
    return -1 if best is None else best[2]


def simulate_staged(policy, model, jobs, load_s=None, comp_s=None):
    """Replay with loading and computation as two stages that each serve their highest-priority ready
    request (Section 3.1: a stage's dispatcher works on the request of highest priority whose lower-level
    blocks are ready): the loading stage picks among the requests that have arrived, the compute
    stage among those whose loading has finished.  Both are non-preemptive.  Decisions are taken in
    time order; when both stages could decide at the same instant, the compute stage goes first."""
    n = len(jobs)
    t_load = [load_s[i] if load_s is not None else estimate(model, jobs[i])[0] for i in range(n)]
    t_comp = [comp_s[i] if comp_s is not None else estimate(model, jobs[i])[1] for i in range(n)]
    start, finish = [0.0] * n, [0.0] * n
    load_end = [math.inf] * n
    taken = [False] * n           # by the loading stage
    done = [False] * n            # by the compute stage
    loader_free = compute_free = -math.inf
    for _ in range(2 * n):
        t_l = math.inf
        if not all(taken):
            t_l = max(loader_free, min(jobs[i][0] for i in range(n) if not taken[i]))
        t_c = math.inf
        ready = [load_end[i] for i in range(n) if taken[i] and not done[i]]
        if ready:
            t_c = max(compute_free, min(ready))
        if t_c <= t_l:
            best = None
            for i in range(n):
                if taken[i] and not done[i] and load_end[i] <= t_c:
                    key = (priority(policy, model, jobs[i]), jobs[i][0], i)
                    if best is None or key < best:
                        best = key
            i = best[2]
            finish[i] = t_c + t_comp[i]
            compute_free = finish[i]
            done[i] = True
        else:
            i = pick(policy, model, jobs, taken, t_l)
            start[i] = t_l
            load_end[i] = t_l + t_load[i]
            loader_free = load_end[i]
            taken[i] = True
    return start, finish


def simulate(policy, model, jobs, load_s=None, comp_s=None, pipelined=False):
    """Replay of the trace on one server; returns (start, finish) lists.  pipelined: False/0 = one
    request at a time; True/1 = loading overlaps the previous request's computation, computation in
    loading order; 2 = simulate_staged."""
    if int(pipelined) == 2:
        return simulate_staged(policy, model, jobs, load_s, comp_s)
    n = len(jobs)
    done = [False] * n
    start, finish = [0.0] * n, [0.0] * n
    loader_free = compute_free = -math.inf
    for _ in range(n):
        free_at = loader_free if pipelined else compute_free
        next_arrival = min(job[0] for i, job in enumerate(jobs) if not done[i])
        now = max(free_at, next_arrival)
        i = pick(policy, model, jobs, done, now)
        t_load = load_s[i] if load_s is not None else estimate(model, jobs[i])[0]
        t_comp = comp_s[i] if comp_s is not None else estimate(model, jobs[i])[1]
        start[i] = now
        load_end = now + t_load
        comp_start = max(load_end, compute_free) if pipelined else load_end
        finish[i] = comp_start + t_comp
        loader_free, compute_free = load_end, finish[i]
        done[i] = True
    return start, finish
