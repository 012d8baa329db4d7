"""Multi-request dispatcher on top of the C ABI (paper Section 3.2): whenever the GPU path is
free, the library's scheduler (calvo_sched_pick) chooses among the requests that have arrived,
and the chosen request is run to its first token.  Sequencing and time keeping only - the
policy arithmetic is in the library, the work in its HIP code.
"""
from __future__ import annotations

import time
from typing import Callable, Optional, Sequence

from . import binding as cb


def serve_trace(policy: int, model: Optional[Sequence[float]], jobs: Sequence[Sequence[float]],
                run_request: Callable[[int], None], clock: Callable[[], float] = time.perf_counter,
                sleep: Callable[[float], None] = time.sleep):
    """Serves every job once, non-preemptively, in the order the policy dictates.

    jobs[i] = (arrival_s, deadline_s, ctx_tokens, query_tokens), arrival relative to the moment this
    function is entered.  run_request(i) must return when request i's first token is ready.
    Returns (start_s, finish_s) lists on the same time axis; TTFT_i = finish_s[i] - arrival_s[i].
    """
    n = len(jobs)
    done = [False] * n
    start, finish = [0.0] * n, [0.0] * n
    t0 = clock()
    for _ in range(n):
        while True:
            now = clock() - t0
            i = cb.calvo_sched_pick(policy, model, jobs, done, now)
            if i >= 0:
                break
            sleep(max(0.0, min(jobs[k][0] for k in range(n) if not done[k]) - now))
        start[i] = now
        run_request(i)
        finish[i] = clock() - t0
        done[i] = True
    return start, finish


def serve_trace_pooled(policy: int, model: Optional[Sequence[float]], jobs: Sequence[Sequence[float]],
                       pool: int, n_blocks: Sequence[int], run_request: Callable[[int, "object"], None],
                       hold_s: Sequence[float], clock: Callable[[], float] = time.perf_counter,
                       sleep: Callable[[float], None] = time.sleep):
    """serve_trace with the KV slots of every request taken from a calvo_pool (paper Section 3.1,
    proactive allocation): the moment a request is picked - when its loading is issued - its
    n_blocks[i] destination slots are requested.  If HBM has room they are granted at once; if not,
    the request waits for slots to come back (reactive allocation) and loading starts then.  Request
    i keeps its slots for hold_s[i] seconds after its first token (the decode phase that follows the
    prefill) and releases them afterwards.

    run_request(i, table) gets the granted slot ids (int32 array of n_blocks[i]).
    Returns (start_s, finish_s, reactive, alloc_wait_s): reactive[i] tells whether request i had to
    wait for slots, alloc_wait_s[i] for how long.
    """
    n = len(jobs)
    done = [False] * n
    start, finish = [0.0] * n, [0.0] * n
    reactive, alloc_wait = [False] * n, [0.0] * n
    holders = []                                       # (release time, table)
    t0 = clock()

    def release_expired(now):
        for when, table in holders:
            if when <= now:
                cb.calvo_pool_release(pool, table)
        holders[:] = [h for h in holders if h[0] > now]

    for _ in range(n):
        while True:
            now = clock() - t0
            release_expired(now)
            i = cb.calvo_sched_pick(policy, model, jobs, done, now)
            if i >= 0:
                break
            sleep(max(0.0, min(jobs[k][0] for k in range(n) if not done[k]) - now))
        table, ticket = cb.calvo_pool_admit(pool, [], int(n_blocks[i]))
        if table is None:                              # HBM short: reactive allocation
            reactive[i] = True
            while table is None:
                if not holders:
                    cb.calvo_pool_cancel(pool, ticket)
                    raise RuntimeError(f"request {i} needs {n_blocks[i]} slots and nothing is left to release")
                wake = min(h[0] for h in holders)
                sleep(max(0.0, wake - (clock() - t0)))
                release_expired(clock() - t0)
                table = cb.calvo_pool_retry(pool, ticket, int(n_blocks[i]))
            alloc_wait[i] = (clock() - t0) - now
        start[i] = clock() - t0
        run_request(i, table)
        finish[i] = clock() - t0
        done[i] = True
        holders.append((finish[i] + float(hold_s[i]), table))
    for _, table in holders:
        cb.calvo_pool_release(pool, table)
    return start, finish, reactive, alloc_wait


def serve_trace_two_stage(policy: int, model: Optional[Sequence[float]], jobs: Sequence[Sequence[float]],
                          try_issue: Callable[[int], bool], load_done: Callable[[int], bool],
                          finished: Callable[[int], bool], clock: Callable[[], float] = time.perf_counter,
                          sleep: Callable[[float], None] = time.sleep, poll_s: float = 1e-4):
    """Loading and computation as two stages that progress on their own (paper Section 3.1): the loading
    stage takes the next request - the policy's pick among those that have arrived - as soon as the
    previous request's blocks are all loaded, while that request (and earlier ones) may still be
    computing; computation follows in the order of loading.

    try_issue(i) queues request i's loading and computation without waiting for either and returns
    True, or returns False if it cannot be queued yet (no room for its blocks: it is tried again);
    load_done(i) tells whether all of i's blocks are loaded; finished(i) whether its first token is
    ready.  Returns (start_s, finish_s) as serve_trace does; a finish time is taken when the loop
    notices it (every poll_s while it idles).
    """
    n = len(jobs)
    issued = [False] * n
    start, finish = [0.0] * n, [0.0] * n
    in_flight = []
    loading = -1
    n_done = 0
    t0 = clock()
    while n_done < n:
        now = clock() - t0
        for i in list(in_flight):
            if finished(i):
                finish[i] = now
                in_flight.remove(i)
                n_done += 1
        if loading >= 0 and load_done(loading):
            loading = -1
        if loading < 0 and not all(issued):
            i = cb.calvo_sched_pick(policy, model, jobs, issued, now)
            if i >= 0 and try_issue(i):
                start[i] = now
                issued[i] = True
                loading = i
                in_flight.append(i)
                continue
            if i < 0 and not in_flight:
                sleep(max(0.0, min(jobs[k][0] for k in range(n) if not issued[k]) - now))
                continue
        sleep(poll_s)
    return start, finish
