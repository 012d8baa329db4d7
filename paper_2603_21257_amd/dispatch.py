"""Callers of the library's multi-request dispatcher (paper Sections 3.1 and 3.2).

The stage threads, the queues, the policy order, the slot admission and the hand-over between the
stages are inside libcalvo (calvo_dispatch_*); this module only keeps time for a trace: it submits
every request at its arrival time and collects the results.  serve_trace_serial is the baseline the
paper's dispatcher is compared with: one request at a time, the library's scheduler choosing the
next one.
"""
from __future__ import annotations

import time
from typing import Callable, Optional, Sequence

from . import binding as cb


class Dispatcher:
    """Handle of a calvo_dispatcher: `with Dispatcher(ctx, policy, ...) as d: d.submit(...); d.wait(i)`."""

    def __init__(self, ctx: Optional[int], policy: int, model=None, **kw):
        self.handle = cb.calvo_dispatch_create(ctx, policy, model, **kw)

    def submit(self, **job) -> int:
        return cb.calvo_dispatch_submit(self.handle, **job)

    def wait(self, job: int) -> dict:
        return cb.calvo_dispatch_wait(self.handle, job)

    def poll(self, job: int):
        return cb.calvo_dispatch_poll(self.handle, job)

    def table(self, job: int):
        return cb.calvo_dispatch_table(self.handle, job)

    def release(self, job: int) -> None:
        cb.calvo_dispatch_release(self.handle, job)

    def stats(self) -> dict:
        return cb.calvo_dispatch_stats_get(self.handle)

    def close(self) -> None:
        if self.handle:
            h, self.handle = self.handle, 0
            cb.calvo_dispatch_destroy(h)

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False


def serve_trace(d: Dispatcher, arrivals: Sequence[float], make_job: Callable[[int], dict], hold_s: Optional[Sequence[float]] = None,
                on_finish: Optional[Callable[[int, int, dict], None]] = None, on_release: Optional[Callable[[int], None]] = None,
                clock: Callable[[], float] = time.perf_counter, sleep: Callable[[float], None] = time.sleep):
    """Submits request i (keyword arguments of calvo_dispatch_submit from make_job(i)) at arrivals[i]
    seconds after entry, in the order of arrivals, and returns the list of results
    (calvo_dispatch_result as dicts, times on the dispatcher's clock) indexed like arrivals.

    hold_s[i]: request i keeps its HBM slots this long after its first token (the decode phase that
    follows the prefill), then they are released; None releases at the first token.  on_finish(i,
    job id, result) runs when request i has finished, before its slots are released; on_release(i) right
    before they are.
    """
    n = len(arrivals)
    order = sorted(range(n), key=lambda i: (arrivals[i], i))
    ids, results = [None] * n, [None] * n
    holders = []                                            # (release time, request)
    pending = []
    t0 = clock()

    def collect():
        # polls: a request that waits for HBM slots only moves on when a finished one is released here
        for i in list(pending):
            res = d.poll(ids[i])
            if res is None:
                continue
            pending.remove(i)
            results[i] = res
            if on_finish:
                on_finish(i, ids[i], res)
            holders.append((clock() - t0 + (float(hold_s[i]) if hold_s is not None else 0.0), i))
        now = clock() - t0
        for when, i in [h for h in holders if h[0] <= now]:
            if on_release:
                on_release(i)
            d.release(ids[i])
            holders.remove((when, i))

    for i in order:
        while True:
            now = clock() - t0
            if now >= arrivals[i]:
                break
            collect()
            sleep(min(arrivals[i] - now, 2e-4))
        ids[i] = d.submit(**make_job(i))
        pending.append(i)
    while pending or holders:
        collect()
        sleep(2e-4)
    return results


def serve_trace_serial(policy: int, model: Optional[Sequence[float]], jobs: Sequence[Sequence[float]],
                       run_request: Callable[[int], None], clock: Callable[[], float] = time.perf_counter,
                       sleep: Callable[[float], None] = time.sleep):
    """One request at a time, non-preemptively, in the order the library's scheduler dictates.

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
