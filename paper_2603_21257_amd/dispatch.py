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
