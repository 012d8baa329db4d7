"""The library's dispatcher (calvo_dispatch_*) as a dry run, without a GPU: with no context the stage
threads run the same queues, policy order and slot admission on the host clock, the loading stage
busy for a job's sim_load_s and the compute stage for its sim_comp_s.  Its decisions are compared
with the scheduling oracle's staged replay (oracle/sched_oracle.py: both stages serve their
highest-priority ready request) on traces whose decisions are separated from the events they depend
on by several milliseconds, so thread wake-up jitter cannot change them; the serial baseline loop of
dispatch.py runs on a virtual clock."""
import math
import time

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import dispatch

MODEL = (2.0e-6, 1.0e-3, 3.0e-5, 2.0e-3)
POLICIES = [cb.CALVO_POLICY_FIFO, cb.CALVO_POLICY_SJF, cb.CALVO_POLICY_SJF_PT, cb.CALVO_POLICY_LSTF, cb.CALVO_POLICY_EDF]
MARGIN = 6e-3


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

    start, fin = dispatch.serve_trace_serial(policy, MODEL, jobs, run, clock=clk, sleep=clk.sleep)
    s0, f0 = cb.calvo_sched_simulate(policy, MODEL, jobs, pipelined=0)
    assert np.allclose(start, s0, atol=1e-9) and np.allclose(fin, f0, atol=1e-9)


def staged_trace(policy, n=6):
    """A small trace (arrival, deadline, ctx tokens, query tokens), stage times of 30..100 ms, whose staged
    replay takes every decision at least MARGIN away from any arrival or end of loading that could
    change it, and between priorities that differ.  Deterministic: the first seed that qualifies."""
    model = (1.0e-6, 0.0, 1.0e-4, 0.0)                     # 30000..100000 ctx tokens, 300..1000 query tokens
    for seed in range(4000):
        rng = np.random.default_rng(seed)
        arr = np.sort(rng.uniform(0.0, 0.3, n))
        arr[0] = 0.0
        jobs = []
        for a in arr:
            ctx, qry = int(rng.integers(30000, 100000)), int(rng.integers(300, 1000))
            jobs.append((float(a), float(a) + float(rng.uniform(0.2, 1.0)), ctx, qry))
        start, fin = so.simulate_staged(policy, model, jobs)
        load_end = [start[i] + so.estimate(model, jobs[i])[0] for i in range(n)]
        comp_start = [fin[i] - so.estimate(model, jobs[i])[1] for i in range(n)]
        events = list(arr[1:]) + load_end
        decisions = start[1:] + comp_start
        gap = min(abs(d - e) for d in decisions for e in events if abs(d - e) > 1e-12)
        pri = sorted(so.priority(policy, model, j) for j in jobs)
        if gap >= MARGIN and min(np.diff(arr)) >= MARGIN and all(b - a > 1e-6 for a, b in zip(pri, pri[1:])):
            return model, jobs
    raise AssertionError("no seed gives a trace with well-separated decisions")


@pytest.mark.parametrize("policy", POLICIES)
def test_dry_run_takes_the_decisions_of_the_staged_replay(policy):
    model, jobs = staged_trace(policy)
    n = len(jobs)
    with dispatch.Dispatcher(None, policy, model) as d:
        t0 = time.perf_counter()
        res = dispatch.serve_trace(
            d, [j[0] for j in jobs],
            lambda i: dict(n_prefix_blocks=jobs[i][2] // 16, suffix_len=jobs[i][3], deadline_s=jobs[i][1] - jobs[i][0],
                           sim_load_s=so.estimate(model, jobs[i])[0], sim_comp_s=so.estimate(model, jobs[i])[1]))
        assert time.perf_counter() - t0 < 5.0
        st = d.stats()
    assert st["jobs_submitted"] == n and st["jobs_done"] == n
    # replay with the submission times the dispatcher saw
    base = res[0]["submit_s"]
    seen = [(r["submit_s"] - base, r["submit_s"] - base + (j[1] - j[0]), j[2], j[3]) for r, j in zip(res, jobs)]
    assert max(abs(s[0] - j[0]) for s, j in zip(seen, jobs)) < MARGIN / 2, "the host could not keep the arrival times"
    start, fin = so.simulate_staged(policy, model, seen)
    got_start = [r["load_start_s"] - base for r in res]
    got_fin = [r["first_token_s"] - base for r in res]
    got_comp = [r["compute_start_s"] - base for r in res]
    assert list(np.argsort(got_start)) == list(np.argsort(start)), "loading stage served another order"
    want_comp = [fin[i] - so.estimate(model, seen[i])[1] for i in range(n)]
    assert list(np.argsort(got_comp)) == list(np.argsort(want_comp)), "compute stage served another order"
    lag = np.array(got_fin) - np.array(fin)                  # threads wake a little late, never early
    assert lag.min() > -1e-3 and lag.max() < MARGIN * 2, lag
    # the library's own staged replay says the same
    s2, f2 = cb.calvo_sched_simulate(policy, model, seen, pipelined=2)
    assert np.allclose(s2, start, atol=1e-12) and np.allclose(f2, fin, atol=1e-12)
    for r in res:
        assert r["status"] == 0 and not r["reactive"]
        assert r["submit_s"] <= r["load_start_s"] <= r["load_end_s"] <= r["compute_start_s"] <= r["first_token_s"]


def test_dry_run_overlaps_loading_with_the_previous_computation():
    """Two stages on different requests at once: n equal jobs take load + n * max(load, comp) + ..., not n * (load + comp)."""
    with dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO) as d:
        ids = [d.submit(suffix_len=1, sim_load_s=0.03, sim_comp_s=0.03) for _ in range(5)]
        res = [d.wait(i) for i in ids]
    span = res[-1]["first_token_s"] - res[0]["load_start_s"]
    assert 0.03 * 6 - 1e-3 <= span < 0.03 * 6 + 0.03, span       # serial service would take 0.30 s
    for a, b in zip(res, res[1:]):
        assert b["load_start_s"] < a["first_token_s"]             # the next request loads while this one computes


def test_dry_run_slot_admission_is_proactive_then_reactive():
    """Three requests of 6 slots on a pool of 10: the first is granted at issue; the second has to wait in the
    loading stage until the first is released, the third until the second is."""
    pool = cb.calvo_pool_create(10)
    try:
        with dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO, pool=pool) as d:
            ids = [d.submit(n_prefix_blocks=5, suffix_len=16, sim_load_s=0.01, sim_comp_s=0.01) for _ in range(3)]
            r0 = d.wait(ids[0])
            t0 = d.table(ids[0])
            assert len(t0) == 6 and len(set(t0.tolist())) == 6 and not r0["reactive"]
            assert cb.calvo_pool_counts(pool)["waiting"] == 1
            assert d.poll(ids[1]) is None
            with pytest.raises(cb.CalvoError):
                d.table(ids[1])                                   # no slots yet
            time.sleep(0.05)
            assert d.poll(ids[1]) is None                         # still waiting: nothing was released
            d.release(ids[0])
            r1 = d.wait(ids[1])
            assert r1["reactive"] and r1["alloc_wait_s"] >= 0.05
            t1 = d.table(ids[1])
            assert len(set(t1.tolist())) == 6
            time.sleep(0.02)
            d.release(ids[1])
            r2 = d.wait(ids[2])
            assert r2["reactive"] and r2["alloc_wait_s"] >= 0.02
            assert r2["load_end_s"] >= r1["first_token_s"]
            with pytest.raises(cb.CalvoError):
                d.release(ids[1])                                 # once per job
            # job 2 is not released by hand: the dispatcher gives its slots back when it goes
        assert cb.calvo_pool_counts(pool) == {"free": 10, "used": 0, "refs": 0, "waiting": 0}
    finally:
        cb.calvo_pool_destroy(pool)


def test_dry_run_shared_run_is_referenced_per_job():
    pool = cb.calvo_pool_create(16)
    try:
        run = cb.calvo_pool_reserve(pool, 4)                      # a resident prefix run, held by its owner
        with dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO, pool=pool) as d:
            a = d.submit(block_table=run, n_prefix_blocks=6, n_shared=4, suffix_len=16, sim_load_s=0.005, sim_comp_s=0.005)
            b = d.submit(block_table=run, n_prefix_blocks=4, n_shared=4, suffix_len=20, sim_load_s=0.005, sim_comp_s=0.005)
            d.wait(a), d.wait(b)
            ta, tb = d.table(a), d.table(b)
            assert list(ta[:4]) == list(run) and list(tb[:4]) == list(run)
            assert len(ta) == 7 and len(tb) == 6 and not set(ta[4:].tolist()) & set(tb[4:].tolist())
            assert cb.calvo_pool_counts(pool)["refs"] == 4 * 3 + 3 + 2
            d.release(a)
            assert cb.calvo_pool_counts(pool)["refs"] == 4 * 2 + 2
            d.release(b)
        assert cb.calvo_pool_counts(pool) == {"free": 12, "used": 4, "refs": 4, "waiting": 0}
        cb.calvo_pool_release(pool, run)
    finally:
        cb.calvo_pool_destroy(pool)


def test_dispatcher_refuses_bad_arguments():
    with pytest.raises(cb.CalvoError):
        cb.calvo_dispatch_create(None, 9)
    with dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO) as d:
        for bad in (dict(n_prefix_blocks=-1), dict(suffix_len=-1), dict(n_prefix_blocks=2, n_shared=3),
                    dict(sim_load_s=math.nan), dict(sim_comp_s=-1.0), dict(sim_load_s=math.inf)):
            with pytest.raises(cb.CalvoError):
                d.submit(**bad)
        with pytest.raises(cb.CalvoError):
            d.wait(0)                                             # nothing was queued by the refused calls
        i = d.submit(sim_load_s=0.02, sim_comp_s=0.0)
        with pytest.raises(cb.CalvoError):
            d.release(i)                                          # not finished yet
        d.wait(i)
        d.release(i)
        with pytest.raises(cb.CalvoError):
            d.poll(7)
    pool = cb.calvo_pool_create(4)
    try:
        with dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO, pool=pool) as d:
            i = d.submit(n_prefix_blocks=8, suffix_len=1, sim_load_s=0.0, sim_comp_s=0.0)     # can never fit
            with pytest.raises(cb.CalvoError):
                d.wait(i)
            with pytest.raises(cb.CalvoError):
                d.poll(i)
    finally:
        cb.calvo_pool_destroy(pool)


def test_destroy_releases_finished_jobs_so_that_waiting_ones_finish():
    """Nobody releases anything: closing the dispatcher gives the finished jobs' slots back one after the other,
    the jobs that wait for them run, and every slot is free afterwards."""
    pool = cb.calvo_pool_create(10)
    try:
        d = dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO, pool=pool)
        ids = [d.submit(n_prefix_blocks=5, suffix_len=16, sim_load_s=0.005, sim_comp_s=0.005) for _ in range(3)]
        d.wait(ids[0])
        t0 = time.perf_counter()
        d.close()
        assert time.perf_counter() - t0 < 5.0
        assert cb.calvo_pool_counts(pool) == {"free": 10, "used": 0, "refs": 0, "waiting": 0}
    finally:
        cb.calvo_pool_destroy(pool)


def test_a_failed_job_reports_what_the_stage_thread_saw():
    pool = cb.calvo_pool_create(4)
    try:
        with dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO, pool=pool) as d:
            run = np.array([9], np.int32)                         # not a slot of this pool: the admission is refused
            i = d.submit(block_table=run, n_prefix_blocks=2, n_shared=1, suffix_len=1, sim_load_s=0.0, sim_comp_s=0.0)
            with pytest.raises(cb.CalvoError) as ei:
                d.wait(i)
            assert ei.value.code == cb.CALVO_EINVAL and f"job {i} failed" in str(ei.value)
            ok = d.submit(n_prefix_blocks=1, suffix_len=1, sim_load_s=0.0, sim_comp_s=0.0)   # the dispatcher goes on
            assert d.wait(ok)["status"] == 0
    finally:
        cb.calvo_pool_destroy(pool)


@pytest.mark.parametrize("policy", POLICIES)
def test_dry_run_random_trace_with_a_tight_pool_drains(policy):
    """60 jobs of random size on a pool that holds about three of them, random hold times: every job gets
    distinct slots while it holds them, every job finishes, nothing is left allocated."""
    rng = np.random.default_rng(100 + policy)
    n = 60
    blocks = rng.integers(1, 40, n)
    suffix = rng.integers(0, 64, n)
    need = [int(b) + -(-int(s) // 16) for b, s in zip(blocks, suffix)]
    arrivals = np.sort(rng.uniform(0.0, 0.15, n))
    deadlines = rng.uniform(0.05, 0.5, n)
    pool = cb.calvo_pool_create(100)
    live = {}
    try:
        with dispatch.Dispatcher(None, policy, (1e-6, 0.0, 1e-5, 0.0), pool=pool) as d:
            def on_finish(i, jid, res):
                t = d.table(jid)
                assert len(t) == need[i] and len(set(t.tolist())) == need[i] and t.min() >= 0 and t.max() < 100
                for j, other in live.items():                      # jobs that still hold slots share none with this one
                    assert not set(t.tolist()) & other, (i, j)
                live[i] = set(t.tolist())

            t0 = time.perf_counter()
            res = dispatch.serve_trace(
                d, list(arrivals),
                lambda i: dict(n_prefix_blocks=int(blocks[i]), suffix_len=int(suffix[i]), deadline_s=float(deadlines[i]),
                               sim_load_s=float(blocks[i]) * 1e-4, sim_comp_s=float(suffix[i]) * 2e-5),
                hold_s=list(rng.uniform(0.0, 0.01, n)), on_finish=on_finish, on_release=lambda i: live.pop(i))
            assert time.perf_counter() - t0 < 20.0
        assert not live and all(r is not None and r["status"] == 0 for r in res)
        assert sum(r["reactive"] for r in res) > 0, "the pool was never short: the case does not test the reactive path"
        assert cb.calvo_pool_counts(pool) == {"free": 100, "used": 0, "refs": 0, "waiting": 0}
    finally:
        cb.calvo_pool_destroy(pool)


def test_destroy_does_not_wait_for_slots_that_are_held_outside():
    """The pool's slots are held by someone else: the job can never be admitted.  Closing the dispatcher fails it
    instead of waiting for ever, and withdraws its admission."""
    pool = cb.calvo_pool_create(8)
    try:
        held = cb.calvo_pool_reserve(pool, 6)
        d = dispatch.Dispatcher(None, cb.CALVO_POLICY_FIFO, pool=pool)
        i = d.submit(n_prefix_blocks=4, suffix_len=1, sim_load_s=0.0, sim_comp_s=0.0)      # 5 slots, 2 free
        time.sleep(0.05)
        assert d.poll(i) is None
        t0 = time.perf_counter()
        d.close()
        assert time.perf_counter() - t0 < 5.0
        assert cb.calvo_pool_counts(pool) == {"free": 2, "used": 6, "refs": 6, "waiting": 0}
        cb.calvo_pool_release(pool, held)
    finally:
        cb.calvo_pool_destroy(pool)
