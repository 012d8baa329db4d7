"""The library's scheduler (host C++ behind the C ABI) against the scheduling oracle: same picks,
same replayed start / finish times, on seeded random traces.  Needs no GPU."""
import math

import numpy as np
import pytest

from oracle import sched_oracle as so
from paper_2603_21257_amd import binding as cb

POLICIES = [(cb.CALVO_POLICY_FIFO, so.FIFO), (cb.CALVO_POLICY_SJF, so.SJF), (cb.CALVO_POLICY_SJF_PT, so.SJF_PT),
            (cb.CALVO_POLICY_LSTF, so.LSTF), (cb.CALVO_POLICY_EDF, so.EDF)]
MODEL = (1.31e-5, 0.0037, 2.4e-5, 0.0011)


def trace(seed, n):
    rng = np.random.default_rng(seed)
    arrivals = np.cumsum(rng.exponential(0.15, n))                  # Poisson arrivals, as in the paper's Section 4.1
    jobs = []
    for a in arrivals:
        ctx = int(rng.choice([0, 8192, 16384, 28672, 61440]) * rng.choice([0.25, 0.5, 0.75, 1.0]))
        query = int(rng.integers(1, 1200))
        solo = sum(so.estimate(MODEL, (0, 0, ctx, query)))
        jobs.append((float(a), float(a + solo * rng.choice([2, 4, 8])), ctx, query))   # SLO = solo TTFT x {2,4,8}
    return jobs


@pytest.mark.parametrize("seed", range(4))
@pytest.mark.parametrize("cpol,opol", POLICIES)
@pytest.mark.parametrize("pipelined", [False, True, 2])
def test_replay_matches_oracle_exactly(seed, cpol, opol, pipelined):
    jobs = trace(seed, 40)
    rng = np.random.default_rng(1000 + seed)
    load = [so.estimate(MODEL, j)[0] * float(rng.uniform(0.9, 1.1)) for j in jobs]   # actual != modelled
    comp = [so.estimate(MODEL, j)[1] * float(rng.uniform(0.9, 1.1)) for j in jobs]
    want_s, want_f = so.simulate(opol, MODEL, jobs, load, comp, pipelined)
    got_s, got_f = cb.calvo_sched_simulate(cpol, MODEL, jobs, load, comp, pipelined)
    assert list(got_s) == want_s and list(got_f) == want_f
    want_s, want_f = so.simulate(opol, MODEL, jobs, None, None, pipelined)            # model's own estimates
    got_s, got_f = cb.calvo_sched_simulate(cpol, MODEL, jobs, None, None, pipelined)
    assert list(got_s) == want_s and list(got_f) == want_f


@pytest.mark.parametrize("cpol,opol", POLICIES)
def test_pick_matches_oracle(cpol, opol):
    jobs = trace(11, 25)
    rng = np.random.default_rng(5)
    for _ in range(60):
        done = [bool(x) for x in rng.integers(0, 2, len(jobs))]
        now = float(rng.uniform(0, jobs[-1][0] * 1.1))
        assert cb.calvo_sched_pick(cpol, MODEL, jobs, done, now) == so.pick(opol, MODEL, jobs, done, now)
    assert cb.calvo_sched_pick(cpol, MODEL, jobs, None, -1.0) == -1
    assert cb.calvo_sched_pick(cpol, MODEL, [], None, 0.0) == -1


def test_cost_fit_and_estimate_match_oracle():
    rng = np.random.default_rng(2)
    x = rng.uniform(1000, 60000, 30)
    y = 1.3e-5 * x + 0.01 + rng.normal(0, 2e-4, 30)
    a, b = cb.calvo_cost_fit(x, y)
    oa, ob = so.fit_line([float(v) for v in x], [float(v) for v in y])
    assert abs(a - oa) <= 1e-15 and abs(b - ob) <= 1e-12
    for job in [(0, 0, 0, 5), (0, 0, 777, 0), (0, 0, 61440, 4096)]:
        assert cb.calvo_cost_estimate(MODEL, job) == so.estimate(MODEL, job)


def test_worked_example_through_the_library():
    """Paper Section 2.3: loading-aware SJF serves R2 first (0.41 s on average instead of 0.49 s)."""
    model = (1e-3, 0.0, 1e-3, 0.0)
    jobs = [(0.0, math.inf, 361, 19), (0.0, math.inf, 199, 25)]
    load, comp = [0.361, 0.199], [0.019, 0.025]
    _, fin = cb.calvo_sched_simulate(cb.CALVO_POLICY_FIFO, model, jobs, load, comp)
    assert round(float(np.mean(fin)), 2) == 0.49
    _, fin = cb.calvo_sched_simulate(cb.CALVO_POLICY_SJF_PT, model, jobs, load, comp)
    assert round(float(np.mean(fin)), 2) == 0.49
    _, fin = cb.calvo_sched_simulate(cb.CALVO_POLICY_SJF, model, jobs, load, comp)
    assert round(float(np.mean(fin)), 2) == 0.41


def test_bad_arguments_are_rejected():
    jobs = [(0.0, 1.0, 10, 10)]
    with pytest.raises(cb.CalvoError):
        cb.calvo_sched_simulate(9, MODEL, jobs)
    with pytest.raises(cb.CalvoError):
        cb.calvo_sched_simulate(cb.CALVO_POLICY_SJF, None, jobs, [0.1], [0.1])      # SJF needs the model
    with pytest.raises(cb.CalvoError):
        cb.calvo_sched_pick(cb.CALVO_POLICY_FIFO, None, [(float("nan"), 1.0, 1, 1)], None, 0.0)
    with pytest.raises(cb.CalvoError):
        cb.calvo_cost_fit([5.0, 5.0], [1.0, 2.0])
    s, f = cb.calvo_sched_simulate(cb.CALVO_POLICY_FIFO, None, jobs, [0.1], [0.2])   # FIFO with given times: no model
    assert list(s) == [0.0] and abs(f[0] - 0.3) < 1e-15


@pytest.mark.parametrize("pipelined", [0, 1, 2])
def test_replay_rejects_unusable_measured_times(pipelined):
    """Measured times that are not finite or negative, and an unknown replay mode, are refused before
    anything is computed (a NaN loading time once left the two-stage replay without a job to pick)."""
    jobs = [(0.0, 1.0, 10, 10), (0.1, 2.0, 20, 5)]
    for load, comp in [([float("nan"), 0.1], [0.1, 0.1]), ([0.1, 0.1], [float("inf"), 0.1]), ([-0.1, 0.1], [0.1, 0.1])]:
        with pytest.raises(cb.CalvoError):
            cb.calvo_sched_simulate(cb.CALVO_POLICY_FIFO, MODEL, jobs, load, comp, pipelined)
    with pytest.raises(cb.CalvoError):
        cb.calvo_sched_simulate(cb.CALVO_POLICY_FIFO, MODEL, jobs, [0.1, 0.1], [0.1, 0.1], 3)
    with pytest.raises(cb.CalvoError):
        cb.calvo_sched_simulate(cb.CALVO_POLICY_FIFO, MODEL, jobs, [0.1, 0.1], [0.1, 0.1], -1)
