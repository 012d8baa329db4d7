"""The policy study (paper Section 4.3 setting, synthetic trace, replayed by the library with both stages
serving their highest-priority ready request) reproduces the paper's qualitative findings on seeded
traces: ordering by the modelled cost beats FIFO, and when every context is fully reusable - all the cost
is loading - ordering by the binary cost model beats ordering by the prefill token count (Fig. 9)."""
import pytest

from paper_2603_21257_amd import sched_study as st


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_loading_aware_sjf_beats_token_count_sjf_when_loading_dominates(seed):
    for model, qps in [(st.MEASURED_MODEL, 16.0), (st.REMOTE_POOL_MODEL, 2.0)]:
        res = st.run(st.make_trace(seed, 400, qps, [1.0], model), model)
        assert res["SJF"][0] < 0.98 * res["SJF-PT"][0] < 0.98 * res["FIFO"][0], res
        assert res["SJF"][1] >= res["FIFO"][1]


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_cost_ordering_beats_fifo_on_mixed_hit_ratios(seed):
    res = st.run(st.make_trace(seed, 400, 3.0, [0.25, 0.5, 0.75, 1.0]))
    assert res["SJF"][0] < 0.7 * res["FIFO"][0], res
    assert res["SJF"][1] > res["FIFO"][1]
    assert res["LSTF"][0] <= res["FIFO"][0] and res["EDF"][0] <= res["FIFO"][0]


def test_an_idle_system_serves_everyone_alike():
    res = st.run(st.make_trace(5, 200, 0.2, [0.5, 1.0]))
    ttft = [v[0] for v in res.values()]
    # Poisson arrivals still collide now and then; the policies differ only on those few requests
    assert max(ttft) - min(ttft) < 0.02 * min(ttft) and all(v[1] >= 0.97 for v in res.values())
