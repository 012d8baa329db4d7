"""Policy comparison on a synthetic request trace, in the setting of the paper's Section 4.3: Poisson
arrivals, contexts of the sizes of its Table 1, a share of every context reusable (the hit ratio), TTFT
deadlines drawn as the request's interference-free TTFT times 2, 4 or 8.  The trace is replayed by the
library (calvo_sched_simulate, loading and computation as two stages that each serve their
highest-priority ready request) under FIFO, SJF on the
prefill token count (SJF-PT), SJF on the binary linear cost model, EDF and LSTF.

No dataset is involved: lengths are drawn around the Table 1 means.  The default cost model holds this
build's own measurements on one MI355X for the Llama-3-8B-shaped stack (loading 128 KiB per token at
56.6 GB/s; 32 layers of attention at about 27 us per computed token over a 32K context) - the
computation part covers attention only, which is all this path computes.

    python -m paper_2603_21257_amd.sched_study [--qps 2.5] [--requests 400] [--seed 1] [--model measured|remote-pool]
"""
from __future__ import annotations

import argparse

import numpy as np

from . import binding as cb

# (load s/token, load fixed s, compute s/token, compute fixed s)
MEASURED_MODEL = (2.32e-6, 1.0e-4, 2.7e-5, 2.0e-4)
# A model in the paper's regime, where loading is the slow part: loading at the rate of its sampled request
# R1 (Section 2.3: 0.361 s for a context of the LooGLE mean length); the computation rate is this study's own
# assumption (a whole-model prefill at 16K tokens per second plus 15 ms), the paper prints none.
REMOTE_POOL_MODEL = (0.361 / 28100, 0.0, 1.0 / 16000, 0.015)
TABLE1_MEANS = [(28100, 28), (28300, 61), (38300, 209)]      # (context, query) tokens: LooGLE, ICL, code
POLICIES = [("FIFO", cb.CALVO_POLICY_FIFO), ("SJF-PT", cb.CALVO_POLICY_SJF_PT), ("SJF", cb.CALVO_POLICY_SJF),
            ("EDF", cb.CALVO_POLICY_EDF), ("LSTF", cb.CALVO_POLICY_LSTF)]


def make_trace(seed: int, n: int, qps: float, hit_ratios, model=MEASURED_MODEL):
    """jobs[i] = (arrival_s, deadline_s, ctx_tokens to load, query_tokens to compute).  Every request
    draws a dataset, a context within +-30 % of its mean, and one of hit_ratios; the part of the
    context that is not reusable is computed together with the query."""
    rng = np.random.default_rng(seed)
    t = 0.0
    jobs = []
    for _ in range(n):
        t += rng.exponential(1.0 / qps)
        ctx, qry = TABLE1_MEANS[int(rng.integers(0, len(TABLE1_MEANS)))]
        ctx = int(ctx * rng.uniform(0.7, 1.3))
        hit = float(hit_ratios[int(rng.integers(0, len(hit_ratios)))])
        load = int(ctx * hit) // 16 * 16
        comp = ctx - load + qry
        t_load, t_comp = cb.calvo_cost_estimate(model, (0.0, 0.0, load, comp))
        slo = (t_load + t_comp) * float(rng.choice([2.0, 4.0, 8.0]))
        jobs.append((t, t + slo, load, comp))
    return jobs


def run(jobs, model=MEASURED_MODEL):
    """{policy: (average TTFT s, share of requests that met their deadline)}"""
    arr = np.array([j[0] for j in jobs])
    ddl = np.array([j[1] for j in jobs])
    res = {}
    for name, pol in POLICIES:
        _, fin = cb.calvo_sched_simulate(pol, model, jobs, pipelined=2)
        res[name] = (float(np.mean(fin - arr)), float(np.mean(fin <= ddl)))
    return res


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--qps", type=float, default=2.5)
    ap.add_argument("--requests", type=int, default=400)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--model", choices=["measured", "remote-pool"], default="measured")
    args = ap.parse_args()
    model = MEASURED_MODEL if args.model == "measured" else REMOTE_POOL_MODEL
    print(f"{args.requests} requests, Poisson arrivals at {args.qps:g} per second, model {model}")
    print(f"{'hit ratios':<22}" + "".join(f"{name:>18}" for name, _ in POLICIES))
    for label, ratios in [("25 %", [0.25]), ("50 %", [0.5]), ("75 %", [0.75]), ("100 %", [1.0]),
                          ("mixed 25-100 %", [0.25, 0.5, 0.75, 1.0])]:
        res = run(make_trace(args.seed, args.requests, args.qps, ratios, model), model)
        print(f"{label:<22}" + "".join(f"{res[n][0] * 1e3:>9.1f} ms {res[n][1] * 100:>4.0f} %" for n, _ in POLICIES))
    print("(average TTFT, share of deadlines met)")


if __name__ == "__main__":
    main()
