"""The scheduling example of the paper's Section 2.3 on the real path: two queued requests, the first
loading-heavy with few query tokens, the second with a quarter of the context to load and four times
the query tokens.  FIFO and token-count SJF serve the first one first; SJF on the fitted binary cost
model serves the second first and lowers the average TTFT.  The cost model is fitted from this GPU's own measured loading / computation times."""
import math
import time

import numpy as np
import pytest
import torch

import hip_harness as hh
from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import dispatch
from paper_2603_21257_amd import hostmem
from paper_2603_21257_amd import workload as wl

pytestmark = pytest.mark.gpu


def test_loading_aware_sjf_lowers_average_ttft_on_the_gpu():
    L, Hq, Hkv, D = 8, 32, 8, 128
    lens = [(49152, 64), (12288, 256)]                       # R1: 3 GiB to load; R2: 0.75 GiB, 4x the query tokens
    shape = wl.Shape(L, Hq, Hkv, D, "bf16", sum(-(-(p + s) // 16) for p, s in lens) + 8)
    w = wl.make_custom(shape, lens, seed=321, with_payload=False)
    s = w.shape
    dev = torch.device("cuda:0")
    arena = hostmem.PinnedBuffer(L * w.host_blocks * s.blk_bytes)
    try:
        host = arena.tensor((L, w.host_blocks, s.blk_elems), torch.bfloat16)
        wl.fill_normal_(host, 1)
        pool = torch.empty((L, s.pool_blocks, s.blk_elems), dtype=torch.bfloat16, device=dev)
        T = w.total_suffix
        q = wl.fill_normal_(torch.empty((L, T, Hq, D), dtype=torch.bfloat16, device=dev), 2)
        ks = wl.fill_normal_(torch.empty((L, T, Hkv, D), dtype=torch.bfloat16, device=dev), 3)
        vs = wl.fill_normal_(torch.empty((L, T, Hkv, D), dtype=torch.bfloat16, device=dev), 4)
        out = torch.empty((L, T, Hq, D), dtype=torch.bfloat16, device=dev)
        ctx = cb.calvo_create(L, Hq, Hkv, D, cb.CALVO_BF16, s.pool_blocks, pool, staging_bytes=128 << 20)
        try:
            reqs = hh.make_requests(w, host)
            cu = w.cu_suffix

            def load_only(i):
                cb.calvo_kv_ingest(ctx, [reqs[i]], 0, L)
                cb.calvo_layer_event(ctx, L - 1, cb.CALVO_EV_HOST_WAIT)

            def compute_only(i):
                a, b = int(cu[i]), int(cu[i + 1])
                for l in range(L):
                    cb.calvo_prefill_attn(ctx, l, q[l, a:b], ks[l, a:b], vs[l, a:b], out[l, a:b], [reqs[i]],
                                          np.array([0, b - a], np.int32), 0.0)
                torch.cuda.synchronize()

            def run_request(i):                              # load and compute overlap inside one request
                a, b = int(cu[i]), int(cu[i + 1])
                cb.calvo_kv_ingest(ctx, [reqs[i]], 0, L)
                for l in range(L):
                    cb.calvo_prefill_attn(ctx, l, q[l, a:b], ks[l, a:b], vs[l, a:b], out[l, a:b], [reqs[i]],
                                          np.array([0, b - a], np.int32), 0.0)
                torch.cuda.synchronize()

            def timed(fn, i):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn(i)
                return time.perf_counter() - t0

            # ---- offline profiling -> binary linear cost model (Section 3.2)
            for i in (0, 1):
                run_request(i)
            load_t = [min(timed(load_only, i) for _ in range(2)) for i in (0, 1)]
            comp_t = [min(timed(compute_only, i) for _ in range(2)) for i in (0, 1)]
            la, lb = cb.calvo_cost_fit([lens[0][0], lens[1][0]], load_t)
            ca, cbb = cb.calvo_cost_fit([lens[0][1], lens[1][1]], comp_t)
            model = (la, lb, ca, cbb)
            print(f"profiled load {load_t}, compute {comp_t} -> model {model}", flush=True)
            assert load_t[0] > 2.5 * load_t[1]

            jobs = [(0.0, math.inf, lens[0][0], lens[0][1]), (0.0, math.inf, lens[1][0], lens[1][1])]
            avg = {}
            for name, pol in [("FIFO", cb.CALVO_POLICY_FIFO), ("SJF_PT", cb.CALVO_POLICY_SJF_PT), ("SJF", cb.CALVO_POLICY_SJF)]:
                start, fin = dispatch.serve_trace(pol, model, jobs, run_request)
                first = int(np.argmin(start))
                avg[name] = (first, float(np.mean(fin)))
                print(f"{name}: first served R{first + 1}, TTFT {fin}, average {np.mean(fin) * 1e3:.1f} ms", flush=True)
            assert avg["FIFO"][0] == 0 and avg["SJF_PT"][0] == 0 and avg["SJF"][0] == 1
            assert avg["SJF"][1] < 0.85 * avg["FIFO"][1] and avg["SJF"][1] < 0.85 * avg["SJF_PT"][1]
            # the replay with the measured per-request times predicts the measured averages
            whole = [timed(run_request, i) for i in (0, 1)]
            for name, pol in [("FIFO", cb.CALVO_POLICY_FIFO), ("SJF", cb.CALVO_POLICY_SJF)]:
                _, fin = cb.calvo_sched_simulate(pol, model, jobs, whole, [0.0, 0.0])
                assert abs(float(np.mean(fin)) - avg[name][1]) < 0.15 * avg[name][1]
        finally:
            cb.calvo_destroy(ctx)
    finally:
        arena.free()
