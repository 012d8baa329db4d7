"""The paper's scheduling comparison (Section 4.3) served for real on one GPU: a seeded trace of
prefix-hit requests with Poisson arrivals is served one request at a time (dispatch.serve_trace_serial)
or through the library's staged dispatcher (--two-stage, --three-stage) under each queue policy, every request running the whole HIP path - load its cached context from
pinned host memory, prefill its query tokens layer by layer - and TTFTs are taken with the wall clock.
The binary linear cost model is fitted from a few profiled requests first (Section 3.2: offline
profiling), deadlines are the model's interference-free TTFT times 2, 4 or 8, and the library's own
replay of the same trace (calvo_sched_simulate) is printed beside the measurement: it shows how well
the cost model predicts the real server.

No dataset is involved: context lengths are drawn log-uniformly between 4K and 48K tokens, query
lengths between 16 and 512 tokens, every context fully reusable; the stack is Llama-3-8B-shaped with
8 layers (the per-request cost scales with the layer count, the comparison does not).  All requests
read the same host bytes and reuse the same pool slots one after the other - service is
non-preemptive and one request at a time, so nothing is shared in time.

    python -m paper_2603_21257_amd.serve_study [--requests 48] [--load 1.2] [--seed 1] [--two-stage | --three-stage]
"""
from __future__ import annotations

import argparse
import math
import time

import numpy as np

from . import binding as cb
from . import dispatch
from . import hostmem
from . import workload as wl

POLICIES = [("FIFO", cb.CALVO_POLICY_FIFO), ("SJF-PT", cb.CALVO_POLICY_SJF_PT), ("SJF", cb.CALVO_POLICY_SJF),
            ("EDF", cb.CALVO_POLICY_EDF), ("LSTF", cb.CALVO_POLICY_LSTF)]
MAX_CTX, MAX_QRY = 49152, 512


def draw_lengths(rng, n):
    """(context tokens, query tokens) per request: contexts log-uniform in [4K, 48K] in whole blocks."""
    ctx = np.exp(rng.uniform(math.log(4096), math.log(MAX_CTX), n)).astype(np.int64) // 16 * 16
    qry = rng.integers(16, MAX_QRY + 1, n)
    return [(int(c), int(q)) for c, q in zip(ctx, qry)]


class Server:
    """One context on cuda:0 that can run any request of up to MAX_CTX + MAX_QRY tokens to its first token."""

    def __init__(self, n_layers=8, seed=7):
        import torch
        self.torch = torch
        self.L, self.Hq, self.Hkv, self.D = n_layers, 32, 8, 128
        slots = (MAX_CTX + MAX_QRY) // 16 + 8
        self.shape = s = wl.Shape(self.L, self.Hq, self.Hkv, self.D, "bf16", slots)
        dev = torch.device("cuda:0")
        self.host_blocks = MAX_CTX // 16
        self.arena = hostmem.PinnedBuffer(self.L * self.host_blocks * s.blk_bytes)
        self.host = wl.fill_normal_(self.arena.tensor((self.L, self.host_blocks, s.blk_elems), torch.bfloat16), seed)
        self.pool = torch.empty((self.L, slots, s.blk_elems), dtype=torch.bfloat16, device=dev)
        self.q = wl.fill_normal_(torch.empty((self.L, MAX_QRY, self.Hq, self.D), dtype=torch.bfloat16, device=dev), seed + 1)
        self.ks = wl.fill_normal_(torch.empty((self.L, MAX_QRY, self.Hkv, self.D), dtype=torch.bfloat16, device=dev), seed + 2)
        self.vs = wl.fill_normal_(torch.empty((self.L, MAX_QRY, self.Hkv, self.D), dtype=torch.bfloat16, device=dev), seed + 3)
        self.out = torch.empty((self.L, MAX_QRY, self.Hq, self.D), dtype=torch.bfloat16, device=dev)
        self.table = np.random.default_rng(seed).permutation(slots).astype(np.int32)
        self.ctx = cb.calvo_create(self.L, self.Hq, self.Hkv, self.D, cb.CALVO_BF16, slots, self.pool,
                                   staging_bytes=256 << 20)

    def close(self):
        if self.ctx:
            cb.calvo_destroy(self.ctx)
            self.ctx = 0
        self.arena.free()

    def request(self, ctx_tokens, qry_tokens):
        nb = ctx_tokens // 16
        stride = self.host_blocks * self.shape.blk_bytes
        return cb.make_request(self.host.data_ptr(), stride, self.table[: nb + -(-qry_tokens // 16)], nb, qry_tokens)

    def load_only(self, ctx_tokens, qry_tokens):
        cb.calvo_kv_ingest(self.ctx, [self.request(ctx_tokens, qry_tokens)], 0, self.L)
        cb.calvo_layer_event(self.ctx, self.L - 1, cb.CALVO_EV_HOST_WAIT)

    def compute_only(self, ctx_tokens, qry_tokens):
        r = self.request(ctx_tokens, qry_tokens)
        cu = np.array([0, qry_tokens], np.int32)
        for l in range(self.L):
            cb.calvo_prefill_attn(self.ctx, l, self.q[l, :qry_tokens], self.ks[l, :qry_tokens], self.vs[l, :qry_tokens],
                                  self.out[l, :qry_tokens], [r], cu, 0.0)
        self.torch.cuda.synchronize()

    def serve(self, ctx_tokens, qry_tokens):
        """Whole request: loading and attention overlap layer by layer; returns when the last layer is done."""
        r = self.request(ctx_tokens, qry_tokens)
        cu = np.array([0, qry_tokens], np.int32)
        cb.calvo_kv_ingest(self.ctx, [r], 0, self.L)
        for l in range(self.L):
            cb.calvo_prefill_attn(self.ctx, l, self.q[l, :qry_tokens], self.ks[l, :qry_tokens], self.vs[l, :qry_tokens],
                                  self.out[l, :qry_tokens], [r], cu, 0.0)
        self.torch.cuda.synchronize()

    def fit_model(self):
        """Offline profiling -> (load s/token, load fixed s, compute s/token, compute fixed s)."""
        def best(fn, c, q):
            ts = []
            for _ in range(3):
                self.torch.cuda.synchronize()
                t0 = time.perf_counter()
                fn(c, q)
                ts.append(time.perf_counter() - t0)
            return min(ts)
        ctxs, qrys = [4096, 12288, 24576, 49152], [16, 128, 256, 512]
        self.serve(8192, 64)                                    # warm up
        load_t = [best(self.load_only, c, 16) for c in ctxs]
        # Inside a request loading and attention overlap layer by layer, so what a request costs beyond
        # its loading is the part of the computation that is left over at the end: that is what the
        # second term of the model is fitted to (whole request minus loading alone, mid-size context).
        comp_t = [max(0.0, best(self.serve, 24576, q) - load_t[2]) for q in qrys]
        la, lb = cb.calvo_cost_fit(ctxs, load_t)
        ca, cbb = cb.calvo_cost_fit(qrys, comp_t)
        return (la, lb, ca, cbb)


class DispatchServer(Server):
    """The same path behind the library's dispatcher (calvo_dispatch_*): loading and computation - and,
    with three_stage, the emulated link below them - are stages of their own that work on different
    requests at the same time (paper Section 3.1).  A request's blocks get slots from the slot
    allocator when its lowest transfer is issued; the pool holds `depth` requests of the largest
    size, so under load some requests find HBM short and are allocated reactively.

    pageable: the cached contexts sit in ordinary host memory (the remote store of the three-stage
    path) instead of page-locked memory."""

    def __init__(self, n_layers=8, seed=7, max_query=MAX_QRY, depth=4, pageable=False, l3_GBps=0.0):
        import torch
        self.torch = torch
        self.L, self.Hq, self.Hkv, self.D = n_layers, 32, 8, 128
        self.max_query, self.pageable, self.l3_GBps = max_query, pageable, l3_GBps
        per_req = (MAX_CTX + max_query) // 16 + 1
        slots = depth * per_req
        self.shape = s = wl.Shape(self.L, self.Hq, self.Hkv, self.D, "bf16", slots)
        dev = torch.device("cuda:0")
        self.host_blocks = MAX_CTX // 16
        if pageable:
            self.arena = None
            self.host = wl.fill_normal_(torch.empty((self.L, self.host_blocks, s.blk_elems), dtype=torch.bfloat16), seed)
        else:
            self.arena = hostmem.PinnedBuffer(self.L * self.host_blocks * s.blk_bytes)
            self.host = wl.fill_normal_(self.arena.tensor((self.L, self.host_blocks, s.blk_elems), torch.bfloat16), seed)
        self.pool = torch.empty((self.L, slots, s.blk_elems), dtype=torch.bfloat16, device=dev)
        mk = lambda h, sd: wl.fill_normal_(torch.empty((self.L, max_query, h, self.D), dtype=torch.bfloat16, device=dev), sd)
        self.q, self.ks, self.vs = mk(self.Hq, seed + 1), mk(self.Hkv, seed + 2), mk(self.Hkv, seed + 3)
        self.out = torch.empty((self.L, max_query, self.Hq, self.D), dtype=torch.bfloat16, device=dev)
        self.table = np.arange(per_req, dtype=np.int32)          # the one-request-at-a-time calls use the first region
        self.ctx = cb.calvo_create(self.L, self.Hq, self.Hkv, self.D, cb.CALVO_BF16, slots, self.pool, staging_bytes=256 << 20)
        self.slots = cb.calvo_pool_create(slots)

    def close(self):
        if self.slots:
            cb.calvo_pool_destroy(self.slots)
            self.slots = 0
        if self.ctx:
            cb.calvo_destroy(self.ctx)
            self.ctx = 0
        if self.arena:
            self.arena.free()

    def _ingest(self, r):
        if self.pageable:
            cb.calvo_kv_ingest_l3(self.ctx, [r], 0, self.L, l3_GBps=self.l3_GBps)
        else:
            cb.calvo_kv_ingest(self.ctx, [r], 0, self.L)

    def load_only(self, ctx_tokens, qry_tokens):
        self._ingest(self.request(ctx_tokens, qry_tokens))
        if self.pageable:
            cb.calvo_l3_wait(self.ctx)
        cb.calvo_layer_event(self.ctx, self.L - 1, cb.CALVO_EV_HOST_WAIT)

    def serve(self, ctx_tokens, qry_tokens):
        r = self.request(ctx_tokens, qry_tokens)
        cu = np.array([0, qry_tokens], np.int32)
        self._ingest(r)
        for l in range(self.L):
            cb.calvo_prefill_attn(self.ctx, l, self.q[l, :qry_tokens], self.ks[l, :qry_tokens], self.vs[l, :qry_tokens],
                                  self.out[l, :qry_tokens], [r], cu, 0.0)
        if self.pageable:
            cb.calvo_l3_wait(self.ctx)
        self.torch.cuda.synchronize()

    def run_trace(self, policy, model, jobs, three_stage=False, on_result=None):
        """The trace through a dispatcher of its own; returns the list of calvo_dispatch_result dicts.
        on_result(i, table, out) sees request i's granted table and its output [L][query][Hq][D] before
        its slots are released."""
        torch = self.torch
        outs = {}
        stride = self.host_blocks * self.shape.blk_bytes
        q_stride = self.max_query * self.Hq * self.D * 2
        kv_stride = self.max_query * self.Hkv * self.D * 2

        with dispatch.Dispatcher(self.ctx, policy, model, three_stage=three_stage, pool=self.slots,
                                 l3_GBps=self.l3_GBps if three_stage else 0.0) as d:
            def make_job(i):
                _, ddl, c, qn = jobs[i]
                outs[i] = torch.empty((self.L, qn, self.Hq, self.D), dtype=torch.bfloat16, device=self.pool.device)
                return dict(host_kv=self.host.data_ptr(), host_layer_stride=stride, n_prefix_blocks=c // 16, suffix_len=qn,
                            q=self.q, k_suffix=self.ks, v_suffix=self.vs, out=outs[i], q_layer_stride=q_stride,
                            kv_layer_stride=kv_stride, deadline_s=(ddl - jobs[i][0]) if math.isfinite(ddl) else 0.0)

            def on_finish(i, jid, res):
                if on_result:
                    on_result(i, d.table(jid), outs[i])
                outs.pop(i)                                   # the output buffer was this request's own

            res = dispatch.serve_trace(d, [j[0] for j in jobs], make_job, on_finish=on_finish)
            self.last_stats = d.stats()
        counts = cb.calvo_pool_counts(self.slots)
        assert counts["used"] == 0 and counts["waiting"] == 0, "slots left allocated after the trace"
        return res


def make_jobs(lengths, model, load, seed):
    """Poisson arrivals at `load` times the server's capacity for these requests (1 = as fast as it can
    serve them on average); deadline = arrival + model TTFT x {2, 4, 8}."""
    rng = np.random.default_rng(seed)
    solo = [sum(cb.calvo_cost_estimate(model, (0.0, 0.0, c, q))) for c, q in lengths]
    rate = load / float(np.mean(solo))
    t, jobs = 0.0, []
    for (c, q), s in zip(lengths, solo):
        t += rng.exponential(1.0 / rate)
        jobs.append((t, t + s * float(rng.choice([2.0, 4.0, 8.0])), c, q))
    return jobs


def study(n_requests=48, load=1.2, seed=1, n_layers=8, log=print):
    """{policy: dict(measured mean TTFT s, replayed mean TTFT s, deadlines met, replayed deadlines met)} and the model."""
    srv = Server(n_layers)
    try:
        model = srv.fit_model()
        log(f"fitted cost model: load {model[0] * 1e6:.3f} us/token + {model[1] * 1e3:.3f} ms, "
            f"compute {model[2] * 1e6:.3f} us/token + {model[3] * 1e3:.3f} ms")
        lengths = draw_lengths(np.random.default_rng(seed), n_requests)
        jobs = make_jobs(lengths, model, load, seed + 1)
        arr = np.array([j[0] for j in jobs])
        ddl = np.array([j[1] for j in jobs])
        res = {}
        for name, pol in POLICIES:
            _, fin = dispatch.serve_trace_serial(pol, model, jobs, lambda i: srv.serve(jobs[i][2], jobs[i][3]))
            fin = np.array(fin)
            _, sim = cb.calvo_sched_simulate(pol, model, jobs, pipelined=0)
            res[name] = {"ttft_s": float(np.mean(fin - arr)), "replay_ttft_s": float(np.mean(sim - arr)),
                         "met": float(np.mean(fin <= ddl)), "replay_met": float(np.mean(sim <= ddl))}
        return res, model
    finally:
        srv.close()


def study_staged(n_requests=48, load=1.2, seed=1, n_layers=8, max_query=MAX_QRY, policies=POLICIES, three_stage=False,
                 l3_GBps=50.0, depth=4, on_result=None, log=print):
    """The same trace once request by request (serve_trace_serial) and once through the library's
    dispatcher with its stages working on different requests at the same time: loading and computation
    (two stages, contexts in page-locked memory), or - three_stage - the emulated link of l3_GBps in
    front of them (contexts in pageable memory; the paper's Section 4.1 link is 400 Gbps = 50 GB/s).
    {policy: dict(serial / staged mean TTFT s, deadlines met, spans, requests allocated reactively,
    link utilisation)} and the model.  on_result(i, (ctx tokens, query tokens), table, out, server) sees
    the granted block table and the output of every request of the untimed first pass (six requests
    queued at once) before its slots are released."""
    srv = DispatchServer(n_layers, max_query=max_query, depth=depth, pageable=three_stage, l3_GBps=l3_GBps if three_stage else 0.0)
    try:
        model = srv.fit_model()
        log(f"fitted cost model: load {model[0] * 1e6:.3f} us/token + {model[1] * 1e3:.3f} ms, "
            f"compute {model[2] * 1e6:.3f} us/token + {model[3] * 1e3:.3f} ms")
        rng = np.random.default_rng(seed)
        lengths = [(c, int(rng.integers(16, max_query + 1))) for c, _ in draw_lengths(rng, n_requests)]
        jobs = make_jobs(lengths, model, load, seed + 1)
        arr = np.array([j[0] for j in jobs])
        ddl = np.array([j[1] for j in jobs])
        res = {}
        # first use of the staged path, untimed: the first requests of the trace, all queued at once; this
        # is the pass whose results on_result sees (a check there would hold up the timed passes)
        warm = [(0.0, math.inf, c, q) for c, q in lengths[:6]]
        srv.run_trace(cb.CALVO_POLICY_FIFO, model, warm, three_stage,
                      on_result=(lambda i, table, o: on_result(i, warm[i][2:], table, o, srv)) if on_result else None)
        for name, pol in policies:
            _, fin1 = dispatch.serve_trace_serial(pol, model, jobs, lambda i: srv.serve(jobs[i][2], jobs[i][3]))
            out = srv.run_trace(pol, model, jobs, three_stage)
            base = min(r["submit_s"] - a for r, a in zip(out, arr))      # the dispatcher's clock at the trace's time zero
            fin1, fin2 = np.array(fin1), np.array([r["first_token_s"] - base for r in out])
            st = srv.last_stats
            res[name] = {"serial_ttft_s": float(np.mean(fin1 - arr)), "staged_ttft_s": float(np.mean(fin2 - arr)),
                         "serial_met": float(np.mean(fin1 <= ddl)), "staged_met": float(np.mean(fin2 <= ddl)),
                         "serial_span_s": float(fin1.max()), "staged_span_s": float(fin2.max()),
                         "reactive": int(sum(r["reactive"] for r in out)),
                         "alloc_wait_s": float(sum(r["alloc_wait_s"] for r in out)),
                         "link_busy": (st["link_busy_s"] / st["link_span_s"]) if st["link_span_s"] > 0 else None}
        return res, model
    finally:
        srv.close()


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--requests", type=int, default=48)
    ap.add_argument("--load", type=float, default=1.2)
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--layers", type=int, default=8)
    ap.add_argument("--two-stage", action="store_true",
                    help="compare request-by-request service with loading and computation as two stages of the library's dispatcher")
    ap.add_argument("--three-stage", action="store_true",
                    help="the same with the emulated link in front: link, PCIe and compute as three stages")
    ap.add_argument("--l3-gbps", type=float, default=50.0, help="rate of the emulated link in 1e9 bytes/s")
    ap.add_argument("--depth", type=int, default=4, help="HBM pool size in requests of the largest size")
    ap.add_argument("--max-query", type=int, default=MAX_QRY)
    args = ap.parse_args()
    if args.two_stage or args.three_stage:
        res, _ = study_staged(args.requests, args.load, args.seed, args.layers, args.max_query, three_stage=args.three_stage,
                              l3_GBps=args.l3_gbps, depth=args.depth)
        what = f"three stages, link {args.l3_gbps:g} GB/s" if args.three_stage else "two stages"
        print(f"{args.requests} requests at {args.load:g} x capacity, {args.layers} layers, queries up to {args.max_query} tokens, "
              f"{what}, pool of {args.depth} requests")
        print(f"{'policy':<8}{'serial TTFT ms':>16}{'staged ms':>12}{'met':>6}{'met':>6}{'serial span ms':>16}{'staged ms':>12}"
              f"{'reactive':>10}{'link busy':>11}")
        for name, _ in POLICIES:
            r = res[name]
            busy = f"{r['link_busy'] * 100:.0f}%" if r["link_busy"] is not None else "-"
            print(f"{name:<8}{r['serial_ttft_s'] * 1e3:>16.1f}{r['staged_ttft_s'] * 1e3:>12.1f}{r['serial_met'] * 100:>5.0f}%"
                  f"{r['staged_met'] * 100:>5.0f}%{r['serial_span_s'] * 1e3:>16.1f}{r['staged_span_s'] * 1e3:>12.1f}"
                  f"{r['reactive']:>10d}{busy:>11}")
        return
    res, _ = study(args.requests, args.load, args.seed, args.layers)
    print(f"{args.requests} requests at {args.load:g} x capacity, {args.layers} layers")
    print(f"{'policy':<8}{'mean TTFT ms':>14}{'replayed ms':>13}{'deadlines met':>15}{'replayed':>10}")
    for name, _ in POLICIES:
        r = res[name]
        print(f"{name:<8}{r['ttft_s'] * 1e3:>14.1f}{r['replay_ttft_s'] * 1e3:>13.1f}{r['met'] * 100:>14.0f}%{r['replay_met'] * 100:>9.0f}%")


if __name__ == "__main__":
    main()
