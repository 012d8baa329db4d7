"""The paper's scheduling comparison (Section 4.3) served for real on one GPU: a seeded trace of
prefix-hit requests with Poisson arrivals goes through the dispatcher loop (dispatch.serve_trace)
under each queue policy, every request running the whole HIP path - load its cached context from
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

    python -m paper_2603_21257_amd.serve_study [--requests 48] [--load 1.2] [--seed 1]
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


class PipelinedServer(Server):
    """The same path with several requests in flight: a request's blocks get slots of their own from
    the slot allocator (paper Section 3.1, allocation at the moment loading is issued), loading and
    attention are queued without waiting, and the next request's loading starts while this one still
    computes.  The compute stream is the caller's, so a request's completion can be polled."""

    def __init__(self, n_layers=8, seed=7, max_query=MAX_QRY, depth=4):
        import torch
        self.torch = torch
        self.L, self.Hq, self.Hkv, self.D = n_layers, 32, 8, 128
        self.max_query = max_query
        per_req = (MAX_CTX + max_query) // 16 + 1
        slots = depth * per_req
        self.shape = s = wl.Shape(self.L, self.Hq, self.Hkv, self.D, "bf16", slots)
        dev = torch.device("cuda:0")
        self.host_blocks = MAX_CTX // 16
        self.arena = hostmem.PinnedBuffer(self.L * self.host_blocks * s.blk_bytes)
        self.host = wl.fill_normal_(self.arena.tensor((self.L, self.host_blocks, s.blk_elems), torch.bfloat16), seed)
        self.pool = torch.empty((self.L, slots, s.blk_elems), dtype=torch.bfloat16, device=dev)
        mk = lambda h, sd: wl.fill_normal_(torch.empty((self.L, max_query, h, self.D), dtype=torch.bfloat16, device=dev), sd)
        self.q, self.ks, self.vs = mk(self.Hq, seed + 1), mk(self.Hkv, seed + 2), mk(self.Hkv, seed + 3)
        self.outs = [torch.empty((self.L, max_query, self.Hq, self.D), dtype=torch.bfloat16, device=dev) for _ in range(depth)]
        self.out = self.outs[0]
        self.table = np.arange(per_req, dtype=np.int32)          # Server's single-request calls (profiling) use the first region
        self.stream = torch.cuda.Stream()
        self.ctx = cb.calvo_create(self.L, self.Hq, self.Hkv, self.D, cb.CALVO_BF16, slots, self.pool,
                                   staging_bytes=256 << 20, compute_stream=self.stream.cuda_stream)
        self.slots = cb.calvo_pool_create(slots)
        self.flight = {}                                         # request -> (table, done event, out index)
        self.free_outs = list(range(depth))
        self.last_issued = -1

    def close(self):
        if self.slots:
            cb.calvo_pool_destroy(self.slots)
            self.slots = 0
        super().close()

    def try_issue(self, i, ctx_tokens, qry_tokens):
        nb = ctx_tokens // 16 + -(-qry_tokens // 16)
        if not self.free_outs or cb.calvo_pool_counts(self.slots)["free"] < nb:
            return False
        table = cb.calvo_pool_reserve(self.slots, nb)
        o = self.free_outs.pop()
        stride = self.host_blocks * self.shape.blk_bytes
        r = cb.make_request(self.host.data_ptr(), stride, table, ctx_tokens // 16, qry_tokens)
        cu = np.array([0, qry_tokens], np.int32)
        cb.calvo_kv_ingest(self.ctx, [r], 0, self.L)
        out = self.outs[o]
        for l in range(self.L):
            cb.calvo_prefill_attn(self.ctx, l, self.q[l, :qry_tokens], self.ks[l, :qry_tokens], self.vs[l, :qry_tokens],
                                  out[l, :qry_tokens], [r], cu, 0.0)
        ev = self.torch.cuda.Event()
        ev.record(self.stream)
        self.flight[i] = (table, ev, o)
        self.last_issued = i
        return True

    def load_done(self, i):
        # only asked about the request issued last: the per-layer events belong to the latest loading call
        assert i == self.last_issued
        return cb.calvo_layer_event(self.ctx, self.L - 1, cb.CALVO_EV_QUERY)

    def finished(self, i):
        table, ev, o = self.flight[i]
        if not ev.query():
            return False
        cb.calvo_pool_release(self.slots, table)
        self.free_outs.append(o)
        del self.flight[i]
        return True

    def compute_only(self, ctx_tokens, qry_tokens):
        super().compute_only(ctx_tokens, qry_tokens)
        self.stream.synchronize()

    def serve(self, ctx_tokens, qry_tokens):
        super().serve(ctx_tokens, qry_tokens)
        self.stream.synchronize()


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
            _, fin = dispatch.serve_trace(pol, model, jobs, lambda i: srv.serve(jobs[i][2], jobs[i][3]))
            fin = np.array(fin)
            _, sim = cb.calvo_sched_simulate(pol, model, jobs, pipelined=0)
            res[name] = {"ttft_s": float(np.mean(fin - arr)), "replay_ttft_s": float(np.mean(sim - arr)),
                         "met": float(np.mean(fin <= ddl)), "replay_met": float(np.mean(sim <= ddl))}
        return res, model
    finally:
        srv.close()


def study_two_stage(n_requests=48, load=1.2, seed=1, n_layers=8, max_query=MAX_QRY, policies=POLICIES, log=print):
    """The same trace on the pipelined server, once request by request (serve_trace) and once with
    loading and computation as two stages (serve_trace_two_stage).
    {policy: dict(serial mean TTFT s, two-stage mean TTFT s, deadlines met by each)} and the model."""
    srv = PipelinedServer(n_layers, max_query=max_query)
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
        warm = [(0.0, math.inf, c, q) for c, q in lengths[:4]]           # first use of the two-stage path: untimed
        dispatch.serve_trace_two_stage(cb.CALVO_POLICY_FIFO, model, warm, lambda i: srv.try_issue(i, warm[i][2], warm[i][3]),
                                       srv.load_done, srv.finished, poll_s=0.0)
        for name, pol in policies:
            _, fin1 = dispatch.serve_trace(pol, model, jobs, lambda i: srv.serve(jobs[i][2], jobs[i][3]))
            # poll_s = 0: the loop spins (yielding the processor) so that a finished loading is noticed at once
            _, fin2 = dispatch.serve_trace_two_stage(pol, model, jobs, lambda i: srv.try_issue(i, jobs[i][2], jobs[i][3]),
                                                     srv.load_done, srv.finished, poll_s=0.0)
            fin1, fin2 = np.array(fin1), np.array(fin2)
            res[name] = {"serial_ttft_s": float(np.mean(fin1 - arr)), "two_stage_ttft_s": float(np.mean(fin2 - arr)),
                         "serial_met": float(np.mean(fin1 <= ddl)), "two_stage_met": float(np.mean(fin2 <= ddl)),
                         "serial_span_s": float(fin1.max()), "two_stage_span_s": float(fin2.max())}
        counts = cb.calvo_pool_counts(srv.slots)
        assert counts["used"] == 0 and not srv.flight, "slots left allocated after the trace"
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
                    help="compare request-by-request service with loading and computation as two stages")
    ap.add_argument("--max-query", type=int, default=MAX_QRY)
    args = ap.parse_args()
    if args.two_stage:
        res, _ = study_two_stage(args.requests, args.load, args.seed, args.layers, args.max_query)
        print(f"{args.requests} requests at {args.load:g} x capacity, {args.layers} layers, queries up to {args.max_query} tokens")
        print(f"{'policy':<8}{'serial TTFT ms':>16}{'two-stage ms':>14}{'met':>6}{'met':>6}{'serial span ms':>16}{'two-stage ms':>14}")
        for name, _ in POLICIES:
            r = res[name]
            print(f"{name:<8}{r['serial_ttft_s'] * 1e3:>16.1f}{r['two_stage_ttft_s'] * 1e3:>14.1f}{r['serial_met'] * 100:>5.0f}%"
                  f"{r['two_stage_met'] * 100:>5.0f}%{r['serial_span_s'] * 1e3:>16.1f}{r['two_stage_span_s'] * 1e3:>14.1f}")
        return
    res, _ = study(args.requests, args.load, args.seed, args.layers)
    print(f"{args.requests} requests at {args.load:g} x capacity, {args.layers} layers")
    print(f"{'policy':<8}{'mean TTFT ms':>14}{'replayed ms':>13}{'deadlines met':>15}{'replayed':>10}")
    for name, _ in POLICIES:
        r = res[name]
        print(f"{name:<8}{r['ttft_s'] * 1e3:>14.1f}{r['replay_ttft_s'] * 1e3:>13.1f}{r['met'] * 100:>14.0f}%{r['replay_met'] * 100:>9.0f}%")


if __name__ == "__main__":
    main()
