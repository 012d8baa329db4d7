#!/usr/bin/env python3
"""Benchmark of the prefix-hit prefill path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic request batch: queue the
ingest of every layer's cached prefix blocks (pinned host -> paged HBM pool), then for each
layer the suffix KV append and the paged causal attention, each layer's attention waiting
on the device for that layer's ingest.  The step time is the GPU-side TTFT of the batch.

Prints ONE JSON line (metric: prefix-hit TTFT in ms at the 64K-context workload) that also
carries the ingest GB/s against the measured host-to-device peak, the attention TFLOP/s
against the bf16 MFMA peak (roofline object) and the CPU oracle timed on a bounded sample
(cpu_baseline object).  Inputs are resident (pinned host KV, device Q / suffix KV) before
the clock starts.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0     # MI355X dense bf16, published


def profiled_traffic(config: int):
    """HBM bytes of one attention launch of workload `config`, from the rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE passes recorded under profiles/ (calibrated there against a plain copy of known size).
    Counters cannot be read from inside this process: the figure is read from the profile's line
    'HBM_BYTES_PER_LAUNCH cfg<N> = <bytes>' (None if no profile of the workload is recorded)."""
    import glob
    import re
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.md"))):
        m = re.search(r"HBM_BYTES_PER_LAUNCH cfg%d = ([0-9.eE+]+)" % config, open(path).read())
        if m:
            return float(m.group(1))
    return None


def alap_schedule(n_layers: int, n_chain: int, rho: float):
    """Which layer's loading signal each layer's attention launch waits for, so that the launches of layers
    0 .. n_chain-1 run back to back and the last of them starts when its own blocks land (layers from n_chain on
    wait for themselves).

    Load-bound step: a layer's attention is shorter than a layer's load (rho = t_att / t_load per layer < 1), so
    launches that each wait for their own layer run with idle gaps between them, and after every gap the clock has
    to ramp up again (measured: --mode attn --gap-ms).  The compute chain loses nothing by starting later.  Layer j
    lands at (j + 1) t_load and the chain has to be at layer l by n t_load - (n - 1 - l) t_att, so layer l waits for
    layer j = n - 1 - ceil((n - 1 - l) rho), never an earlier one than itself.  The caller takes rho a few percent
    high: the first launches after the idle start are slow."""
    import math
    rho = min(1.0, max(0.0, rho))
    n = min(n_chain, n_layers)
    return [max(l, n - 1 - math.ceil((n - 1 - l) * rho)) if l < n else l for l in range(n_layers)]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=3, help="workload recipe 1..7 (default 3: 64K context)")
    ap.add_argument("--staging-mib", type=int, default=-1,
                    help="size of each device staging buffer of the copy-engine ingest; 0 = zero-copy kernel "
                         "ingest; -1 = one layer of the workload's prefix bytes (at most 512 MiB)")
    ap.add_argument("--mode", choices=["full", "attn", "ingest"], default="full",
                    help="attn / ingest: run only that stage `steps` times (for profiling); no JSON contract line")
    ap.add_argument("--n-staging", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--custom", type=str, default="",
                    help="replace the workload's requests by 'P:S[,P:S...]' (prefix:suffix tokens) on the same model shape, "
                         "e.g. 32768:64 for a long-context short-query point; the JSON line then describes that workload")
    ap.add_argument("--no-three-stage", action="store_true",
                    help="skip the extra measurement with the emulated remote store in front (L3 -> L2 -> L1 -> compute)")
    ap.add_argument("--l3-whole-layers", action="store_true",
                    help="three-stage measurement: attention waits for whole layers instead of following the loader's chunks")
    ap.add_argument("--l3-gbps", type=float, default=50.0, help="emulated L3 link rate (paper Section 4.1: 400 Gbps)")
    ap.add_argument("--sample-rows", type=int, default=512)
    ap.add_argument("--tail-chunks", type=int, default=-1,
                    help="load each of the last --tail-layers layers in this many chunks with one readiness signal each, so "
                         "that their attention starts on the chunks that have landed (0 = whole layers only; -1 = 4 if loading "
                         "alone takes longer than attention alone on this workload but less than twice as long, else 0)")
    ap.add_argument("--tail-layers", type=int, default=6)
    ap.add_argument("--no-cfg4-leg", action="store_true",
                    help="skip the short run of the attention-bound 8-request batch (workload 4) that the default run appends")
    ap.add_argument("--zero-data", action="store_true",
                    help="diagnostic, with --mode attn: all inputs zero instead of N(0,1) - the matrix pipes then run at the "
                         "nominal clock, which shows the kernel's structural duty apart from the power limit")
    ap.add_argument("--gap-ms", type=float, default=0.0,
                    help="diagnostic, with --mode attn: the GPU idles this long before every attention launch (the clock "
                         "has to ramp up again after an idle gap; the kernel time is reported)")
    ap.add_argument("--no-alap", action="store_true",
                    help="queue every layer's attention behind its own layer's loading signal.  Default for load-bound "
                         "steps with large layers whose tail is loaded in chunks: the whole-layer attention launches are "
                         "queued so that they run back to back and reach the chunked tail when it lands")
    ap.add_argument("--leg", action="store_true", help="(internal) run as the appended leg: timing of the step only")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1")
        sys.exit(2)

    import torch
    from paper_2603_21257_amd import binding as cb
    from paper_2603_21257_amd import workload as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(2)
    dev = torch.device("cuda:0")
    w = wl.make_config(args.config, with_payload=False)
    if args.custom:
        lens = [tuple(int(x) for x in item.split(":")) for item in args.custom.split(",")]
        need = sum(-(-(p + q) // 16) for p, q in lens)
        base = w.shape
        shape = wl.Shape(base.n_layers, base.n_q_heads, base.n_kv_heads, base.head_dim, base.dtype, need + 16)
        w = wl.make_custom(shape, lens, seed=w.seed, with_payload=False)
        w.name = f"custom {args.custom} on the shape of cfg{args.config}"
    s = w.shape
    tdt = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    L, T = s.n_layers, w.total_suffix
    log(f"[bench] {w.name}: ingest {w.ingest_bytes() / 2**30:.2f} GiB, attention {w.attn_flop():.3e} flop")

    # ---- resident inputs
    t_setup = time.perf_counter()
    from paper_2603_21257_amd import hostmem
    arena = hostmem.PinnedBuffer(L * w.host_blocks * s.blk_bytes)       # exact size, page-locked
    host = arena.tensor((L, w.host_blocks, s.blk_elems), tdt)
    wl.fill_normal_(host, w.seed + 10)
    pool = torch.empty((L, s.pool_blocks, s.blk_elems), dtype=tdt, device=dev)
    q = wl.fill_normal_(torch.empty((L, T, s.n_q_heads, s.head_dim), dtype=tdt, device=dev), w.seed + 11)
    ks = wl.fill_normal_(torch.empty((L, T, s.n_kv_heads, s.head_dim), dtype=tdt, device=dev), w.seed + 12)
    vs = wl.fill_normal_(torch.empty((L, T, s.n_kv_heads, s.head_dim), dtype=tdt, device=dev), w.seed + 13)
    out = torch.empty((L, T, s.n_q_heads, s.head_dim), dtype=tdt, device=dev)
    if args.zero_data:
        if args.mode != "attn":
            sys.exit("--zero-data is a diagnostic of --mode attn")
        for t in (host, q, ks, vs):
            t.zero_()
    torch.cuda.synchronize()
    log(f"[bench] inputs resident after {time.perf_counter() - t_setup:.1f} s")

    # ---- measured host-to-device peak (plain pinned -> device copy, best of 3)
    nprobe = min(host.numel(), (1 << 30) // host.element_size())
    probe_dst = torch.empty(nprobe, dtype=tdt, device=dev)
    flat_host = host.view(-1)
    h2d_peak = 0.0
    for _ in range(4):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        probe_dst.copy_(flat_host[:nprobe], non_blocking=True)
        torch.cuda.synchronize()
        h2d_peak = max(h2d_peak, nprobe * host.element_size() / (time.perf_counter() - t0) / 1e9)
    del probe_dst
    log(f"[bench] measured pinned H2D peak {h2d_peak:.2f} GB/s")

    if args.staging_mib < 0:      # one copy-engine transfer per layer (several small layers per transfer): fewest gaps on the PCIe link
        args.staging_mib = max(256, min(512, -(-w.ingest_bytes() // L // (1 << 20))))
    stride = w.host_blocks * s.blk_bytes
    reqs = [cb.make_request(host.data_ptr() + r.host_block_start * s.blk_bytes, stride, r.table,
                            r.n_prefix_blocks, r.suffix_len, r.first_ingest_block) for r in w.requests]
    ctx = cb.calvo_create(L, s.n_q_heads, s.n_kv_heads, s.head_dim,
                          cb.CALVO_BF16 if s.dtype == "bf16" else cb.CALVO_F32, s.pool_blocks, pool,
                          staging_bytes=args.staging_mib << 20, n_staging=args.n_staging)

    # the batch is validated, planned and described to the device once; every layer of every step re-uses it
    batch = cb.calvo_batch_prepare(ctx, reqs, w.cu_suffix)

    def poison():
        pool.view(torch.int16 if tdt == torch.bfloat16 else torch.int32).fill_(0x7FC1 if tdt == torch.bfloat16 else 0x7FC12345)
        torch.cuda.synchronize()

    # chunk-granular readiness for the last layers: their attention cannot hide behind the loading of
    # later layers, and starting it on landed chunks moves compute-stream work forward
    plan = {"chunk_blocks": None}

    def set_tail_chunks(n, head=False):
        """n chunks per layer for the last --tail-layers layers, or (head) for the first layer only."""
        longest = max(r.n_prefix_blocks for r in w.requests)
        if n <= 0 or L < 1 or longest < 2:
            plan["chunk_blocks"] = None
            return
        per = max(2, -(-longest // n))
        per += per & 1
        if head:
            plan["chunk_blocks"] = [per] + [0] * (L - 1)
        else:
            nt = max(1, min(L, args.tail_layers))
            plan["chunk_blocks"] = [0] * (L - nt) + [per] * nt

    host_trace = []
    # after[l]: the layer whose loading signal layer l's attention waits for (l itself: as soon as its own blocks are in)
    plan["after"] = list(range(L))

    def set_alap(t_ing_ms, t_att_ms):
        cbs = plan["chunk_blocks"] or [0] * L
        n = next((l for l in range(L) if cbs[l]), L)
        plan["after"] = alap_schedule(L, n, 1.06 * t_att_ms / max(t_ing_ms, 1e-9))

    def step():
        t0 = time.perf_counter()
        if plan["chunk_blocks"] is None:
            cb.calvo_kv_ingest(ctx, reqs, 0, L)
        else:
            cb.calvo_kv_ingest_chunked(ctx, reqs, 0, L, plan["chunk_blocks"])
        t1 = time.perf_counter()
        for l in range(L):
            if plan["after"][l] > l:
                cb.calvo_layer_event(ctx, plan["after"][l], cb.CALVO_EV_STREAM_WAIT)      # on the compute stream
            cb.calvo_prefill_attn_batch(ctx, batch, l, q[l], ks[l], vs[l], out[l], 0.0)
        t2 = time.perf_counter()
        torch.cuda.synchronize()
        host_trace.append((t1 - t0, t2 - t1, time.perf_counter() - t2))

    def ingest_only():
        cb.calvo_kv_ingest(ctx, reqs, 0, L)
        cb.calvo_layer_event(ctx, L - 1, cb.CALVO_EV_HOST_WAIT)
        torch.cuda.synchronize()

    def attn_only():
        for l in range(L):
            cb.calvo_prefill_attn_batch(ctx, batch, l, q[l], ks[l], vs[l], out[l], 0.0)
        torch.cuda.synchronize()

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        return (time.perf_counter() - t0) * 1e3

    try:
        poison()
        if args.mode != "full":
            fn = attn_only if args.mode == "attn" else ingest_only
            if args.mode == "attn":
                ingest_only()                      # attention needs a resident prefix
            for _ in range(args.warmup):
                fn()
            if args.mode == "attn" and args.gap_ms > 0:
                kt = []
                for _ in range(max(args.steps, 1)):
                    for l in range(L):
                        torch.cuda.synchronize()
                        t_end = time.perf_counter() + args.gap_ms * 1e-3
                        while time.perf_counter() < t_end:
                            pass
                        cb.calvo_prefill_attn_batch(ctx, batch, l, q[l], ks[l], vs[l], out[l], 0.0)
                        kt.append(cb.calvo_attn_kernel_ms(ctx, l))
                log(f"[bench] mode attn, {args.gap_ms:g} ms idle before every launch: kernel {statistics.mean(kt):.3f} ms "
                    f"(min {min(kt):.3f} max {max(kt):.3f}) = {w.attn_flop() / L / statistics.mean(kt) / 1e9:.1f} TFLOP/s")
                return
            t = [timed(fn) for _ in range(args.steps)]
            log(f"[bench] mode {args.mode}{' (zero data)' if args.zero_data else ''}: {statistics.mean(t):.3f} ms per pass over {L} layers"
                + (f" = {w.attn_flop() / statistics.mean(t) / 1e9:.1f} TFLOP/s" if args.mode == "attn" else ""))
            return
        # ---- stage times in isolation (context for the overlap figure, and the choice of the chunked tail)
        ingest_only()
        t_ing = min(timed(ingest_only) for _ in range(2))
        t_att = min(timed(attn_only) for _ in range(2))
        head_chunks = False
        if args.tail_chunks < 0:
            # The last layers in chunks pay when loading bounds the step and a layer's attention is a sizeable
            # part of a layer's load.  When attention bounds the step, the first layer in chunks lets it start
            # after a quarter of that layer's load (single requests: a batch would trade its one transfer per
            # layer for one per request and chunk).
            args.tail_chunks = 4 if t_ing > t_att >= 0.5 * t_ing else 0
            head_chunks = t_att > t_ing and L > 1 and len(w.requests) == 1
        set_tail_chunks(4 if head_chunks else args.tail_chunks, head=head_chunks)
        # Only where it pays and cannot hurt: attention a sizeable part of the loading time (the same condition as
        # the chunked tail, which the chain ends at), and every layer a transfer of its own (small layers share
        # transfers, and a layer's signal then fires with its group's).
        if not args.no_alap and args.tail_chunks > 0 and not head_chunks and w.ingest_bytes() / L >= (128 << 20):
            set_alap(t_ing, t_att)
            # the chain must not cost TTFT: two untimed steps each way decide (the stage times it was derived from
            # were measured in isolation)
            chain, plain = plan["after"], list(range(L))
            if chain != plain:
                step()
                t_chain = min(timed(step) for _ in range(2))
                plan["after"] = plain
                t_plain = min(timed(step) for _ in range(2))
                keep = t_chain <= 1.002 * t_plain
                plan["after"] = chain if keep else plain
                log(f"[bench] attention launches queued back to back: step {t_chain:.2f} ms against {t_plain:.2f} ms with one launch "
                    f"per landed layer: {'kept' if keep else 'dropped'}")
        # the interpreter's cyclic collector would otherwise run a full pass (tens of milliseconds with torch
        # loaded) in the middle of some step's enqueue loop
        import gc
        gc.collect()
        gc.disable()
        for _ in range(args.warmup):
            step()
        # ---- the timed steps
        step_ms, kern_ms = [], []
        for _ in range(args.steps):
            poison()
            step_ms.append(timed(step))
            # whole-layer launches only: the event pair of a chunk-granular layer also spans its waits
            cbs = plan["chunk_blocks"]
            kern_ms.extend(cb.calvo_attn_kernel_ms(ctx, l) for l in range(L) if not (cbs and cbs[l]))
        gc.enable()
        if kern_ms:
            ks_sorted = sorted(kern_ms)
            log(f"[bench] attention launch inside the timed steps: min {ks_sorted[0]:.3f} median {ks_sorted[len(ks_sorted) // 2]:.3f} "
                f"max {ks_sorted[-1]:.3f} ms; first step, layers 0-7: " + " ".join(f"{x:.3f}" for x in kern_ms[:8]))
        kernel_id, kernel_wgs = cb.calvo_attn_kernel_info(ctx, 0)
        ms = statistics.mean(step_ms)
        # every layer chunk-granular: no whole-layer launch inside the steps, take the launches of the attention-only pass
        k_ms = statistics.mean(kern_ms) if kern_ms else t_att / L
        log("[bench] host time per step, warm-up steps first (ingest call, attention calls, final wait) ms: " +
            ", ".join("(%.2f %.2f %.2f)" % tuple(1e3 * x for x in t) for t in host_trace))
        flop_per_launch = w.attn_flop() / L
        att_tflops = flop_per_launch / (k_ms * 1e-3) / 1e12
        ing_gbps = w.ingest_bytes() / (t_ing * 1e-3) / 1e9
        t_ing_l = w.ingest_bytes() / L / (h2d_peak * 1e9) * 1e3
        t_att_l = flop_per_launch / (MFMA_BF16_PEAK_TFLOPS * 1e12) * 1e3
        ttft_lb = max(L * t_ing_l + t_att_l, t_ing_l + L * t_att_l)
        overlap = 1.0 - (ms - max(t_ing, t_att)) / max(min(t_ing, t_att), 1e-9)

        result = {
            "metric": "prefix-hit TTFT ms @64K ctx; KV ingest GB/s; prefill-attn % bf16 MFMA peak",
            "value": round(ms, 3), "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(ms, 3), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": s.dtype, "data": "synthetic",
            "config": {"workload": w.name, "layers": L, "q_heads": s.n_q_heads, "kv_heads": s.n_kv_heads,
                       "head_dim": s.head_dim, "block_tokens": s.block_tokens,
                       "prefix_tokens": [r.prefix_len for r in w.requests],
                       "suffix_tokens": [r.suffix_len for r in w.requests],
                       "attention_waits_for_layer": plan["after"],
                       "ingest": "zero-copy kernel" if args.staging_mib == 0 else f"copy engine, {args.staging_mib} MiB staging x{args.n_staging or 2}",
                       "chunked_layers": ("first layer x 4 chunks" if head_chunks else
                                          f"last {args.tail_layers} layers x {args.tail_chunks} chunks" if args.tail_chunks else "none")},
            "ttft_ms": {"mean": round(ms, 3), "median": round(statistics.median(step_ms), 3),
                        "min": round(min(step_ms), 3), "each": [round(x, 3) for x in step_ms], "lower_bound": round(ttft_lb, 3),
                        "frac_of_lower_bound": round(ttft_lb / ms, 4)},
            "ingest": {"GBps": round(ing_gbps, 2), "h2d_peak_GBps": round(h2d_peak, 2),
                       "frac_of_h2d_peak": round(ing_gbps / h2d_peak, 4), "alone_ms": round(t_ing, 3),
                       "bytes": w.ingest_bytes()},
            "attention": {"TFLOPs": round(att_tflops, 1), "alone_ms_all_layers": round(t_att, 3),
                          "frac_of_bf16_mfma_peak": round(att_tflops / MFMA_BF16_PEAK_TFLOPS, 4)},
            "overlap": round(overlap, 4),
            "roofline": {"bound": "mfma", "achieved": round(att_tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": round(att_tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                         "traffic": profiled_traffic(args.config) if kernel_id == 3 and not args.custom else None,
                         "kernel": cb.ATTN_KERNEL_NAMES.get(kernel_id, f"calvo::attn_mfma_kernel (variant {kernel_id})"),
                         "workgroups_per_launch": kernel_wgs, "flop_per_launch": flop_per_launch,
                         "avg_launch_ms": round(k_ms, 4)},
        }
        if not args.leg:
            # what the matrix pipes sustain on MFMAs alone (the published peak assumes the top clock; the
            # part is power limited and the sustained rate depends on the operand data)
            peak = measured_mfma_peak(cb, torch, dev)
            result["mfma_measured_peak_TFLOPs"] = peak
            result["roofline"]["frac_of_measured_mfma_peak"] = round(att_tflops / peak["normal_operands"], 4)
        if not args.no_three_stage and not args.leg and w.ingest_bytes() <= (16 << 30):
            result["three_stage"] = three_stage(args, cb, ctx, w, host, reqs, q, ks, vs, out, poison, timed, t_att)
        if not args.no_cpu_baseline and not args.leg:
            result["cpu_baseline"] = cpu_baseline(w, host, q, ks, vs, out, args.sample_rows)
    finally:
        cb.calvo_batch_destroy(batch)
        cb.calvo_destroy(ctx)
    if not args.leg and not args.no_cfg4_leg and args.config == 3 and not args.custom and args.mode == "full":
        # release this workload's buffers before the leg allocates its own (78 GiB pool)
        del pool, q, ks, vs, out, host
        arena.free()
        torch.cuda.empty_cache()
        result["attention_bound_leg"] = cfg4_leg()
    print(json.dumps(result), flush=True)


def measured_mfma_peak(cb, torch, dev):
    """calvo_mfma_peak with normally distributed and with all-zero bf16 operands, for the MFMA shape the attention
    kernels use (16x16x32) and, for comparison, the 32x32x16 shape."""
    sink = torch.empty(512 * 1024, dtype=torch.float32, device=dev)
    out = {}
    for name, fill in (("normal_operands", lambda t: t.normal_(0.0, 1.0)), ("zero_operands", lambda t: t.zero_())):
        ops = torch.empty(8192, dtype=torch.bfloat16, device=dev)
        fill(ops)
        torch.cuda.synchronize()
        for shape, key in ((cb.CALVO_MFMA_16x16x32, name), (cb.CALVO_MFMA_32x32x16, name + "_32x32x16")):
            tf, ms = cb.calvo_mfma_peak(ops, sink, iters=20000, repeats=3, shape=shape)
            out[key] = round(tf, 1)
            log(f"[bench] MFMA-only peak, {key}: {tf:.0f} TFLOP/s ({ms:.2f} ms per launch)")
    out["kernel"] = "v_mfma_f32_16x16x32_bf16 only (the attention kernels' shape), two waves per SIMD, register operands"
    return out


def cfg4_leg():
    """The 8-request batch of workload 4 (attention bound: the step the attention kernel's speed
    moves), 3 timed steps in a process of its own.  Extra keys of the JSON line, never `value`."""
    import subprocess
    cmd = [sys.executable, os.path.abspath(__file__), "--config", "4", "--steps", "3", "--warmup", "1", "--leg"]
    t0 = time.perf_counter()
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=600)
    for ln in res.stderr.splitlines():
        log("[cfg4 leg] " + ln)
    if res.returncode != 0:
        return {"error": f"exit code {res.returncode}"}
    d = json.loads(res.stdout.strip().splitlines()[-1])
    return {"workload": d["config"]["workload"], "steps": d["steps"], "ttft_ms": d["ttft_ms"]["mean"],
            "lower_bound_ms": d["ttft_ms"]["lower_bound"], "frac_of_lower_bound": d["ttft_ms"]["frac_of_lower_bound"],
            "ingest_alone_ms": d["ingest"]["alone_ms"], "attention_alone_ms": d["attention"]["alone_ms_all_layers"],
            "attention_TFLOPs": d["attention"]["TFLOPs"], "frac_of_bf16_mfma_peak": d["attention"]["frac_of_bf16_mfma_peak"],
            "avg_launch_ms": d["roofline"]["avg_launch_ms"], "kernel": d["roofline"]["kernel"],
            "wall_s": round(time.perf_counter() - t0, 1)}


def three_stage(args, cb, ctx, w, host, reqs, q, ks, vs, out, poison, timed, t_att):
    """The same step with the cached prefix in pageable host memory behind an emulated remote link:
    a loader thread copies it chunk by chunk into a small pinned ring (L3 -> L2, rate limited), every
    landed chunk goes through the copy engine and the scatter kernel (L2 -> L1), and each layer's
    attention waits for that layer only.  Reported beside the headline number, never as `value`."""
    import torch
    s, L = w.shape, w.shape.n_layers
    remote = torch.empty(host.shape, dtype=host.dtype)           # pageable
    remote.copy_(host)
    stride = w.host_blocks * s.blk_bytes
    rreqs = [cb.make_request(remote.data_ptr() + r.host_block_start * s.blk_bytes, stride, r.table,
                             r.n_prefix_blocks, r.suffix_len, r.first_ingest_block) for r in w.requests]
    chunk = 64 << 20
    stats = {}
    link_ms = w.ingest_bytes() / (args.l3_gbps * 1e9) * 1e3 if args.l3_gbps > 0 else 0.0
    # attention follows the loader's chunks when the link clearly bounds the step; piecewise attention costs a
    # few percent of attention time, which a compute-bound step cannot hide
    per_chunk = not args.l3_whole_layers and t_att < 0.8 * link_ms

    def step_l3():
        cb.calvo_kv_ingest_l3(ctx, rreqs, 0, L, chunk_bytes=chunk, n_slots=4, n_threads=8, l3_GBps=args.l3_gbps,
                              chunk_ready=per_chunk)
        for l in range(L):
            cb.calvo_prefill_attn(ctx, l, q[l], ks[l], vs[l], out[l], rreqs, w.cu_suffix, 0.0)
        stats.update(cb.calvo_l3_wait(ctx))
        torch.cuda.synchronize()

    poison()
    step_l3()
    t = []
    for _ in range(2):
        poison()
        t.append(timed(step_l3))
    ms = sum(t) / len(t)
    log(f"[bench] three-stage (emulated L3 at {args.l3_gbps:g} GB/s, 64 MiB chunks, 4-slot pinned ring = 256 MiB): "
        f"TTFT {ms:.2f} ms, link alone {link_ms:.2f} ms, ring wait {stats['ring_wait_s'] * 1e3:.1f} ms")
    return {"ttft_ms": round(ms, 3), "l3_GBps": args.l3_gbps, "link_alone_ms": round(link_ms, 3),
            "frac_of_link_bound": round(link_ms / ms, 4) if ms > 0 else None,
            "pinned_ring_MiB": 4 * chunk >> 20, "chunk_MiB": chunk >> 20, "host_threads": 8,
            "readiness": "per chunk" if per_chunk else "whole layers",
            "l3_busy_ms": round(stats["l3_busy_s"] * 1e3, 2), "loader_total_ms": round(stats["total_s"] * 1e3, 2), "ring_wait_ms": round(stats["ring_wait_s"] * 1e3, 2)}


def cpu_baseline(w, host, q, ks, vs, out, n_rows):
    """Times the oracle as it stands on a bounded sample (first / middle / last layer, a seeded
    set of suffix rows per request, all heads) and checks the GPU output on that sample."""
    import torch
    from threadpoolctl import threadpool_info
    from oracle import calvo_oracle as orc

    s = w.shape
    B = s.block_tokens
    L = s.n_layers

    def stored(t):
        t = t.detach().cpu().contiguous()
        return t.view(torch.int16).numpy().view(np.uint16) if s.dtype == "bf16" else t.numpy()

    host_np = (host.view(torch.int16).numpy().view(np.uint16) if s.dtype == "bf16" else host.numpy())
    layers = sorted({0, L // 2, L - 1})
    rng = np.random.default_rng(w.seed + 99)
    per_req = max(4, n_rows // len(w.requests))
    # keep the sample near 10-20 s of oracle time whatever the shape: about 3.5e9 (row, key, head) triples
    ctx_sum = sum(r.prefix_len + r.suffix_len / 2 for r in w.requests if r.suffix_len)
    per_req = max(8, min(per_req, int(3.5e9 / (len(layers) * s.n_q_heads * max(ctx_sum, 1)))))
    pairs = 0
    worst_max, means = 0.0, []
    t0 = time.perf_counter()
    for l in layers:
        pool_l = np.zeros((1, s.pool_blocks, s.blk_elems), host_np.dtype)
        for r in w.requests:
            orc.kv_ingest(pool_l, host_np[l:l + 1], r.table, r.n_prefix_blocks, r.first_ingest_block,
                          r.host_block_start)
        view = pool_l.reshape(s.pool_blocks, 2, B, s.n_kv_heads, s.head_dim)
        ks_l, vs_l, q_l, out_l = stored(ks[l]), stored(vs[l]), stored(q[l]), stored(out[l])
        for ri, r in enumerate(w.requests):
            a, b = int(w.cu_suffix[ri]), int(w.cu_suffix[ri + 1])
            if b == a:
                continue
            orc.suffix_append(view, ks_l[a:b], vs_l[a:b], r.table, r.prefix_len, B)
            S = r.suffix_len
            fixed = {0, S - 1, min(15, S - 1), min(16, S - 1), S // 2}
            rows = sorted(fixed | set(rng.integers(0, S, size=max(0, per_req - len(fixed))).tolist()))
            want = orc.prefill_attn_sampled(view, q_l[a:b], r.table, r.prefix_len, S, B, rows)
            got = orc.widen(out_l[a:b][rows]) if s.dtype == "bf16" else out_l[a:b][rows].astype(np.float64)
            d = np.abs(got - want)
            worst_max = max(worst_max, float(d.max()))
            means.append(float(d.mean()))
            pairs += sum(r.prefix_len + i + 1 for i in rows)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    total_pairs = w.attn_pairs() * L
    extrapolated_ms = dt * 1e3 * total_pairs / max(pairs, 1)
    # the same oracle on one thread, on a sixth of the rows of the last sampled layer's first request
    from threadpoolctl import threadpool_limits
    r0 = next(r for r in w.requests if r.suffix_len)
    ri0 = w.requests.index(r0)
    a0, b0 = int(w.cu_suffix[ri0]), int(w.cu_suffix[ri0 + 1])
    rows1 = sorted(set(rng.integers(0, r0.suffix_len, size=max(4, per_req // 6)).tolist()))
    with threadpool_limits(limits=1):
        t1 = time.perf_counter()
        orc.prefill_attn_sampled(view, q_l[a0:b0], r0.table, r0.prefix_len, r0.suffix_len, B, rows1)
        dt1 = time.perf_counter() - t1
    pairs1 = sum(r0.prefix_len + i + 1 for i in rows1)
    single_ms = dt1 * 1e3 * total_pairs / max(pairs1, 1)
    cores = len(os.sched_getaffinity(0))
    model = "unknown"
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                model = ln.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    log(f"[bench] oracle sample: {dt:.1f} s for {pairs} (row,key) pairs x {s.n_q_heads} heads on {threads} BLAS threads "
        f"({cores} cores in the affinity mask, {model}); one thread: {dt1:.1f} s for {pairs1} pairs; "
        f"GPU vs oracle on the sample: max-abs {worst_max:.3e}, mean-abs {max(means):.3e}")
    return {"value": round(extrapolated_ms, 1), "unit": "ms", "cores": cores, "kind": "oracle",
            "threads_used": int(threads), "cpu_model": model,
            "sample": f"layers {layers}, {per_req} suffix rows per request x all {s.n_q_heads} heads "
                      f"(incl. oracle ingest + suffix append of those layers), {dt:.1f} s measured on {threads} BLAS threads, "
                      f"extrapolated by unmasked (query,key) pairs to the whole step",
            "measured_s": round(dt, 2),
            "single_thread": {"value": round(single_ms, 1), "unit": "ms", "measured_s": round(dt1, 2),
                              "sample": f"{len(rows1)} suffix rows of one request x all heads, one layer, BLAS limited to 1 thread"},
            "gpu_vs_oracle_on_sample": {"max_abs": worst_max, "mean_abs": max(means)}}


if __name__ == "__main__":
    main()
