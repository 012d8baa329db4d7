"""ctypes binding of libcalvo.so: same names as the C ABI, argument marshalling only.

Every step of the path (scatter, suffix append, attention, events) runs inside
the library's HIP code; nothing here computes.  PyTorch is used by callers for
device memory, pinned memory and streams; this module accepts raw addresses
(ints) or objects with a data_ptr() method.

The library must have been built (python -m paper_2603_21257_amd.build, or
__graft_entry__.build()); loading fails loudly otherwise - there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

CALVO_OK, CALVO_EINVAL, CALVO_ENOMEM, CALVO_EHIP, CALVO_ENOTREADY = 0, -1, -2, -3, -4
CALVO_BF16, CALVO_F32 = 0, 1
CALVO_EV_QUERY, CALVO_EV_HOST_WAIT, CALVO_EV_STREAM_WAIT = 0, 1, 2

# CALVO_LIB names another build of the library (A/B timing of two builds); default: the in-tree one
LIB_PATH = os.environ.get("CALVO_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcalvo.so")
EXPORTS = ["calvo_create", "calvo_destroy", "calvo_kv_ingest", "calvo_kv_ingest_chunked", "calvo_chunk_count",
           "calvo_chunk_event", "calvo_kv_ingest_l3", "calvo_l3_wait", "calvo_layer_event", "calvo_prefill_attn", "calvo_prefill_attn_noalloc", "calvo_batch_prepare", "calvo_batch_destroy", "calvo_prefill_attn_batch", "calvo_attn_kernel_ms", "calvo_mfma_peak", "calvo_attn_kernel_info", "calvo_attn_plan", "calvo_attn_plan_items", "calvo_ingest_plan", "calvo_cost_fit", "calvo_cost_estimate",
           "calvo_sched_pick", "calvo_sched_simulate", "calvo_pool_create", "calvo_pool_destroy", "calvo_pool_reserve",
           "calvo_pool_retain", "calvo_pool_release", "calvo_pool_counts", "calvo_pool_admit", "calvo_pool_retry",
           "calvo_pool_cancel", "calvo_dispatch_create", "calvo_dispatch_submit", "calvo_dispatch_wait", "calvo_dispatch_poll",
           "calvo_dispatch_table", "calvo_dispatch_release", "calvo_dispatch_stats_get", "calvo_dispatch_destroy",
           "calvo_last_error"]
CALVO_POLICY_FIFO, CALVO_POLICY_SJF, CALVO_POLICY_SJF_PT, CALVO_POLICY_LSTF, CALVO_POLICY_EDF = range(5)


class calvo_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("block_tokens", C.c_int32), ("dtype", C.c_int32),
                ("pool_blocks", C.c_int64), ("pool", C.c_void_p), ("staging_bytes", C.c_size_t),
                ("n_staging", C.c_int32), ("n_copy_streams", C.c_int32), ("compute_stream", C.c_void_p)]


class calvo_request(C.Structure):
    _fields_ = [("host_kv", C.c_void_p), ("host_layer_stride", C.c_int64), ("block_table", C.POINTER(C.c_int32)),
                ("n_prefix_blocks", C.c_int32), ("first_ingest_block", C.c_int32), ("suffix_len", C.c_int32)]


class calvo_l3_config(C.Structure):
    _fields_ = [("chunk_bytes", C.c_size_t), ("n_slots", C.c_int32), ("n_threads", C.c_int32), ("l3_GBps", C.c_double),
                ("chunk_ready", C.c_int32), ("reserved", C.c_int32)]


class calvo_l3_stats(C.Structure):
    _fields_ = [("bytes", C.c_int64), ("chunks", C.c_int32), ("l3_busy_s", C.c_double), ("ring_wait_s", C.c_double),
                ("total_s", C.c_double)]


class calvo_cost_model(C.Structure):
    _fields_ = [("load_per_token_s", C.c_double), ("load_fixed_s", C.c_double), ("comp_per_token_s", C.c_double),
                ("comp_fixed_s", C.c_double)]


class calvo_job(C.Structure):
    _fields_ = [("arrival_s", C.c_double), ("deadline_s", C.c_double), ("ctx_tokens", C.c_int64),
                ("query_tokens", C.c_int64)]


class calvo_dispatch_config(C.Structure):
    _fields_ = [("policy", C.c_int32), ("three_stage", C.c_int32), ("model", calvo_cost_model), ("l3", calvo_l3_config),
                ("pool", C.c_void_p)]


class calvo_dispatch_job(C.Structure):
    _fields_ = [("host_kv", C.c_void_p), ("host_layer_stride", C.c_int64), ("block_table", C.POINTER(C.c_int32)),
                ("n_prefix_blocks", C.c_int32), ("n_shared", C.c_int32), ("suffix_len", C.c_int32), ("reserved", C.c_int32),
                ("q", C.c_void_p), ("k_suffix", C.c_void_p), ("v_suffix", C.c_void_p), ("out", C.c_void_p),
                ("q_layer_stride", C.c_int64), ("kv_layer_stride", C.c_int64), ("out_layer_stride", C.c_int64), ("scale", C.c_float), ("reserved2", C.c_float), ("deadline_s", C.c_double), ("sim_load_s", C.c_double),
                ("sim_comp_s", C.c_double)]


class calvo_dispatch_result(C.Structure):
    _fields_ = [("submit_s", C.c_double), ("load_start_s", C.c_double), ("load_end_s", C.c_double),
                ("compute_start_s", C.c_double), ("first_token_s", C.c_double), ("alloc_wait_s", C.c_double),
                ("reactive", C.c_int32), ("status", C.c_int32)]


class calvo_dispatch_stats(C.Structure):
    _fields_ = [("link_busy_s", C.c_double), ("link_span_s", C.c_double), ("ring_wait_s", C.c_double), ("bytes", C.c_int64),
                ("jobs_submitted", C.c_int64), ("jobs_done", C.c_int64)]


class CalvoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"calvo error {code}: {msg}")
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_21257_amd.build` "
                               "(there is no CPU fallback for the HIP path)")
        L = C.CDLL(LIB_PATH)
        L.calvo_create.argtypes = [C.POINTER(calvo_config), C.POINTER(C.c_void_p)]
        L.calvo_destroy.argtypes = [C.c_void_p]
        L.calvo_kv_ingest.argtypes = [C.c_void_p, C.POINTER(calvo_request), C.c_int, C.c_int, C.c_int]
        L.calvo_kv_ingest_chunked.argtypes = [C.c_void_p, C.POINTER(calvo_request), C.c_int, C.c_int, C.c_int,
                                              C.POINTER(C.c_int32)]
        L.calvo_chunk_count.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int)]
        L.calvo_chunk_event.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.calvo_kv_ingest_l3.argtypes = [C.c_void_p, C.POINTER(calvo_request), C.c_int, C.c_int, C.c_int,
                                         C.POINTER(calvo_l3_config)]
        L.calvo_l3_wait.argtypes = [C.c_void_p, C.POINTER(calvo_l3_stats)]
        L.calvo_layer_event.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.calvo_prefill_attn.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.POINTER(calvo_request), C.c_int, C.POINTER(C.c_int32), C.c_float]
        L.calvo_prefill_attn_noalloc.argtypes = L.calvo_prefill_attn.argtypes
        L.calvo_batch_prepare.argtypes = [C.c_void_p, C.POINTER(calvo_request), C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_void_p)]
        L.calvo_batch_destroy.argtypes = [C.c_void_p]
        L.calvo_prefill_attn_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.c_float]
        L.calvo_mfma_peak.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.calvo_attn_kernel_ms.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_float)]
        L.calvo_attn_plan.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int32,
                                      C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.calvo_attn_plan_items.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                            C.c_int32, C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.POINTER(C.c_int32)]
        L.calvo_ingest_plan.argtypes = [C.POINTER(calvo_request), C.c_int32, C.c_int32, C.c_int32, C.c_int64, C.c_int64,
                                        C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.calvo_attn_kernel_info.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]
        dp = C.POINTER(C.c_double)
        L.calvo_cost_fit.argtypes = [dp, dp, C.c_int, dp, dp]
        L.calvo_cost_estimate.argtypes = [C.POINTER(calvo_cost_model), C.POINTER(calvo_job), dp, dp]
        L.calvo_sched_pick.argtypes = [C.c_int, C.POINTER(calvo_cost_model), C.POINTER(calvo_job), C.POINTER(C.c_ubyte),
                                       C.c_int, C.c_double, C.POINTER(C.c_int)]
        L.calvo_sched_simulate.argtypes = [C.c_int, C.POINTER(calvo_cost_model), C.POINTER(calvo_job), C.c_int, dp, dp,
                                           C.c_int, dp, dp]
        i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
        L.calvo_pool_create.argtypes = [C.c_int64, C.POINTER(C.c_void_p)]
        L.calvo_pool_destroy.argtypes = [C.c_void_p]
        L.calvo_pool_reserve.argtypes = [C.c_void_p, C.c_int32, i32p]
        L.calvo_pool_retain.argtypes = [C.c_void_p, i32p, C.c_int32]
        L.calvo_pool_release.argtypes = [C.c_void_p, i32p, C.c_int32]
        L.calvo_pool_counts.argtypes = [C.c_void_p, i64p, i64p, i64p, i64p]
        L.calvo_pool_admit.argtypes = [C.c_void_p, i32p, C.c_int32, C.c_int32, i32p, i64p]
        L.calvo_pool_retry.argtypes = [C.c_void_p, C.c_int64, i32p]
        L.calvo_pool_cancel.argtypes = [C.c_void_p, C.c_int64]
        L.calvo_dispatch_create.argtypes = [C.c_void_p, C.POINTER(calvo_dispatch_config), C.POINTER(C.c_void_p)]
        L.calvo_dispatch_submit.argtypes = [C.c_void_p, C.POINTER(calvo_dispatch_job), i64p]
        L.calvo_dispatch_wait.argtypes = [C.c_void_p, C.c_int64, C.POINTER(calvo_dispatch_result)]
        L.calvo_dispatch_poll.argtypes = [C.c_void_p, C.c_int64, C.POINTER(calvo_dispatch_result)]
        L.calvo_dispatch_table.argtypes = [C.c_void_p, C.c_int64, i32p, C.c_int32, i32p]
        L.calvo_dispatch_release.argtypes = [C.c_void_p, C.c_int64]
        L.calvo_dispatch_stats_get.argtypes = [C.c_void_p, C.POINTER(calvo_dispatch_stats)]
        L.calvo_dispatch_destroy.argtypes = [C.c_void_p]
        L.calvo_last_error.argtypes = []
        L.calvo_last_error.restype = C.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def calvo_last_error() -> str:
    return lib().calvo_last_error().decode()


def _check(rc: int, ok=(CALVO_OK,)) -> int:
    if rc not in ok:
        raise CalvoError(rc, calvo_last_error())
    return rc


def make_request(host_kv, host_layer_stride: int, block_table: np.ndarray, n_prefix_blocks: int,
                 suffix_len: int, first_ingest_block: int = 0) -> calvo_request:
    """Marshal one request.  The returned struct keeps the table array alive."""
    tab = np.ascontiguousarray(block_table, dtype=np.int32)
    r = calvo_request(_ptr(host_kv), int(host_layer_stride), tab.ctypes.data_as(C.POINTER(C.c_int32)),
                      int(n_prefix_blocks), int(first_ingest_block), int(suffix_len))
    r._keep = tab
    return r


def _req_array(reqs: Sequence[calvo_request]):
    arr = (calvo_request * max(len(reqs), 1))()
    for i, r in enumerate(reqs):
        arr[i] = r
    arr._keep = list(reqs)
    return arr


def calvo_create(n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int, dtype: int, pool_blocks: int,
                 pool, staging_bytes: int = 0, n_staging: int = 0, n_copy_streams: int = 0,
                 compute_stream=None, block_tokens: int = 16) -> int:
    """Returns the context handle (an address)."""
    cfg = calvo_config(n_layers, n_q_heads, n_kv_heads, head_dim, block_tokens, dtype, pool_blocks, _ptr(pool),
                       staging_bytes, n_staging, n_copy_streams,
                       None if compute_stream is None else int(compute_stream))
    out = C.c_void_p()
    _check(lib().calvo_create(C.byref(cfg), C.byref(out)))
    return out.value


def calvo_destroy(ctx: int) -> None:
    _check(lib().calvo_destroy(ctx))


def calvo_kv_ingest(ctx: int, reqs: Sequence[calvo_request], layer_begin: int, layer_end: int) -> None:
    _check(lib().calvo_kv_ingest(ctx, _req_array(reqs), len(reqs), layer_begin, layer_end))


def calvo_kv_ingest_chunked(ctx: int, reqs: Sequence[calvo_request], layer_begin: int, layer_end: int,
                            chunk_blocks) -> None:
    """chunk_blocks: one even block count per layer of the range (0 = load that layer as a whole)."""
    cb = np.ascontiguousarray(chunk_blocks, dtype=np.int32)
    if cb.shape != (layer_end - layer_begin,):
        raise ValueError("chunk_blocks needs one entry per layer of the range")
    _check(lib().calvo_kv_ingest_chunked(ctx, _req_array(reqs), len(reqs), layer_begin, layer_end,
                                         cb.ctypes.data_as(C.POINTER(C.c_int32))))


def calvo_chunk_count(ctx: int, layer: int) -> int:
    n = C.c_int(0)
    _check(lib().calvo_chunk_count(ctx, layer, C.byref(n)))
    return n.value


def calvo_chunk_event(ctx: int, layer: int, chunk: int, mode: int, stream=None) -> bool:
    """True when the chunk is resident (always, for the two waiting modes)."""
    rc = lib().calvo_chunk_event(ctx, layer, chunk, mode, None if stream is None else int(stream))
    return _check(rc, ok=(CALVO_OK, CALVO_ENOTREADY)) == CALVO_OK


def calvo_kv_ingest_l3(ctx: int, reqs: Sequence[calvo_request], layer_begin: int, layer_end: int,
                       chunk_bytes: int = 0, n_slots: int = 0, n_threads: int = 0, l3_GBps: float = 0.0,
                       chunk_ready: bool = False) -> None:
    """host_kv of the requests may be pageable host memory; it must stay alive until calvo_l3_wait."""
    cfg = calvo_l3_config(int(chunk_bytes), int(n_slots), int(n_threads), float(l3_GBps), 1 if chunk_ready else 0, 0)
    _check(lib().calvo_kv_ingest_l3(ctx, _req_array(reqs), len(reqs), layer_begin, layer_end, C.byref(cfg)))


def calvo_l3_wait(ctx: int) -> dict:
    st = calvo_l3_stats()
    _check(lib().calvo_l3_wait(ctx, C.byref(st)))
    return {name: getattr(st, name) for name, _ in calvo_l3_stats._fields_}


def calvo_layer_event(ctx: int, layer: int, mode: int, stream=None) -> bool:
    """True when the layer is ready (always, for the two waiting modes)."""
    rc = lib().calvo_layer_event(ctx, layer, mode, None if stream is None else int(stream))
    return _check(rc, ok=(CALVO_OK, CALVO_ENOTREADY)) == CALVO_OK


def calvo_prefill_attn(ctx: int, layer: int, q, k_suffix, v_suffix, out, reqs: Sequence[calvo_request],
                       cu_suffix: np.ndarray, scale: float = 0.0) -> None:
    cu = np.ascontiguousarray(cu_suffix, dtype=np.int32)
    _check(lib().calvo_prefill_attn(ctx, layer, _ptr(q), _ptr(k_suffix), _ptr(v_suffix), _ptr(out),
                                    _req_array(reqs), len(reqs), cu.ctypes.data_as(C.POINTER(C.c_int32)),
                                    float(scale)))


def calvo_prefill_attn_noalloc(ctx: int, layer: int, q, k_suffix, v_suffix, out, reqs: Sequence[calvo_request],
                               cu_suffix: np.ndarray, scale: float = 0.0) -> None:
    """calvo_prefill_attn without any allocation inside the call (fixed-size static device array)."""
    cu = np.ascontiguousarray(cu_suffix, dtype=np.int32)
    _check(lib().calvo_prefill_attn_noalloc(ctx, layer, _ptr(q), _ptr(k_suffix), _ptr(v_suffix), _ptr(out),
                                            _req_array(reqs), len(reqs), cu.ctypes.data_as(C.POINTER(C.c_int32)),
                                            float(scale)))


def calvo_batch_prepare(ctx: int, reqs: Sequence[calvo_request], cu_suffix: np.ndarray) -> int:
    """Validates, plans and uploads the batch once; returns the handle for calvo_prefill_attn_batch."""
    cu = np.ascontiguousarray(cu_suffix, dtype=np.int32)
    out = C.c_void_p()
    _check(lib().calvo_batch_prepare(ctx, _req_array(reqs), len(reqs), cu.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(out)))
    return out.value


def calvo_batch_destroy(batch: int) -> None:
    _check(lib().calvo_batch_destroy(batch))


def calvo_prefill_attn_batch(ctx: int, batch: int, layer: int, q, k_suffix, v_suffix, out, scale: float = 0.0) -> None:
    _check(lib().calvo_prefill_attn_batch(ctx, batch, layer, _ptr(q), _ptr(k_suffix), _ptr(v_suffix), _ptr(out), float(scale)))


CALVO_MFMA_16x16x32, CALVO_MFMA_32x32x16 = 0, 1


def calvo_mfma_peak(operands, sink, iters: int = 20000, repeats: int = 3, shape: int = CALVO_MFMA_16x16x32):
    """(TFLOP/s, ms) the matrix pipes sustain on bf16 MFMAs of one shape alone with the given operand data (device buffers)."""
    tf, ms = C.c_double(), C.c_double()
    _check(lib().calvo_mfma_peak(_ptr(operands), _ptr(sink), int(iters), int(repeats), int(shape), C.byref(tf), C.byref(ms)))
    return tf.value, ms.value


def _darr(x):
    a = np.ascontiguousarray(x, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _job_array(jobs):
    """jobs: sequence of (arrival_s, deadline_s, ctx_tokens, query_tokens)."""
    arr = (calvo_job * max(len(jobs), 1))()
    for i, (a, d, c, q) in enumerate(jobs):
        arr[i] = calvo_job(float(a), float(d), int(c), int(q))
    return arr


def _sched_check(rc: int):
    if rc != CALVO_OK:
        raise CalvoError(rc, "invalid scheduling argument")


def calvo_cost_fit(tokens, seconds):
    """Returns (per_token_s, fixed_s)."""
    t, tp = _darr(tokens)
    y, yp = _darr(seconds)
    a, b = C.c_double(), C.c_double()
    _sched_check(lib().calvo_cost_fit(tp, yp, min(len(t), len(y)), C.byref(a), C.byref(b)))
    return a.value, b.value


def calvo_cost_estimate(model, job):
    m = calvo_cost_model(*model)
    j = calvo_job(float(job[0]), float(job[1]), int(job[2]), int(job[3]))
    a, b = C.c_double(), C.c_double()
    _sched_check(lib().calvo_cost_estimate(C.byref(m), C.byref(j), C.byref(a), C.byref(b)))
    return a.value, b.value


def calvo_sched_pick(policy: int, model, jobs, done, now: float) -> int:
    m = calvo_cost_model(*model) if model is not None else None
    d = (C.c_ubyte * max(len(jobs), 1))(*[1 if x else 0 for x in done]) if done is not None else None
    out = C.c_int(-2)
    _sched_check(lib().calvo_sched_pick(policy, C.byref(m) if m is not None else None, _job_array(jobs), d, len(jobs),
                                        float(now), C.byref(out)))
    return out.value


def calvo_sched_simulate(policy: int, model, jobs, load_s=None, comp_s=None, pipelined=False):
    """Returns (start_s, finish_s) as numpy arrays.  pipelined: 0 / False, 1 / True, or 2 (see the header)."""
    m = calvo_cost_model(*model) if model is not None else None
    n = len(jobs)
    start, sp = _darr(np.zeros(max(n, 1)))
    fin, fp = _darr(np.zeros(max(n, 1)))
    la = _darr(load_s) if load_s is not None else (None, None)
    ca = _darr(comp_s) if comp_s is not None else (None, None)
    _sched_check(lib().calvo_sched_simulate(policy, C.byref(m) if m is not None else None, _job_array(jobs), n, la[1], ca[1],
                                            int(pipelined), sp, fp))
    return start[:n], fin[:n]


ATTN_KERNEL_NAMES = {3: "calvo::pipe::attn_pipe_kernel", 4: "calvo::duo::attn_duo_kernel", -1: "calvo::attn_simple_kernel"}


def calvo_attn_plan(n_q_heads: int, n_kv_heads: int, n_cus: int, prefix_blocks, suffix_lens) -> dict:
    """What calvo_prefill_attn would launch for these lengths: kernel id, tile size, pieces per tile, workgroups."""
    pb = np.ascontiguousarray(prefix_blocks, dtype=np.int32)
    sl = np.ascontiguousarray(suffix_lens, dtype=np.int32)
    if pb.shape != sl.shape:
        raise ValueError("prefix_blocks and suffix_lens need one entry per request")
    out = [C.c_int32() for _ in range(4)]
    rc = lib().calvo_attn_plan(n_q_heads, n_kv_heads, n_cus, pb.ctypes.data_as(C.POINTER(C.c_int32)),
                               sl.ctypes.data_as(C.POINTER(C.c_int32)), len(pb), *[C.byref(o) for o in out])
    if rc != CALVO_OK:
        raise CalvoError(rc, "invalid planning argument")
    return dict(zip(("kernel", "tile_tokens", "pieces", "workgroups"), (o.value for o in out)))


def calvo_attn_plan_items(n_q_heads: int, n_kv_heads: int, n_cus: int, prefix_blocks, suffix_lens,
                          chunk_blocks: int = 0) -> np.ndarray:
    """The work items of that launch, in launch order: int32 array [n][6] of (request, tile, first sub-tile,
    end sub-tile, pieces of the tile, launch index); chunk_blocks > 0: the layer was loaded in such chunks."""
    pb = np.ascontiguousarray(prefix_blocks, dtype=np.int32)
    sl = np.ascontiguousarray(suffix_lens, dtype=np.int32)
    if pb.shape != sl.shape:
        raise ValueError("prefix_blocks and suffix_lens need one entry per request")
    i32p = C.POINTER(C.c_int32)
    n = C.c_int32()
    args = (n_q_heads, n_kv_heads, n_cus, pb.ctypes.data_as(i32p), sl.ctypes.data_as(i32p), len(pb), chunk_blocks)
    rc = lib().calvo_attn_plan_items(*args, None, 0, C.byref(n))
    if rc not in (CALVO_OK, CALVO_ENOMEM):
        raise CalvoError(rc, "invalid planning argument")
    out = np.zeros((n.value, 6), np.int32)
    if n.value:
        rc = lib().calvo_attn_plan_items(*args, out.ctypes.data_as(i32p), n.value, C.byref(n))
        if rc != CALVO_OK:
            raise CalvoError(rc, "invalid planning argument")
    return out


def calvo_ingest_plan(reqs, layer_begin: int, layer_end: int, block_bytes: int, staging_blocks: int,
                      merge_bytes: int = 256 << 20, chunk_blocks=None):
    """(transfer group of every layer, runs of every layer) as the ingest calls would move them; reqs as for calvo_kv_ingest."""
    n = layer_end - layer_begin
    arr = _req_array(reqs)
    i32p = C.POINTER(C.c_int32)
    cbk = None if chunk_blocks is None else np.ascontiguousarray(chunk_blocks, dtype=np.int32)
    if cbk is not None and len(cbk) != n:
        raise ValueError("chunk_blocks needs one entry per layer")
    groups, runs = np.zeros(max(n, 1), np.int32), np.zeros(max(n, 1), np.int32)
    rc = lib().calvo_ingest_plan(arr, len(reqs), layer_begin, layer_end, block_bytes, staging_blocks, merge_bytes,
                                 None if cbk is None else cbk.ctypes.data_as(i32p), groups.ctypes.data_as(i32p),
                                 runs.ctypes.data_as(i32p))
    if rc != CALVO_OK:
        raise CalvoError(rc, "invalid planning argument")
    return groups[:n], runs[:n]


def calvo_attn_kernel_info(ctx: int, layer: int):
    """(kernel id, number of workgroups) of the layer's most recent attention launch."""
    k, n = C.c_int(), C.c_int()
    _check(lib().calvo_attn_kernel_info(ctx, layer, C.byref(k), C.byref(n)))
    return k.value, n.value


def calvo_attn_kernel_ms(ctx: int, layer: int) -> float:
    ms = C.c_float()
    _check(lib().calvo_attn_kernel_ms(ctx, layer, C.byref(ms)))
    return ms.value


# ---- slot allocation (host code; no GPU needed)

def _pool_check(rc: int, ok=(CALVO_OK,)) -> int:
    if rc not in ok:
        raise CalvoError(rc, "slot allocation call refused")
    return rc


def _i32(a):
    arr = np.ascontiguousarray(a, dtype=np.int32)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int32))


def calvo_pool_create(n_blocks: int) -> int:
    out = C.c_void_p()
    _pool_check(lib().calvo_pool_create(int(n_blocks), C.byref(out)))
    return out.value


def calvo_pool_destroy(pool: int) -> None:
    _pool_check(lib().calvo_pool_destroy(pool))


def calvo_pool_reserve(pool: int, n: int):
    """n free slots as an int32 array, or None if fewer than n are free."""
    arr, ap = _i32(np.zeros(max(n, 1)))
    rc = _pool_check(lib().calvo_pool_reserve(pool, n, ap), ok=(CALVO_OK, CALVO_ENOMEM))
    return arr[:n].copy() if rc == CALVO_OK else None


def calvo_pool_retain(pool: int, slots) -> None:
    arr, ap = _i32(slots)
    _pool_check(lib().calvo_pool_retain(pool, ap, len(arr)))


def calvo_pool_release(pool: int, slots) -> None:
    arr, ap = _i32(slots)
    _pool_check(lib().calvo_pool_release(pool, ap, len(arr)))


def calvo_pool_counts(pool: int) -> dict:
    v = [C.c_int64() for _ in range(4)]
    _pool_check(lib().calvo_pool_counts(pool, *[C.byref(x) for x in v]))
    return dict(zip(("free", "used", "refs", "waiting"), (x.value for x in v)))


def calvo_pool_admit(pool: int, shared, n_own: int):
    """(table, 0) when the slots were granted at once (proactive), (None, ticket) when the request
    was queued for reactive allocation."""
    sh, sp = _i32(shared)
    table, tp = _i32(np.zeros(max(len(sh) + n_own, 1)))
    ticket = C.c_int64()
    rc = _pool_check(lib().calvo_pool_admit(pool, sp, len(sh), n_own, tp, C.byref(ticket)), ok=(CALVO_OK, CALVO_ENOTREADY))
    return (table[:len(sh) + n_own].copy(), 0) if rc == CALVO_OK else (None, ticket.value)


def calvo_pool_retry(pool: int, ticket: int, n_table: int):
    """The table of a queued admission once it can be served, else None."""
    table, tp = _i32(np.zeros(max(n_table, 1)))
    rc = _pool_check(lib().calvo_pool_retry(pool, ticket, tp), ok=(CALVO_OK, CALVO_ENOTREADY))
    return table[:n_table].copy() if rc == CALVO_OK else None


def calvo_pool_cancel(pool: int, ticket: int) -> None:
    _pool_check(lib().calvo_pool_cancel(pool, ticket))


# ---- the multi-request dispatcher (stage threads inside the library)

def _fields(st) -> dict:
    return {name: getattr(st, name) for name, _ in st._fields_}


def calvo_dispatch_create(ctx: Optional[int], policy: int, model=None, three_stage: bool = False, pool: int = 0,
                          chunk_bytes: int = 0, n_slots: int = 0, n_threads: int = 0, l3_GBps: float = 0.0) -> int:
    """ctx None: a dry run of the stage logic (jobs carry sim_load_s / sim_comp_s).  Returns the handle."""
    cfg = calvo_dispatch_config(int(policy), 1 if three_stage else 0, calvo_cost_model(*(model or (0.0, 0.0, 0.0, 0.0))),
                                calvo_l3_config(int(chunk_bytes), int(n_slots), int(n_threads), float(l3_GBps), 0, 0),
                                pool or None)
    out = C.c_void_p()
    _check(lib().calvo_dispatch_create(ctx, C.byref(cfg), C.byref(out)))
    return out.value


def calvo_dispatch_submit(d: int, host_kv=None, host_layer_stride: int = 0, block_table=(), n_prefix_blocks: int = 0,
                          n_shared: int = 0, suffix_len: int = 0, q=None, k_suffix=None, v_suffix=None, out=None,
                          scale: float = 0.0, deadline_s: float = 0.0, sim_load_s: float = 0.0, sim_comp_s: float = 0.0,
                          q_layer_stride: int = 0, kv_layer_stride: int = 0, out_layer_stride: int = 0) -> int:
    """Queues one job (q, k_suffix, v_suffix, out: [L][S][H][D] device arrays) and returns its id."""
    tab, tp = _i32(block_table)
    job = calvo_dispatch_job(_ptr(host_kv), int(host_layer_stride), tp if len(tab) else None, int(n_prefix_blocks), int(n_shared),
                             int(suffix_len), 0, _ptr(q), _ptr(k_suffix), _ptr(v_suffix), _ptr(out), int(q_layer_stride), int(kv_layer_stride), int(out_layer_stride),
                             float(scale), 0.0,
                             float(deadline_s), float(sim_load_s), float(sim_comp_s))
    jid = C.c_int64(-1)
    _check(lib().calvo_dispatch_submit(d, C.byref(job), C.byref(jid)))
    return jid.value


def calvo_dispatch_wait(d: int, job: int) -> dict:
    res = calvo_dispatch_result()
    _check(lib().calvo_dispatch_wait(d, job, C.byref(res)))
    return _fields(res)


def calvo_dispatch_poll(d: int, job: int):
    """The job's result once it has finished, else None."""
    res = calvo_dispatch_result()
    rc = _check(lib().calvo_dispatch_poll(d, job, C.byref(res)), ok=(CALVO_OK, CALVO_ENOTREADY))
    return _fields(res) if rc == CALVO_OK else None


def calvo_dispatch_table(d: int, job: int) -> np.ndarray:
    n = C.c_int32(0)
    rc = lib().calvo_dispatch_table(d, job, None, 0, C.byref(n))
    if rc not in (CALVO_OK, CALVO_ENOMEM):
        _check(rc)
    table, tp = _i32(np.zeros(max(n.value, 1)))
    if n.value:
        _check(lib().calvo_dispatch_table(d, job, tp, n.value, C.byref(n)))
    return table[:n.value].copy()


def calvo_dispatch_release(d: int, job: int) -> None:
    _check(lib().calvo_dispatch_release(d, job))


def calvo_dispatch_stats_get(d: int) -> dict:
    st = calvo_dispatch_stats()
    _check(lib().calvo_dispatch_stats_get(d, C.byref(st)))
    return _fields(st)


def calvo_dispatch_destroy(d: int) -> None:
    _check(lib().calvo_dispatch_destroy(d))
