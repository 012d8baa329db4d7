"""calvo_prefill_attn_noalloc (the entry point for callers that cannot allocate device memory)
against calvo_prefill_attn: same pool bytes, same attention output, on two calls in a row that
share the library's static device array - the second one smaller - and both against the oracle."""
import os

import numpy as np
import pytest

import hip_harness as hh
from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import workload as wl

pytestmark = pytest.mark.gpu


def _both(w, **kw):
    pool_a, out_a = hh.run_hip(w, **kw)
    pool_n, out_n = hh.run_hip(w, attn_fn=cb.calvo_prefill_attn_noalloc, **kw)
    return (pool_a, out_a), (pool_n, out_n)


def _check(w, ref, new):
    hh.assert_pool_bit_exact(new[0], ref[0])
    # same kernels, same launch plan: the two entry points differ only in where descriptors and
    # partial results live, so the outputs agree to the bar of the parity tests (and in fact bit for bit)
    g = hh.orc.widen(new[1]) if new[1].dtype == np.uint16 else new[1].astype(np.float64)
    e = hh.orc.widen(ref[1]) if ref[1].dtype == np.uint16 else ref[1].astype(np.float64)
    tmx, tmean = hh.TOL[w.shape.dtype]
    d = np.abs(g - e)
    assert np.isfinite(g).all()
    assert d.max() <= tmx and d.mean() <= tmean, (d.max(), d.mean())
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(new[0], pool_o)
    hh.assert_attn_close(new[1], out_o, w.shape.dtype)


def test_noalloc_matches_prefill_attn_twice_second_smaller(monkeypatch):
    # first call: split tiles (partial results go through the static array), two requests
    monkeypatch.setenv("CALVO_ATTN_SPLITS", "3")
    shape = wl.Shape(2, 8, 2, 128, "bf16", 700)
    big = wl.make_custom(shape, [(4096, 70), (2048, 33)], seed=71)
    ref, new = _both(big)
    _check(big, ref, new)
    # second call, smaller, no cut tiles: stale descriptors and partial results of the first call
    # are still in the array and must not matter
    monkeypatch.delenv("CALVO_ATTN_SPLITS")
    small = wl.make_custom(wl.Shape(1, 8, 2, 128, "bf16", 64), [(256, 40)], seed=72)
    ref, new = _both(small)
    _check(small, ref, new)


def test_noalloc_fp32_path_and_repeat_in_one_context():
    # the vector-ALU kernel (fp32 pool) reads its descriptors from the same array
    w = wl.make_custom(wl.Shape(1, 8, 2, 64, "f32", 96), [(512, 50)], seed=73)
    ref, new = _both(w)
    _check(w, ref, new)


def test_noalloc_rejects_what_does_not_fit(monkeypatch):
    import torch
    monkeypatch.setenv("CALVO_ATTN_SPLITS", "8")
    shape = wl.Shape(1, 8, 2, 128, "bf16", 1200)
    w = wl.make_custom(shape, [(8192, 4096)], seed=74, with_payload=False)
    pool = torch.zeros((shape.pool_blocks * shape.blk_elems,), dtype=torch.bfloat16, device="cuda:0")
    q = torch.zeros((4096, 8, 128), dtype=torch.bfloat16, device="cuda:0")
    out = torch.full_like(q, 7.0)
    ctx = cb.calvo_create(1, 8, 2, 128, cb.CALVO_BF16, shape.pool_blocks, pool)
    try:
        r = w.requests[0]
        req = cb.make_request(None, 0, r.table, r.n_prefix_blocks, r.suffix_len, r.n_prefix_blocks)
        with pytest.raises(cb.CalvoError) as ei:
            cb.calvo_prefill_attn_noalloc(ctx, 0, q, None, None, out, [req], w.cu_suffix)
        assert ei.value.code == cb.CALVO_ENOMEM and "partial-result slots" in str(ei.value)
        torch.cuda.synchronize()
        assert bool((out == 7.0).all())          # nothing was queued
    finally:
        cb.calvo_destroy(ctx)
