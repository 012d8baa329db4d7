"""Chunk-granular readiness: layers loaded in chunks of block indices, one signal per chunk, attention
started chunk by chunk on what has landed (paper Section 3.1, the per-block signal between stages).

The result is defined by the same oracle as the whole-layer path: pool bytes bit exact, attention
within the stated tolerance, element by element.
"""
import pytest
import torch

import hip_harness as hh
from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import workload as wl

pytestmark = pytest.mark.gpu


def check(w, chunk_blocks, **kw):
    print(f"[case] chunks={chunk_blocks} shape={w.shape} lens={[(r.prefix_len, r.suffix_len) for r in w.requests]} kw={kw}",
          flush=True)
    pool_g, out_g = hh.run_hip(w, chunk_blocks=chunk_blocks, **kw)
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    return hh.assert_attn_close(out_g, out_o, w.shape.dtype)


@pytest.mark.parametrize("cb_", [2, 6, 16, 40, 64, 1000])
def test_single_request_any_chunk_size(cb_):
    """Chunks of one sub-tile up to more than the whole prefix; 63 prefix blocks (an odd count: the last
    prefix block shares a 32-key sub-tile with the suffix) and a ragged suffix."""
    shape = wl.Shape(2, 8, 2, 128, "bf16", 128)
    w = wl.make_custom(shape, [(63 * 16, 77)], seed=1200 + cb_)
    check(w, [cb_, cb_])


def test_mixed_layers_and_staged_copy_engine():
    """Only the last layer in chunks (the case that pays when loading bounds the request), copy-engine
    ingest with staging buffers smaller than a chunk."""
    shape = wl.Shape(3, 8, 2, 128, "bf16", 300)
    w = wl.make_custom(shape, [(200 * 16, 150)], seed=1301)
    check(w, [0, 0, 48], staging_bytes=20 * shape.blk_bytes, n_staging=3)


def test_batch_with_shared_run_and_empty_prefix():
    """Four requests: a shared run of 8 blocks that only request 0 loads, different prefix lengths, one
    request without a prefix, one without a suffix; chunk boundaries inside and outside the shared run."""
    shape = wl.Shape(2, 8, 2, 128, "bf16", 400)
    lens = [(40 * 16, 100), (8 * 16, 33), (101 * 16, 0), (64 * 16, 257)]
    w = wl.make_custom(shape, lens, seed=1302, shared_blocks=8)
    check(w, [6, 30])
    w2 = wl.make_custom(shape, [(0, 90), (32 * 16, 5)], seed=1303)
    check(w2, [10, 10])


def test_group_sizes_other_than_four():
    for Hq, Hkv in [(10, 2), (4, 4), (6, 2)]:
        shape = wl.Shape(1, Hq, Hkv, 128, "bf16", 200)
        w = wl.make_custom(shape, [(96 * 16, 300)], seed=1304 + Hq)
        check(w, [32])


def test_fp32_pool_loads_in_chunks_and_attends_per_layer():
    """The vector-ALU kernel (fp32 pools, other head dims) has no partial results: chunked loads still
    give the same bytes and attention waits for the whole layer."""
    shape = wl.Shape(2, 8, 2, 64, "f32", 96)
    w = wl.make_custom(shape, [(48 * 16, 40)], seed=1305)
    check(w, [8, 0])


def test_chunk_events_and_argument_checks():
    shape = wl.Shape(3, 8, 2, 128, "bf16", 64)
    w = wl.make_custom(shape, [(40 * 16, 16)], seed=1306)
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(shape), shape, dev)
    host = hh.to_torch(w.host_kv, shape, pin=True)
    ctx = cb.calvo_create(3, 8, 2, 128, cb.CALVO_BF16, 64, pool)
    try:
        reqs = hh.make_requests(w, host)
        assert cb.calvo_chunk_count(ctx, 1) == 0
        for bad in ([3, 4, 4], [-2, 0, 0]):
            with pytest.raises(cb.CalvoError) as ei:
                cb.calvo_kv_ingest_chunked(ctx, reqs, 0, 3, bad)
            assert ei.value.code == cb.CALVO_EINVAL
        with pytest.raises(ValueError):
            cb.calvo_kv_ingest_chunked(ctx, reqs, 0, 3, [4, 4])
        hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, shape), hh.sentinel_pool_np(shape))   # nothing written
        cb.calvo_kv_ingest_chunked(ctx, reqs, 0, 3, [16, 0, 6])
        assert [cb.calvo_chunk_count(ctx, l) for l in range(3)] == [3, 0, 7]
        assert cb.calvo_chunk_event(ctx, 2, 6, cb.CALVO_EV_HOST_WAIT)
        for k in range(7):
            assert cb.calvo_chunk_event(ctx, 2, k, cb.CALVO_EV_QUERY)          # chunks fire in order
        assert cb.calvo_layer_event(ctx, 2, cb.CALVO_EV_HOST_WAIT)
        s = torch.cuda.Stream()
        assert cb.calvo_chunk_event(ctx, 0, 1, cb.CALVO_EV_STREAM_WAIT, s.cuda_stream)
        s.synchronize()
        for layer, chunk in [(1, 0), (0, 3), (2, -1), (5, 0)]:
            with pytest.raises(cb.CalvoError) as ei:
                cb.calvo_chunk_event(ctx, layer, chunk, cb.CALVO_EV_QUERY)
            assert ei.value.code == cb.CALVO_EINVAL
        cb.calvo_kv_ingest(ctx, reqs, 0, 1)                                     # a whole-layer load forgets the chunks
        assert cb.calvo_chunk_count(ctx, 0) == 0
    finally:
        cb.calvo_destroy(ctx)
    want = hh.sentinel_pool_after_ingest(w)
    hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, shape), want)


def test_attention_of_a_chunk_sees_only_landed_bytes():
    """A long load in a NaN-poisoned pool with attention queued right behind it, no host wait: every
    chunk's launch must wait for its own chunk (a launch that ran early would read NaN patterns)."""
    shape = wl.Shape(3, 8, 2, 128, "bf16", 1300)
    w = wl.make_custom(shape, [(1200 * 16, 40)], seed=1307)            # 3 x 75 MiB
    pool_g, out_g = hh.run_hip(w, chunk_blocks=[300, 0, 150], staging_bytes=64 * shape.blk_bytes)
    pool_o, _ = hh.run_oracle(w, attn=False)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    rows = [0, 15, 16, 39]
    view = pool_o.reshape(3, 1300, 2, 16, 2, 128)
    r = w.requests[0]
    for l in range(3):
        want = hh.orc.prefill_attn_sampled(view[l], w.q[l], r.table, r.prefix_len, r.suffix_len, 16, rows)
        hh.assert_attn_close(out_g[l][rows], want, "bf16")


@pytest.mark.parametrize("second", ["chunked", "whole"])
def test_two_requests_interleaved_through_one_context(second):
    """The readiness state of a layer belongs to the most recent loading call.  Here the second request's
    loading call (another chunk size, or whole layers) is queued before the first request's attention
    calls: the first request's launches are then planned with the later call's chunk geometry and wait
    for the later call's events - later than necessary, never too early, because the loads are in order
    on one stream.  Both requests' outputs and the pool bytes are the oracle's."""
    shape = wl.Shape(3, 8, 2, 128, "bf16", 256)
    w = wl.make_custom(shape, [(97 * 16, 45), (40 * 16, 70)], seed=1400)
    s = w.shape
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(s), s, dev)
    host = hh.to_torch(w.host_kv, s, pin=True)
    q, ks, vs = (hh.to_torch(a, s, dev) for a in (w.q, w.k_suffix, w.v_suffix))
    out = torch.full((s.n_layers, w.total_suffix, s.n_q_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    ctx = cb.calvo_create(s.n_layers, s.n_q_heads, s.n_kv_heads, s.head_dim, cb.CALVO_BF16, s.pool_blocks, pool,
                          staging_bytes=24 * s.blk_bytes)
    try:
        reqs = hh.make_requests(w, host)
        cb.calvo_kv_ingest_chunked(ctx, [reqs[0]], 0, s.n_layers, [16, 16, 0])
        if second == "chunked":
            cb.calvo_kv_ingest_chunked(ctx, [reqs[1]], 0, s.n_layers, [6, 0, 10])
        else:
            cb.calvo_kv_ingest(ctx, [reqs[1]], 0, s.n_layers)
        for i in (0, 1):
            a, b = int(w.cu_suffix[i]), int(w.cu_suffix[i + 1])
            for l in range(s.n_layers):
                cb.calvo_prefill_attn(ctx, l, q[l, a:b], ks[l, a:b], vs[l, a:b], out[l, a:b], [reqs[i]], [0, b - a], 0.0)
    finally:
        cb.calvo_destroy(ctx)
    torch.cuda.synchronize()
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, s), pool_o)
    hh.assert_attn_close(hh.to_numpy_stored(out, s), out_o, "bf16")
