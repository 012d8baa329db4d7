"""Three-stage loading (emulated remote store -> pinned ring -> HBM) through the C ABI: the pool
must hold exactly the bytes the oracle's ingest puts there, attention over it must match the
oracle, and the hand-over / readiness signals must behave as the header says."""
import time

import pytest
import torch

import hip_harness as hh
from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import workload as wl

pytestmark = pytest.mark.gpu


def run_l3(w, staging_bytes, wait_before_attn=False, **l3):
    """Like hip_harness.run_hip, but the cached prefix sits in pageable host memory and is loaded
    with calvo_kv_ingest_l3.  Returns (pool, out, loader stats)."""
    s = w.shape
    dev = torch.device("cuda:0")
    dt = hh.torch_dtype(s)
    pool = hh.to_torch(hh.sentinel_pool_np(s), s, dev)
    remote = hh.to_torch(w.host_kv, s)                       # ordinary (pageable) CPU tensor
    assert not remote.is_pinned()
    T = w.total_suffix
    q, ks, vs = hh.to_torch(w.q, s, dev), hh.to_torch(w.k_suffix, s, dev), hh.to_torch(w.v_suffix, s, dev)
    out = torch.full((s.n_layers, max(T, 1), s.n_q_heads, s.head_dim), float("nan"), dtype=dt, device=dev)
    torch.cuda.synchronize()
    ctx = cb.calvo_create(s.n_layers, s.n_q_heads, s.n_kv_heads, s.head_dim,
                          cb.CALVO_BF16 if s.dtype == "bf16" else cb.CALVO_F32, s.pool_blocks, pool,
                          staging_bytes=staging_bytes)
    try:
        reqs = hh.make_requests(w, remote)
        cb.calvo_kv_ingest_l3(ctx, reqs, 0, s.n_layers, **l3)
        if wait_before_attn:
            stats = cb.calvo_l3_wait(ctx)
        for l in range(s.n_layers):                          # attention is queued while loading proceeds
            cb.calvo_prefill_attn(ctx, l, q[l], ks[l], vs[l], out[l], reqs, w.cu_suffix, 0.0)
        stats = cb.calvo_l3_wait(ctx)
        for l in range(s.n_layers):
            assert cb.calvo_layer_event(ctx, l, cb.CALVO_EV_HOST_WAIT)
    finally:
        cb.calvo_destroy(ctx)
    torch.cuda.synchronize()
    return hh.to_numpy_stored(pool, s), hh.to_numpy_stored(out[:, :T], s), stats


@pytest.mark.parametrize("chunk_blocks,n_slots,n_threads", [(1, 2, 1), (3, 3, 4), (7, 8, 2), (0, 0, 0)])
def test_three_stage_ingest_is_bit_exact_and_attention_matches(chunk_blocks, n_slots, n_threads):
    shape = wl.Shape(3, 8, 2, 128, "bf16", 96)
    w = wl.make_custom(shape, [(21 * 16, 40), (9 * 16, 20), (16 * 16, 70)], seed=77, shared_blocks=3)
    print(f"[case] three-stage chunk_blocks={chunk_blocks} n_slots={n_slots} n_threads={n_threads}", flush=True)
    pool_g, out_g, st = run_l3(w, staging_bytes=5 * shape.blk_bytes, chunk_bytes=chunk_blocks * shape.blk_bytes,
                               n_slots=n_slots, n_threads=n_threads)
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    hh.assert_attn_close(out_g, out_o, "bf16")
    assert st["bytes"] == w.ingest_bytes()
    eff = min(chunk_blocks or 5, 5)                          # chunks never exceed the device staging buffer
    want_chunks = shape.n_layers * sum(-(-(r.n_prefix_blocks - r.first_ingest_block) // eff) for r in w.requests)
    assert st["chunks"] == want_chunks


def test_three_stage_fp32_and_full_wait_first():
    w = wl.make_config(1)
    pool_g, out_g, st = run_l3(w, staging_bytes=16 * w.shape.blk_bytes, wait_before_attn=True, n_threads=3)
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    hh.assert_attn_close(out_g, out_o, "f32")


@pytest.mark.timing
def test_link_rate_is_respected_and_layers_become_ready_in_order():
    """2 layers x 32 MiB at an emulated 1 GB/s: at least 64 ms on the link; while the loader works
    on layer 0 a query of layer 1 says 'not ready', and its event fires only after the loader is done."""
    shape = wl.Shape(2, 8, 8, 128, "bf16", 600)              # 64 KiB blocks
    w = wl.make_custom(shape, [(512 * 16, 16)], seed=5)
    s = w.shape
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(s), s, dev)
    remote = hh.to_torch(w.host_kv, s)
    ctx = cb.calvo_create(s.n_layers, s.n_q_heads, s.n_kv_heads, s.head_dim, cb.CALVO_BF16, s.pool_blocks, pool,
                          staging_bytes=8 << 20)
    try:
        reqs = hh.make_requests(w, remote)
        t0 = time.perf_counter()
        cb.calvo_kv_ingest_l3(ctx, reqs, 0, 2, chunk_bytes=4 << 20, n_slots=3, n_threads=2, l3_GBps=1.0)
        t_call = time.perf_counter() - t0
        assert cb.calvo_layer_event(ctx, 1, cb.CALVO_EV_QUERY) is False        # still on the link
        assert cb.calvo_layer_event(ctx, 0, cb.CALVO_EV_HOST_WAIT)
        t_l0 = time.perf_counter() - t0
        assert cb.calvo_layer_event(ctx, 1, cb.CALVO_EV_HOST_WAIT)
        t_l1 = time.perf_counter() - t0
        st = cb.calvo_l3_wait(ctx)
        assert cb.calvo_layer_event(ctx, 1, cb.CALVO_EV_QUERY) is True
    finally:
        cb.calvo_destroy(ctx)
    nbytes = w.ingest_bytes()
    assert nbytes == 2 * 32 * 2 ** 20
    print(f"call returned after {t_call * 1e3:.1f} ms, layer 0 after {t_l0 * 1e3:.1f} ms, layer 1 after {t_l1 * 1e3:.1f} ms, "
          f"link busy {st['l3_busy_s'] * 1e3:.1f} ms, ring wait {st['ring_wait_s'] * 1e3:.1f} ms")
    assert t_call < 0.5 * nbytes / 1e9                        # the call only starts the loader (it returns long before layer 0 is in)
    assert t_l0 >= 0.5 * nbytes / 1e9 * 0.98 and t_l1 >= nbytes / 1e9 * 0.98
    assert st["l3_busy_s"] >= nbytes / 1e9 * 0.98
    assert t_l1 < nbytes / 1e9 * 3.0                          # and the other stages add little on top (margin for a slow box)
    # suffix slots were never written here: prefix slots hold the host bytes, the rest the sentinel
    hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, s), hh.sentinel_pool_after_ingest(w))


def test_l3_call_rejects_bad_arguments_and_zero_copy_contexts():
    shape = wl.Shape(1, 8, 2, 128, "bf16", 32)
    w = wl.make_custom(shape, [(4 * 16, 8)], seed=6)
    s = w.shape
    pool = hh.to_torch(hh.sentinel_pool_np(s), s, torch.device("cuda:0"))
    remote = hh.to_torch(w.host_kv, s)
    ctx0 = cb.calvo_create(1, 8, 2, 128, cb.CALVO_BF16, 32, pool, staging_bytes=0)
    ctx1 = cb.calvo_create(1, 8, 2, 128, cb.CALVO_BF16, 32, pool, staging_bytes=4 * s.blk_bytes)
    try:
        reqs = hh.make_requests(w, remote)
        for ctx, kw, frag in [(ctx0, {}, "staging buffers"), (ctx1, dict(n_slots=1), "n_slots"),
                              (ctx1, dict(n_threads=40), "n_threads"), (ctx1, dict(l3_GBps=-1.0), "l3_GBps"),
                              (ctx1, dict(chunk_bytes=100), "smaller than one block")]:
            with pytest.raises(cb.CalvoError) as ei:
                cb.calvo_kv_ingest_l3(ctx, reqs, 0, 1, **kw)
            assert ei.value.code == cb.CALVO_EINVAL and frag in str(ei.value)
        assert cb.calvo_l3_wait(ctx1)["chunks"] == 0
        torch.cuda.synchronize()
        assert (hh.to_numpy_stored(pool, s) == hh.SENTINEL_BF16).all()          # nothing was written
    finally:
        cb.calvo_destroy(ctx0)
        cb.calvo_destroy(ctx1)


@pytest.mark.parametrize("chunk_blocks", [2, 6, 12])
def test_three_stage_with_chunk_granular_readiness(chunk_blocks):
    """The loader signals every chunk of block indices as it hands it to the L2 -> L1 stage and
    attention follows chunk by chunk (queued while the loader is still working): same bytes, same
    attention result; a batch with a shared run, an odd block count and a request without prefix."""
    shape = wl.Shape(3, 8, 2, 128, "bf16", 160)
    w = wl.make_custom(shape, [(33 * 16, 50), (9 * 16, 20), (48 * 16, 70)], seed=78, shared_blocks=5)
    print(f"[case] three-stage chunk-ready chunk_blocks={chunk_blocks}", flush=True)
    pool_g, out_g, st = run_l3(w, staging_bytes=16 * shape.blk_bytes, chunk_bytes=chunk_blocks * shape.blk_bytes,
                               n_slots=3, n_threads=2, chunk_ready=True, l3_GBps=2.0)
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    hh.assert_attn_close(out_g, out_o, "bf16")
    assert st["bytes"] == w.ingest_bytes()


@pytest.mark.timing
def test_chunk_signals_follow_the_loader():
    """1 layer x 48 MiB in 8 MiB chunks at an emulated 1 GB/s: early chunks report ready while later
    ones are still on the link, and a chunk the loader has not reached says 'not ready'."""
    shape = wl.Shape(1, 8, 8, 128, "bf16", 800)              # 64 KiB blocks
    w = wl.make_custom(shape, [(768 * 16, 16)], seed=6)
    s = w.shape
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(s), s, dev)
    remote = hh.to_torch(w.host_kv, s)
    ctx = cb.calvo_create(1, 8, 8, 128, cb.CALVO_BF16, 800, pool, staging_bytes=8 << 20)
    try:
        reqs = hh.make_requests(w, remote)
        t0 = time.perf_counter()
        cb.calvo_kv_ingest_l3(ctx, reqs, 0, 1, chunk_bytes=8 << 20, l3_GBps=1.0, chunk_ready=True)
        assert cb.calvo_chunk_count(ctx, 0) == 6
        assert not cb.calvo_chunk_event(ctx, 0, 5, cb.CALVO_EV_QUERY)        # 48 ms away
        assert cb.calvo_chunk_event(ctx, 0, 1, cb.CALVO_EV_HOST_WAIT)
        t1 = time.perf_counter() - t0
        assert 0.014 < t1 < 0.2, t1                                          # two chunks of 8 ms each on the link (upper bound: a slow box)
        assert not cb.calvo_chunk_event(ctx, 0, 5, cb.CALVO_EV_QUERY)
        assert not cb.calvo_layer_event(ctx, 0, cb.CALVO_EV_QUERY)
        assert cb.calvo_chunk_event(ctx, 0, 5, cb.CALVO_EV_HOST_WAIT)
        assert time.perf_counter() - t0 > 0.046
        cb.calvo_l3_wait(ctx)
        assert cb.calvo_layer_event(ctx, 0, cb.CALVO_EV_HOST_WAIT)
    finally:
        cb.calvo_destroy(ctx)
    hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, s), hh.sentinel_pool_after_ingest(w))


def test_loader_failure_is_reported_once_and_the_context_loads_again(monkeypatch):
    """A failure inside the loader thread (injected from the host: no device fault) comes back from the
    first call that depends on it and from no later one; the layers it did not hand over count as
    never loaded, and a plain calvo_kv_ingest through the same context then fills the pool correctly."""
    monkeypatch.setenv("CALVO_TEST_L3_FAIL_CHUNK", "3")
    shape = wl.Shape(3, 8, 2, 128, "bf16", 96)
    w = wl.make_custom(shape, [(12 * 16, 40)], seed=91)
    s = w.shape
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(s), s, dev)
    remote = hh.to_torch(w.host_kv, s)
    pinned = hh.to_torch(w.host_kv, s, pin=True)
    T = w.total_suffix
    q, ks, vs = hh.to_torch(w.q, s, dev), hh.to_torch(w.k_suffix, s, dev), hh.to_torch(w.v_suffix, s, dev)
    out = torch.full((s.n_layers, T, s.n_q_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=dev)
    ctx = cb.calvo_create(s.n_layers, s.n_q_heads, s.n_kv_heads, s.head_dim, cb.CALVO_BF16, s.pool_blocks, pool,
                          staging_bytes=4 * s.blk_bytes)
    try:
        cb.calvo_kv_ingest_l3(ctx, hh.make_requests(w, remote), 0, s.n_layers, chunk_bytes=4 * s.blk_bytes)
        with pytest.raises(cb.CalvoError) as ei:                 # chunk 3 is the first one of layer 1
            cb.calvo_prefill_attn(ctx, 2, q[2], ks[2], vs[2], out[2], hh.make_requests(w, remote), w.cu_suffix, 0.0)
        assert ei.value.code == cb.CALVO_EHIP and "injected" in str(ei.value)
        st = cb.calvo_l3_wait(ctx)                               # reported once: not again
        assert cb.calvo_layer_event(ctx, 2, cb.CALVO_EV_QUERY)   # un-marked: counts as never loaded
        monkeypatch.delenv("CALVO_TEST_L3_FAIL_CHUNK")
        reqs = hh.make_requests(w, pinned)
        cb.calvo_kv_ingest(ctx, reqs, 0, s.n_layers)
        for l in range(s.n_layers):
            cb.calvo_prefill_attn(ctx, l, q[l], ks[l], vs[l], out[l], reqs, w.cu_suffix, 0.0)
        for l in range(s.n_layers):
            assert cb.calvo_layer_event(ctx, l, cb.CALVO_EV_HOST_WAIT)
    finally:
        cb.calvo_destroy(ctx)
    torch.cuda.synchronize()
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, s), pool_o)
    hh.assert_attn_close(hh.to_numpy_stored(out, s), out_o, "bf16")
