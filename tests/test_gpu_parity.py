"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI.

Sizes are small enough for the full oracle yet span several 64-key tiles, several query
tiles, ragged tails and partial last blocks.  Pool bytes must be bit exact (including every
slot the path must not touch); attention must meet the stated tolerance.
"""
import numpy as np
import pytest
import torch

import hip_harness as hh
from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import workload as wl

pytestmark = pytest.mark.gpu


def check(w, **kw):
    print(f"[case] {w.name} shape={w.shape} lens={[(r.prefix_len, r.suffix_len) for r in w.requests]} kw={kw}",
          flush=True)
    pool_g, out_g = hh.run_hip(w, **kw)
    pool_o, out_o = hh.run_oracle(w, scale=kw.get("scale") or None)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    return hh.assert_attn_close(out_g, out_o, w.shape.dtype)


def test_config1_fp32_full():
    """Workload 1 in full: fp32, 8Q/2KV heads, D=64, P=1024, S=128, pool of 256 slots."""
    w = wl.make_config(1)
    mx, mean = check(w)
    print(f"cfg1 fp32 max {mx:.2e} mean {mean:.2e}")


@pytest.mark.parametrize("P,S", [(160, 77), (0, 130), (1024, 64), (48, 1), (256, 200)])
def test_bf16_mfma_single_request(P, S):
    shape = wl.Shape(2, 8, 2, 128, "bf16", 128)
    w = wl.make_custom(shape, [(P, S)], seed=100 + P + S)
    check(w)


@pytest.mark.parametrize("lens,shared,chunks", [
    ([(160, 77)], 0, None), ([(1024, 64), (48, 1), (0, 130)], 0, None), ([(8192, 40)], 0, None),
    ([(17 * 16, 40), (9 * 16, 20)], 2, None), ([(64 * 16, 90)], 0, [8, 0]), ([(64 * 16, 90)], 0, [8, 24]), ([(320, 0)], 0, None)])
def test_prepared_batch_gives_the_result_of_the_per_call_path(lens, shared, chunks):
    """calvo_batch_prepare + calvo_prefill_attn_batch (validation, planning and descriptor upload
    once per batch) against the oracle, and bit for bit against calvo_prefill_attn: single requests,
    a batch, split-KV pieces, a shared run, a layer loaded in chunks (planned per call), an empty suffix."""
    shape = wl.Shape(2, 8, 2, 128, "bf16", sum(-(-(p + s) // 16) for p, s in lens) + 8)
    w = wl.make_custom(shape, lens, seed=311 + len(lens), shared_blocks=shared)
    kw = dict(staging_bytes=16 * shape.blk_bytes, chunk_blocks=chunks)
    pool_p, out_p = hh.run_hip(w, prepared=True, **kw)
    pool_c, out_c = hh.run_hip(w, **kw)
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(pool_p, pool_o)
    hh.assert_attn_close(out_p, out_o, "bf16")
    assert np.array_equal(out_p, out_c)


def test_prepared_batch_is_reused_over_steps_and_chunk_geometries():
    """One prepared batch serves several steps whose layers are loaded whole or in chunks of different sizes:
    the launches that follow a chunking are planned the first time it is seen and found again afterwards.
    Every step gives the oracle's result."""
    shape = wl.Shape(3, 8, 2, 128, "bf16", 160)
    w = wl.make_custom(shape, [(70 * 16, 50), (33 * 16, 17)], seed=77)
    s = w.shape
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(s), s, dev)
    host = hh.to_torch(w.host_kv, s, pin=True)
    q, ks, vs = (hh.to_torch(a, s, dev) for a in (w.q, w.k_suffix, w.v_suffix))
    out = torch.empty((s.n_layers, w.total_suffix, s.n_q_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
    pool_o, out_o = hh.run_oracle(w)
    ctx = cb.calvo_create(s.n_layers, s.n_q_heads, s.n_kv_heads, s.head_dim, cb.CALVO_BF16, s.pool_blocks, pool,
                          staging_bytes=32 * s.blk_bytes)
    try:
        reqs = hh.make_requests(w, host)
        batch = cb.calvo_batch_prepare(ctx, reqs, w.cu_suffix)
        try:
            for step, chunks in enumerate([[8, 8, 20], None, [0, 12, 12], [8, 0, 20], [8, 8, 20]]):
                pool.copy_(hh.to_torch(hh.sentinel_pool_np(s), s, dev))
                out.fill_(float("nan"))
                torch.cuda.synchronize()
                if chunks is None:
                    cb.calvo_kv_ingest(ctx, reqs, 0, s.n_layers)
                else:
                    cb.calvo_kv_ingest_chunked(ctx, reqs, 0, s.n_layers, chunks)
                for l in range(s.n_layers):
                    cb.calvo_prefill_attn_batch(ctx, batch, l, q[l], ks[l], vs[l], out[l], 0.0)
                torch.cuda.synchronize()
                hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, s), pool_o)
                hh.assert_attn_close(hh.to_numpy_stored(out, s), out_o, "bf16")
        finally:
            cb.calvo_batch_destroy(batch)
    finally:
        cb.calvo_destroy(ctx)


def test_prepared_batch_fp32_and_bad_requests():
    w = wl.make_custom(wl.Shape(2, 6, 3, 40, "f32", 64), [(64, 37), (0, 50), (160, 5)], seed=19)
    pool_p, out_p = hh.run_hip(w, prepared=True, scale=0.2)
    pool_o, out_o = hh.run_oracle(w, scale=0.2)
    hh.assert_pool_bit_exact(pool_p, pool_o)
    hh.assert_attn_close(out_p, out_o, "f32")
    # a slot outside the pool is refused when the batch is prepared: no handle, nothing queued
    pool = torch.zeros(64 * w.shape.blk_elems * 2, dtype=torch.float32, device="cuda:0")
    ctx = cb.calvo_create(2, 6, 3, 40, cb.CALVO_F32, 64, pool)
    try:
        bad = cb.make_request(None, 0, np.array([1, 2, 64], np.int32), 2, 5, 2)
        with pytest.raises(cb.CalvoError) as ei:
            cb.calvo_batch_prepare(ctx, [bad], np.array([0, 5], np.int32))
        assert ei.value.code == cb.CALVO_EINVAL and "outside the pool" in str(ei.value)
    finally:
        cb.calvo_destroy(ctx)


def _scale_prefix_keys(w, gain):
    """Multiply the K rows of the cached prefix by gain(position) (re-rounded to bf16), in place."""
    from oracle import calvo_oracle as orc
    s = w.shape
    B = s.block_tokens
    for r in w.requests:
        for j in range(r.n_prefix_blocks):
            blk = w.host_kv[:, r.host_block_start + j].reshape(s.n_layers, 2, B, s.n_kv_heads * s.head_dim)
            g = np.array([gain(j * B + i) for i in range(B)], np.float64)[None, :, None]
            blk[:, 0] = wl.f32_to_bf16_bits((orc.widen(blk[:, 0]) * g).astype(np.float32))


@pytest.mark.parametrize("pattern", ["growing", "spike", "shrinking"])
def test_bf16_scores_that_outgrow_the_softmax_reference(pattern):
    """The pipelined kernel keeps a softmax reference that it raises only when a weight gets too
    large.  Keys whose scores grow along the sequence (or jump once) force that path in the
    middle of the pipelined loop; keys that shrink leave an early large reference in place."""
    shape = wl.Shape(2, 8, 2, 128, "bf16", 192)
    P, S = 2048, 96
    w = wl.make_custom(shape, [(P, S)], seed=900 + len(pattern))
    gain = {"growing": lambda pos: 1.0 + 60.0 * (pos / P) ** 2,
            "spike": lambda pos: 80.0 if pos == 1037 else 1.0,
            "shrinking": lambda pos: 60.0 * (1.0 - pos / P) ** 2 + 0.05}[pattern]
    _scale_prefix_keys(w, gain)
    check(w)


@pytest.mark.parametrize("lens", [[(16384, 20)], [(8192, 64)], [(12000, 1)], [(4096, 3), (8192, 70), (2048, 0), (6144, 130)]])
def test_bf16_short_suffix_over_long_context_uses_split_kv(lens):
    """Few suffix tokens over a long context: the library cuts every tile's context into pieces that run
    as separate workgroups and merges them (the paper's regime: long reused context, short query)."""
    shape = wl.Shape(2, 8, 2, 128, "bf16", sum(-(-(p + s) // 16) for p, s in lens) + 5)
    w = wl.make_custom(shape, lens, seed=700 + len(lens) + lens[0][1])
    check(w)


@pytest.mark.parametrize("n_splits", [2, 5, 64])
def test_bf16_forced_context_splits(n_splits, monkeypatch):
    """Every tile cut into n pieces (down to single 32-key sub-tiles), including the pieces that hold
    the causal diagonal and the ragged end of the context."""
    monkeypatch.setenv("CALVO_ATTN_SPLITS", str(n_splits))
    shape = wl.Shape(2, 8, 2, 128, "bf16", 128)
    w = wl.make_custom(shape, [(1024, 200), (48, 77), (0, 130)], seed=800 + n_splits)
    check(w)


@pytest.mark.parametrize("variant", [3, 4])
def test_bf16_both_pipelined_kernels_on_the_same_batches(variant, monkeypatch):
    """The library picks one of two pipelined kernels per call (8-wave workgroups with 64-token tiles,
    or two 4-wave workgroups per CU with 32-token tiles); here each is forced on batches the other
    would have served: ragged suffixes, a forced split, group sizes 1 and 2, chunk-granular loading."""
    monkeypatch.setenv("CALVO_ATTN_VARIANT", str(variant))
    shape = wl.Shape(2, 8, 2, 128, "bf16", 400)
    check(wl.make_custom(shape, [(1024, 200), (48, 77), (0, 130), (2048, 28), (512, 64)], seed=2000 + variant))
    check(wl.make_custom(wl.Shape(1, 10, 2, 128, "bf16", 300), [(96 * 16, 300)], seed=2010 + variant))
    check(wl.make_custom(wl.Shape(1, 4, 2, 128, "bf16", 300), [(64 * 16, 150), (32 * 16, 31)], seed=2020 + variant))
    check(wl.make_custom(wl.Shape(2, 8, 2, 128, "bf16", 600), [(8192, 40)], seed=2030 + variant))   # automatic split-KV
    pool_g, out_g = hh.run_hip(wl.make_custom(shape, [(63 * 16, 77)], seed=2040), chunk_blocks=[6, 16])
    pool_o, out_o = hh.run_oracle(wl.make_custom(shape, [(63 * 16, 77)], seed=2040))
    hh.assert_pool_bit_exact(pool_g, pool_o)
    hh.assert_attn_close(out_g, out_o, "bf16")


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (16, 2), (6, 2), (12, 4)])
def test_bf16_mfma_gqa_group_sizes(Hq, Hkv):
    shape = wl.Shape(1, Hq, Hkv, 128, "bf16", 64)
    w = wl.make_custom(shape, [(192, 150)], seed=7 * Hq + Hkv)
    check(w)


def test_bf16_mfma_varlen_batch_with_shared_run():
    shape = wl.Shape(2, 8, 2, 128, "bf16", 256)
    w = wl.make_custom(shape, [(256, 90), (128, 257), (512, 33), (64, 0), (128, 64)], seed=5, shared_blocks=4)
    check(w)


def test_bf16_generic_kernel_other_head_dims():
    for D in (64, 96, 256):
        shape = wl.Shape(1, 4, 2, D, "bf16", 64)
        w = wl.make_custom(shape, [(96, 70)], seed=D)
        check(w)


def test_fp32_varlen_and_explicit_scale():
    shape = wl.Shape(2, 6, 3, 40, "f32", 64)
    w = wl.make_custom(shape, [(64, 37), (0, 50), (160, 5)], seed=17)
    check(w, scale=0.2)


@pytest.mark.parametrize("staging_blocks,n_staging,n_copy", [(1, 2, 1), (3, 2, 0), (5, 4, 1), (64, 2, 1)])
def test_staged_copy_engine_ingest_is_bit_exact(staging_blocks, n_staging, n_copy):
    shape = wl.Shape(3, 8, 2, 128, "bf16", 128)
    w = wl.make_custom(shape, [(17 * 16, 40), (9 * 16, 20)], seed=23, shared_blocks=2)
    check(w, staging_bytes=staging_blocks * shape.blk_bytes, n_staging=n_staging, n_copy_streams=n_copy)


@pytest.mark.parametrize("hook,us", [("CALVO_TEST_SCATTER_DELAY_US", 300), ("CALVO_INGEST_DELAY_US", 200)])
def test_staging_ring_reuse_under_adverse_timing(hook, us, monkeypatch):
    """Two staging buffers of one block each and 26 blocks per layer: every transfer re-uses a buffer
    that an earlier scatter has read.  With a bounded delay kernel in front of every scatter the
    copy engine is far ahead of the scatter stream (a transfer into a buffer the scatter has not read
    yet would show as wrong pool bytes); with the host sleeping before every transfer the scatter
    stream runs dry between transfers instead."""
    monkeypatch.setenv(hook, str(us))
    shape = wl.Shape(2, 8, 2, 128, "bf16", 64)
    w = wl.make_custom(shape, [(17 * 16, 40), (9 * 16, 20)], seed=29)
    check(w, staging_bytes=shape.blk_bytes, n_staging=2)


@pytest.mark.parametrize("n_layers,lens,shared,staging_blocks", [
    (6, [(160, 40)], 0, 64),                               # groups of 1, 2, 1, 1, 1 layers
    (9, [(96, 20)], 0, 200),                               # 1, 2, 2, 2, 1, 1
    (12, [(64, 10), (128, 33), (96, 5)], 2, 64),           # a batch that loads as one run per layer: 1, 2, 3, 2, 2, 1, 1
    (5, [(160, 40)], 0, 15),                               # staging holds one layer and a half: no merge
])
def test_small_layers_share_a_transfer(n_layers, lens, shared, staging_blocks):
    """Layers that are one run each and follow each other in host memory cross PCIe together when
    the staging buffer holds several of them; every layer still gets its own scatter and event."""
    need = sum(p // 16 + -(-s // 16) for p, s in lens) - shared * (len(lens) - 1)
    shape = wl.Shape(n_layers, 8, 2, 128, "bf16", need + 20)
    w = wl.make_custom(shape, lens, seed=31 * n_layers + staging_blocks, shared_blocks=shared)
    check(w, staging_bytes=staging_blocks * shape.blk_bytes, n_staging=2)


@pytest.mark.parametrize("order", ["as laid out", "reversed", "interleaved"])
@pytest.mark.parametrize("staging_blocks", [0, 7, 64])
def test_batch_ingest_in_any_request_order(order, staging_blocks):
    """Requests whose host blocks follow each other are loaded as one run per layer (one transfer, one
    scatter); given in another order, or with a request in between that has nothing to load, they are
    separate runs.  The pool must hold the same bytes either way."""
    shape = wl.Shape(3, 8, 2, 128, "bf16", 160)
    w = wl.make_custom(shape, [(10 * 16, 10), (0, 20), (20 * 16, 5), (6 * 16, 7), (33 * 16, 0)], seed=3100, shared_blocks=0)
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(shape), shape, dev)
    host = hh.to_torch(w.host_kv, shape, pin=True)
    ctx = cb.calvo_create(3, 8, 2, 128, cb.CALVO_BF16, 160, pool, staging_bytes=staging_blocks * shape.blk_bytes)
    try:
        reqs = hh.make_requests(w, host)
        idx = {"as laid out": [0, 1, 2, 3, 4], "reversed": [4, 3, 2, 1, 0], "interleaved": [2, 0, 4, 1, 3]}[order]
        cb.calvo_kv_ingest(ctx, [reqs[i] for i in idx], 0, 3)
        assert cb.calvo_layer_event(ctx, 2, cb.CALVO_EV_HOST_WAIT)
    finally:
        cb.calvo_destroy(ctx)
    hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, shape), hh.sentinel_pool_after_ingest(w))


def test_no_suffix_and_no_prefix_edge_cases():
    shape = wl.Shape(1, 8, 2, 128, "bf16", 64)
    w = wl.make_custom(shape, [(128, 0)], seed=3)           # nothing to compute: ingest only
    pool_g, out_g = hh.run_hip(w)
    pool_o, _ = hh.run_oracle(w, attn=False)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    assert out_g.size == 0
    w = wl.make_custom(shape, [(0, 1)], seed=4)             # single token, no hit: O = V[0]
    pool_g, out_g = hh.run_hip(w)
    pool_o, out_o = hh.run_oracle(w)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    assert np.array_equal(hh.orc.widen(out_g)[0, 0, :, :],
                          np.repeat(hh.orc.widen(w.v_suffix[0, 0]), shape.group, axis=0))


def test_permuted_block_table_gives_same_output_bits():
    """Moving the same KV to other slots must not change a single output bit on the GPU either."""
    shape = wl.Shape(1, 8, 2, 128, "bf16", 96)
    w = wl.make_custom(shape, [(320, 100)], seed=31)
    _, out_a = hh.run_hip(w)
    rng = np.random.default_rng(1)
    w.requests[0].table = rng.permutation(shape.pool_blocks)[:len(w.requests[0].table)].astype(np.int32)
    _, out_b = hh.run_hip(w)
    assert np.array_equal(out_a, out_b)


def test_prefix_hit_equals_full_recompute_on_gpu():
    """Same tokens served as (P=256 hit, S=96) and as (P=0, S=352): suffix rows agree within tolerance."""
    shape = wl.Shape(1, 8, 2, 128, "bf16", 64)
    w_hit = wl.make_custom(shape, [(256, 96)], seed=41)
    _, out_hit = hh.run_hip(w_hit)
    B, r = 16, w_hit.requests[0]
    # rebuild the same sequence as one no-hit request: K/V of the prefix come from the host blocks
    blocks = w_hit.host_kv[0].reshape(16, 2, B, 2, 128)
    k_pre = blocks[:, 0].reshape(256, 2, 128)
    v_pre = blocks[:, 1].reshape(256, 2, 128)
    w_full = wl.make_custom(shape, [(0, 352)], seed=42)
    w_full.k_suffix = np.concatenate([k_pre, w_hit.k_suffix[0]])[None]
    w_full.v_suffix = np.concatenate([v_pre, w_hit.v_suffix[0]])[None]
    qf = w_full.q.copy()
    qf[0, 256:] = w_hit.q[0]
    w_full.q = qf
    _, out_full = hh.run_hip(w_full)
    a = hh.orc.widen(out_hit[0])
    b = hh.orc.widen(out_full[0, 256:])
    assert np.abs(a - b).max() <= 2e-2
    # and both equal the oracle of the hit formulation
    _, out_o = hh.run_oracle(w_hit)
    hh.assert_attn_close(out_full[:, 256:], out_o, "bf16")


def test_layer_events_and_layer_ranges():
    shape = wl.Shape(4, 8, 2, 128, "bf16", 64)
    w = wl.make_custom(shape, [(256, 16)], seed=51)
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(shape), shape, dev)
    host = hh.to_torch(w.host_kv, shape, pin=True)
    ctx = cb.calvo_create(4, 8, 2, 128, cb.CALVO_BF16, 64, pool)
    try:
        reqs = hh.make_requests(w, host)
        assert cb.calvo_layer_event(ctx, 2, cb.CALVO_EV_QUERY)          # never ingested: ready
        cb.calvo_kv_ingest(ctx, reqs, 1, 3)
        assert cb.calvo_layer_event(ctx, 1, cb.CALVO_EV_HOST_WAIT)
        assert cb.calvo_layer_event(ctx, 2, cb.CALVO_EV_HOST_WAIT)
        assert cb.calvo_layer_event(ctx, 2, cb.CALVO_EV_QUERY)
        s = torch.cuda.Stream()
        assert cb.calvo_layer_event(ctx, 2, cb.CALVO_EV_STREAM_WAIT, s.cuda_stream)
        s.synchronize()
    finally:
        cb.calvo_destroy(ctx)
    got = hh.to_numpy_stored(pool, shape)
    want = hh.sentinel_pool_np(shape)
    r = w.requests[0]
    hh.orc.kv_ingest(want, w.host_kv, r.table, r.n_prefix_blocks, layer_begin=1, layer_end=3)
    hh.assert_pool_bit_exact(got, want)                                  # layers 0 and 3 untouched


def test_invalid_requests_write_nothing():
    shape = wl.Shape(2, 8, 2, 128, "bf16", 32)
    w = wl.make_custom(shape, [(128, 16)], seed=61)
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(shape), shape, dev)
    host = hh.to_torch(w.host_kv, shape, pin=True)
    ctx = cb.calvo_create(2, 8, 2, 128, cb.CALVO_BF16, 32, pool)
    try:
        r = w.requests[0]
        stride = w.host_blocks * shape.blk_bytes
        bad = r.table.copy(); bad[3] = 32                               # destination not allocated
        dup = r.table.copy(); dup[5] = dup[1]
        pageable = np.zeros(w.host_kv.size, np.uint16)
        cases = [
            ([cb.make_request(host, stride, bad, r.n_prefix_blocks, r.suffix_len)], 0, 2),
            ([cb.make_request(host, stride, dup, r.n_prefix_blocks, r.suffix_len)], 0, 2),
            ([cb.make_request(host, stride, r.table, r.n_prefix_blocks, r.suffix_len)], 0, 3),
            ([cb.make_request(host, stride, r.table, r.n_prefix_blocks, r.suffix_len, first_ingest_block=9)], 0, 2),
            ([cb.make_request(None, stride, r.table, r.n_prefix_blocks, r.suffix_len)], 0, 2),
            ([cb.make_request(pageable.ctypes.data, stride, r.table, r.n_prefix_blocks, r.suffix_len)], 0, 2),
            ([cb.make_request(host, 16, r.table, r.n_prefix_blocks, r.suffix_len)], 0, 2),
        ]
        for reqs, lb, le in cases:
            with pytest.raises(cb.CalvoError) as ei:
                cb.calvo_kv_ingest(ctx, reqs, lb, le)
            assert ei.value.code == cb.CALVO_EINVAL, ei.value
        big = np.arange(40, dtype=np.int32)
        with pytest.raises(cb.CalvoError) as ei:
            cb.calvo_kv_ingest(ctx, [cb.make_request(host, stride, big, 40, 0)], 0, 2)
        assert ei.value.code == cb.CALVO_ENOMEM
        q = torch.zeros(16, 8, 128, dtype=torch.bfloat16, device=dev)
        with pytest.raises(cb.CalvoError):
            cb.calvo_prefill_attn(ctx, 0, q, None, None, q.clone(),
                                  [cb.make_request(host, stride, r.table, r.n_prefix_blocks, r.suffix_len)],
                                  np.array([0, 15], np.int32))
        with pytest.raises(cb.CalvoError):
            cb.calvo_prefill_attn(ctx, 5, q, None, None, q.clone(),
                                  [cb.make_request(host, stride, r.table, r.n_prefix_blocks, r.suffix_len)],
                                  np.array([0, 16], np.int32))
    finally:
        cb.calvo_destroy(ctx)
    hh.assert_pool_bit_exact(hh.to_numpy_stored(pool, shape), hh.sentinel_pool_np(shape))


def test_attention_waits_for_ingest_of_its_layer():
    """Compute must see fully loaded bytes even when it is queued right behind a long ingest:
    a large prefix in a NaN-poisoned pool, attention queued immediately, no host wait in between."""
    shape = wl.Shape(6, 8, 2, 128, "bf16", 1200)
    w = wl.make_custom(shape, [(1024 * 16, 32)], seed=71)              # 6 x 16 MiB to load
    pool_g, out_g = hh.run_hip(w)
    rows = [0, 15, 16, 31]
    B = 16
    pool_o, _ = hh.run_oracle(w, attn=False)
    hh.assert_pool_bit_exact(pool_g, pool_o)
    view = pool_o.reshape(6, 1200, 2, B, 2, 128)
    r = w.requests[0]
    for l in (0, 5):
        want = hh.orc.prefill_attn_sampled(view[l], w.q[l], r.table, r.prefix_len, r.suffix_len, B, rows)
        hh.assert_attn_close(out_g[l][rows], want, "bf16")


def test_caller_owned_compute_stream_orders_the_output():
    """With a caller's stream as the compute stream, work queued on that stream after
    calvo_prefill_attn sees the finished output (no host synchronisation in between), the inputs may
    be produced on that stream right before the call, and calvo_destroy leaves the stream usable."""
    shape = wl.Shape(3, 8, 2, 128, "bf16", 96)
    w = wl.make_custom(shape, [(512, 90), (256, 33)], seed=77)
    dev = torch.device("cuda:0")
    pool = hh.to_torch(hh.sentinel_pool_np(shape), shape, dev)
    host = hh.to_torch(w.host_kv, shape, pin=True)
    q_src, ks_src, vs_src = (hh.to_torch(a, shape, dev) for a in (w.q, w.k_suffix, w.v_suffix))
    T = w.total_suffix
    out = torch.full((3, T, 8, 128), float("nan"), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    ctx = cb.calvo_create(3, 8, 2, 128, cb.CALVO_BF16, 96, pool, staging_bytes=8 * shape.blk_bytes,
                          compute_stream=st.cuda_stream)
    snaps = []
    try:
        reqs = hh.make_requests(w, host)
        cb.calvo_kv_ingest(ctx, reqs, 0, 3)
        with torch.cuda.stream(st):
            for l in range(3):
                q, ks, vs = q_src[l].clone(), ks_src[l].clone(), vs_src[l].clone()     # produced on the stream, just before
                cb.calvo_prefill_attn(ctx, l, q, ks, vs, out[l], reqs, w.cu_suffix, 0.0)
                snaps.append(out[l].clone())                                           # consumed on the stream, right after
        st.synchronize()
        got = torch.stack(snaps)
    finally:
        cb.calvo_destroy(ctx)
    with torch.cuda.stream(st):                     # the stream is the caller's: still there
        again = got.float().sum()
    st.synchronize()
    assert torch.isfinite(again)
    _, out_o = hh.run_oracle(w)
    hh.assert_attn_close(hh.to_numpy_stored(got, shape), out_o, "bf16")
