"""Pins for the byte-level oracles (ingest scatter, suffix append) and the byte accounting."""
import os

import numpy as np

from oracle import calvo_oracle as orc
from paper_2603_21257_amd import workload as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_kv_footprint_matches_paper_statement():
    """Section 2.2: 10 M tokens of Llama-3.1-8B KVCache take more than 1 TB (and not, say, 2 TB)."""
    with open(os.path.join(GOLDEN, "kv_footprint.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    name, tokens, lower = rows[0][0], int(rows[0][1]), int(rows[0][2])
    assert name == "llama-3.1-8b"
    shape = wl.Shape(32, 32, 8, 128, "bf16", 1)
    per_token = shape.tok_bytes * shape.n_layers
    assert per_token == 131072
    total = per_token * tokens
    assert lower < total < 2 * lower
    # the workload's own accounting uses the same per-token figure
    w = wl.make_config(3, with_payload=False)
    assert w.ingest_bytes() == 61440 * per_token
    assert w.ingest_bytes() == int(7.5 * 2 ** 30)


def test_work_accounting_closed_forms():
    w2 = wl.make_config(2, with_payload=False)
    assert w2.ingest_bytes() == 2 * 2 ** 30
    assert w2.attn_pairs() == 2048 * 16384 + 2048 * 2049 // 2
    assert abs(w2.attn_flop() / 1.869e13 - 1) < 1e-3
    w3 = wl.make_config(3, with_payload=False)
    assert abs(w3.attn_flop() / 1.363e14 - 1) < 1e-3
    w5 = wl.make_config(5, with_payload=False)
    assert w5.ingest_bytes() == int(37.5 * 2 ** 30)
    assert abs(w5.attn_flop() / 2.727e15 - 1) < 1e-3
    w1 = wl.make_config(1)
    assert w1.ingest_bytes() == 2 ** 20
    assert abs(w1.attn_flop() / 2.85e8 - 1) < 2e-3


def test_ingest_is_a_byte_permutation_and_leaves_other_slots_alone():
    shape = wl.Shape(3, 4, 2, 8, "f32", 32, block_tokens=4)
    w = wl.make_custom(shape, [(24, 5)], seed=7)
    r = w.requests[0]
    sentinel = np.float32(-123.25)
    pool = np.full((3, 32, shape.blk_elems), sentinel, np.float32)
    moved = orc.kv_ingest(pool, w.host_kv, r.table, r.n_prefix_blocks)
    assert moved == w.ingest_bytes() == 6 * shape.blk_bytes * 3
    used = set(int(s) for s in r.table[:r.n_prefix_blocks])
    for l in range(3):
        for j in range(r.n_prefix_blocks):
            assert pool[l, r.table[j]].tobytes() == w.host_kv[l, j].tobytes()
        for s in range(32):
            if s not in used:
                assert np.all(pool[l, s] == sentinel)      # includes the (not yet written) suffix slots
    # multiset of bytes is preserved: sort both sides
    got = np.sort(pool[:, sorted(used)].reshape(-1).view(np.uint32))
    want = np.sort(w.host_kv.reshape(-1).view(np.uint32))
    assert np.array_equal(got, want)


def test_ingest_layer_range_and_first_block():
    shape = wl.Shape(4, 2, 1, 8, "bf16", 16, block_tokens=4)
    w = wl.make_custom(shape, [(16, 4)], seed=8)
    r = w.requests[0]
    pool = np.zeros((4, 16, shape.blk_elems), np.uint16)
    orc.kv_ingest(pool, w.host_kv, r.table, r.n_prefix_blocks, first_ingest_block=2, layer_begin=1, layer_end=3)
    for l in range(4):
        for j in range(4):
            moved = (1 <= l < 3) and j >= 2
            same = np.array_equal(pool[l, r.table[j]], w.host_kv[l, j])
            assert same == moved


def test_ingest_of_a_batch_reads_each_request_from_its_own_host_blocks():
    """Two requests staged back to back in one host area, the second sharing a run of slots with the
    first: request r's block j comes from host block host_block_start_r + j, and shared blocks are
    loaded once (first_ingest_block)."""
    shape = wl.Shape(2, 2, 1, 8, "bf16", 32, block_tokens=4)
    w = wl.make_custom(shape, [(20, 3), (28, 2)], seed=14, shared_blocks=2)
    r0, r1 = w.requests
    assert r0.host_block_start == 0 and r1.host_block_start > 0 and r1.first_ingest_block == 2
    pool = np.full((2, 32, shape.blk_elems), 0xFFFF, np.uint16)
    moved = sum(orc.kv_ingest(pool, w.host_kv, r.table, r.n_prefix_blocks, r.first_ingest_block, r.host_block_start)
                for r in w.requests)
    assert moved == w.ingest_bytes()
    # independent statement: whole-array fancy indexing per request
    for r in w.requests:
        js = np.arange(r.first_ingest_block, r.n_prefix_blocks)
        assert np.array_equal(pool[:, r.table[js]], w.host_kv[:, r.host_block_start + js])
    assert np.array_equal(r0.table[:2], r1.table[:2])          # the shared run names the same slots
    assert not np.array_equal(w.host_kv[:, 2], w.host_kv[:, r1.host_block_start + 2])   # distinct payloads per request


def test_ingest_preserves_nan_payloads_and_negative_zero():
    shape = wl.Shape(1, 2, 1, 8, "f32", 8, block_tokens=4)
    w = wl.make_custom(shape, [(8, 1)], seed=9)
    raw = w.host_kv.view(np.uint32)
    raw[0, 0, 0] = 0x7FC12345      # quiet NaN with payload
    raw[0, 0, 1] = 0xFF800001      # signalling NaN
    raw[0, 0, 2] = 0x80000000      # -0.0
    pool = np.zeros((1, 8, shape.blk_elems), np.float32)
    r = w.requests[0]
    orc.kv_ingest(pool, w.host_kv, r.table, r.n_prefix_blocks)
    assert pool[0, r.table[0]].tobytes() == w.host_kv[0, 0].tobytes()


def test_ingest_rejects_unallocated_destination():
    shape = wl.Shape(1, 2, 1, 8, "f32", 8, block_tokens=4)
    w = wl.make_custom(shape, [(8, 1)], seed=10)
    pool = np.zeros((1, 8, shape.blk_elems), np.float32)
    bad = w.requests[0].table.copy()
    bad[1] = 8
    try:
        orc.kv_ingest(pool, w.host_kv, bad, 2)
    except AssertionError:
        return
    raise AssertionError("out-of-range slot was accepted")


def test_suffix_append_places_tokens_at_absolute_positions():
    B, Hkv, D = 4, 2, 8
    rng = np.random.default_rng(12)
    P, S = 8, 6
    table = rng.permutation(16)[:4].astype(np.int32)
    pool = np.full((16, 2, B, Hkv, D), np.nan, np.float32)
    ks = rng.standard_normal((S, Hkv, D)).astype(np.float32)
    vs = rng.standard_normal((S, Hkv, D)).astype(np.float32)
    orc.suffix_append(pool, ks, vs, table, P, B)
    # independent statement of the same placement
    flatk = pool[table[2:], 0].reshape(-1, Hkv, D)
    flatv = pool[table[2:], 1].reshape(-1, Hkv, D)
    assert np.array_equal(flatk[:S], ks) and np.array_equal(flatv[:S], vs)
    assert np.isnan(flatk[S:]).all()                 # tail of the partial block untouched
    assert np.isnan(pool[table[:2]]).all()           # prefix slots untouched
    untouched = [s for s in range(16) if s not in set(table[2:].tolist())]
    assert np.isnan(pool[untouched]).all()


def test_varlen_batch_recipe_properties():
    shape, reqs = wl.config_shape_and_requests(4)
    assert len(reqs) == 8
    shared = reqs[0].table[:256]
    seen = set(shared.tolist())
    assert len(seen) == 256
    for i, r in enumerate(reqs):
        total = r.prefix_len + r.suffix_len
        assert 8192 <= total <= 32768
        assert r.prefix_len % 16 == 0 and r.prefix_len >= 4096
        assert np.array_equal(r.table[:256], shared)
        own = r.table[256:].tolist()
        assert len(r.table) == r.n_prefix_blocks + r.n_suffix_blocks
        assert not (set(own) & seen)                # distinct outside the shared run
        seen |= set(own)
        assert r.first_ingest_block == (0 if i == 0 else 256)
    assert max(seen) < shape.pool_blocks
    # host regions tile the host buffer exactly once
    w = wl.make_config(4, with_payload=False)
    cover = np.zeros(w.host_blocks, np.int32)
    for r in reqs:
        cover[r.host_block_start + r.first_ingest_block: r.host_block_start + r.n_prefix_blocks] += 1
    assert np.all(cover == 1)
