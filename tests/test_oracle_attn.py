"""Pins for the attention oracle: none of them re-uses the oracle's own formula path.

Each test is chosen so that a plausible mistake (dropped scale, wrong causal
boundary, transposed operand, wrong GQA group, wrong block index, reading the
tail of a partial block) fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

from oracle import calvo_oracle as orc
from paper_2603_21257_amd import workload as wl


def build_pool(shape, req, k_all, v_all, fill=np.nan):
    """Place contiguous K/V [T][Hkv][D] (fp32) into a pool through req.table (test-side helper,
    written independently of oracle.suffix_append: whole-array indexing, not a token loop)."""
    B = shape.block_tokens
    pool = np.full((shape.pool_blocks, 2, B, shape.n_kv_heads, shape.head_dim), fill, np.float32)
    T = k_all.shape[0]
    for b in range(-(-T // B)):
        n = min(B, T - b * B)
        pool[req.table[b], 0, :n] = k_all[b * B:b * B + n]
        pool[req.table[b], 1, :n] = v_all[b * B:b * B + n]
    return pool


def tiny(seed=0, P=8, S=5, Hq=4, Hkv=2, D=8, B=4, pool_blocks=16):
    shape = wl.Shape(1, Hq, Hkv, D, "f32", pool_blocks, block_tokens=B)
    rng = np.random.default_rng(seed)
    nblk = P // B + -(-S // B)
    table = rng.permutation(pool_blocks)[:nblk].astype(np.int32)
    req = wl.Request(P, S, table, block_tokens=B)
    k = rng.standard_normal((P + S, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((P + S, Hkv, D)).astype(np.float32)
    q = rng.standard_normal((S, Hq, D)).astype(np.float32)
    return shape, req, q, k, v


def brute_force(q, k, v, P, scale):
    """Contiguous, unpaged, scalar triple loop in Python floats (fp64)."""
    S, Hq, D = q.shape
    G = Hq // k.shape[1]
    out = np.zeros((S, Hq, D))
    for i in range(S):
        for h in range(Hq):
            g = h // G
            scores = []
            for t in range(P + i + 1):
                acc = 0.0
                for d in range(D):
                    acc += float(q[i, h, d]) * float(k[t, g, d])
                scores.append(acc * scale)
            m = max(scores)
            ws = [math.exp(s - m) for s in scores]
            z = sum(ws)
            for d in range(D):
                out[i, h, d] = sum(w * float(v[t, g, d]) for t, w in enumerate(ws)) / z
    return out


@pytest.mark.parametrize("seed,P,S,B", [(0, 8, 5, 4), (1, 0, 7, 4), (2, 12, 1, 4), (3, 16, 6, 8)])
def test_paged_equals_bruteforce_contiguous(seed, P, S, B):
    shape, req, q, k, v = tiny(seed, P=P, S=S, B=B)
    pool = build_pool(shape, req, k, v)
    got = orc.prefill_attn(pool, q, req.table, P, S, B)
    scale = float(np.float32(1.0) / np.sqrt(np.float32(shape.head_dim)))
    want = brute_force(q, k, v, P, scale)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


@pytest.mark.parametrize("seed,P,S,Hq,Hkv,D", [(5, 48, 19, 8, 2, 16), (6, 0, 33, 4, 4, 32), (7, 32, 32, 6, 1, 8)])
def test_matches_library_sdpa_float64(seed, P, S, Hq, Hkv, D):
    """Special case that reduces to a library routine: dense SDPA with an explicit boolean mask."""
    shape, req, q, k, v = tiny(seed, P=P, S=S, Hq=Hq, Hkv=Hkv, D=D, B=16, pool_blocks=32)
    pool = build_pool(shape, req, k, v)
    got = orc.prefill_attn(pool, q, req.table, P, S, 16)
    G = Hq // Hkv
    tq = torch.from_numpy(q.astype(np.float64)).permute(1, 0, 2)[None]            # [1,Hq,S,D]
    tk = torch.from_numpy(k.astype(np.float64)).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    tv = torch.from_numpy(v.astype(np.float64)).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    cols = torch.arange(P + S)[None, :]
    rows = torch.arange(S)[:, None]
    mask = cols <= (P + rows)
    scale = float(np.float32(1.0) / np.sqrt(np.float32(D)))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    ref = ref[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_block_table_permutation_invariance_is_bit_exact():
    shape, req, q, k, v = tiny(11, P=16, S=9, B=4, pool_blocks=32)
    pool_a = build_pool(shape, req, k, v)
    out_a = orc.prefill_attn(pool_a, q, req.table, 16, 9, 4)
    rng = np.random.default_rng(99)
    req_b = wl.Request(16, 9, rng.permutation(32)[:len(req.table)].astype(np.int32), block_tokens=4)
    assert not np.array_equal(req_b.table, req.table)
    pool_b = build_pool(shape, req_b, k, v)
    out_b = orc.prefill_attn(pool_b, q, req_b.table, 16, 9, 4)
    assert np.array_equal(out_a, out_b)


def test_prefix_hit_equals_full_recompute():
    """Rows P..P+S-1 of a no-hit prefill over the whole sequence equal the prefix-hit result."""
    rng = np.random.default_rng(21)
    P, S, Hq, Hkv, D, B = 32, 11, 4, 2, 16, 8
    shape = wl.Shape(1, Hq, Hkv, D, "f32", 16, block_tokens=B)
    k = rng.standard_normal((P + S, Hkv, D)).astype(np.float32)
    v = rng.standard_normal((P + S, Hkv, D)).astype(np.float32)
    q_full = rng.standard_normal((P + S, Hq, D)).astype(np.float32)
    nblk = -(-(P + S) // B)
    table = rng.permutation(16)[:nblk].astype(np.int32)
    req = wl.Request(P, S, table, block_tokens=B)
    pool = build_pool(shape, req, k, v)
    hit = orc.prefill_attn(pool, q_full[P:], table, P, S, B)
    full = orc.prefill_attn(pool, q_full, table, 0, P + S, B)
    np.testing.assert_allclose(hit, full[P:], rtol=0, atol=1e-14)


def test_convex_combination_bounds():
    shape, req, q, k, v = tiny(31, P=12, S=6, B=4)
    pool = build_pool(shape, req, k, v)
    out = orc.prefill_attn(pool, q, req.table, 12, 6, 4)
    G = shape.group
    for i in range(6):
        for h in range(shape.n_q_heads):
            vis = v[:12 + i + 1, h // G].astype(np.float64)
            assert np.all(out[i, h] <= vis.max(0) + 1e-12)
            assert np.all(out[i, h] >= vis.min(0) - 1e-12)


def test_zero_keys_give_running_mean_of_values():
    shape, req, q, k, v = tiny(41, P=8, S=7, B=4)
    k[:] = 0
    pool = build_pool(shape, req, k, v)
    out = orc.prefill_attn(pool, q, req.table, 8, 7, 4)
    G = shape.group
    for i in range(7):
        for h in range(shape.n_q_heads):
            want = v[:8 + i + 1, h // G].astype(np.float64).mean(0)
            np.testing.assert_allclose(out[i, h], want, rtol=0, atol=1e-14)


def test_constant_values_and_single_key():
    shape, req, q, k, v = tiny(42, P=8, S=4, B=4)
    v[:] = np.float32(0.375)
    pool = build_pool(shape, req, k, v)
    out = orc.prefill_attn(pool, q, req.table, 8, 4, 4)
    np.testing.assert_allclose(out, 0.375, rtol=0, atol=1e-15)
    # P=0, S=1: the only visible key is the token itself
    shape, req, q, k, v = tiny(43, P=0, S=1, B=4)
    pool = build_pool(shape, req, k, v)
    out = orc.prefill_attn(pool, q, req.table, 0, 1, 4)
    for h in range(shape.n_q_heads):
        assert np.array_equal(out[0, h], v[0, h // shape.group].astype(np.float64))


def test_dominant_key_selects_its_value_row():
    """One key with a score margin >= 50 takes all the weight (to ~e^-50)."""
    shape, req, q, k, v = tiny(44, P=8, S=3, Hq=2, Hkv=1, D=8, B=4)
    q[:] = 0
    q[:, :, 0] = 1.0
    k[:] = 0
    k[5, 0, 0] = np.float32(200.0)          # score = 200/sqrt(8) = 70.7 for key 5, 0 for the others
    pool = build_pool(shape, req, k, v)
    out = orc.prefill_attn(pool, q, req.table, 8, 3, 4)
    for i in range(3):
        np.testing.assert_allclose(out[i, 0], v[5, 0].astype(np.float64), rtol=0, atol=1e-20 + 1e-28)


def test_scale_is_applied_default_and_explicit():
    """Scores scale: doubling D by zero-padding must change the result unless the scale is passed."""
    shape, req, q, k, v = tiny(45, P=8, S=3, D=8, B=4)
    pool = build_pool(shape, req, k, v)
    base = orc.prefill_attn(pool, q, req.table, 8, 3, 4)
    explicit = orc.prefill_attn(pool, q, req.table, 8, 3, 4, scale=np.float32(1 / math.sqrt(8)))
    np.testing.assert_allclose(base, explicit, rtol=0, atol=1e-15)
    other = orc.prefill_attn(pool, q, req.table, 8, 3, 4, scale=np.float32(1.0))
    assert np.abs(other - base).max() > 1e-3
    # scale 0 -> uniform weights -> running mean
    unif = orc.prefill_attn(pool, q, req.table, 8, 3, 4, scale=np.float32(0.0))
    np.testing.assert_allclose(unif[2, 0], v[:11, 0].astype(np.float64).mean(0), atol=1e-14)


def test_nan_in_masked_positions_never_reaches_output():
    B = 4
    shape, req, q, k, v = tiny(51, P=8, S=6, B=B, pool_blocks=16)   # S=6: last block holds 2 of 4 tokens
    pool = build_pool(shape, req, k, v, fill=np.nan)                # unused slots and the block tail are NaN
    out = orc.prefill_attn(pool, q, req.table, 8, 6, B)
    assert np.isfinite(out).all()
    # future tokens: poison tokens after row i and recompute row i only
    for i in range(5):
        k2, v2 = k.copy(), v.copy()
        k2[8 + i + 1:] = np.nan
        v2[8 + i + 1:] = np.nan
        pool2 = build_pool(shape, req, k2, v2, fill=np.nan)
        row = orc.prefill_attn(pool2, q, req.table, 8, 6, B, rows=[i])
        assert np.array_equal(row[0], out[i])


def test_gqa_head_mapping():
    shape, req, q, k, v = tiny(61, P=8, S=4, Hq=4, Hkv=2, D=8, B=4)
    q[:, 1] = q[:, 0]
    q[:, 3] = q[:, 2]
    q[:, 2] = q[:, 0]                         # heads 0,1 use KV head 0; heads 2,3 use KV head 1
    q[:, 3] = q[:, 0]
    pool = build_pool(shape, req, k, v)
    out = orc.prefill_attn(pool, q, req.table, 8, 4, 4)
    assert np.array_equal(out[:, 0], out[:, 1])
    assert np.array_equal(out[:, 2], out[:, 3])
    assert np.abs(out[:, 0] - out[:, 2]).max() > 1e-3
    # swapping the two KV heads swaps the groups' outputs
    pool_sw = build_pool(shape, req, k[:, ::-1], v[:, ::-1])
    out_sw = orc.prefill_attn(pool_sw, q, req.table, 8, 4, 4)
    assert np.array_equal(out_sw[:, 0], out[:, 2])
    assert np.array_equal(out_sw[:, 2], out[:, 0])


def test_rows_and_heads_sampling_matches_full():
    shape, req, q, k, v = tiny(71, P=16, S=9, B=4, pool_blocks=32)
    pool = build_pool(shape, req, k, v)
    full = orc.prefill_attn(pool, q, req.table, 16, 9, 4)
    part = orc.prefill_attn(pool, q, req.table, 16, 9, 4, rows=[0, 3, 8], heads=[1, 2])
    assert np.array_equal(part, full[[0, 3, 8]][:, [1, 2]])


def test_token_gather_equals_block_gather():
    shape, req, q, k, v = tiny(72, P=16, S=7, B=4, pool_blocks=32)
    pool = build_pool(shape, req, k, v)
    for g in range(shape.n_kv_heads):
        for n in (1, 4, 17, 23):
            Ka, Va = orc.gather_kv(pool, req.table, n, g, 4)
            Kb, Vb = orc.gather_kv_blocks(pool, req.table, n, g, 4)
            assert np.array_equal(Ka, Kb) and np.array_equal(Va, Vb)
            assert np.array_equal(Ka, k[:n, g].astype(np.float64))


def test_bf16_widening_is_exact():
    vals = np.array([0.0, -0.0, 1.0, -2.5, 3.140625, 1e-3, 65280.0, np.inf], np.float32)
    bits = wl.f32_to_bf16_bits(vals)
    wide = orc.widen(bits)
    back = torch.tensor(vals).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(wide, back)
    assert np.signbit(wide[1])
    # rounding to nearest even of the generator agrees with the library's conversion
    x = np.random.default_rng(3).standard_normal(4096).astype(np.float32)
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.f32_to_bf16_bits(x), lib)


def test_bf16_storage_path():
    """Same request in bf16 storage: the oracle must equal the fp32-storage oracle fed the rounded values."""
    shape, req, q, k, v = tiny(81, P=16, S=5, B=4, pool_blocks=32)
    def rt(x):
        return orc.widen(wl.f32_to_bf16_bits(x)).astype(np.float32)
    pool32 = build_pool(shape, req, rt(k), rt(v), fill=0.0)
    want = orc.prefill_attn(pool32, rt(q), req.table, 16, 5, 4)
    pool16 = wl.f32_to_bf16_bits(pool32)
    got = orc.prefill_attn(pool16, wl.f32_to_bf16_bits(q), req.table, 16, 5, 4)
    assert np.array_equal(got, want)


def test_batch_is_concatenation_of_requests():
    shape = wl.Shape(1, 4, 2, 8, "f32", 64, block_tokens=4)
    w = wl.make_custom(shape, [(8, 5), (16, 3), (8, 9)], seed=5, shared_blocks=2)
    pool = np.full((64, 2, 4, 2, 8), np.nan, np.float32)
    flat = pool.reshape(1, 64, -1)
    for r in w.requests:
        orc.kv_ingest(flat, w.host_kv, r.table, r.n_prefix_blocks, r.first_ingest_block, r.host_block_start)
    for ri, r in enumerate(w.requests):
        a, b = w.cu_suffix[ri], w.cu_suffix[ri + 1]
        orc.suffix_append(pool, w.k_suffix[0, a:b], w.v_suffix[0, a:b], r.table, r.prefix_len, 4)
    reqs = [(r.table, r.prefix_len, r.suffix_len) for r in w.requests]
    out = orc.prefill_attn_batch(pool, w.q[0], reqs, w.cu_suffix, 4)
    assert np.isfinite(out).all()
    for ri, r in enumerate(w.requests):
        a, b = w.cu_suffix[ri], w.cu_suffix[ri + 1]
        one = orc.prefill_attn(pool, w.q[0, a:b], r.table, r.prefix_len, r.suffix_len, 4)
        assert np.array_equal(out[a:b], one)
    # shared run: request 1's first two blocks are request 0's bytes
    k0, _ = orc.gather_kv(pool, w.requests[0].table, 8, 0, 4)
    k1, _ = orc.gather_kv(pool, w.requests[1].table, 8, 0, 4)
    assert np.array_equal(k0, k1)


def test_matrix_form_equals_row_form():
    shape, req, q, k, v = tiny(91, P=48, S=21, Hq=4, Hkv=2, D=16, B=16, pool_blocks=32)
    pool = build_pool(shape, req, k, v)
    rows = [0, 1, 7, 15, 16, 20]
    a = orc.prefill_attn(pool, q, req.table, 48, 21, 16, rows=rows)
    b = orc.prefill_attn_sampled(pool, q, req.table, 48, 21, 16, rows)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-14)
    # and against the brute-force loops directly
    want = brute_force(q, k, v, 48, float(np.float32(1.0) / np.sqrt(np.float32(16))))
    np.testing.assert_allclose(b, want[rows], rtol=0, atol=1e-13)
