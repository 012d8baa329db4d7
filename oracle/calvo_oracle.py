"""CPU oracle for the prefix-hit prefill path.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this file.  It shares no code with the HIP library and is deliberately plain
and slow: numpy, fp64, one query row and one head at a time, no blocking, no
fusion, no reordering.

What it defines
---------------
kv_ingest       The L2->L1 loading stage of the paper (Section 3.1: a block is
                moved once its source is ready and its destination space is
                allocated).  A KVCache block is moved as raw bytes from the
                host staging area to the pool slot its block table names.  The
                result has a plain definition (a permutation of 64-KiB byte
                strings), so the oracle is that definition.
suffix_append   The prefill step builds the KVCache of the prompt (Section 2.1): the
                K/V of the tokens that are computed, not loaded, are written
                to the request's remaining slots.  Plain definition again.
prefill_attn    Causal attention of the query (suffix) tokens over the reused
                prefix plus the suffix itself (Section 2.1 prefill; Section 2.1 on
                prefix caching: cached KV is reused as it is).  The paper
                inherits this operation from its serving engine and prints no
                formula; the textbook definition is used: for row i at absolute
                position p = P + i and query head h,
                    s_t = scale * <q[i,h,:], K[t,g,:]>,  t = 0..p,  g = h // (Hq/Hkv)
                    O[i,h,:] = sum_t softmax(s)_t * V[t,g,:].

Readings taken where the paper is silent: 16-token blocks; softmax scale
1/sqrt(D) given as an fp32 number; causal mask aligned to the end of the
sequence (row i sees keys 0..P+i inclusive); contiguous GQA groups; no
positional encoding inside the operation; block layout [K|V][token][kv_head][dim];
tokens stored after position P+S-1 in the last slot are undefined and never read.

Pins (tests/test_oracle_*.py): brute-force contiguous triple loop, the float64
scaled_dot_product_attention routine of a library with an explicit mask,
block-table permutation invariance, prefix-hit == full recomputation, convex
combination bounds, closed forms (zero keys -> running mean, constant values,
single key, dominant key), NaN planted in every masked position, GQA head
mapping, byte accounting against the KV footprint the paper prints
(Section 2.2: Llama-3.1-8B, 10 M tokens, more than 1 TB).
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------
# element handling
# --------------------------------------------------------------------------

def widen(stored: np.ndarray) -> np.ndarray:
    """Stored element values, exactly, as fp64.

    fp32 arrays widen directly.  bf16 is carried as uint16 bit patterns: a bf16
    number is the fp32 number with the same upper 16 bits and zero lower bits.
    """
    if stored.dtype == np.float32 or stored.dtype == np.float64:
        return stored.astype(np.float64)
    if stored.dtype == np.uint16:
        return (stored.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    raise TypeError(f"unsupported stored dtype {stored.dtype}")


# --------------------------------------------------------------------------
# ingest (bytes)
# --------------------------------------------------------------------------

def kv_ingest(pool: np.ndarray, host_kv: np.ndarray, table, n_prefix_blocks: int,
              first_ingest_block: int = 0, host_block_start: int = 0,
              layer_begin: int = 0, layer_end=None) -> int:
    """pool[l][table[j]] <- host_kv[l][host_block_start + j] for the prefix blocks
    j in [first_ingest_block, n_prefix_blocks) and layers in [layer_begin, layer_end).

    pool is [L][pool_blocks][block bytes or elements], host_kv is
    [L][host_blocks][same]; both are modified / read as they are (a byte move:
    NaN payloads and negative zeros survive).  Returns the bytes moved.
    """
    L = pool.shape[0]
    if layer_end is None:
        layer_end = L
    assert pool.dtype == host_kv.dtype and pool.shape[2:] == host_kv.shape[2:]
    moved = 0
    for l in range(layer_begin, layer_end):
        for j in range(first_ingest_block, n_prefix_blocks):
            slot = int(table[j])
            assert 0 <= slot < pool.shape[1], "destination slot is not allocated"
            pool[l, slot] = host_kv[l, host_block_start + j]
            moved += pool[l, slot].nbytes
    return moved


def suffix_append(pool_layer: np.ndarray, k_suffix: np.ndarray, v_suffix: np.ndarray,
                  table, prefix_len: int, block_tokens: int) -> None:
    """Write the suffix tokens' K and V into their slots of one layer.

    pool_layer is [pool_blocks][2][B][Hkv][D]; k_suffix, v_suffix are [S][Hkv][D].
    Token i of the suffix sits at absolute position prefix_len + i.
    """
    S = k_suffix.shape[0]
    for i in range(S):
        t = prefix_len + i
        slot = int(table[t // block_tokens])
        pool_layer[slot, 0, t % block_tokens] = k_suffix[i]
        pool_layer[slot, 1, t % block_tokens] = v_suffix[i]


# --------------------------------------------------------------------------
# attention
# --------------------------------------------------------------------------

def gather_kv(pool_layer: np.ndarray, table, n_tokens: int, kv_head: int, block_tokens: int):
    """K[t], V[t] for t in [0, n_tokens) of one KV head, through the block table, in fp64."""
    D = pool_layer.shape[-1]
    K = np.empty((n_tokens, D), np.float64)
    V = np.empty((n_tokens, D), np.float64)
    for t in range(n_tokens):
        slot = int(table[t // block_tokens])
        K[t] = widen(pool_layer[slot, 0, t % block_tokens, kv_head])
        V[t] = widen(pool_layer[slot, 1, t % block_tokens, kv_head])
    return K, V


def gather_kv_blocks(pool_layer: np.ndarray, table, n_tokens: int, kv_head: int, block_tokens: int):
    """Same result as gather_kv, taking one block per step instead of one token
    (used for long contexts; checked against gather_kv in the tests)."""
    nblk = -(-n_tokens // block_tokens)
    slots = np.asarray(table[:nblk], dtype=np.int64)
    K = widen(pool_layer[slots, 0, :, kv_head, :]).reshape(nblk * block_tokens, -1)[:n_tokens]
    V = widen(pool_layer[slots, 1, :, kv_head, :]).reshape(nblk * block_tokens, -1)[:n_tokens]
    return K, V


def attn_row(q_row: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """softmax(scale * K q) V for one query row over the keys it may see (all rows of K)."""
    s = scale * (K @ q_row)
    m = np.max(s)
    w = np.exp(s - m)
    return (w @ V) / np.sum(w)


def prefill_attn(pool_layer: np.ndarray, q: np.ndarray, table, prefix_len: int, suffix_len: int,
                 block_tokens: int, scale=None, rows=None, heads=None) -> np.ndarray:
    """Attention output of one request in one layer, fp64.

    pool_layer [pool_blocks][2][B][Hkv][D] must already hold the prefix AND the
    suffix K/V (see suffix_append).  q is [S][Hq][D] (stored dtype).  rows /
    heads restrict the computation to a sample (default: everything).  Returns
    [len(rows)][len(heads)][D].
    """
    S, Hq, D = q.shape
    assert S == suffix_len
    Hkv = pool_layer.shape[3]
    assert Hq % Hkv == 0
    G = Hq // Hkv
    if scale is None:
        scale = np.float32(1.0) / np.sqrt(np.float32(D))
    scale = float(np.float32(scale))          # the fp32 number the kernel is handed, as fp64
    rows = list(range(S)) if rows is None else [int(r) for r in rows]
    heads = list(range(Hq)) if heads is None else [int(h) for h in heads]
    out = np.zeros((len(rows), len(heads), D), np.float64)
    if not rows:
        return out
    n_max = prefix_len + max(rows) + 1
    qf = widen(q)
    for g in sorted({h // G for h in heads}):
        K, V = gather_kv_blocks(pool_layer, table, n_max, g, block_tokens)
        for hi, h in enumerate(heads):
            if h // G != g:
                continue
            for ri, i in enumerate(rows):
                n = prefix_len + i + 1            # keys 0 .. P+i inclusive
                out[ri, hi] = attn_row(qf[i, h], K[:n], V[:n], scale)
    return out


def attn_rows(q_rows: np.ndarray, K: np.ndarray, V: np.ndarray, n_visible, scale: float) -> np.ndarray:
    """The same definition for several query rows of one head at once, in matrix form:
    scores = scale * Q K^T, keys at index >= n_visible[r] are excluded from row r, softmax
    along keys, times V.  q_rows is [R][D] fp64, n_visible[r] = P + i_r + 1.  No running
    maximum, no tiling: every row's full score vector is formed."""
    n_visible = np.asarray(n_visible, dtype=np.int64)
    n_max = int(n_visible.max())
    s = scale * (q_rows @ K[:n_max].T)                        # [R][n_max]
    hidden = np.arange(n_max)[None, :] >= n_visible[:, None]
    s[hidden] = -np.inf
    w = np.exp(s - s.max(axis=1, keepdims=True))
    return (w @ V[:n_max]) / w.sum(axis=1, keepdims=True)


def prefill_attn_sampled(pool_layer: np.ndarray, q: np.ndarray, table, prefix_len: int, suffix_len: int,
                         block_tokens: int, rows, scale=None) -> np.ndarray:
    """prefill_attn restricted to the suffix rows in `rows`, all heads, using attn_rows
    (one matrix product per head).  Meant for long contexts where only a sample of the
    output rows is checked.  Returns [len(rows)][Hq][D]."""
    S, Hq, D = q.shape
    assert S == suffix_len
    Hkv = pool_layer.shape[3]
    G = Hq // Hkv
    if scale is None:
        scale = np.float32(1.0) / np.sqrt(np.float32(D))
    scale = float(np.float32(scale))
    rows = np.asarray([int(r) for r in rows], dtype=np.int64)
    out = np.zeros((len(rows), Hq, D), np.float64)
    n_vis = prefix_len + rows + 1
    qf = widen(q[rows])
    for g in range(Hkv):
        K, V = gather_kv_blocks(pool_layer, table, int(n_vis.max()), g, block_tokens)
        for h in range(g * G, (g + 1) * G):
            out[:, h] = attn_rows(qf[:, h], K, V, n_vis, scale)
    return out


def prefill_attn_batch(pool_layer, q, requests, cu_suffix, block_tokens, scale=None):
    """All requests of a batch; q is [sum S][Hq][D], requests is a list of
    (table, prefix_len, suffix_len).  Returns [sum S][Hq][D] fp64."""
    out = np.zeros(q.shape, np.float64)
    for r, (table, P, S) in enumerate(requests):
        a, b = int(cu_suffix[r]), int(cu_suffix[r + 1])
        assert b - a == S
        out[a:b] = prefill_attn(pool_layer, q[a:b], table, P, S, block_tokens, scale)
    return out
