"""Seeded synthetic inputs for the prefix-hit prefill path.

This module only draws shapes, block tables and random tensor values.  It holds
none of the method's arithmetic (no scatter, no attention, no softmax): both the
HIP path and the CPU oracle are fed from here and neither imports the other.

A request is a reusable context whose KVCache blocks already exist plus a query
that still has to be computed (paper, Section 2.2, "long context, short
query").  The paper never states a block size, a precision or a memory layout;
the values used here (16-token blocks, bf16 or fp32 elements, block layout
[K|V][token][kv_head][dim]) are this build's reading and are the single place
where they are written down for the input side.

The five workload recipes follow the model shapes the paper serves
(Llama-3.1-8B class, Section 4.1) and its context/query length regime
(Table 1: contexts of 28K-38K tokens, short queries); values are i.i.d. N(0,1)
because the paper's datasets and trained weights are not available.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

BASE_SEED = 260321257
BLOCK_TOKENS = 16


@dataclass(frozen=True)
class Shape:
    """Static attention-stack shape.  dtype is 'bf16' or 'f32'."""
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str
    pool_blocks: int
    block_tokens: int = BLOCK_TOKENS

    @property
    def elt_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def tok_bytes(self) -> int:
        """Bytes of K and V of one token in one layer."""
        return 2 * self.n_kv_heads * self.head_dim * self.elt_bytes

    @property
    def blk_bytes(self) -> int:
        """Bytes of one KVCache block in one layer."""
        return self.block_tokens * self.tok_bytes

    @property
    def blk_elems(self) -> int:
        return self.blk_bytes // self.elt_bytes

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


@dataclass
class Request:
    """One request: P cached-prefix tokens (whole blocks) and S suffix tokens.

    table holds P/B prefix slot ids followed by ceil(S/B) suffix slot ids.
    host_block_start is the index, inside the batch's shared host buffer, that
    this request's block 0 maps to; blocks below first_ingest_block are already
    resident in the pool (a shared run) and are never read from the host.
    """
    prefix_len: int
    suffix_len: int
    table: np.ndarray
    first_ingest_block: int = 0
    host_block_start: int = 0
    block_tokens: int = BLOCK_TOKENS

    @property
    def n_prefix_blocks(self) -> int:
        return self.prefix_len // self.block_tokens

    @property
    def n_suffix_blocks(self) -> int:
        return -(-self.suffix_len // self.block_tokens)


@dataclass
class Workload:
    name: str
    shape: Shape
    requests: List[Request]
    host_blocks: int                      # blocks per layer in the host buffer
    seed: int
    # numpy payloads (small workloads only; large ones are filled by fill_normal_)
    host_kv: Optional[np.ndarray] = None  # [L, host_blocks, blk_elems] stored dtype
    q: Optional[np.ndarray] = None        # [L, sumS, Hq, D]
    k_suffix: Optional[np.ndarray] = None  # [L, sumS, Hkv, D]
    v_suffix: Optional[np.ndarray] = None
    cu_suffix: np.ndarray = field(default_factory=lambda: np.zeros(1, np.int32))

    @property
    def total_suffix(self) -> int:
        return int(self.cu_suffix[-1])

    def ingest_bytes(self) -> int:
        """Unique bytes that cross from host to pool over all layers."""
        blocks = sum(r.n_prefix_blocks - r.first_ingest_block for r in self.requests)
        return blocks * self.shape.blk_bytes * self.shape.n_layers

    def attn_pairs(self) -> int:
        """Unmasked (query, key) pairs per head per layer."""
        return sum(r.suffix_len * r.prefix_len + r.suffix_len * (r.suffix_len + 1) // 2
                   for r in self.requests)

    def attn_flop(self) -> int:
        """4*D*Hq*pairs per layer, times layers (QK^T and PV, 2 flop per MAC)."""
        s = self.shape
        return 4 * s.head_dim * s.n_q_heads * self.attn_pairs() * s.n_layers


# --------------------------------------------------------------------------
# value generators
# --------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest even) and return the 16-bit patterns."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def normal_values(rng: np.random.Generator, shape, dtype: str) -> np.ndarray:
    """N(0,1) values stored as fp32, or as bf16 bit patterns in a uint16 array."""
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def child_rng(seed: int, *key: int) -> np.random.Generator:
    """Independent stream per (workload, tensor) key."""
    return np.random.default_rng(np.random.SeedSequence([seed, *key]))


def fill_normal_(dst, seed: int, chunk_elems: int = 1 << 26):
    """Fill a torch tensor (any device, bf16 or fp32, contiguous) with N(0,1).

    Used for the multi-GiB buffers: values are drawn on dst's own device when it
    is a GPU tensor, otherwise on the GPU (if any) and copied over, chunk by
    chunk, so a pinned host buffer is filled at PCIe speed instead of at the
    speed of a host generator.  The oracle reads the bytes that end up in the
    buffer, so any fixed fill is a valid input.
    """
    import torch

    flat = dst.view(-1)
    n = flat.numel()
    dev = dst.device if dst.is_cuda else (torch.device("cuda:0") if torch.cuda.is_available()
                                          else torch.device("cpu"))
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    for off in range(0, n, chunk_elems):
        m = min(chunk_elems, n - off)
        x = torch.randn(m, generator=gen, device=dev, dtype=torch.float32).to(dst.dtype)
        flat[off:off + m].copy_(x)
    if dev.type == "cuda":
        torch.cuda.synchronize()
    return dst


# --------------------------------------------------------------------------
# request / table draws
# --------------------------------------------------------------------------

def single_request(shape: Shape, prefix_len: int, suffix_len: int, seed: int) -> List[Request]:
    assert prefix_len % shape.block_tokens == 0
    nblk = prefix_len // shape.block_tokens + -(-suffix_len // shape.block_tokens)
    assert nblk <= shape.pool_blocks
    rng = child_rng(seed, 1)
    table = rng.permutation(shape.pool_blocks)[:nblk].astype(np.int32)
    return [Request(prefix_len, suffix_len, table, block_tokens=shape.block_tokens)]


def varlen_batch(shape: Shape, seed: int, n_req: int = 8, lo: int = 8192, hi: int = 32768,
                 shared_tokens: int = 4096) -> List[Request]:
    """Batch of requests that share one common prefix run of whole blocks.

    total length uniform in [lo, hi], hit ratio uniform in [0.5, 0.95]; the
    first shared_tokens/B entries of every table are the same slots and only
    request 0 ingests them.
    """
    B = shape.block_tokens
    rng = child_rng(seed, 4)
    totals = rng.integers(lo, hi, size=n_req, endpoint=True)
    hits = rng.uniform(0.5, 0.95, size=n_req)
    shared_blocks = shared_tokens // B
    plen = [max(shared_tokens, int(t * h) // B * B) for t, h in zip(totals, hits)]
    slen = [int(t) - p for t, p in zip(totals, plen)]
    need = shared_blocks + sum(p // B - shared_blocks + -(-s // B) for p, s in zip(plen, slen))
    assert need <= shape.pool_blocks
    slots = rng.permutation(shape.pool_blocks)[:need].astype(np.int32)
    shared = slots[:shared_blocks]
    cur = shared_blocks
    host_cur = 0
    reqs = []
    for r in range(n_req):
        own = plen[r] // B - shared_blocks + -(-slen[r] // B)
        table = np.concatenate([shared, slots[cur:cur + own]]).astype(np.int32)
        cur += own
        first = 0 if r == 0 else shared_blocks
        # request r's block j lives at host block host_block_start + j
        start = host_cur - first
        reqs.append(Request(plen[r], slen[r], table, first, start, B))
        host_cur += plen[r] // B - first
    return reqs


CONFIG_NAMES = {
    1: "cfg1: 1 layer, 8Q/2KV heads, D=64, fp32, P=1024, S=128, pool 256",
    2: "cfg2: Llama-3-8B-shaped stack, 32 layers, 32Q/8KV, D=128, bf16, P=16384, S=2048",
    3: "cfg3: Llama-3-8B-shaped stack, 32 layers, 32Q/8KV, D=128, bf16, P=61440, S=4096 (64K ctx)",
    4: "cfg4: same shape, 8 varlen requests sharing a 4096-token run, pool 40000",
    5: "cfg5: Qwen2.5-72B-shaped stack, 80 layers, 64Q/8KV, D=128, bf16, P=122880, S=8192",
    6: "cfg6: Qwen2.5-14B-shaped stack, 48 layers, 40Q/8KV (group of 5), D=128, bf16, P=61440, S=4096",
    7: "cfg7: Llama-3-8B-shaped stack, 3 requests with the mean context/query lengths of the paper's Table 1 "
       "(28096+28, 28304+61, 38304+209)",
}

# Mean (context, query) token counts of the three datasets in the paper's Table 1, contexts
# rounded down to whole 16-token blocks: long context, short query.
TABLE1_MEAN_LENGTHS = [(28096, 28), (28304, 61), (38304, 209)]


def config_shape_and_requests(cfg: int, seed: int = BASE_SEED, n_layers: Optional[int] = None):
    """Shapes, tables and lengths of one of the workload recipes (no payload)."""
    if cfg == 1:
        shape = Shape(1, 8, 2, 64, "f32", 256)
        reqs = single_request(shape, 1024, 128, seed)
    elif cfg in (2, 3):
        P, S = (16384, 2048) if cfg == 2 else (61440, 4096)
        need = (P + S) // BLOCK_TOKENS
        shape = Shape(n_layers or 32, 32, 8, 128, "bf16", need * 5 // 4)
        reqs = single_request(shape, P, S, seed)
    elif cfg == 4:
        shape = Shape(n_layers or 32, 32, 8, 128, "bf16", 40000)
        reqs = varlen_batch(shape, seed)
    elif cfg == 5:
        P, S = 122880, 8192
        need = (P + S) // BLOCK_TOKENS
        shape = Shape(n_layers or 80, 64, 8, 128, "bf16", need * 5 // 4)
        reqs = single_request(shape, P, S, seed)
    elif cfg == 6:
        # second model family of the paper's evaluation (Section 4.1): 48 layers, 40 query heads in
        # 8 KV groups of 5 - a group size the 4-heads-per-workgroup tiling does not divide
        P, S = 61440, 4096
        need = (P + S) // BLOCK_TOKENS
        shape = Shape(n_layers or 48, 40, 8, 128, "bf16", need * 5 // 4)
        reqs = single_request(shape, P, S, seed)
    elif cfg == 7:
        need = sum(p // BLOCK_TOKENS + -(-q // BLOCK_TOKENS) for p, q in TABLE1_MEAN_LENGTHS)
        shape = Shape(n_layers or 32, 32, 8, 128, "bf16", need * 5 // 4)
        return shape, make_custom(shape, TABLE1_MEAN_LENGTHS, seed, with_payload=False).requests
    else:
        raise ValueError(f"unknown config {cfg}")
    return shape, reqs


def _finish(name, shape, reqs, seed, with_payload) -> Workload:
    host_blocks = sum(r.n_prefix_blocks - r.first_ingest_block for r in reqs)
    cu = np.zeros(len(reqs) + 1, np.int32)
    cu[1:] = np.cumsum([r.suffix_len for r in reqs])
    w = Workload(name, shape, reqs, host_blocks, seed, cu_suffix=cu)
    if with_payload:
        L, T = shape.n_layers, int(cu[-1])
        w.host_kv = normal_values(child_rng(seed, 10), (L, host_blocks, shape.blk_elems), shape.dtype)
        w.q = normal_values(child_rng(seed, 11), (L, T, shape.n_q_heads, shape.head_dim), shape.dtype)
        w.k_suffix = normal_values(child_rng(seed, 12), (L, T, shape.n_kv_heads, shape.head_dim), shape.dtype)
        w.v_suffix = normal_values(child_rng(seed, 13), (L, T, shape.n_kv_heads, shape.head_dim), shape.dtype)
    return w


def make_config(cfg: int, seed: int = BASE_SEED, n_layers: Optional[int] = None,
                with_payload: Optional[bool] = None) -> Workload:
    """Workload recipe cfg (1..7).  Payload arrays are drawn with numpy only when
    asked for (default: config 1 only); large payloads are produced with
    fill_normal_ into buffers the caller allocates."""
    shape, reqs = config_shape_and_requests(cfg, seed, n_layers)
    if with_payload is None:
        with_payload = cfg == 1
    return _finish(CONFIG_NAMES[cfg], shape, reqs, seed, with_payload)


def make_custom(shape: Shape, lengths, seed: int, shared_blocks: int = 0, with_payload: bool = True) -> Workload:
    """Test workload: lengths is a list of (prefix_len, suffix_len).  with_payload=False leaves the
    value arrays out (large cases fill caller-allocated buffers with fill_normal_).

    shared_blocks > 0 makes every request's first shared_blocks table entries the
    same slots (ingested by request 0 only), as in the varlen batch recipe.
    """
    B = shape.block_tokens
    rng = child_rng(seed, 2)
    need = shared_blocks + sum(p // B - shared_blocks + -(-s // B) for p, s in lengths)
    assert need <= shape.pool_blocks, (need, shape.pool_blocks)
    slots = rng.permutation(shape.pool_blocks)[:need].astype(np.int32)
    shared = slots[:shared_blocks]
    cur, host_cur, reqs = shared_blocks, 0, []
    for r, (p, s) in enumerate(lengths):
        assert p % B == 0 and p // B >= shared_blocks
        own = p // B - shared_blocks + -(-s // B)
        table = np.concatenate([shared, slots[cur:cur + own]]).astype(np.int32)
        cur += own
        first = 0 if r == 0 else shared_blocks
        reqs.append(Request(p, s, table, first, host_cur - first, B))
        host_cur += p // B - first
    return _finish("custom", shape, reqs, seed, with_payload)
