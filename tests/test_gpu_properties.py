"""Two properties the paper reports for its system, checked on this path (no oracle involved: they are
statements about time, not about values).

* Loading time is a linear function of the number of context tokens (paper Fig. 6, the premise of
  the binary linear cost model of Section 3.2).
* With the total length fixed, TTFT falls as the cache hit ratio rises (paper Fig. 11; hit ratios
  25-100 % as in Section 4.3) - true whenever loading a token's KV is cheaper than recomputing it.
"""
import time

import numpy as np
import pytest
import torch

from paper_2603_21257_amd import binding as cb
from paper_2603_21257_amd import hostmem
from paper_2603_21257_amd import workload as wl

pytestmark = pytest.mark.gpu

L, HQ, HKV, D = 8, 32, 8, 128


class Stack:
    """An 8-layer Llama-3-8B-shaped attention stack with room for a 32K-token request."""

    def __init__(self, max_tokens=32768 + 64):
        self.shape = wl.Shape(L, HQ, HKV, D, "bf16", max_tokens // 16 + 8)
        s = self.shape
        dev = torch.device("cuda:0")
        self.arena = hostmem.PinnedBuffer(L * (max_tokens // 16) * s.blk_bytes)
        self.host = self.arena.tensor((L, max_tokens // 16, s.blk_elems), torch.bfloat16)
        wl.fill_normal_(self.host, 5)
        self.pool = torch.empty((L, s.pool_blocks, s.blk_elems), dtype=torch.bfloat16, device=dev)
        self.q = wl.fill_normal_(torch.empty((L, max_tokens, HQ, D), dtype=torch.bfloat16, device=dev), 6)
        self.kv = wl.fill_normal_(torch.empty((2, L, max_tokens, HKV, D), dtype=torch.bfloat16, device=dev), 7)
        self.out = torch.empty((L, max_tokens, HQ, D), dtype=torch.bfloat16, device=dev)
        self.ctx = cb.calvo_create(L, HQ, HKV, D, cb.CALVO_BF16, s.pool_blocks, self.pool, staging_bytes=128 << 20)
        self.stride = (max_tokens // 16) * s.blk_bytes
        self.table = np.random.default_rng(3).permutation(s.pool_blocks).astype(np.int32)

    def close(self):
        cb.calvo_destroy(self.ctx)
        self.arena.free()

    def request(self, P, S):
        return cb.make_request(self.host, self.stride, self.table[:P // 16 + -(-S // 16)], P // 16, S)

    def load_s(self, P):
        req = self.request(P, 0)
        best = 1e9
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            cb.calvo_kv_ingest(self.ctx, [req], 0, L)
            cb.calvo_layer_event(self.ctx, L - 1, cb.CALVO_EV_HOST_WAIT)
            best = min(best, time.perf_counter() - t0)
        return best

    def ttft_s(self, P, S):
        req = self.request(P, S)
        cu = np.array([0, S], np.int32)
        best = 1e9
        for _ in range(3):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            cb.calvo_kv_ingest(self.ctx, [req], 0, L)
            for l in range(L):
                cb.calvo_prefill_attn(self.ctx, l, self.q[l, :S], self.kv[0, l, :S], self.kv[1, l, :S], self.out[l, :S],
                                      [req], cu, 0.0)
            torch.cuda.synchronize()
            best = min(best, time.perf_counter() - t0)
        return best


@pytest.fixture(scope="module")
def stack():
    s = Stack()
    yield s
    s.close()


@pytest.mark.timing
def test_loading_time_is_linear_in_the_context_tokens(stack):
    tokens = [2048, 4096, 8192, 12288, 16384, 24576, 32768]
    secs = [stack.load_s(p) for p in tokens]
    per_token, fixed = cb.calvo_cost_fit(tokens, secs)
    pred = np.array(tokens) * per_token + fixed
    ss_res = float(np.sum((np.array(secs) - pred) ** 2))
    ss_tot = float(np.sum((np.array(secs) - np.mean(secs)) ** 2))
    r2 = 1.0 - ss_res / ss_tot
    rate = L * stack.shape.tok_bytes / per_token / 1e9
    print(f"load seconds {['%.4f' % x for x in secs]} -> {per_token * 1e9:.2f} ns/token + {fixed * 1e6:.0f} us, "
          f"R^2 {r2:.5f}, slope = {rate:.1f} GB/s", flush=True)
    assert r2 > 0.995
    assert 15.0 < rate < 80.0            # the slope is the link rate: PCIe Gen5 x16 (55-57 GB/s measured; wide margins for another box)
    assert fixed < 0.5 * secs[0]         # and the fixed part is small next to even the shortest load


@pytest.mark.timing
def test_ttft_falls_as_the_hit_ratio_rises(stack):
    total = 32768
    ratios = [0.25, 0.5, 0.75, 0.95, 0.998]
    ttft = []
    for r in ratios:
        P = int(total * r) // 16 * 16
        ttft.append(stack.ttft_s(P, total - P))
    print("hit ratio -> TTFT ms: " + ", ".join(f"{r:.3f}: {t * 1e3:.2f}" for r, t in zip(ratios, ttft)), flush=True)
    # Asserted up to 95 %: there the step has become load bound on this path, which recomputes attention
    # only (not the rest of the model forward), and the last 5 % of hits add bytes to load without taking
    # a matching amount of compute away; the 99.8 % point is printed, not asserted.
    for a, b in zip(ttft[:4], ttft[1:4]):
        assert b < a
    assert ttft[3] < 0.5 * ttft[0]
