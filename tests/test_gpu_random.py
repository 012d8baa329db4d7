"""Seeded random batches through the whole HIP path against the CPU oracle: head layouts,
request counts, prefix / suffix lengths (empty, one token, ragged, partial last block),
staging sizes, chunk-granular loading, the softmax scale, the attention kernel and forced context splits drawn at random.  Every case is valid input; pool
bytes must be bit exact and attention within the bf16 tolerance."""
import numpy as np
import pytest

import hip_harness as hh
from paper_2603_21257_amd import workload as wl

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    hkv = int(rng.choice([1, 2, 4]))
    group = int(rng.choice([1, 2, 4, 8]))
    n_layers = int(rng.integers(1, 4))
    n_reqs = int(rng.integers(1, 5))
    shared = int(rng.choice([0, 0, 2, 6]))
    lens = []
    for _ in range(n_reqs):
        kind = rng.integers(0, 5)
        p_blocks = int(rng.integers(shared, 161)) if kind else shared            # kind 0: no prefix beyond the shared run
        s_len = int(rng.choice([0, 1, 15, 16, 17, 33])) if kind == 1 else int(rng.integers(1, 261))
        lens.append((16 * p_blocks, s_len))
    if all(s == 0 for _, s in lens):
        lens[0] = (lens[0][0], 40)
    need = sum(p // 16 + -(-s // 16) for p, s in lens) - shared * (n_reqs - 1)
    shape = wl.Shape(n_layers, hkv * group, hkv, 128, "bf16", int(need * 1.3) + 8)
    kw = {}
    if rng.integers(0, 2):
        kw["staging_bytes"] = int(rng.integers(1, 40)) * shape.blk_bytes
        kw["n_staging"] = int(rng.choice([2, 3]))
    if rng.integers(0, 2):
        kw["chunk_blocks"] = [int(2 * rng.integers(0, 17)) for _ in range(n_layers)]     # 0 = that layer as a whole
    if rng.integers(0, 3) == 0:
        kw["scale"] = float(rng.choice([0.03, 0.2]))                 # explicit softmax scale instead of 1 / sqrt(D)
    env = {}
    pick = int(rng.integers(0, 4))
    if pick == 1:
        env["CALVO_ATTN_VARIANT"] = str(rng.choice([3, 4]))          # one of the two pipelined kernels, whatever the lengths
    elif pick == 2:
        env["CALVO_ATTN_SPLITS"] = str(rng.choice([2, 3, 7]))        # every tile's context cut into pieces
    return shape, lens, shared, kw, env


@pytest.mark.parametrize("seed", range(32))
def test_random_batch(seed, monkeypatch):
    shape, lens, shared, kw, env = draw_case(seed)
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    w = wl.make_custom(shape, lens, seed=9000 + seed, shared_blocks=shared)
    print(f"[case] seed={seed} shape={shape} lens={lens} shared={shared} kw={kw} env={env}", flush=True)
    pool_g, out_g = hh.run_hip(w, **kw)
    pool_o, out_o = hh.run_oracle(w, scale=kw.get("scale"))
    hh.assert_pool_bit_exact(pool_g, pool_o)
    hh.assert_attn_close(out_g, out_o, "bf16")
