"""Host-side planning of an attention launch (calvo_attn_plan): which kernel, how many split-KV pieces.
Runs without a GPU.  The expectations are properties of the plan, not of any timing: pieces cover a tile
and are never shorter than 48 sub-tiles, nothing is cut when the chip is full anyway, short suffixes get
the small-tile kernel, and a launch just above a whole number of rounds is cut."""
import numpy as np
import pytest

from paper_2603_21257_amd import binding as cb

CUS = 256


def plan(hq, hkv, lens, cus=CUS, monkeypatch=None):
    pb = [p // 16 for p, _ in lens]
    sl = [s for _, s in lens]
    return cb.calvo_attn_plan(hq, hkv, cus, pb, sl)


def test_long_suffix_fills_the_chip_and_is_not_cut():
    r = plan(32, 8, [(61440, 4096)])                      # 64 tiles x 8 head groups = 2 rounds of 256
    assert r == {"kernel": 3, "tile_tokens": 64, "pieces": 1, "workgroups": 512}
    r = plan(64, 8, [(122880, 8192)])                     # 8 rounds
    assert r["kernel"] == 3 and r["pieces"] == 1 and r["workgroups"] == 128 * 16


def test_short_suffix_gets_small_tiles_and_pieces():
    """The paper's Table 1 lengths: 28, 61, 209 query tokens over 28K-38K cached tokens."""
    r = plan(32, 8, [(28096, 28), (28304, 61), (38304, 209)])
    assert r["kernel"] == 4 and r["tile_tokens"] == 32
    assert r["pieces"] > 1
    tiles = 1 + 2 + 7
    assert tiles * 8 < r["workgroups"] <= tiles * 8 * r["pieces"]
    # pieces are never shorter than 48 sub-tiles: at most n_sub / 48 per tile
    assert r["workgroups"] <= 8 * sum(((p + min((t + 1) * 32, s) + 31) // 32) // 48
                                      for p, s in [(28096, 28), (28304, 61), (38304, 209)] for t in range(-(-s // 32)))


def test_single_token_and_single_tile():
    r = plan(32, 8, [(32768, 1)])
    assert r["kernel"] == 4 and r["pieces"] > 1 and r["workgroups"] > 8
    r = plan(32, 8, [(0, 64)])                            # nothing to cut: 2 sub-tiles
    assert r["pieces"] == 1 or r["workgroups"] == 8


def test_group_of_five_is_cut_to_fill_the_last_round():
    """40 query heads in 8 KV groups: one head per workgroup, 256-token tiles, 16 x 40 = 640 equal
    workgroups = 2.5 rounds on 256 CUs; cut in two they run as 5 half-length rounds."""
    r = plan(40, 8, [(61440, 4096)])
    assert r["kernel"] == 3 and r["tile_tokens"] == 256
    assert r["pieces"] == 2 and r["workgroups"] == 1280
    # on a device with 320 CUs the 640 workgroups are exactly two rounds: no cut
    assert plan(40, 8, [(61440, 4096)], cus=320)["pieces"] == 1


def test_plan_is_monotone_in_device_size_for_tiny_batches():
    small = plan(32, 8, [(65536, 16)], cus=64)
    big = plan(32, 8, [(65536, 16)], cus=256)
    assert big["workgroups"] >= small["workgroups"]


def test_no_requests_and_bad_arguments():
    assert cb.calvo_attn_plan(32, 8, CUS, [], [])["workgroups"] == 0
    for args in [(32, 5, CUS, [1], [1]), (0, 8, CUS, [1], [1]), (32, 8, 0, [1], [1]), (32, 8, CUS, [-1], [1]),
                 (32, 8, CUS, [1], [-4])]:
        with pytest.raises(cb.CalvoError):
            cb.calvo_attn_plan(*args)
    with pytest.raises(ValueError):
        cb.calvo_attn_plan(32, 8, CUS, [1, 2], [1])


def test_random_batches_give_consistent_plans():
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(1, 9))
        lens = [(int(rng.integers(0, 4096)) * 16, int(rng.integers(0, 3000))) for _ in range(n)]
        hq, hkv = [(32, 8), (40, 8), (8, 8), (16, 8), (64, 8)][int(rng.integers(0, 5))]
        r = plan(hq, hkv, lens)
        hw = 4 if (hq // hkv) % 4 == 0 else 2 if (hq // hkv) % 2 == 0 else 1
        assert r["kernel"] in (3, 4) and r["tile_tokens"] == 32 * ((8 if r["kernel"] == 3 else 4) // hw)
        tiles = sum(-(-s // r["tile_tokens"]) for _, s in lens)
        assert 1 <= r["pieces"] <= 64
        assert tiles * (hq // hw) <= r["workgroups"] <= tiles * (hq // hw) * r["pieces"]


def _random_batch(rng):
    n = int(rng.integers(1, 6))
    lens = []
    for _ in range(n):
        p_blocks = int(rng.integers(0, 2500))
        s = int(rng.choice([0, 1, 31, 32, 33, 64, 100])) if rng.integers(0, 3) == 0 else int(rng.integers(1, 3000))
        lens.append((p_blocks, s))
    if all(s == 0 for _, s in lens):
        lens[0] = (lens[0][0], 17)
    return lens


def _check_partition(items, lens, tile_tokens):
    """Every tile of every request appears once; its pieces follow each other, agree on their count and
    partition [0, n_sub) with n_sub = ceil(keys the tile's last row sees / 32)."""
    seen = {}
    i = 0
    while i < len(items):
        req, tile, b, e, n, _ = items[i]
        assert (req, tile) not in seen and n >= 1
        p_blocks, s = lens[req]
        assert 0 <= tile < -(-s // tile_tokens)
        n_sub = -(-(16 * p_blocks + min((tile + 1) * tile_tokens, s)) // 32)
        at = 0
        for k in range(n):
            r2, t2, b2, e2, n2, _ = items[i + k]
            assert (r2, t2, n2) == (req, tile, n) and b2 == at and e2 > b2
            at = e2
        assert at == n_sub
        seen[(req, tile)] = n
        i += n
    assert len(seen) == sum(-(-s // tile_tokens) for _, s in lens)
    return seen


@pytest.mark.parametrize("seed", range(12))
def test_work_items_partition_every_tile(seed):
    rng = np.random.default_rng(4200 + seed)
    lens = _random_batch(rng)
    hq, hkv = [(32, 8), (40, 8), (8, 8), (16, 2)][seed % 4]
    pb, sl = [p for p, _ in lens], [s for _, s in lens]
    r = cb.calvo_attn_plan(hq, hkv, CUS, pb, sl)
    items = cb.calvo_attn_plan_items(hq, hkv, CUS, pb, sl)
    seen = _check_partition(items, lens, r["tile_tokens"])
    group = hq // hkv
    hw = 4 if group % 4 == 0 else 2 if group % 2 == 0 else 1
    assert len(items) * (hq // hw) == r["workgroups"]
    assert max(seen.values()) <= r["pieces"] and (items[:, 5] == 0).all()
    # heaviest tile first
    first = [it for it in items if it[2] == 0]
    spans = [-(-(16 * lens[q][0] + min((t + 1) * r["tile_tokens"], lens[q][1])) // 32) for q, t, *_ in first]
    assert spans == sorted(spans, reverse=True)


@pytest.mark.parametrize("seed", range(12))
def test_work_items_of_a_chunked_layer_follow_the_chunks(seed):
    """Piece k of a tile reads blocks below (k + 1) * chunk_blocks only and is in launch k; the last piece
    (end of the prefix, suffix) is in the launch that waits for the whole layer."""
    rng = np.random.default_rng(4300 + seed)
    lens = _random_batch(rng)
    hq, hkv = [(32, 8), (40, 8)][seed % 2]
    cbk = int(2 * rng.integers(1, 400))
    pb, sl = [p for p, _ in lens], [s for _, s in lens]
    r = cb.calvo_attn_plan(hq, hkv, CUS, pb, sl)
    items = cb.calvo_attn_plan_items(hq, hkv, CUS, pb, sl, chunk_blocks=cbk)
    _check_partition(items, lens, r["tile_tokens"])
    n_chunks = -(-max(pb) // cbk)
    for req, tile, b, e, n, launch in items:
        assert 0 <= launch <= n_chunks
        if launch < n_chunks:
            assert 2 * e <= min((launch + 1) * cbk, pb[req])      # sub-tile j = blocks 2j, 2j+1: all inside chunk <= launch
            assert 2 * b >= launch * cbk
        else:
            assert b == pb[req] // 2                               # everything wholly inside the prefix came before
    # launches are served in order: the items of launch k precede nothing of an earlier tile's later launch
    for req in range(len(lens)):
        mine = [it for it in items if it[0] == req and it[1] == 0]
        assert [it[5] for it in mine] == sorted(it[5] for it in mine)


def test_plan_items_argument_checks():
    with pytest.raises(cb.CalvoError):
        cb.calvo_attn_plan_items(32, 8, CUS, [10], [5], chunk_blocks=3)       # odd chunk
    with pytest.raises(cb.CalvoError):
        cb.calvo_attn_plan_items(32, 5, CUS, [10], [5])
    assert cb.calvo_attn_plan_items(32, 8, CUS, [], []).shape == (0, 6)
