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
