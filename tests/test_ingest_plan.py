"""Host-side planning of the loading stage's transfers (calvo_ingest_plan): which requests of a batch
load as one run, which consecutive layers share a transfer.  Runs without a GPU; host addresses are
made up (the planner only compares them)."""
import numpy as np
import pytest

from paper_2603_21257_amd import binding as cb

BLK = 65536
BASE = 0x7F0000000000


def req(addr, stride, n_blocks, first=0):
    return cb.make_request(addr, stride, np.arange(n_blocks, dtype=np.int32), n_blocks, 0, first)


def groups_of(transfer_of_layer):
    """Sizes of the transfer groups, in order."""
    sizes, prev = [], None
    for g in transfer_of_layer:
        if g == prev and g >= 0:
            sizes[-1] += 1
        else:
            sizes.append(1)
        prev = g
    return sizes


def test_one_request_small_layers_ramp_up_and_down():
    nb = 256                                                   # 16 MiB per layer
    r = [req(BASE, nb * BLK, nb)]
    g, runs = cb.calvo_ingest_plan(r, 0, 32, BLK, staging_blocks=4096)        # 256 MiB staging
    sizes = groups_of(g)
    assert sum(sizes) == 32 and (runs == 1).all()
    assert sizes[0] == 1 and sizes[1] == 2 and sizes[2] == 4                  # ramp-up: the first layer arrives at once
    assert sizes[-1] == 1 and sizes[-2] == 1                                  # the last layers travel alone
    layer = 0
    for i, k in enumerate(sizes):
        assert k <= 2 ** i and k * nb * BLK <= 256 << 20 and k * nb <= 4096
        assert k <= (32 - layer + 2) // 3                                     # never more than a third of what is left
        layer += k
    assert (np.diff(g) >= 0).all() and g[0] == 0 and g[-1] == len(sizes) - 1


def test_large_layers_and_small_staging_are_not_merged():
    nb = 3840                                                  # 240 MiB per layer
    g, _ = cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 0, 32, BLK, staging_blocks=4096)
    assert groups_of(g) == [1] * 32
    nb = 256
    g, _ = cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 0, 12, BLK, staging_blocks=400)   # one layer and a half
    assert groups_of(g) == [1] * 12
    g, _ = cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 0, 12, BLK, staging_blocks=0)     # zero-copy mode
    assert groups_of(g) == [1] * 12
    g, _ = cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 0, 12, BLK, staging_blocks=4096, merge_bytes=0)
    assert groups_of(g) == [1] * 12


def test_layers_with_a_gap_between_them_are_not_merged():
    nb = 128
    g, _ = cb.calvo_ingest_plan([req(BASE, (nb + 1) * BLK, nb)], 0, 12, BLK, staging_blocks=4096)   # stride leaves a hole
    assert groups_of(g) == [1] * 12
    g, _ = cb.calvo_ingest_plan([req(BASE, nb * BLK, nb, first=8)], 0, 12, BLK, staging_blocks=4096)  # resident head: hole
    assert groups_of(g) == [1] * 12


def test_batch_contiguous_requests_are_one_run_and_merge_across_layers():
    n = [40, 24, 64]
    total = sum(n)
    stride = total * BLK
    reqs, at = [], 0
    for k in n:
        reqs.append(req(BASE + at * BLK, stride, k))
        at += k
    g, runs = cb.calvo_ingest_plan(reqs, 0, 12, BLK, staging_blocks=1024)
    assert (runs == 1).all()
    assert groups_of(g)[:3] == [1, 2, 3] and groups_of(g)[-2:] == [1, 1]
    # the same requests in reversed order: three runs per layer, nothing shared across layers
    g, runs = cb.calvo_ingest_plan(reqs[::-1], 0, 12, BLK, staging_blocks=1024)
    assert (runs == 3).all() and groups_of(g) == [1] * 12
    # separate host buffers per request
    sep = [req(BASE + i * (1 << 32), k * BLK, k) for i, k in enumerate(n)]
    g, runs = cb.calvo_ingest_plan(sep, 0, 6, BLK, staging_blocks=1024)
    assert (runs == 3).all() and groups_of(g) == [1] * 6


def test_shared_run_is_loaded_once_and_the_batch_stays_one_run():
    """Requests 1.. skip the shared blocks (first_ingest_block): their own blocks follow in host memory."""
    shared, own = 16, [20, 30, 10]
    stride = (shared + sum(own)) * BLK
    reqs = [req(BASE, stride, shared + own[0])]
    at = shared + own[0]
    for k in own[1:]:
        # block j >= shared of this request sits at host block at + (j - shared)
        reqs.append(req(BASE + (at - shared) * BLK, stride, shared + k, first=shared))
        at += k
    g, runs = cb.calvo_ingest_plan(reqs, 0, 9, BLK, staging_blocks=2048)
    assert (runs == 1).all() and groups_of(g)[0:2] == [1, 2]


def test_chunked_layers_stand_alone_and_stop_a_group():
    nb = 128
    cbk = [0] * 8 + [32, 32] + [0] * 2
    g, _ = cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 0, 12, BLK, staging_blocks=4096, chunk_blocks=cbk)
    assert list(g[8:10]) == [-1, -1]
    assert all(x >= 0 for x in list(g[:8]) + list(g[10:]))
    sizes = groups_of(g)
    assert sum(sizes) == 12
    # no group reaches across the chunked layers
    assert g[7] != g[10]


def test_layer_subrange_and_argument_checks():
    nb = 64
    g, runs = cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 4, 10, BLK, staging_blocks=4096)
    assert len(g) == 6 and groups_of(g) == [1, 2, 1, 1, 1]
    with pytest.raises(cb.CalvoError):
        cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 3, 2, BLK, 64)
    with pytest.raises(cb.CalvoError):
        cb.calvo_ingest_plan([req(BASE, nb * BLK, nb)], 0, 2, BLK, 64, chunk_blocks=[3, 0])
    g, runs = cb.calvo_ingest_plan([], 0, 3, BLK, 64)
    assert list(runs) == [0, 0, 0]


def test_back_to_back_attention_chain_schedule():
    """bench.alap_schedule: every launch waits for its own layer or a later one, in non-decreasing order; the chain
    is feasible (the awaited layer lands no later than a back-to-back chain ending with the last chain layer would
    reach the launch), as late as a whole layer allows, and rho >= 1 degenerates to one launch per landed layer."""
    import math
    import bench
    for L, n, rho in [(32, 26, 0.78), (32, 32, 0.45), (48, 42, 0.93), (8, 8, 0.0), (5, 3, 0.5), (4, 0, 0.7)]:
        after = bench.alap_schedule(L, n, rho)
        assert len(after) == L and all(a >= l for l, a in enumerate(after)) and after == sorted(after)
        assert after[n:] == list(range(n, L))
        for l in range(min(n, L)):
            lands = after[l] + 1                                   # in units of one layer's load
            due = n - (n - 1 - l) * rho                            # when the chain has to start launch l
            assert lands <= due + 1e-9 or after[l] == l
            assert after[l] == l or lands + 1 > due - 1e-9         # not a whole layer earlier than needed
        if n:
            assert after[n - 1] == n - 1
    assert bench.alap_schedule(6, 6, 1.0) == list(range(6)) and bench.alap_schedule(6, 6, 1.7) == list(range(6))
    assert bench.alap_schedule(6, 6, 0.0) == [5] * 6
