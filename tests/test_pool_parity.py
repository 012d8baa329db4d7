"""The library's slot allocator (calvo_pool_*) against the oracle on the same operation sequences.
Host code: runs without a GPU.  Which free slot is handed out is not defined, so each side releases
and shares the slots it was given itself; outcomes and counts must agree exactly, and the library's
slots must be valid (distinct, in range, not in use)."""
import random

import numpy as np
import pytest

from oracle import pool_oracle as po
from paper_2603_21257_amd import binding as cb


class LibPool:
    """The library behind the oracle's call shapes."""

    def __init__(self, n):
        self.h = cb.calvo_pool_create(n)

    def close(self):
        cb.calvo_pool_destroy(self.h)

    def counts(self):
        return cb.calvo_pool_counts(self.h)

    def _rc(self, fn, *a):
        try:
            return po.OK, fn(*a)
        except cb.CalvoError as e:
            return e.code, None

    def reserve(self, n):
        rc, v = self._rc(cb.calvo_pool_reserve, self.h, n)
        if rc == po.OK and v is None:
            return po.ENOMEM, None
        return rc, (v.tolist() if v is not None else None)

    def retain(self, slots):
        return self._rc(cb.calvo_pool_retain, self.h, slots)[0]

    def release(self, slots):
        return self._rc(cb.calvo_pool_release, self.h, slots)[0]

    def admit(self, shared, n_own):
        rc, v = self._rc(cb.calvo_pool_admit, self.h, shared, n_own)
        if rc != po.OK:
            return rc, None, 0
        table, ticket = v
        return (po.OK, table.tolist(), 0) if table is not None else (po.ENOTREADY, None, ticket)

    def retry(self, ticket, n_table):
        rc, v = self._rc(cb.calvo_pool_retry, self.h, ticket, n_table)
        if rc != po.OK:
            return rc, None
        return (po.OK, v.tolist()) if v is not None else (po.ENOTREADY, None)

    def cancel(self, ticket):
        return self._rc(cb.calvo_pool_cancel, self.h, ticket)[0]


def test_short_pool_scenario_matches_the_oracle():
    lib, ref = LibPool(10), po.PoolModel(10)
    try:
        a = lib.admit([], 6); b = ref.admit([], 6)
        assert a[0] == b[0] == po.OK and len(set(a[1])) == 6
        a2 = lib.admit([], 6); b2 = ref.admit([], 6)
        assert a2[0] == b2[0] == po.ENOTREADY
        a3 = lib.admit([], 2); b3 = ref.admit([], 2)
        assert a3[0] == b3[0] == po.ENOTREADY
        assert lib.retry(a3[2], 2)[0] == ref.retry(b3[2])[0] == po.ENOTREADY
        assert lib.release(a[1]) == ref.release(b[1]) == po.OK
        assert lib.retry(a3[2], 2)[0] == ref.retry(b3[2])[0] == po.ENOTREADY
        assert lib.retry(a2[2], 6)[0] == ref.retry(b2[2])[0] == po.OK
        assert lib.retry(a3[2], 2)[0] == ref.retry(b3[2])[0] == po.OK
        assert lib.counts() == ref.counts() == {"free": 2, "used": 8, "refs": 8, "waiting": 0}
    finally:
        lib.close()


@pytest.mark.parametrize("seed", range(8))
def test_random_sequences_match_the_oracle(seed):
    rng = random.Random(77000 + seed)
    n = rng.randint(3, 64)
    lib, ref = LibPool(n), po.PoolModel(n)
    # request id -> its table on each side; waiting: id -> (tickets, shared ids prefix, n_own)
    live_l, live_r, waiting = {}, {}, {}
    next_id = 0
    try:
        for step in range(600):
            op = rng.random()
            if op < 0.35:
                src, n_sh = None, 0
                if live_l and rng.random() < 0.4:
                    src = rng.choice(list(live_l))
                    n_sh = rng.randint(0, len(live_l[src]))
                n_own = rng.randint(0, n // 2 + 1) if rng.random() < 0.9 else n + rng.randint(1, 3)
                sh_l = live_l[src][:n_sh] if src is not None else []
                sh_r = live_r[src][:n_sh] if src is not None else []
                a, b = lib.admit(sh_l, n_own), ref.admit(sh_r, n_own)
                assert a[0] == b[0], (step, a, b)
                if a[0] == po.OK:
                    own = a[1][n_sh:]
                    held = {s for t in live_l.values() for s in t}
                    assert a[1][:n_sh] == sh_l and len(a[1]) == len(b[1]) == n_sh + n_own
                    assert len(set(own)) == n_own and not set(own) & held and all(0 <= s < n for s in own)
                    live_l[next_id], live_r[next_id] = a[1], b[1]
                    next_id += 1
                elif a[0] == po.ENOTREADY:
                    waiting[next_id] = (a[2], b[2], n_sh + n_own)
                    next_id += 1
            elif op < 0.6 and live_l:
                rid = rng.choice(list(live_l))
                assert lib.release(live_l.pop(rid)) == ref.release(live_r.pop(rid)) == po.OK
            elif op < 0.8 and waiting:
                rid = rng.choice(list(waiting))
                kl, kr, nt = waiting[rid]
                a, b = lib.retry(kl, nt), ref.retry(kr)
                assert a[0] == b[0], (step, a, b)
                if a[0] == po.OK:
                    held = {s for t in live_l.values() for s in t}
                    assert len(a[1]) == len(b[1]) == nt and all(0 <= s < n for s in a[1])
                    live_l[rid], live_r[rid] = a[1], b[1]
                    del waiting[rid]
            elif op < 0.85 and waiting:
                rid = rng.choice(list(waiting))
                kl, kr, _ = waiting.pop(rid)
                assert lib.cancel(kl) == ref.cancel(kr) == po.OK
            elif op < 0.9 and live_l:
                rid = rng.choice(list(live_l))
                k = rng.randint(0, len(live_l[rid]))
                assert lib.retain(live_l[rid][:k]) == ref.retain(live_r[rid][:k]) == po.OK
                live_l[next_id], live_r[next_id] = live_l[rid][:k], live_r[rid][:k]
                next_id += 1
            elif op < 0.95:
                # refusals: a slot nobody holds, a double release, a bad ticket
                free_l = sorted(set(range(n)) - {s for t in live_l.values() for s in t})
                free_r = sorted(set(range(n)) - {s for t in live_r.values() for s in t})
                # (slots held only by waiting requests are not free: skip them on both sides alike)
                if free_l and free_r and not waiting:
                    assert lib.retain(free_l[:1]) == ref.retain(free_r[:1]) == po.EINVAL
                    assert lib.release(free_l[:1]) == ref.release(free_r[:1]) == po.EINVAL
                assert lib.cancel(10**6) == ref.cancel(10**6) == po.EINVAL
                assert lib.release([n]) == ref.release([n]) == po.EINVAL
            else:
                k = rng.randint(0, 4)
                a, b = lib.reserve(k), ref.reserve(k)
                assert a[0] == b[0]
                if a[0] == po.OK:
                    live_l[next_id], live_r[next_id] = a[1], b[1]
                    next_id += 1
            assert lib.counts() == ref.counts(), step
        for rid in list(live_l):
            assert lib.release(live_l.pop(rid)) == ref.release(live_r.pop(rid)) == po.OK
        for kl, kr, _ in waiting.values():
            assert lib.cancel(kl) == ref.cancel(kr) == po.OK
        assert lib.counts() == ref.counts() == {"free": n, "used": 0, "refs": 0, "waiting": 0}
    finally:
        lib.close()


def test_argument_checks():
    with pytest.raises(cb.CalvoError):
        cb.calvo_pool_create(0)
    with pytest.raises(cb.CalvoError):
        cb.calvo_pool_create(2**31)
    h = cb.calvo_pool_create(5)
    try:
        with pytest.raises(cb.CalvoError) as ei:
            cb.calvo_pool_admit(h, [], 6)
        assert ei.value.code == cb.CALVO_ENOMEM
        assert cb.calvo_pool_reserve(h, 6) is None
        t = cb.calvo_pool_reserve(h, 5)
        assert sorted(t.tolist()) == [0, 1, 2, 3, 4]
        with pytest.raises(cb.CalvoError):
            cb.calvo_pool_release(h, np.array([0, 0], np.int32))
        assert cb.calvo_pool_counts(h) == {"free": 0, "used": 5, "refs": 5, "waiting": 0}
    finally:
        cb.calvo_pool_destroy(h)
