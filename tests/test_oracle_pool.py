"""Pins of the slot-allocation oracle (oracle/pool_oracle.py): the short-pool scenario behind the
paper's "degrades to the reactive allocation" remark (Section 3.1, footnote) written out by hand, and
counts recomputed from first principles on random operation sequences."""
import random

from oracle import pool_oracle as po


def test_short_pool_scenario_by_hand():
    """Pool of 10 blocks.  R1 (6 blocks) asks when its transfer is issued and is served at once
    (proactive).  R2 (6 blocks) finds 4 free: it waits (reactive).  R3 (2 blocks) would fit but may not
    overtake R2.  When R1 lets go, R2 is served, then R3."""
    p = po.PoolModel(10)
    rc, t1, _ = p.admit([], 6)
    assert rc == po.OK and len(set(t1)) == 6 and p.counts() == {"free": 4, "used": 6, "refs": 6, "waiting": 0}
    rc, t2, k2 = p.admit([], 6)
    assert rc == po.ENOTREADY and t2 is None and k2 > 0 and p.counts()["free"] == 4
    rc, t3, k3 = p.admit([], 2)
    assert rc == po.ENOTREADY and k3 > k2 and p.counts() == {"free": 4, "used": 6, "refs": 6, "waiting": 2}
    assert p.retry(k2) == (po.ENOTREADY, None)           # still short
    assert p.retry(k3) == (po.ENOTREADY, None)           # would fit, but R2 is ahead
    assert p.release(t1) == po.OK and p.counts()["free"] == 10
    assert p.retry(k3) == (po.ENOTREADY, None)           # order is kept after the release too
    rc, t2 = p.retry(k2)
    assert rc == po.OK and len(set(t2)) == 6
    rc, t3 = p.retry(k3)
    assert rc == po.OK and len(set(t3)) == 2 and not set(t2) & set(t3)
    assert p.counts() == {"free": 2, "used": 8, "refs": 8, "waiting": 0}
    assert p.retry(k2)[0] == po.EINVAL                   # a ticket is good once


def test_shared_run_is_counted_per_request_and_survives_its_first_owner():
    p = po.PoolModel(12)
    _, owner, _ = p.admit([], 8)
    run = owner[:4]
    rc, other, _ = p.admit(run, 3)
    assert rc == po.OK and other[:4] == run and not set(other[4:]) & set(owner)
    assert p.counts() == {"free": 1, "used": 11, "refs": 15, "waiting": 0}
    assert p.release(owner) == po.OK                      # the run stays: the second request holds it
    assert p.counts() == {"free": 5, "used": 7, "refs": 7, "waiting": 0}
    # a waiting request holds the run too
    rc, _, k = p.admit(run, 6)
    assert rc == po.ENOTREADY and p.counts()["refs"] == 11
    assert p.release(other) == po.OK
    assert p.counts() == {"free": 8, "used": 4, "refs": 4, "waiting": 1}
    assert p.cancel(k) == po.OK and p.counts() == {"free": 12, "used": 0, "refs": 0, "waiting": 0}


def test_exact_fit_is_served():
    """A request for exactly the free space is served, one more is not."""
    p = po.PoolModel(7)
    rc, a = p.reserve(3)
    assert rc == po.OK and p.counts()["free"] == 4
    assert p.reserve(5) == (po.ENOMEM, None)
    rc, b = p.reserve(4)
    assert rc == po.OK and sorted(a + b) == list(range(7)) and p.counts()["free"] == 0
    assert p.release(b) == po.OK
    rc, t, _ = p.admit(a[:2], 4)
    assert rc == po.OK and t[:2] == a[:2] and sorted(t[2:]) == sorted(b)
    assert p.admit([], 1)[0] == po.ENOTREADY


def test_refusals_change_nothing():
    p = po.PoolModel(4)
    _, t, _ = p.admit([], 3)
    before = p.counts()
    assert p.reserve(2) == (po.ENOMEM, None)
    assert p.admit([], 5)[0] == po.ENOMEM                 # larger than the whole pool: can never be served
    free_slot = ({0, 1, 2, 3} - set(t)).pop()
    assert p.retain([free_slot]) == po.EINVAL
    assert p.release([t[0], t[0]]) == po.EINVAL           # one reference, released twice
    assert p.release([free_slot]) == po.EINVAL
    assert p.admit([free_slot], 0)[0] == po.EINVAL        # shared slot that nobody holds
    assert p.admit([t[0], t[0]], 0)[0] == po.EINVAL
    assert p.cancel(99) == po.EINVAL
    assert p.counts() == before


def test_counts_equal_what_the_live_tables_say():
    """Random operation sequences; after every step the model's counts must equal those recomputed
    from the list of live tables alone: a slot's count is the number of live tables (plus waiting
    requests' shared runs) that contain it, used = slots with a count, free = the rest."""
    rng = random.Random(2603)
    for trial in range(40):
        n = rng.randint(4, 40)
        p = po.PoolModel(n)
        live, waiting = [], {}                            # granted tables; ticket -> (shared, n_own)
        for _ in range(300):
            op = rng.random()
            if op < 0.35:
                shared = []
                if live and rng.random() < 0.4:
                    src = rng.choice(live)
                    shared = src[:rng.randint(0, len(src))]
                n_own = rng.randint(0, max(1, n // 3))
                rc, table, k = p.admit(shared, n_own)
                if rc == po.OK:
                    assert table[:len(shared)] == shared and len(table) == len(shared) + n_own
                    held = {s for t in live for s in t} | {s for sh, _ in waiting.values() for s in sh}
                    assert not set(table[len(shared):]) & held, "a slot that is in use was handed out"
                    assert len(set(table[len(shared):])) == n_own and all(0 <= s < n for s in table)
                    live.append(table)
                elif rc == po.ENOTREADY:
                    waiting[k] = (shared, n_own)
            elif op < 0.6 and live:
                t = live.pop(rng.randrange(len(live)))
                assert p.release(t) == po.OK
            elif op < 0.8 and waiting:
                k = rng.choice(list(waiting))
                rc, table = p.retry(k)
                oldest = min(waiting)
                fits = waiting[oldest][1] <= p.counts()["free"] if rc != po.OK else True
                if rc == po.OK:
                    assert k == oldest, "a younger request was served ahead of an older one"
                    sh, n_own = waiting.pop(k)
                    assert table[:len(sh)] == sh and len(table) == len(sh) + n_own
                    live.append(table)
                else:
                    assert k != oldest or not fits
            elif op < 0.85 and waiting:
                k = rng.choice(list(waiting))
                assert p.cancel(k) == po.OK
                del waiting[k]
            else:
                rc, slots = p.reserve(rng.randint(0, 3))
                if rc == po.OK:
                    live.append(slots)
            refs = {}
            for t in live:
                for s in t:
                    refs[s] = refs.get(s, 0) + 1
            for sh, _ in waiting.values():
                for s in sh:
                    refs[s] = refs.get(s, 0) + 1
            c = p.counts()
            assert c["used"] == len(refs) and c["free"] == n - len(refs), (trial, c, refs)
            assert c["refs"] == sum(refs.values()) and c["waiting"] == len(waiting)
        for t in live:
            assert p.release(t) == po.OK
        for k in list(waiting):
            assert p.cancel(k) == po.OK
        assert p.counts() == {"free": n, "used": 0, "refs": 0, "waiting": 0}
