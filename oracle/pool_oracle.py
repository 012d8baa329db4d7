"""CPU oracle for the slot allocation of the paged KV space.  TEST INFRASTRUCTURE ONLY.

Only tests/ may import this file.  Plain Python, one dictionary of reference counts; shares no code
with the library.

What it follows (paper Section 3.1, proactive higher-level allocation): the destination blocks of a
request are requested at the moment its lower-level transfer is issued; when the higher level is
short of space the scheme degrades to reactive allocation (footnote of that section): the request
gets its blocks later, when space has been released.

Readings taken where the paper is silent: a reservation is all or nothing; a block shared by several
requests (a common prefix run) is counted once per request and is free again when the last one lets
go; requests that could not be served at once are served strictly in the order in which they asked,
and while one is waiting no later request is served ahead of it, however small; a waiting request
holds a reference on the shared blocks it maps from the moment it asks.  Which free block a request
receives is not defined: callers of this model compare counts and outcomes, never block numbers
(the model hands out the lowest free numbers).

Pins (tests/test_oracle_pool.py): the two-requests-in-a-short-pool scenario of the footnote written
out by hand, and - on random operation sequences - the counts recomputed from nothing but the list of
tables that are alive (a block's count is the number of live tables that contain it).
"""
from __future__ import annotations

OK, EINVAL, ENOMEM, ENOTREADY = 0, -1, -2, -4


class PoolModel:
    def __init__(self, n_blocks: int):
        assert n_blocks > 0
        self.n = n_blocks
        self.refs = {}                # slot -> count (> 0)
        self.waiting = []             # [ticket, shared slots, n_own], oldest first
        self.next_ticket = 1

    # ---- counts
    def n_free(self) -> int:
        return self.n - len(self.refs)

    def counts(self) -> dict:
        return {"free": self.n_free(), "used": len(self.refs), "refs": sum(self.refs.values()),
                "waiting": len(self.waiting)}

    def _take(self, n: int):
        out = []
        s = 0
        while len(out) < n:
            if s not in self.refs:
                self.refs[s] = 1
                out.append(s)
            s += 1
        return out

    # ---- plain reservations
    def reserve(self, n: int):
        if n < 0:
            return EINVAL, None
        if n > self.n_free():
            return ENOMEM, None
        return OK, self._take(n)

    def retain(self, slots):
        if any(s not in self.refs for s in slots):
            return EINVAL
        for s in slots:
            self.refs[s] += 1
        return OK

    def release(self, slots):
        need = {}
        for s in slots:
            need[s] = need.get(s, 0) + 1
        if any(self.refs.get(s, 0) < k for s, k in need.items()):
            return EINVAL
        for s, k in need.items():
            self.refs[s] -= k
            if self.refs[s] == 0:
                del self.refs[s]
        return OK

    # ---- admission: proactive when possible, reactive otherwise
    def admit(self, shared, n_own: int):
        """(OK, table, 0) | (ENOTREADY, None, ticket) | (ENOMEM / EINVAL, None, 0)"""
        shared = list(shared)
        if n_own < 0:
            return EINVAL, None, 0
        if n_own > self.n:
            return ENOMEM, None, 0
        if any(s not in self.refs for s in shared) or len(set(shared)) != len(shared):
            return EINVAL, None, 0
        for s in shared:
            self.refs[s] += 1
        if not self.waiting and n_own <= self.n_free():
            return OK, shared + self._take(n_own), 0
        t = self.next_ticket
        self.next_ticket += 1
        self.waiting.append([t, shared, n_own])
        return ENOTREADY, None, t

    def retry(self, ticket: int):
        pos = [i for i, w in enumerate(self.waiting) if w[0] == ticket]
        if not pos:
            return EINVAL, None
        if pos[0] != 0 or self.waiting[0][2] > self.n_free():
            return ENOTREADY, None
        _, shared, n_own = self.waiting.pop(0)
        return OK, shared + self._take(n_own)

    def cancel(self, ticket: int):
        pos = [i for i, w in enumerate(self.waiting) if w[0] == ticket]
        if not pos:
            return EINVAL
        _, shared, _ = self.waiting.pop(pos[0])
        for s in shared:
            self.refs[s] -= 1
            if self.refs[s] == 0:
                del self.refs[s]
        return OK
