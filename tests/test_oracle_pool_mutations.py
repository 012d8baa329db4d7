"""Sharpness of the slot-allocation pins: one plausible mistake at a time is planted in a private
copy of oracle/pool_oracle.py and at least one pin of tests/test_oracle_pool.py must fail."""
import pathlib
import types

import pytest

import test_oracle_pool
from oracle import pool_oracle

SOURCE = pathlib.Path(pool_oracle.__file__).read_text()

MUTANTS = [
    ("a waiting request may be overtaken", "if not self.waiting and n_own <= self.n_free():", "if n_own <= self.n_free():", 1),
    ("queued requests served out of order", "if pos[0] != 0 or self.waiting[0][2] > self.n_free():",
     "if self.waiting[pos[0]][2] > self.n_free():", 1),
    ("reservation hands out fewer slots than fit exactly", "if n > self.n_free():", "if n >= self.n_free():", 1),
    ("shared run not referenced by the new request", "        for s in shared:\n            self.refs[s] += 1\n        if not self.waiting",
     "        if not self.waiting", 1),
    ("release frees a slot that is still referenced", "            if self.refs[s] == 0:\n                del self.refs[s]\n        return OK\n\n    # ---- admission",
     "            del self.refs[s]\n        return OK\n\n    # ---- admission", 1),
    ("double release accepted", "if any(self.refs.get(s, 0) < k for s, k in need.items()):", "if any(s not in self.refs for s in need):", 1),
    ("cancel keeps the shared references", "        for s in shared:\n            self.refs[s] -= 1\n            if self.refs[s] == 0:\n                del self.refs[s]\n        return OK\n",
     "        return OK\n", 1),
    ("a used slot is handed out again", "            if s not in self.refs:\n                self.refs[s] = 1\n                out.append(s)",
     "            if self.refs.get(s, 0) <= 1:\n                self.refs[s] = 1\n                out.append(s)", 1),
    ("request larger than the pool queues forever", "if n_own > self.n:\n            return ENOMEM, None, 0", "if n_own > 10 ** 9:\n            return ENOMEM, None, 0", 1),
    ("ticket stays valid after it was served", "_, shared, n_own = self.waiting.pop(0)\n        return OK, shared + self._take(n_own)",
     "_, shared, n_own = self.waiting[0]\n        return OK, shared + self._take(n_own)", 1),
]

PINS = [fn for name, fn in sorted(vars(test_oracle_pool).items()) if name.startswith("test_") and callable(fn)]


def failing_pins(module):
    saved = test_oracle_pool.po
    test_oracle_pool.po = module
    failed = []
    try:
        for fn in PINS:
            try:
                fn()
            except Exception:
                failed.append(fn.__name__)
    finally:
        test_oracle_pool.po = saved
    return failed


def test_unmutated_copy_passes_every_pin():
    clean = types.ModuleType("pool_copy")
    exec(compile(SOURCE, "pool_copy", "exec"), clean.__dict__)
    assert len(PINS) >= 4 and failing_pins(clean) == []


@pytest.mark.parametrize("name,old,new,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, count):
    assert SOURCE.count(old) == count, f"mutation site for '{name}' not found {count}x"
    mutant = types.ModuleType("pool_mutant")
    exec(compile(SOURCE.replace(old, new), "pool_mutant", "exec"), mutant.__dict__)
    failed = failing_pins(mutant)
    assert failed, f"no pin notices the mistake: {name}"
