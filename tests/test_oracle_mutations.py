"""Are the oracle's pins sharp?  Plant one plausible mistake at a time in a private copy of the
oracle's source (on the CPU, never in the shipped file) and require that at least one pin test of
tests/test_oracle_attn.py / tests/test_oracle_ingest.py fails for it.

A mutant that survives would mean a mistake of that kind could sit in the oracle unnoticed.
"""
import inspect
import pathlib
import types

import pytest

import test_oracle_attn
import test_oracle_ingest
from oracle import calvo_oracle

SOURCE = pathlib.Path(calvo_oracle.__file__).read_text()

# (name, text in the oracle, replacement, expected number of occurrences)
MUTANTS = [
    ("causal boundary excludes the row's own key", "n = prefix_len + i + 1", "n = prefix_len + i", 1),
    ("causal boundary sees one key too many", "n = prefix_len + i + 1", "n = min(prefix_len + i + 2, n_max)", 1),
    ("scale dropped", "s = scale * (K @ q_row)", "s = (K @ q_row)", 1),
    ("default scale 1/D instead of 1/sqrt(D)", "scale = np.float32(1.0) / np.sqrt(np.float32(D))\n    scale = float(np.float32(scale))          #",
     "scale = np.float32(1.0) / np.float32(D)\n    scale = float(np.float32(scale))          #", 1),
    ("softmax not normalised", "return (w @ V) / np.sum(w)", "return (w @ V)", 1),
    ("GQA group by modulo instead of contiguous groups", "h // G", "h % Hkv", 2),
    ("K and V halves swapped in the block gather", "K = widen(pool_layer[slots, 0, :, kv_head, :])", "K = widen(pool_layer[slots, 1, :, kv_head, :])", 1),
    ("block gather ignores the block table", "slots = np.asarray(table[:nblk], dtype=np.int64)", "slots = np.arange(nblk, dtype=np.int64)", 1),
    ("block gather drops the partial last block", "nblk = -(-n_tokens // block_tokens)", "nblk = max(1, n_tokens // block_tokens)", 1),
    ("token gather uses the wrong row inside a block", "K[t] = widen(pool_layer[slot, 0, t % block_tokens, kv_head])",
     "K[t] = widen(pool_layer[slot, 0, (t + 1) % block_tokens, kv_head])", 1),
    ("matrix form shows one hidden key", "hidden = np.arange(n_max)[None, :] >= n_visible[:, None]", "hidden = np.arange(n_max)[None, :] > n_visible[:, None]", 1),
    ("sampled rows use the wrong visibility", "n_vis = prefix_len + rows + 1", "n_vis = prefix_len + rows", 1),
    ("ingest ignores the block table", "pool[l, slot] = host_kv[l, host_block_start + j]", "pool[l, j] = host_kv[l, host_block_start + j]", 1),
    ("ingest ignores the request's first host block", "pool[l, slot] = host_kv[l, host_block_start + j]", "pool[l, slot] = host_kv[l, j]", 1),
    ("ingest reloads blocks that are already resident", "for j in range(first_ingest_block, n_prefix_blocks):", "for j in range(0, n_prefix_blocks):", 1),
    ("ingest ignores the layer range", "for l in range(layer_begin, layer_end):", "for l in range(0, L):", 1),
    ("suffix tokens placed from position 0", "t = prefix_len + i\n", "t = i\n", 1),
    ("suffix V written with K", "pool_layer[slot, 1, t % block_tokens] = v_suffix[i]", "pool_layer[slot, 1, t % block_tokens] = k_suffix[i]", 1),
    ("bf16 widened from the wrong half", "<< np.uint32(16)", "<< np.uint32(15)", 1),
    ("batch mixes up the requests' query rows", "out[a:b] = prefill_attn(pool_layer, q[a:b], table, P, S, block_tokens, scale)",
     "out[a:b] = prefill_attn(pool_layer, q[:S], table, P, S, block_tokens, scale)", 1),
]


def pin_cases():
    """Every pin test of the two modules as a (label, callable) list, parametrisations expanded."""
    cases = []
    for mod in (test_oracle_attn, test_oracle_ingest):
        for name, fn in sorted(vars(mod).items()):
            if not name.startswith("test_") or not callable(fn):
                continue
            marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
            if not marks:
                assert not inspect.signature(fn).parameters, name
                cases.append((name, fn))
                continue
            assert len(marks) == 1, name
            argnames, argvalues = marks[0].args[0], marks[0].args[1]
            n_args = len([a for a in argnames.split(",") if a.strip()])
            for vals in argvalues:
                vals = tuple(vals) if n_args > 1 else (vals,)
                cases.append((f"{name}{list(vals)}", lambda fn=fn, vals=vals: fn(*vals)))
    return cases


def run_pins_against(module):
    """Point both test modules at `module` instead of the oracle; return the labels of the pins that fail."""
    saved = (test_oracle_attn.orc, test_oracle_ingest.orc)
    test_oracle_attn.orc = module
    test_oracle_ingest.orc = module
    failed = []
    try:
        for label, call in pin_cases():
            try:
                call()
            except Exception:                      # assertion, index or shape error: the pin noticed
                failed.append(label)
    finally:
        test_oracle_attn.orc, test_oracle_ingest.orc = saved
    return failed


def test_unmutated_copy_passes_every_pin():
    clean = types.ModuleType("oracle_copy")
    exec(compile(SOURCE, "oracle_copy", "exec"), clean.__dict__)
    assert len(pin_cases()) >= 25
    assert run_pins_against(clean) == []


@pytest.mark.parametrize("name,old,new,count", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planted_mistake_is_caught(name, old, new, count):
    assert SOURCE.count(old) == count, f"mutation site for '{name}' not found {count}x in the oracle source"
    mutant = types.ModuleType("oracle_mutant")
    exec(compile(SOURCE.replace(old, new), "oracle_mutant", "exec"), mutant.__dict__)
    failed = run_pins_against(mutant)
    print(f"{name}: caught by {len(failed)} pins, e.g. {failed[:3]}")
    assert failed, f"no pin notices the mistake: {name}"
