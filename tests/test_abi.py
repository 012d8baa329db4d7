"""The C-ABI library loads and exports every symbol include/calvo.h declares; argument checks that
run before any device work behave as documented (no GPU needed, no compute calls)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2603_21257_amd import binding as cb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "calvo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(calvo_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"calvo_kv_ingest", "calvo_prefill_attn", "calvo_layer_event"} <= set(names)
    lib = ctypes.CDLL(cb.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in calvo.h but not exported"
    assert sorted(cb.EXPORTS) == names, "binding and header disagree on the entry points"


def test_struct_layouts_match_header_order():
    assert [f[0] for f in cb.calvo_config._fields_] == [
        "n_layers", "n_q_heads", "n_kv_heads", "head_dim", "block_tokens", "dtype", "pool_blocks", "pool",
        "staging_bytes", "n_staging", "n_copy_streams", "compute_stream"]
    assert [f[0] for f in cb.calvo_request._fields_] == [
        "host_kv", "host_layer_stride", "block_table", "n_prefix_blocks", "first_ingest_block", "suffix_len"]
    assert ctypes.sizeof(cb.calvo_config) == 64
    assert ctypes.sizeof(cb.calvo_request) == 40
    assert [f[0] for f in cb.calvo_l3_config._fields_] == ["chunk_bytes", "n_slots", "n_threads", "l3_GBps", "chunk_ready", "reserved"]
    assert [f[0] for f in cb.calvo_l3_stats._fields_] == ["bytes", "chunks", "l3_busy_s", "ring_wait_s", "total_s"]
    assert ctypes.sizeof(cb.calvo_l3_config) == 32
    assert ctypes.sizeof(cb.calvo_l3_stats) == 40


def test_struct_layouts_match_what_a_c_compiler_makes_of_the_header(tmp_path):
    """Size and every field offset of every struct of the binding against gcc's view of include/calvo.h."""
    import subprocess
    structs = [cb.calvo_config, cb.calvo_request, cb.calvo_l3_config, cb.calvo_l3_stats, cb.calvo_cost_model, cb.calvo_job,
               cb.calvo_dispatch_config, cb.calvo_dispatch_job, cb.calvo_dispatch_result, cb.calvo_dispatch_stats]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "calvo.h"', 'int main(void) {']
    for st in structs:
        lines.append(f'  printf("{st.__name__} %zu\\n", sizeof({st.__name__}));')
        for name, _ in st._fields_:
            lines.append(f'  printf("{st.__name__}.{name} %zu\\n", offsetof({st.__name__}, {name}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = dict(ln.split() for ln in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for st in structs:
        assert int(out[st.__name__]) == ctypes.sizeof(st), st.__name__
        for name, _ in st._fields_:
            assert int(out[f"{st.__name__}.{name}"]) == getattr(st, name).offset, f"{st.__name__}.{name}"


@pytest.mark.parametrize("kw,frag", [
    (dict(pool=0), "pool is NULL"),
    (dict(n_q_heads=8, n_kv_heads=3), "multiple of n_kv_heads"),
    (dict(head_dim=100), "head_dim"),
    (dict(block_tokens=32), "block_tokens"),
    (dict(dtype=7), "dtype"),
    (dict(pool_blocks=0), "pool_blocks"),
    (dict(pool=4104), "16-byte aligned"),
    (dict(n_staging=1, staging_bytes=1 << 20), "n_staging"),
    (dict(staging_bytes=100), "smaller than one block"),
    (dict(n_layers=0), "n_layers"),
])
def test_create_rejects_bad_config_before_touching_the_device(kw, frag):
    args = dict(n_layers=2, n_q_heads=8, n_kv_heads=2, head_dim=128, dtype=cb.CALVO_BF16, pool_blocks=16, pool=4096)
    args.update(kw)
    with pytest.raises(cb.CalvoError) as ei:
        cb.calvo_create(**args)
    assert ei.value.code == cb.CALVO_EINVAL
    assert frag in str(ei.value)


def test_null_context_is_an_error_not_a_crash():
    lib = cb.lib()
    assert lib.calvo_destroy(None) == cb.CALVO_EINVAL
    assert lib.calvo_kv_ingest(None, None, 0, 0, 0) == cb.CALVO_EINVAL
    assert lib.calvo_kv_ingest_l3(None, None, 0, 0, 0, None) == cb.CALVO_EINVAL
    assert lib.calvo_l3_wait(None, None) == cb.CALVO_EINVAL
    assert lib.calvo_layer_event(None, 0, 0, None) == cb.CALVO_EINVAL
    assert lib.calvo_prefill_attn(None, 0, None, None, None, None, None, 0, None, ctypes.c_float(0)) == cb.CALVO_EINVAL
    assert "NULL" in cb.calvo_last_error()


def test_make_request_marshals_table():
    tab = np.array([5, 3, 9], np.int64)
    r = cb.make_request(4096, 1 << 20, tab, 2, 7, 1)
    assert (r.n_prefix_blocks, r.suffix_len, r.first_ingest_block, r.host_layer_stride) == (2, 7, 1, 1 << 20)
    assert [r.block_table[i] for i in range(3)] == [5, 3, 9]
