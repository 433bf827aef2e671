"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol include/*.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1804_06609_amd as dba
from paper_1804_06609_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_WS = 1 << 20          # an aligned fake device address: argument checks come before any use


def _declared_symbols(headers=("dba.h", "dba_debug.h")):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"DBA_API\s+[\w\s\*]+?\b(dba_\w+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_boundary():
    names = _declared_symbols(("dba.h",))
    for must in ("dba_init", "dba_step", "dba_finalize", "dba_workspace_bytes", "dba_destroy"):
        assert must in names
    assert not [n for n in names if n.startswith("dba_debug_")]      # diagnostics have a header of their own
    assert all(n.startswith("dba_debug_") for n in _declared_symbols(("dba_debug.h",)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(binding._SIGNATURES) == _declared_symbols()


def test_workspace_bytes():
    assert dba.dba_workspace_bytes(64, 20, 32000, 100, 32) > 64 * 20 * 64 * 8
    assert dba.dba_workspace_bytes(1, 1, 1, 1, 0) > 0
    for bad in [(0, 5, 100, 10, 0), (1, 0, 100, 10, 0), (1, 65, 100, 10, 0), (1, 5, 4, 10, 0),
                (1, 5, 100, 0, 0), (1, 5, 100, 10, 65), (1, 5, 100, 10, -1)]:
        assert dba.dba_workspace_bytes(*bad) == 0


def _init(B=1, k=5, V=1000, N=10, eos=2, pad=0, toks=(5, 6), poff=(0, 2), soff=(0, 1), ws=FAKE_WS,
          nbytes=1 << 30):
    return dba.dba_init(B, k, V, N, eos, pad, np.array(toks, np.int32), np.array(poff, np.int32),
                        np.array(soff, np.int32), ws, nbytes)


@pytest.mark.parametrize("kw,frag", [
    (dict(k=0), "1 <= k"),
    (dict(k=65), "1 <= k"),
    (dict(k=5, V=4), "k <= V"),
    (dict(N=0), "N"),
    (dict(eos=1000), "eos_id"),
    (dict(eos=0, pad=0), "distinct"),
    (dict(toks=(5, 2)), "cannot be a constraint"),
    (dict(toks=(0, 6)), "cannot be a constraint"),
    (dict(toks=(5, 1000)), "outside"),
    (dict(toks=(5, -1)), "outside"),
    (dict(poff=(0, 0), soff=(0, 1)), "empty"),
    (dict(poff=(1, 2)), "start at 0"),
    (dict(ws=FAKE_WS + 8), "aligned"),
    (dict(ws=0), "NULL"),
    (dict(nbytes=1024), "workspace has"),
    (dict(toks=tuple(range(4, 69 + 4)), poff=(0, 69)), "more than 64"),
    (dict(k=64, V=600000, toks=tuple(range(4, 68)), poff=(0, 64)), "exceed the 32-bit"),
])
def test_init_rejects_bad_arguments(kw, frag):
    with pytest.raises(dba.DbaError) as ei:
        _init(**kw)
    assert ei.value.code in (dba.DBA_EINVAL, dba.DBA_ENOMEM)
    assert frag in str(ei.value)


def test_null_ctx_calls_fail_cleanly():
    lib = binding.load()
    assert lib.dba_step(None, None, None, None, None, None) == dba.DBA_EINVAL
    assert lib.dba_finalize(None, None, None, None, None) == dba.DBA_EINVAL
    assert lib.dba_get_state(None, None, None, None, None, None, None) == dba.DBA_EINVAL
    assert lib.dba_steps_done(None) == dba.DBA_EINVAL
    lib.dba_destroy(None)
    assert isinstance(dba.dba_last_error(None), str)


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asked for more it says so and exits (before touching any GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    for extra_env, argv in (({}, ["--gpus", "2"]), ({"WORLD_SIZE": "4"}, [])):
        env = dict(os.environ, **extra_env)
        r = subprocess.run([sys.executable, os.path.join(root, "bench.py")] + argv, capture_output=True, text=True,
                           env=env, timeout=120)
        assert r.returncode != 0
        assert "ONE GPU" in r.stderr
        assert r.stdout.strip() == ""
