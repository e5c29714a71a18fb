"""CPU-only: the C-ABI library loads and exports every symbol the header declares; host-side
argument checks run without a GPU (they return before any HIP call)."""
import ctypes as C
import os
import re

import pytest

from paper_2509_10406_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "muse.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(?:int|const char\*)\s+(\w+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    if not os.path.exists(mb.LIB_PATH):
        import __graft_entry__ as g
        g.build()
    lib = mb.load()
    names = _declared()
    assert names == sorted(mb.SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_strerror_and_host_side_validation():
    assert mb.muse_strerror(0) == "ok"
    assert "workspace" in mb.muse_strerror(-3)
    good = mb.Params(1, 16, 16, 65536, 64, Cq=256, Ck=1024, r=8)
    mn, pref = mb.muse_workspace_bytes(good, mb.WS_CLUSTER)
    assert mn > 0 and pref >= mn
    for bad, msg in ((dict(causal=0), "unsupported"), (dict(D=80), "unsupported"), (dict(Hkv=3), "invalid"),
                     (dict(block=1000), "invalid"), (dict(r=2000), "invalid"), (dict(Ck=4096), "unsupported"),
                     (dict(flags=16), "invalid")):
        import dataclasses
        with pytest.raises(mb.MuseError, match=msg):
            mb.muse_workspace_bytes(dataclasses.replace(good, **bad), mb.WS_FWD)
    # NULL pointers are rejected on the host, nothing is launched
    pc = good.c()
    rc = mb.load().muse_fwd(C.byref(pc), *([C.c_void_p(0)] * 11), C.c_size_t(0), C.c_void_p(0))
    assert rc == -1
