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
    import dataclasses
    for bad, msg in ((dict(causal=0), "unsupported"), (dict(D=80), "unsupported"), (dict(Hkv=3), "invalid"),
                     (dict(block=1000), "invalid"), (dict(r=2000), "invalid"), (dict(Ck=4096), "unsupported"),
                     (dict(flags=32), "invalid"), (dict(flags=mb.FLAG_DIPOLE), "unsupported")):  # dipole needs r = 0
        with pytest.raises(mb.MuseError, match=msg):
            mb.muse_workspace_bytes(dataclasses.replace(good, **bad), mb.WS_FWD)
    assert mb.muse_workspace_bytes(dataclasses.replace(good, r=0, flags=mb.FLAG_DIPOLE), mb.WS_FWD)[0] > \
        mb.muse_workspace_bytes(dataclasses.replace(good, r=0), mb.WS_FWD)[0]
    with pytest.raises(mb.MuseError, match="unsupported"):      # no backward is defined for the dipole correction
        mb.muse_workspace_bytes(dataclasses.replace(good, r=0, flags=mb.FLAG_DIPOLE), mb.WS_BWD)
    # NULL pointers are rejected on the host, nothing is launched
    pc = good.c()
    rc = mb.load().muse_fwd(C.byref(pc), *([C.c_void_p(0)] * 11), C.c_size_t(0), C.c_void_p(0))
    assert rc == -1


def test_kmeans_stream_rejects_bad_arguments_on_the_host():
    """muse_kmeans_stream: side must be 0 or 1, the row and centroid pointers and the workspace must be given;
    nothing is launched (no GPU here)."""
    good = mb.Params(1, 16, 16, 65536, 64, Cq=256, Ck=1024, r=8)
    pc = good.c()
    lib = mb.load()
    null = C.c_void_p(0)
    fake = C.c_void_p(4096)  # never dereferenced: every call below fails a host check first
    assert lib.muse_kmeans_stream(C.byref(pc), C.c_int(2), fake, null, fake, null, null, fake, C.c_size_t(1 << 40), null) == -1
    assert lib.muse_kmeans_stream(C.byref(pc), C.c_int(0), null, null, fake, null, null, fake, C.c_size_t(1 << 40), null) == -1
    assert lib.muse_kmeans_stream(C.byref(pc), C.c_int(1), fake, null, null, null, null, fake, C.c_size_t(1 << 40), null) == -1
    assert lib.muse_kmeans_stream(C.byref(pc), C.c_int(1), fake, null, fake, null, null, null, C.c_size_t(1 << 40), null) == -1
    assert lib.muse_kmeans_stream(C.byref(pc), C.c_int(1), fake, null, fake, null, null, fake, C.c_size_t(16), null) == -3
