"""CPU oracle for MuSe (test infrastructure only).

Plain fp64 implementation of what the hot path computes, written from the
paper (see the header of ``muse_oracle.c`` for the passage each function
follows).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the GPU library
shares no code with it and never calls it.
"""
from .api import (  # noqa: F401
    MuseParams,
    balanced_assign,
    build,
    exact_bwd,
    exact_fwd,
    kmeans,
    kmeans_stream,
    muse_bwd,
    muse_fwd,
    round_bf16,
    round_fp16,
    summaries,
)
