"""ctypes front end of the C oracle (test infrastructure only).

Every function works on ONE (batch, head): Q, K, V are float64 arrays [N, D]
holding the values the GPU sees (already rounded to the storage type).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "muse_oracle.c")
_LIB = os.path.join(_HERE, "libmuse_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no hand SIMD, no threads)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


class _P(C.Structure):
    _fields_ = [
        ("N", C.c_int32), ("D", C.c_int32), ("Bs", C.c_int32), ("Cq", C.c_int32),
        ("Ck", C.c_int32), ("r", C.c_int32), ("k2", C.c_int32), ("scale", C.c_double),
        ("frozen_weights", C.c_int32), ("dipole", C.c_int32), ("Kw", C.c_void_p),
    ]


@dataclass
class MuseParams:
    N: int
    D: int
    Bs: int
    Cq: int
    Ck: int
    r: int
    k2: int = 1
    scale: float = 0.0  # 0 -> 1/sqrt(D)
    frozen_weights: bool = False  # backward: aggregation weights and mu-bar are constants (App. C)
    dipole: int = 0  # forward, r = 0 only (App. B): 1 per-cell tilted dipole, 2 pre-merged untilted dipole

    def c(self, Kw=None) -> _P:
        """Kw: float64 [N, D] array (kept alive by the caller) of the keys inside the tilted weights."""
        sc = self.scale if self.scale != 0.0 else 1.0 / np.sqrt(self.D)
        return _P(self.N, self.D, self.Bs, self.Cq, self.Ck, self.r, self.k2, sc, int(self.frozen_weights),
                  int(self.dipole), None if Kw is None else Kw.ctypes.data)

    @property
    def nb(self) -> int:
        return self.N // self.Bs

    @property
    def k2e(self) -> int:
        return self.k2 if self.k2 > 0 else max(self.nb - 1, 1)


def _L():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_round_bf16.restype = C.c_double
        _lib.oracle_round_bf16.argtypes = [C.c_double]
        _lib.oracle_round_fp16.restype = C.c_double
        _lib.oracle_round_fp16.argtypes = [C.c_double]
        _lib.oracle_muse_fwd.restype = C.c_int
        _lib.oracle_muse_bwd.restype = C.c_int
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _rows(rows):
    if rows is None:
        return None, 0, None
    r, rp = _i(rows)
    return r, int(r.size), rp


def round_bf16(x):
    """Round-to-nearest-even to bfloat16, returned as float64 (vectorised)."""
    f = np.asarray(x, dtype=np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64).reshape(f.shape)


def exact_fwd(Q, K, V, scale, rows=None):
    Q, Qp = _d(Q); K, Kp = _d(K); V, Vp = _d(V)
    N, D = Q.shape
    O = np.zeros((N, D)); LSE = np.zeros(N)
    r, nr, rp = _rows(rows)
    _L().oracle_exact_fwd(C.c_int(N), C.c_int(D), C.c_double(scale), Qp, Kp, Vp, C.c_int(nr), rp,
                          _d(O)[1], _d(LSE)[1])
    return O, LSE


def exact_bwd(Q, K, V, O, LSE, dO, scale, rows=None):
    Q, Qp = _d(Q); K, Kp = _d(K); V, Vp = _d(V); O, Op = _d(O); LSE, Lp = _d(LSE); dO, gp = _d(dO)
    N, D = Q.shape
    dQ = np.zeros((N, D)); dK = np.zeros((N, D)); dV = np.zeros((N, D))
    r, nr, rp = _rows(rows)
    _L().oracle_exact_bwd(C.c_int(N), C.c_int(D), C.c_double(scale), Qp, Kp, Vp, Op, Lp, gp,
                          C.c_int(nr), rp, _d(dQ)[1], _d(dK)[1], _d(dV)[1])
    return dQ, dK, dV


def kmeans(X, Cn, T, init_idx=None, cent0=None, round_mode=0):
    """Lloyd K-means, T iterations + final assignment.

    round_mode 0: centroids scored as binary32; 1: rounded to bfloat16 for scoring.
    Returns dict(cent [C,D] (binary32 values), assign, margin (relative), counts, objective[T+1]).
    """
    X, Xp = _d(X)
    N, D = X.shape
    cent = np.zeros((Cn, D)) if cent0 is None else np.array(cent0, dtype=np.float64, copy=True)
    assign = np.zeros(N, dtype=np.int32); margin = np.zeros(N)
    counts = np.zeros(Cn, dtype=np.int32); obj = np.zeros(T + 1)
    ip = None
    if init_idx is not None:
        ii, ip = _i(init_idx)
    else:
        assert cent0 is not None
    _L().oracle_kmeans(C.c_int(N), C.c_int(D), C.c_int(Cn), C.c_int(T), C.c_int(round_mode), Xp, ip,
                       _d(cent)[1], _i(assign)[1], _d(margin)[1], _i(counts)[1], _d(obj)[1])
    return dict(cent=cent, assign=assign, margin=margin, counts=counts, objective=obj)


def round_fp16(x):
    """x rounded to IEEE binary16 (nearest even) by the oracle's own routine, elementwise."""
    f = _L().oracle_round_fp16
    return np.array([f(float(v)) for v in np.asarray(x, dtype=np.float64).ravel()]).reshape(np.shape(x))


def kmeans_stream(X, Cn, init_idx, mb=64, beta=0.9, forced=None):
    """Streaming centroid pass of App. C "Centroid Computation" (one pass, minibatches of mb rows).

    forced [N]: assignments to follow instead of the nearest centroid (regret reports how far each is from
    the best).  Returns dict(cent [C,D], t [C,D], c [C], assign [N] (as taken during the pass),
    margin [N], regret [N])."""
    X, Xp = _d(X)
    N, D = X.shape
    cent = np.zeros((Cn, D)); t = np.zeros((Cn, D)); c = np.zeros(Cn)
    assign = np.zeros(N, dtype=np.int32); margin = np.zeros(N); regret = np.zeros(N)
    ii, ip = _i(init_idx)
    fp = None
    if forced is not None:
        ff, fp = _i(forced)
    _L().oracle_kmeans_stream(C.c_int(N), C.c_int(D), C.c_int(Cn), C.c_int(mb), C.c_double(beta), Xp, ip, fp,
                              _d(cent)[1], _d(t)[1], _d(c)[1], _i(assign)[1], _d(margin)[1], _d(regret)[1])
    return dict(cent=cent, t=t, c=c, assign=assign, margin=margin, regret=regret)


def balanced_assign(X, cent, Bs, cap, round_mode=0, forced=None, tol=1e-5):
    """Final assignment under the per-block cap of App. C "Balanced Assignment" (two phases in position order).
    forced: replay along this assignment and check it.  Returns dict(assign, regret, broken)."""
    X, Xp = _d(X); cent, cp = _d(cent)
    N, D = X.shape
    Cn = cent.shape[0]
    assert Cn * cap >= min(Bs, N), "the cap leaves no room for every row of a block"
    assign = np.zeros(N, dtype=np.int32); rep = np.zeros(2)
    fp = None
    if forced is not None:
        ff, fp = _i(forced)
    _L().oracle_balanced_assign(C.c_int(N), C.c_int(D), C.c_int(Cn), C.c_int(Bs), C.c_int(cap), C.c_int(round_mode),
                                Xp, cp, fp, C.c_double(tol), _i(assign)[1], _d(rep)[1])
    return dict(assign=assign, regret=float(rep[0]), broken=int(rep[1]))


def summaries(p: MuseParams, K, V, qc, ak, i):
    """Per-block and accumulated summaries of query cluster i, each [Ck, nb(, D)]."""
    K, Kp = _d(K); V, Vp = _d(V); qc, qp = _d(qc); ak, ap = _i(ak)
    nb = p.nb
    mu = np.zeros((p.Ck, nb)); kb = np.zeros((p.Ck, nb, p.D)); vb = np.zeros((p.Ck, nb, p.D))
    Amu = np.zeros((p.Ck, nb)); Akb = np.zeros((p.Ck, nb, p.D)); Avb = np.zeros((p.Ck, nb, p.D))
    pc = p.c()
    _L().oracle_summaries(C.byref(pc), Kp, Vp, qp, ap, C.c_int(i), _d(mu)[1], _d(kb)[1], _d(vb)[1],
                          _d(Amu)[1], _d(Akb)[1], _d(Avb)[1])
    return dict(mu=mu, kb=kb, vb=vb, Amu=Amu, Akb=Akb, Avb=Avb)


def muse_fwd(p: MuseParams, Q, K, V, qc, aq, ak, rows=None, sel=None, weight_keys=None):
    """MuSe forward.  sel = (selc [N,r], selb [N,r,k2e]) teacher-forces the selections.
    weight_keys: keys used inside the tilted weights of the summaries instead of K (for the pins).
    margin_c / margin_b [N]: relative gap between the last selected and the best left-out cluster score /
    the smallest such gap over the row's block selections (+inf when nothing is left out).  With sel given
    they are the slack of THAT selection by the same formula: negative when a better candidate was left out,
    -inf when the selection is malformed (out of range, repeated, not a candidate, too few entries)."""
    Q, Qp = _d(Q); K, Kp = _d(K); V, Vp = _d(V); qc, qp = _d(qc)
    Kw = None if weight_keys is None else np.ascontiguousarray(weight_keys, dtype=np.float64)
    aq, aqp = _i(aq); ak, akp = _i(ak)
    N, D = Q.shape
    O = np.zeros((N, D)); LSE = np.zeros(N)
    if sel is None:
        selc = np.full((N, max(p.r, 1)), -1, dtype=np.int32)[:, : p.r]
        selc = np.ascontiguousarray(selc)
        selb = np.full((N, p.r, p.k2e), -1, dtype=np.int32)
        given = 0
    else:
        selc = np.array(sel[0], dtype=np.int32, copy=True).reshape(N, p.r)
        selb = np.array(sel[1], dtype=np.int32, copy=True).reshape(N, p.r, p.k2e)
        given = 1
    mc = np.full(N, np.inf); mb = np.full(N, np.inf); mass = np.zeros((N, 4))
    r, nr, rp = _rows(rows)
    pc = p.c(Kw)
    rc = _L().oracle_muse_fwd(C.byref(pc), Qp, Kp, Vp, qp, aqp, akp, C.c_int(nr), rp, C.c_int(given),
                              _d(O)[1], _d(LSE)[1], _i(selc)[1], _i(selb)[1], _d(mc)[1], _d(mb)[1],
                              _d(mass)[1])
    if rc == -2:
        raise ValueError("the dipole correction is defined for the monopole-only mode (r = 0)")
    assert rc == 0
    return dict(O=O, LSE=LSE, selc=selc, selb=selb, margin_c=mc, margin_b=mb, mass=mass)


def muse_bwd(p: MuseParams, Q, K, V, qc, aq, ak, O, LSE, dO, selc, selb, rows=None):
    Q, Qp = _d(Q); K, Kp = _d(K); V, Vp = _d(V); qc, qp = _d(qc)
    aq, aqp = _i(aq); ak, akp = _i(ak)
    O, Op = _d(O); LSE, Lp = _d(LSE); dO, gp = _d(dO)
    selc, scp = _i(selc); selb, sbp = _i(selb)
    N, D = Q.shape
    dQ = np.zeros((N, D)); dK = np.zeros((N, D)); dV = np.zeros((N, D))
    r, nr, rp = _rows(rows)
    pc = p.c()
    rc = _L().oracle_muse_bwd(C.byref(pc), Qp, Kp, Vp, qp, aqp, akp, C.c_int(nr), rp, Op, Lp, gp,
                              scp, sbp, _d(dQ)[1], _d(dK)[1], _d(dV)[1])
    assert rc == 0
    return dQ, dK, dV
