"""ctypes binding of libmuse.so: argument marshalling only.

Same names as the C ABI (include/muse.h).  PyTorch supplies device memory and the
stream; every step of the path runs in the library's kernels.  There is no
fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import math
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmuse.so")
_lib = None

FP32, BF16 = 0, 1
FLAG_KEEP_FWD_STATE = 1
FLAG_FROZEN_WEIGHTS = 2
FLAG_STREAMING_KMEANS = 4
FLAG_BALANCED_ASSIGN = 8
FLAG_DIPOLE = 16
WS_CLUSTER, WS_FWD, WS_BWD, WS_EXACT_FWD, WS_EXACT_BWD = range(5)
SYMBOLS = ["muse_workspace_bytes", "muse_cluster", "muse_kmeans_stream", "muse_fwd", "muse_bwd", "exact_attn_fwd", "exact_attn_bwd",
           "exact_attn_bwd_static", "muse_profile_enable", "muse_profile_report", "muse_probe_peaks", "muse_strerror"]
STATIC_SCRATCH_BYTES = 64 << 20


class MuseError(RuntimeError):
    pass


class _Params(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("B", "Hq", "Hkv", "N", "D", "Cq", "Ck", "r", "k2", "block", "kmeans_iters", "dtype", "grad_dtype",
                 "causal")] + [("flags", C.c_uint32), ("scale", C.c_float)]


@dataclass
class Params:
    B: int
    Hq: int
    Hkv: int
    N: int
    D: int
    Cq: int = 1
    Ck: int = 1
    r: int = 0
    k2: int = 1
    block: int = 0
    kmeans_iters: int = 10
    dtype: int = BF16
    grad_dtype: int = FP32
    causal: int = 1
    flags: int = 0
    scale: float = 0.0

    def c(self) -> _Params:
        return _Params(self.B, self.Hq, self.Hkv, self.N, self.D, self.Cq, self.Ck, self.r, self.k2, self.block,
                       self.kmeans_iters, self.dtype, self.grad_dtype, self.causal, self.flags, self.scale)

    @property
    def Bs(self) -> int:
        return self.block if self.block else self.N // 8

    @property
    def nb(self) -> int:
        return self.N // self.Bs

    @property
    def k2e(self) -> int:
        return self.k2 if self.k2 > 0 else max(self.nb - 1, 1)

    @property
    def eff_scale(self) -> float:
        return self.scale if self.scale > 0 else 1.0 / math.sqrt(self.D)

    @property
    def torch_dtype(self):
        return torch.bfloat16 if self.dtype == BF16 else torch.float32

    @property
    def torch_grad_dtype(self):
        return torch.bfloat16 if self.grad_dtype == BF16 else torch.float32


def load():
    """Loads libmuse.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MuseError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        lib = C.CDLL(LIB_PATH)
        lib.muse_strerror.restype = C.c_char_p
        lib.muse_strerror.argtypes = [C.c_int]
        for n in SYMBOLS[:-1]:
            getattr(lib, n).restype = C.c_int
        _lib = lib
    return _lib


def muse_strerror(code: int) -> str:
    return load().muse_strerror(code).decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise MuseError(f"{what}: {muse_strerror(rc)} ({rc})")


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def muse_workspace_bytes(p: Params, which: int):
    mn, pref = C.c_size_t(0), C.c_size_t(0)
    pc = p.c()
    _check(load().muse_workspace_bytes(C.byref(pc), C.c_int(which), C.byref(mn), C.byref(pref)), "muse_workspace_bytes")
    return mn.value, pref.value


_ws_cache: dict = {}


def workspace(p: Params, which: int, device="cuda", limit_bytes: int | None = None) -> torch.Tensor:
    """A cached uint8 device buffer of the preferred size (capped by limit_bytes, never below the minimum)."""
    mn, pref = muse_workspace_bytes(p, which)
    size = pref if limit_bytes is None else max(mn, min(pref, limit_bytes))
    # under MUSE_FLAG_KEEP_FWD_STATE the backward must be handed the very buffer the forward filled
    shared = (p.flags & FLAG_KEEP_FWD_STATE) and which in (WS_FWD, WS_BWD)
    device = torch.device(device)
    if device.index is None:   # "cuda" and "cuda:<current>" are one device: one buffer
        device = torch.device(device.type, torch.cuda.current_device())
    key = (str(device), "fwd+bwd" if shared else which)
    buf = _ws_cache.get(key)
    if buf is None or buf.numel() < size:
        _ws_cache.pop(key, None)
        buf = torch.empty(size, dtype=torch.uint8, device=device)
        _ws_cache[key] = buf
    return buf


def free_workspaces():
    _ws_cache.clear()


def muse_cluster(p: Params, Q, K, q_init_idx, k_init_idx, q_centroids=None, k_centroids=None, ws=None):
    """Returns (q_centroids, q_assign, k_centroids, k_assign); a side is skipped when its tensor is None."""
    dev = (Q if Q is not None else K).device
    ws = ws if ws is not None else workspace(p, WS_CLUSTER, dev)
    qa = ka = None
    if Q is not None:
        if q_centroids is None:
            q_centroids = torch.empty(p.B, p.Hq, p.Cq, p.D, dtype=torch.float32, device=dev)
        qa = torch.empty(p.B, p.Hq, p.N, dtype=torch.int32, device=dev)
    if K is not None:
        if k_centroids is None:
            k_centroids = torch.empty(p.B, p.Hkv, p.Ck, p.D, dtype=torch.float32, device=dev)
        ka = torch.empty(p.B, p.Hkv, p.N, dtype=torch.int32, device=dev)
    pc = p.c()
    _check(load().muse_cluster(C.byref(pc), _ptr(Q), _ptr(K), _ptr(q_init_idx), _ptr(k_init_idx), _ptr(q_centroids),
                               _ptr(qa), _ptr(k_centroids), _ptr(ka), _ptr(ws), C.c_size_t(ws.numel()), _stream()),
           "muse_cluster")
    return q_centroids, qa, k_centroids, ka


def muse_kmeans_stream(p: Params, side: int, X, init_idx, centroids=None, ws=None):
    """The streaming centroid pass alone.  side 0: query rows, 1: key rows.
    Returns (centroids, stream_assign, counts)."""
    dev = X.device
    H, Cn = (p.Hkv, p.Ck) if side else (p.Hq, p.Cq)
    ws = ws if ws is not None else workspace(p, WS_CLUSTER, dev)
    if centroids is None:
        centroids = torch.empty(p.B, H, Cn, p.D, dtype=torch.float32, device=dev)
    sa = torch.empty(p.B, H, p.N, dtype=torch.int32, device=dev)
    cnt = torch.empty(p.B, H, Cn, dtype=torch.float32, device=dev)
    pc = p.c()
    _check(load().muse_kmeans_stream(C.byref(pc), C.c_int(side), _ptr(X), _ptr(init_idx), _ptr(centroids), _ptr(sa),
                                     _ptr(cnt), _ptr(ws), C.c_size_t(ws.numel()), _stream()), "muse_kmeans_stream")
    return centroids, sa, cnt


def muse_fwd(p: Params, Q, K, V, q_centroids, q_assign, k_assign, ws=None, out=None):
    """Returns (O, LSE, sel_clusters, sel_blocks)."""
    dev = Q.device
    ws = ws if ws is not None else workspace(p, WS_FWD, dev)
    if out is None:
        O = torch.empty(p.B, p.Hq, p.N, p.D, dtype=p.torch_dtype, device=dev)
        LSE = torch.empty(p.B, p.Hq, p.N, dtype=torch.float32, device=dev)
        selc = torch.empty(p.B, p.Hq, p.N, max(p.r, 1), dtype=torch.int32, device=dev)
        selb = torch.empty(p.B, p.Hq, p.N, max(p.r, 1), p.k2e, dtype=torch.int32, device=dev)
    else:
        O, LSE, selc, selb = out
    pc = p.c()
    _check(load().muse_fwd(C.byref(pc), _ptr(Q), _ptr(K), _ptr(V), _ptr(q_centroids), _ptr(q_assign), _ptr(k_assign),
                           _ptr(O), _ptr(LSE), _ptr(selc), _ptr(selb), _ptr(ws), C.c_size_t(ws.numel()), _stream()),
           "muse_fwd")
    return O, LSE, selc, selb


def muse_bwd(p: Params, Q, K, V, O, LSE, dO, q_centroids, q_assign, k_assign, sel_clusters, sel_blocks, ws=None,
             out=None):
    """Returns (dQ, dK, dV)."""
    dev = Q.device
    ws = ws if ws is not None else workspace(p, WS_BWD, dev)
    if out is None:
        dQ = torch.empty(p.B, p.Hq, p.N, p.D, dtype=p.torch_grad_dtype, device=dev)
        dK = torch.empty(p.B, p.Hkv, p.N, p.D, dtype=p.torch_grad_dtype, device=dev)
        dV = torch.empty(p.B, p.Hkv, p.N, p.D, dtype=p.torch_grad_dtype, device=dev)
    else:
        dQ, dK, dV = out
    pc = p.c()
    _check(load().muse_bwd(C.byref(pc), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO), _ptr(q_centroids),
                           _ptr(q_assign), _ptr(k_assign), _ptr(sel_clusters), _ptr(sel_blocks), _ptr(dQ), _ptr(dK),
                           _ptr(dV), _ptr(ws), C.c_size_t(ws.numel()), _stream()), "muse_bwd")
    return dQ, dK, dV


def exact_attn_fwd(p: Params, Q, K, V, ws=None, out=None):
    """Returns (O, LSE)."""
    dev = Q.device
    ws = ws if ws is not None else workspace(p, WS_EXACT_FWD, dev)
    if out is None:
        O = torch.empty(p.B, p.Hq, p.N, p.D, dtype=p.torch_dtype, device=dev)
        LSE = torch.empty(p.B, p.Hq, p.N, dtype=torch.float32, device=dev)
    else:
        O, LSE = out
    pc = p.c()
    _check(load().exact_attn_fwd(C.byref(pc), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(ws),
                                 C.c_size_t(ws.numel()), _stream()), "exact_attn_fwd")
    return O, LSE


def exact_attn_bwd(p: Params, Q, K, V, O, LSE, dO, ws=None, out=None):
    """Returns (dQ, dK, dV)."""
    dev = Q.device
    ws = ws if ws is not None else workspace(p, WS_EXACT_BWD, dev)
    if out is None:
        dQ = torch.empty(p.B, p.Hq, p.N, p.D, dtype=p.torch_grad_dtype, device=dev)
        dK = torch.empty(p.B, p.Hkv, p.N, p.D, dtype=p.torch_grad_dtype, device=dev)
        dV = torch.empty(p.B, p.Hkv, p.N, p.D, dtype=p.torch_grad_dtype, device=dev)
    else:
        dQ, dK, dV = out
    pc = p.c()
    _check(load().exact_attn_bwd(C.byref(pc), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO), _ptr(dQ),
                                 _ptr(dK), _ptr(dV), _ptr(ws), C.c_size_t(ws.numel()), _stream()), "exact_attn_bwd")
    return dQ, dK, dV


def exact_attn_bwd_static(p: Params, Q, K, V, O, LSE, dO, out):
    """exact_attn_bwd on the library's static scratch: no workspace, nothing allocated by the call.
    out = (dQ, dK, dV), allocated by the caller beforehand."""
    dQ, dK, dV = out
    pc = p.c()
    _check(load().exact_attn_bwd_static(C.byref(pc), _ptr(Q), _ptr(K), _ptr(V), _ptr(O), _ptr(LSE), _ptr(dO), _ptr(dQ),
                                        _ptr(dK), _ptr(dV), _stream()), "exact_attn_bwd_static")
    return dQ, dK, dV


def muse_profile_enable(on: bool):
    _check(load().muse_profile_enable(C.c_int(1 if on else 0)), "muse_profile_enable")


def muse_profile_report() -> dict:
    """{kernel name: (launches, total ms)} of everything launched since muse_profile_enable(True)."""
    buf = C.create_string_buffer(1 << 16)
    _check(load().muse_profile_report(buf, C.c_size_t(len(buf))), "muse_profile_report")
    out = {}
    for line in buf.value.decode().splitlines():
        name, cnt, ms = line.split()
        out[name] = (int(cnt), float(ms))
    return out


def muse_probe_peaks(buf) -> dict:
    """{"copy_GBps", "mfma_bf16_TFLOPs"}: what a plain copy inside the device tensor `buf` (>= 1 GiB, overwritten) and
    a loop of independent bf16 MFMAs reach on this device."""
    gbps, tfl = C.c_double(0.0), C.c_double(0.0)
    _check(load().muse_probe_peaks(_ptr(buf), C.c_size_t(buf.numel() * buf.element_size()), C.byref(gbps), C.byref(tfl),
                                   _stream()), "muse_probe_peaks")
    return {"copy_GBps": gbps.value, "mfma_bf16_TFLOPs": tfl.value}


def params_for(w, **kw) -> Params:
    """Params of a workload from paper_2509_10406_amd.inputs."""
    d = dict(B=w.B, Hq=w.Hq, Hkv=w.Hkv, N=w.N, D=w.D, Cq=w.Cq, Ck=w.Ck, r=w.r, k2=w.k2, block=w.block,
             kmeans_iters=w.kmeans_iters, dtype=BF16 if w.dtype == "bf16" else FP32, grad_dtype=FP32)
    d.update(kw)
    return Params(**d)
