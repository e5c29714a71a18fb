"""Seeded synthetic workloads (host side, no method arithmetic in here).

The paper measures on activations of its own trained models; none of those
are available, so these generators stand in for them, keeping only the shapes
(heads, head dim, sequence length, GQA ratio) and the coarse structure
(clustered representations, non-zero query mean, rotary phase).

Every tensor is drawn on the host in float32 from a seeded generator, rounded
once to the storage type and returned as float32 holding exactly those rounded
values, so the CPU oracle and the GPU library see identical inputs.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import torch


@dataclass
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    N: int
    D: int
    Cq: int
    Ck: int
    r: int
    dtype: str  # "fp32" | "bf16"
    k2: int = 1
    block: int = 0  # 0 -> N // 8
    kmeans_iters: int = 10
    backward: bool = True
    gen: str = "mixture"  # "mixture" | "embed" | "lowrank_rope"
    gen_args: dict = field(default_factory=dict)
    seed: int = 1000

    @property
    def Bs(self) -> int:
        return self.block if self.block else self.N // 8

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)


CONFIGS = {
    "cfg1": Workload("cfg1", 1, 1, 1, 2048, 64, 16, 32, 2, "fp32", backward=False, gen="mixture",
                     gen_args=dict(components=16, sd=0.3), seed=1001),
    "cfg2": Workload("cfg2", 1, 8, 8, 16384, 64, 64, 256, 4, "bf16", gen="embed",
                     gen_args=dict(embed=512, components=256, sd=0.3), seed=1002),
    "cfg3": Workload("cfg3", 1, 16, 16, 65536, 64, 256, 1024, 8, "bf16", gen="embed",
                     gen_args=dict(embed=1024, components=1024, sd=0.3), seed=1003),
    "cfg4": Workload("cfg4", 1, 32, 8, 65536, 64, 256, 1024, 8, "bf16", gen="lowrank_rope",
                     gen_args=dict(rank=16, amp=2.0, base=1.0e5), seed=1004),
    "cfg5": Workload("cfg5", 1, 32, 8, 131072, 128, 512, 2048, 16, "bf16", gen="lowrank_rope",
                     gen_args=dict(rank=32, amp=2.0, base=1.0e5), seed=1005),
    # the paper's operating ratio C = N/512 at the shape of cfg3 (Sec. 4: 128 query and 128 key clusters, 8
    # retrieved clusters, 8 blocks of 8k): about 64 keys per retrieved (cluster, block) pair
    "cfg3_qk128": Workload("cfg3_qk128", 1, 16, 16, 65536, 64, 128, 128, 8, "bf16", gen="embed",
                           gen_args=dict(embed=1024, components=1024, sd=0.3), seed=1003),
}


def small(name: str, **kw) -> Workload:
    """A reduced copy of a named config (same generator, smaller sizes) for tests."""
    import dataclasses

    return dataclasses.replace(CONFIGS[name], **kw)


def _round(x: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return x.to(torch.bfloat16).to(torch.float32)
    return x.to(torch.float32)


def _mixture(g, n, dim, components, sd):
    centres = torch.randn(components, dim, generator=g)
    comp = torch.randint(0, components, (n,), generator=g)
    return centres[comp] + sd * torch.randn(n, dim, generator=g), comp


def _rope(x: torch.Tensor, base: float) -> torch.Tensor:
    """Rotary phase at position n on pairs (2t, 2t+1), theta_t = base^(-2t/D).  x: [H, N, D]."""
    H, N, D = x.shape
    t = torch.arange(D // 2, dtype=torch.float64)
    theta = base ** (-2.0 * t / D)
    ang = torch.arange(N, dtype=torch.float64)[:, None] * theta[None, :]
    cs, sn = torch.cos(ang).float(), torch.sin(ang).float()
    xe, xo = x[..., 0::2], x[..., 1::2]
    out = torch.empty_like(x)
    out[..., 0::2] = xe * cs - xo * sn
    out[..., 1::2] = xe * sn + xo * cs
    return out


def generate(w: Workload, need_dO: bool | None = None):
    """Returns dict of float32 CPU tensors: Q [B,Hq,N,D], K,V [B,Hkv,N,D], dO [B,Hq,N,D],
    q_init_idx [B,Hq,Cq] int32, k_init_idx [B,Hkv,Ck] int32, labels (mixture generators)."""
    g = torch.Generator().manual_seed(w.seed)
    B, Hq, Hkv, N, D = w.B, w.Hq, w.Hkv, w.N, w.D
    out = {}
    if w.gen == "mixture":
        a = w.gen_args
        Q = torch.empty(B, Hq, N, D); K = torch.empty(B, Hkv, N, D)
        lq = torch.empty(B, Hq, N, dtype=torch.int64); lk = torch.empty(B, Hkv, N, dtype=torch.int64)
        for b in range(B):
            for h in range(Hkv):
                K[b, h], lk[b, h] = _mixture(g, N, D, a["components"], a["sd"])
            for h in range(Hq):
                Q[b, h], lq[b, h] = _mixture(g, N, D, a["components"], a["sd"])
        V = torch.randn(B, Hkv, N, D, generator=g)
        out["q_labels"], out["k_labels"] = lq, lk
    elif w.gen == "embed":
        a = w.gen_args
        E = a["embed"]
        Q = torch.empty(B, Hq, N, D); K = torch.empty(B, Hkv, N, D)
        for b in range(B):
            emb, _ = _mixture(g, N, E, a["components"], a["sd"])
            Wq = torch.randn(E, Hq * D, generator=g) / math.sqrt(E)
            Wk = torch.randn(E, Hkv * D, generator=g) / math.sqrt(E)
            Q[b] = (emb @ Wq).view(N, Hq, D).permute(1, 0, 2)
            K[b] = (emb @ Wk).view(N, Hkv, D).permute(1, 0, 2)
        V = torch.randn(B, Hkv, N, D, generator=g)
    elif w.gen == "lowrank_rope":
        a = w.gen_args

        def lowrank(H):
            x = torch.empty(B, H, N, D)
            for b in range(B):
                for h in range(H):
                    U, _ = torch.linalg.qr(torch.randn(D, a["rank"], generator=g))
                    coef = torch.randn(N, a["rank"], generator=g)
                    x[b, h] = torch.randn(N, D, generator=g) + a["amp"] * coef @ U.T
            return x

        Q = lowrank(Hq); K = lowrank(Hkv); V = lowrank(Hkv)
        for b in range(B):
            Q[b] = _rope(Q[b], a["base"])
            K[b] = _rope(K[b], a["base"])
    else:
        raise ValueError(w.gen)
    out["Q"], out["K"], out["V"] = _round(Q, w.dtype), _round(K, w.dtype), _round(V, w.dtype)
    if need_dO if need_dO is not None else w.backward:
        out["dO"] = _round(torch.randn(B, Hq, N, D, generator=g), w.dtype)
    out["q_init_idx"] = init_indices(g, B, Hq, N, w.Cq)
    out["k_init_idx"] = init_indices(g, B, Hkv, N, w.Ck)
    return out


def init_indices(g: torch.Generator, B: int, H: int, N: int, C: int) -> torch.Tensor:
    """Seeded shuffle of the positions, then every floor(N/C)-th one (App. C initialisation)."""
    idx = torch.empty(B, H, C, dtype=torch.int32)
    stride = N // C
    for b in range(B):
        for h in range(H):
            perm = torch.randperm(N, generator=g)
            idx[b, h] = perm[torch.arange(C) * stride].to(torch.int32)
    return idx
