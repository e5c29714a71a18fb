"""One small end-to-end pass on cuda:0 through the C ABI, checked against the CPU oracle.

Used by __graft_entry__.smoke().  The oracle is test infrastructure: it is imported here for the
check only and is never on the product path.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as mb
from .inputs import generate, small


def run_small_case(verbose: bool = False) -> dict:
    import oracle as orc

    if not torch.cuda.is_available():
        raise RuntimeError("smoke() needs a GPU")
    mb.load()
    w = small("cfg2", N=1024, Hq=2, Hkv=1, Cq=8, Ck=32, r=3, block=128, kmeans_iters=3)
    d = generate(w, need_dO=True)
    p = mb.params_for(w)
    Q, K, V, dO = (d[x].to(p.torch_dtype).cuda().contiguous() for x in ("Q", "K", "V", "dO"))
    qc, qa, kc, ka = mb.muse_cluster(p, Q, K, d["q_init_idx"].cuda(), d["k_init_idx"].cuda())
    O, LSE, selc, selb = mb.muse_fwd(p, Q, K, V, qc, qa, ka)
    dQ, dK, dV = mb.muse_bwd(p, Q, K, V, O, LSE, dO, qc, qa, ka, selc, selb)
    torch.cuda.synchronize()
    op = orc.MuseParams(w.N, w.D, w.Bs, w.Cq, w.Ck, w.r, w.k2, p.eff_scale)
    G = w.Hq // w.Hkv
    errs = {}
    wantK = np.zeros((w.Hkv, w.N, w.D)); wantV = np.zeros((w.Hkv, w.N, w.D))
    f64 = lambda t: t.float().cpu().double().numpy()
    for h in range(w.Hq):
        q, k, v, g = f64(Q[0, h]), f64(K[0, h // G]), f64(V[0, h // G]), f64(dO[0, h])
        # nearest-centroid assignment of the GPU must be the oracle's for the GPU's centroids
        chk = orc.kmeans(q, w.Cq, 0, cent0=f64(qc[0, h]), round_mode=1)
        safe = chk["margin"] > 1e-5
        assert (qa[0, h].cpu().numpy()[safe] == chk["assign"][safe]).all(), "assignment mismatch"
        sc, sb = selc[0, h].cpu().numpy(), selb[0, h].cpu().numpy()
        free = orc.muse_fwd(op, q, k, v, f64(qc[0, h]), qa[0, h].cpu().numpy(), ka[0, h // G].cpu().numpy())
        ok = free["margin_c"] > 1e-5
        assert (np.sort(sc[ok], 1) == np.sort(free["selc"][ok], 1)).all(), "retrieved clusters mismatch"
        forced = orc.muse_fwd(op, q, k, v, f64(qc[0, h]), qa[0, h].cpu().numpy(), ka[0, h // G].cpu().numpy(), sel=(sc, sb))
        gq, gk, gv = orc.muse_bwd(op, q, k, v, f64(qc[0, h]), qa[0, h].cpu().numpy(), ka[0, h // G].cpu().numpy(),
                                  forced["O"], forced["LSE"], g, sc, sb)
        errs[f"O{h}"] = np.abs(f64(O[0, h]) - forced["O"]).max()
        errs[f"dQ{h}"] = np.abs(f64(dQ[0, h]) - gq).max() / max(1.0, np.abs(gq).max())
        wantK[h // G] += gk; wantV[h // G] += gv
    for hk in range(w.Hkv):
        errs[f"dK{hk}"] = np.abs(f64(dK[0, hk]) - wantK[hk]).max() / max(1.0, np.abs(wantK[hk]).max())
        errs[f"dV{hk}"] = np.abs(f64(dV[0, hk]) - wantV[hk]).max() / max(1.0, np.abs(wantV[hk]).max())
    worst = max(errs.values())
    if verbose:
        print("smoke: max errors vs oracle:", {k: f"{v:.2e}" for k, v in errs.items()})
    assert worst <= 2e-2, errs
    return errs
