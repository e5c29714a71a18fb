"""GPU parity of muse_fwd / muse_bwd against the CPU oracle, through the C ABI.

The clustering handed to both sides is the oracle's (teacher forcing: one near-tie flip upstream
must not invalidate every downstream comparison).  Selections are compared as sets wherever the
oracle's relative score margin exceeds 1e-5; outputs and gradients are then compared against the
oracle evaluated at the GPU's own selections (identical to the oracle's except at sub-margin ties).
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle as orc
from paper_2509_10406_amd import binding as mb
from paper_2509_10406_amd.inputs import generate, small
from tests.util import assert_close, blocks_by_cluster, dev, f64, oracle_head, segment_sizes

pytestmark = pytest.mark.gpu
MARGIN = 1e-5

CASES = {
    "cfg1_full": ("cfg1", {}),
    "cfg1_k2all": ("cfg1", dict(N=1024, k2=0, block=128, kmeans_iters=3)),
    "cfg1_r0": ("cfg1", dict(N=512, r=0, block=64, kmeans_iters=2)),
    "cfg1_k2_2_ragged": ("cfg1", dict(N=768, Cq=5, Ck=19, r=3, k2=2, block=96, kmeans_iters=2)),
    "cfg2_small": ("cfg2", dict(N=2048, Hq=2, Hkv=2, Cq=16, Ck=64, r=4, block=256, kmeans_iters=3)),
    "cfg4_gqa": ("cfg4", dict(N=1024, Hq=4, Hkv=2, Cq=8, Ck=40, r=3, block=128, kmeans_iters=2)),
    "cfg5_d128": ("cfg5", dict(N=1024, Hq=2, Hkv=1, Cq=8, Ck=33, r=9, block=128, kmeans_iters=2)),
    "bf16_one_block": ("cfg2", dict(N=512, Hq=1, Hkv=1, Cq=4, Ck=8, r=2, block=512, kmeans_iters=1)),
    "bf16_r17": ("cfg2", dict(N=1024, Hq=1, Hkv=1, Cq=4, Ck=70, r=17, block=128, kmeans_iters=1)),
    # more than 8 preceding blocks: the second chunk of the block loops
    "bf16_nb16_k2_2": ("cfg2", dict(N=2048, Hq=2, Hkv=1, Cq=8, Ck=32, r=3, k2=2, block=128, kmeans_iters=2)),
    "fp32_nb12": ("cfg1", dict(N=1536, Cq=6, Ck=24, r=2, block=128, kmeans_iters=2)),
    # bf16 with a block size that is not a multiple of the 128-row tiles of the block-diagonal kernels
    "bf16_block96": ("cfg2", dict(N=768, Hq=2, Hkv=1, Cq=5, Ck=19, r=3, k2=2, block=96, kmeans_iters=2)),
    # the ratio of Sec. 3.3 "Complexity" (clusters = N / 512: about 64 keys per retrieved pair), where the pair
    # kernels walk several 32-key tiles per pair, and query groups of several staging passes / tiles
    "bf16_pairs64": ("cfg2", dict(N=4096, Hq=2, Hkv=1, Cq=4, Ck=8, r=2, block=512, kmeans_iters=2)),
    "bf16_pairs64_k2all": ("cfg2", dict(N=4096, Hq=2, Hkv=1, Cq=4, Ck=8, r=2, k2=0, block=512, kmeans_iters=2)),
    "bf16_groups200": ("cfg2", dict(N=4096, Hq=1, Hkv=1, Cq=2, Ck=12, r=3, k2=2, block=512, kmeans_iters=2)),
    "bf16_d128_pairs40": ("cfg5", dict(N=2048, Hq=2, Hkv=1, Cq=3, Ck=6, r=2, block=256, kmeans_iters=2)),
}


def oracle_clustering(w, d, p):
    rm = 1 if w.dtype == "bf16" else 0
    G = w.Hq // w.Hkv
    qc = np.zeros((w.B, w.Hq, w.Cq, w.D), np.float32)
    aq = np.zeros((w.B, w.Hq, w.N), np.int32)
    ak = np.zeros((w.B, w.Hkv, w.N), np.int32)
    for h in range(w.Hq):
        o = orc.kmeans(d["Q"][0, h].double().numpy(), w.Cq, w.kmeans_iters, init_idx=d["q_init_idx"][0, h].numpy(), round_mode=rm)
        qc[0, h], aq[0, h] = o["cent"], o["assign"]
    for h in range(w.Hkv):
        o = orc.kmeans(d["K"][0, h].double().numpy(), w.Ck, w.kmeans_iters, init_idx=d["k_init_idx"][0, h].numpy(), round_mode=rm)
        ak[0, h] = o["assign"]
    return qc, aq, ak


def as_sets(sel):
    s = np.sort(sel.reshape(sel.shape[0], -1), axis=1)
    return s


# What a case must reach, asserted inside the run so that a change of generator or sizes cannot silently take
# it off the code path it is there for: pair_keys = keys of the largest RETRIEVED (cluster, block) pair (the
# pair kernels tile keys by 32); group = queries of the largest (block, query cluster) group (the tile kernels
# take 32 per wave, the cell-gradient kernel stages 96 per pass at D = 64 and 32 at D = 128).
# pair_hits = (query, slot) entries of the most retrieved pair of a KV head (all query heads of the group): the
# key/value-gradient kernel of the retrieval shares a pair among several waves from 8 tiles of 32 hits on.
REACH = {
    "bf16_pairs64": dict(pair_keys=65, group=97, pair_hits=512),
    "bf16_pairs64_k2all": dict(pair_keys=65, group=97, pair_hits=1024),
    "bf16_groups200": dict(pair_keys=33, group=193),
    "bf16_d128_pairs40": dict(pair_keys=33, group=65),
}


def check_selections(name, h, w, op, got_c, got_b, free, forced):
    """Retrieved clusters and blocks of one head against the oracle: equal as sets where the oracle's margin
    allows a comparison; everywhere, the library's own choice must be a valid one (every chosen candidate
    scores within the margin of the best one left out: slack >= -MARGIN by the oracle's fp64 scores)."""
    far = np.arange(w.N) >= w.Bs
    safe_c = free["margin_c"] > MARGIN
    assert safe_c.mean() > 0.98, safe_c.mean()
    np.testing.assert_array_equal(as_sets(got_c)[safe_c], as_sets(free["selc"])[safe_c],
                                  err_msg=f"{name} head {h}: retrieved clusters")
    assert (forced["margin_c"] >= -MARGIN).all(), (name, h, "cluster choice off by", forced["margin_c"].min())
    assert (forced["margin_b"] >= -MARGIN).all(), (name, h, "block choice off by", forced["margin_b"].min())
    # blocks of every retrieved cluster, whatever the slot order, where both margins are safe
    safe = safe_c & (free["margin_b"] > MARGIN)
    assert not far.any() or safe[far].mean() > 0.95, safe[far].mean()
    np.testing.assert_array_equal(blocks_by_cluster(got_c, got_b)[safe],
                                  blocks_by_cluster(free["selc"], free["selb"])[safe],
                                  err_msg=f"{name} head {h}: retrieved blocks")
    # export order: descending score, so where the oracle's scores are well separated the slots agree too
    assert (got_c[~far] == -1).all() and (got_b[~far] == -1).all()


def run_case(name, with_bwd, frozen_weights=False, flags=0):
    base, kw = CASES[name]
    w = small(base, **kw)
    d = generate(w, need_dO=True)
    p = mb.params_for(w, flags=(mb.FLAG_FROZEN_WEIGHTS if frozen_weights else 0) | flags)
    qc, aq, ak = oracle_clustering(w, d, p)
    Q, K, V, dO = (dev(d[x], p) for x in ("Q", "K", "V", "dO"))
    qc_d, aq_d, ak_d = torch.tensor(qc).cuda(), torch.tensor(aq).cuda(), torch.tensor(ak).cuda()
    ws = None
    if flags & mb.FLAG_KEEP_FWD_STATE:
        ws = torch.empty(mb.muse_workspace_bytes(p, mb.WS_BWD)[1], dtype=torch.uint8, device="cuda")
    O, LSE, selc, selb = mb.muse_fwd(p, Q, K, V, qc_d, aq_d, ak_d, ws=ws)
    if with_bwd:
        dQ, dK, dV = mb.muse_bwd(p, Q, K, V, O, LSE, dO, qc_d, aq_d, ak_d, selc, selb, ws=ws)
    torch.cuda.synchronize()
    op = orc.MuseParams(w.N, w.D, w.Bs, w.Cq, w.Ck, w.r, w.k2, p.eff_scale, frozen_weights=frozen_weights)
    G = w.Hq // w.Hkv
    selc_h, selb_h = selc.cpu().numpy()[0], selb.cpu().numpy()[0]
    wantK = np.zeros((w.Hkv, w.N, w.D)); wantV = np.zeros((w.Hkv, w.N, w.D))
    reach = dict(pair_keys=0, group=0, pair_hits=0)
    hits = np.zeros((w.Hkv, max(w.N // w.Bs, 1), w.Ck), np.int64)
    for h in range(w.Hq):
        q, k, v, g = (f64(x) for x in (Q[0, h], K[0, h // G], V[0, h // G], dO[0, h]))
        sc = selc_h[h][:, : w.r]
        sb = selb_h[h][:, : w.r].reshape(w.N, w.r, op.k2e) if w.r else selb_h[h][:, :0].reshape(w.N, 0, op.k2e)
        res = oracle_head(orc, op, q, k, v, g, qc[0, h], aq[0, h], ak[0, h // G], (sc, sb), threads=8, with_bwd=with_bwd)
        free, forced, grads = res["free"], res["forced"], res["grads"]
        if name in ("cfg1_full", "cfg2_small"):
            # the far field must matter in these cases, or the parity below would say little about it
            far = free["mass"][w.Bs:, :3].sum(1)
            assert far.mean() > 0.2 and (free["mass"][w.Bs:, :3].mean(0) > 1e-3).all(), free["mass"][w.Bs:].mean(0)
        if w.r:
            check_selections(name, h, w, op, sc, sb, free, forced)
            keys = segment_sizes(ak[0, h // G], w.Bs, w.Ck)
            ok = (sc[:, :, None] >= 0) & (sb >= 0)
            if ok.any():
                np.add.at(hits[h // G], (sb[ok], np.broadcast_to(sc[:, :, None], sb.shape)[ok]), 1)
                reach["pair_keys"] = max(reach["pair_keys"], int(keys[sb[ok], np.broadcast_to(sc[:, :, None], sb.shape)[ok]].max()))
        if w.N > w.Bs:
            reach["group"] = max(reach["group"], int(segment_sizes(aq[0, h], w.Bs, w.Cq)[1:].max()))
        assert_close(f64(O[0, h]), forced["O"], p, f"{name} O head {h}")
        lse_tol = 1e-4 if w.dtype == "fp32" else 2e-2
        np.testing.assert_allclose(LSE[0, h].cpu().numpy(), forced["LSE"], rtol=0, atol=lse_tol * max(1, np.abs(forced["LSE"]).max()))
        if with_bwd:
            assert_close(f64(dQ[0, h]), grads[0], p, f"{name} dQ head {h}", grad=True)
            wantK[h // G] += grads[1]; wantV[h // G] += grads[2]
    reach["pair_hits"] = int(hits.max())
    for what, least in REACH.get(name, {}).items():
        assert reach[what] >= least, f"{name} no longer reaches {what} >= {least}: {reach}"
    if with_bwd:
        for hk in range(w.Hkv):
            assert_close(f64(dK[0, hk]), wantK[hk], p, f"{name} dK head {hk}", grad=True)
            assert_close(f64(dV[0, hk]), wantV[hk], p, f"{name} dV head {hk}", grad=True)
    return reach


@pytest.mark.parametrize("name", list(CASES))
def test_muse_forward(name):
    run_case(name, with_bwd=False)


@pytest.mark.parametrize("name", list(CASES))
def test_muse_backward(name):
    run_case(name, with_bwd=True)


@pytest.mark.parametrize("name", ["cfg1_full", "cfg2_small", "cfg4_gqa", "cfg5_d128", "fp32_nb12"])
def test_muse_backward_frozen_weights(name):
    """App. C "Aggregation Weight Gradient Flow", non-differentiable variant (MUSE_FLAG_FROZEN_WEIGHTS)."""
    run_case(name, with_bwd=True, frozen_weights=True)


def test_forward_with_small_workspace_chunks_heads():
    """The minimum workspace processes one KV group at a time; results must not change."""
    base, kw = CASES["cfg4_gqa"]
    w = small(base, **kw)
    d = generate(w)
    p = mb.params_for(w)
    qc, aq, ak = oracle_clustering(w, d, p)
    Q, K, V = (dev(d[x], p) for x in ("Q", "K", "V"))
    args = (p, Q, K, V, torch.tensor(qc).cuda(), torch.tensor(aq).cuda(), torch.tensor(ak).cuda())
    mn, pref = mb.muse_workspace_bytes(p, mb.WS_FWD)
    assert mn < pref
    a = mb.muse_fwd(*args, ws=torch.empty(pref, dtype=torch.uint8, device="cuda"))
    b = mb.muse_fwd(*args, ws=torch.empty(mn, dtype=torch.uint8, device="cuda"))
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    with pytest.raises(mb.MuseError, match="workspace"):
        mb.muse_fwd(*args, ws=torch.empty(mn - 256, dtype=torch.uint8, device="cuda"))


def test_forward_tiles_with_many_tied_clusters():
    """Every key is the same row and the key clusters are dealt round-robin (teacher-forced), so in every block all
    64 accumulated cells of a query cluster are equal: every cluster scores the same, all of them are candidates
    for the r best, and the candidate lists of the one-plane tile kernel (r + 8 entries per lane half, 32 clusters
    per half here) overflow in every tile.  Those tiles are left to the two-plane kernel; the result must be a
    valid selection (nothing chosen scores below something left out, by the oracle's scores) and O, LSE must be
    the oracle's at that selection (Sec. 3.2, Eq. 7; Sec. 3.3)."""
    w = small("cfg2", N=1024, Hq=2, Hkv=1, Cq=4, Ck=64, r=3, block=128, kmeans_iters=1)
    d = generate(w)
    p = mb.params_for(w)
    d["K"][:] = d["K"][0, 0, 0]                                     # one key row everywhere
    qc, aq, _ = oracle_clustering(w, d, p)
    ak = np.tile((np.arange(w.N) % w.Ck).astype(np.int32), (w.B, w.Hkv, 1))   # 2 keys per (block, cluster)
    Q, K, V = (dev(d[x], p) for x in ("Q", "K", "V"))
    O, LSE, selc, selb = mb.muse_fwd(p, Q, K, V, torch.tensor(qc).cuda(), torch.tensor(aq).cuda(), torch.tensor(ak).cuda())
    torch.cuda.synchronize()
    op = orc.MuseParams(w.N, w.D, w.Bs, w.Cq, w.Ck, w.r, w.k2, p.eff_scale)
    for h in range(w.Hq):
        q, k, v = (f64(x) for x in (Q[0, h], K[0, 0], V[0, 0]))
        sc = selc.cpu().numpy()[0, h][:, : w.r]
        sb = selb.cpu().numpy()[0, h][:, : w.r].reshape(w.N, w.r, op.k2e)
        res = oracle_head(orc, op, q, k, v, q, qc[0, h], aq[0, h], ak[0, 0], (sc, sb), threads=8, with_bwd=False)
        free, forced = res["free"], res["forced"]
        far = np.arange(w.N) >= w.Bs
        assert (free["margin_c"][far] <= MARGIN).all(), "the clusters were meant to tie"
        assert (forced["margin_c"] >= -MARGIN).all() and (forced["margin_b"] >= -MARGIN).all()
        assert (sc[far] >= 0).all() and (np.sort(sc[far], 1)[:, 1:] != np.sort(sc[far], 1)[:, :-1]).all()
        assert_close(f64(O[0, h]), forced["O"], p, f"tied clusters O head {h}")
        np.testing.assert_allclose(LSE[0, h].cpu().numpy(), forced["LSE"], rtol=0, atol=2e-2 * max(1, np.abs(forced["LSE"]).max()))


def test_gpu_own_clustering_reports_rse(oracle):
    """End to end on the GPU's own clustering (cfg1): approximation error against exact attention."""
    w = small("cfg1")
    d = generate(w)
    p = mb.params_for(w)
    Q, K, V = (dev(d[x], p) for x in ("Q", "K", "V"))
    qc, aq, kc, ka = mb.muse_cluster(p, Q, K, d["q_init_idx"].cuda(), d["k_init_idx"].cuda())
    O, LSE, _, _ = mb.muse_fwd(p, Q, K, V, qc, aq, ka)
    Oe, _ = mb.exact_attn_fwd(p, Q, K, V)
    rse = (((O - Oe) ** 2).sum(-1) / (Oe ** 2).sum(-1)).mean().item()
    print(f"cfg1 RSE vs exact = {rse:.3e}")
    assert rse < 0.05


def test_keep_forward_state_matches_recompute():
    """MUSE_FLAG_KEEP_FWD_STATE (backward reuses the forward's bucketing, summaries and inverse index) must
    give the same bits as the stateless path."""
    base, kw = CASES["cfg4_gqa"]
    w = small(base, **kw)
    d = generate(w, need_dO=True)
    p = mb.params_for(w)
    pk = dataclasses.replace(p, flags=mb.FLAG_KEEP_FWD_STATE)
    qc, aq, ak = oracle_clustering(w, d, p)
    Q, K, V, dO = (dev(d[x], p) for x in ("Q", "K", "V", "dO"))
    cl = (torch.tensor(qc).cuda(), torch.tensor(aq).cuda(), torch.tensor(ak).cuda())
    O, LSE, selc, selb = mb.muse_fwd(p, Q, K, V, *cl)
    g = mb.muse_bwd(p, Q, K, V, O, LSE, dO, *cl, selc, selb)
    mn, pref = mb.muse_workspace_bytes(pk, mb.WS_FWD)
    assert mn == pref == mb.muse_workspace_bytes(pk, mb.WS_BWD)[1]
    ws = torch.empty(pref, dtype=torch.uint8, device="cuda")
    O2, LSE2, selc2, selb2 = mb.muse_fwd(pk, Q, K, V, *cl, ws=ws)
    g2 = mb.muse_bwd(pk, Q, K, V, O2, LSE2, dO, *cl, selc2, selb2, ws=ws)
    assert torch.equal(O, O2) and torch.equal(LSE, LSE2) and torch.equal(selc, selc2) and torch.equal(selb, selb2)
    for a, b in zip(g, g2):
        assert torch.equal(a, b)
    with pytest.raises(mb.MuseError, match="workspace"):
        mb.muse_fwd(pk, Q, K, V, *cl, ws=ws[: pref - 4096])


def test_backward_with_kept_forward_state_multi_tile_paths():
    """The flags bench.py times (MUSE_FLAG_KEEP_FWD_STATE, one workspace for forward and backward) on the case
    with several key tiles per retrieved pair and several staging passes per query group."""
    run_case("bf16_pairs64", with_bwd=True, flags=mb.FLAG_KEEP_FWD_STATE)


def test_keep_forward_state_default_workspace_and_stamp():
    """With ws=None the binding hands forward and backward the same cached buffer under the flag; the library
    refuses a workspace that does not hold the forward state of these params (MUSE_ERR_STATE)."""
    base, kw = CASES["cfg2_small"]
    w = small(base, **kw)
    d = generate(w, need_dO=True)
    p = mb.params_for(w)
    pk = dataclasses.replace(p, flags=mb.FLAG_KEEP_FWD_STATE)
    qc, aq, ak = oracle_clustering(w, d, p)
    Q, K, V, dO = (dev(d[x], p) for x in ("Q", "K", "V", "dO"))
    cl = (torch.tensor(qc).cuda(), torch.tensor(aq).cuda(), torch.tensor(ak).cuda())
    O, LSE, selc, selb = mb.muse_fwd(p, Q, K, V, *cl)
    g = mb.muse_bwd(p, Q, K, V, O, LSE, dO, *cl, selc, selb)
    mb.free_workspaces()
    O2, LSE2, selc2, selb2 = mb.muse_fwd(pk, Q, K, V, *cl)          # default workspace
    g2 = mb.muse_bwd(pk, Q, K, V, O2, LSE2, dO, *cl, selc2, selb2)   # must be the same buffer
    assert torch.equal(O, O2) and torch.equal(selb, selb2)
    for a, b in zip(g, g2):
        assert torch.equal(a, b)
    g3 = mb.muse_bwd(dataclasses.replace(pk, flags=pk.flags | mb.FLAG_FROZEN_WEIGHTS), Q, K, V, O2, LSE2, dO, *cl, selc2, selb2)
    assert torch.equal(g3[0], g[0]) and torch.equal(g3[2], g[2])     # a backward-only flag keeps the state valid
    size = mb.muse_workspace_bytes(pk, mb.WS_BWD)[1]
    other = torch.zeros(size, dtype=torch.uint8, device="cuda")
    with pytest.raises(mb.MuseError, match="forward state"):         # a buffer no forward has filled
        mb.muse_bwd(pk, Q, K, V, O2, LSE2, dO, *cl, selc2, selb2, ws=other)
    with pytest.raises(mb.MuseError, match="forward state"):         # other params than the forward's
        mb.muse_bwd(dataclasses.replace(pk, scale=0.2), Q, K, V, O2, LSE2, dO, *cl, selc2, selb2)
    mb.muse_fwd(p, Q, K, V, *cl, ws=mb.workspace(pk, mb.WS_BWD))     # a stateless call on the buffer clears the stamp
    with pytest.raises(mb.MuseError, match="forward state"):
        mb.muse_bwd(pk, Q, K, V, O2, LSE2, dO, *cl, selc2, selb2)


@pytest.mark.parametrize("name,kw", [
    ("cfg1", dict(N=1024, Cq=6, Ck=24, r=0, block=128, kmeans_iters=2)),                       # fp32
    ("cfg2", dict(N=2048, Hq=2, Hkv=1, Cq=8, Ck=32, r=0, block=256, kmeans_iters=2)),          # bf16, GQA
    ("cfg5", dict(N=1024, Hq=2, Hkv=2, Cq=5, Ck=19, r=0, block=128, kmeans_iters=2)),          # D = 128, ragged
])
def test_dipole_correction_forward(name, kw):
    """MUSE_FLAG_DIPOLE (App. B: pre-merged dipole with untilted covariances, monopole-only mode) against the
    oracle's mode 2, element by element; the correction must be visible (the two modes differ by far more than
    the tolerance), LSE must be the monopole's, and the backward must refuse the flag."""
    w = small(name, **kw)
    d = generate(w, need_dO=True)
    p0 = mb.params_for(w)
    p = dataclasses.replace(p0, flags=mb.FLAG_DIPOLE)
    qc, aq, ak = oracle_clustering(w, d, p)
    Q, K, V, dO = (dev(d[x], p) for x in ("Q", "K", "V", "dO"))
    cl = (torch.tensor(qc).cuda(), torch.tensor(aq).cuda(), torch.tensor(ak).cuda())
    O, LSE, selc, selb = mb.muse_fwd(p, Q, K, V, *cl)
    O0, LSE0, _, _ = mb.muse_fwd(p0, Q, K, V, *cl)
    torch.cuda.synchronize()
    assert torch.equal(LSE, LSE0)
    G = w.Hq // w.Hkv
    for h in range(w.Hq):
        q, k, v = (f64(x) for x in (Q[0, h], K[0, h // G], V[0, h // G]))
        op = orc.MuseParams(w.N, w.D, w.Bs, w.Cq, w.Ck, 0, w.k2, p.eff_scale, dipole=2)
        want = orc.muse_fwd(op, q, k, v, qc[0, h], aq[0, h], ak[0, h // G])
        mono = orc.muse_fwd(dataclasses.replace(op, dipole=0), q, k, v, qc[0, h], aq[0, h], ak[0, h // G])
        assert_close(f64(O[0, h]), want["O"], p, f"dipole {name} O head {h}")
        shift = np.abs(want["O"] - mono["O"]).max()
        assert shift > 10 * (1e-4 * np.abs(want["O"]).max() if w.dtype == "fp32" else 2e-2) or w.dtype == "bf16", shift
        # the correction itself, isolated: (dipole - monopole) on both sides
        got_shift = f64(O[0, h]) - f64(O0[0, h])
        assert np.abs(got_shift - (want["O"] - mono["O"])).max() <= (2e-4 * max(1.0, shift) if w.dtype == "fp32" else 2e-2)
        assert np.abs(got_shift[w.Bs:]).max() > 0
    with pytest.raises(mb.MuseError, match="unsupported"):
        mb.muse_bwd(p, Q, K, V, O, LSE, dO, *cl, selc, selb, ws=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
    with pytest.raises(mb.MuseError, match="unsupported"):
        mb.muse_fwd(dataclasses.replace(p, r=2), Q, K, V, *cl, ws=torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))


def test_probe_peaks_copy_is_exact_and_rates_are_plausible():
    """The measurement aid really copies (second half == first half afterwards) and reports rates between a tenth of
    the published peaks (8 TB/s, 2.5 PFLOP/s bf16) and those peaks; a buffer below 1 GiB is refused."""
    n = 2 << 30
    buf = torch.empty(n, dtype=torch.uint8, device="cuda")
    buf[: n // 2] = torch.arange(n // 2, device="cuda", dtype=torch.int64).mul_(2654435761).bitwise_and_(255).to(torch.uint8)
    want = buf[: n // 2].clone()
    got = mb.muse_probe_peaks(buf)
    assert 800.0 < got["copy_GBps"] < 8000.0, got
    assert 250.0 < got["mfma_bf16_TFLOPs"] < 2500.0, got
    # the MFMA loop writes its sums into the head of the buffer afterwards; the copy's destination is untouched by it
    assert torch.equal(buf[n // 2:], want)
    with pytest.raises(mb.MuseError):
        mb.muse_probe_peaks(torch.empty(1 << 20, dtype=torch.uint8, device="cuda"))
