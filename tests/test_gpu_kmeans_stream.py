"""GPU parity of the streaming centroid pass (App. C "Centroid Computation", step 2) against the CPU oracle,
through the C ABI.

The pass is sequential and chaotic: one different assignment changes a centroid and everything after it.  So
the oracle replays the pass along the library's own assignments (teacher forcing) and checks two things:
every assignment the library took is a nearest centroid (its score is within MARGIN of the best one, relative,
evaluated exactly on the same binary16 values), and, given those assignments, the decayed counts and the
centroids are bit-identical (the state arithmetic is fp32 fused multiply-adds and one division on both sides).
"""
import dataclasses

import numpy as np
import pytest
import torch

from paper_2509_10406_amd import binding as mb
from paper_2509_10406_amd.inputs import CONFIGS, generate, small
from tests.util import dev, f64

pytestmark = pytest.mark.gpu

MARGIN = 1e-5

CASES = {
    "fp32_cfg1": ("cfg1", dict(N=2048)),
    "fp32_ragged": ("cfg1", dict(N=1000, Cq=5, Ck=37, block=125)),
    "fp32_one_cluster": ("cfg1", dict(N=300, Cq=1, Ck=2, block=300)),
    "bf16_cfg2": ("cfg2", dict(N=4096, Hq=2, Hkv=2, Cq=48, Ck=200, block=512)),
    "bf16_gqa": ("cfg4", dict(N=2048, Hq=4, Hkv=2, Cq=32, Ck=96, block=256)),
    "bf16_d128": ("cfg5", dict(N=2080, Hq=2, Hkv=1, Cq=40, Ck=130, block=260)),
    "bf16_many_tiles": ("cfg2", dict(N=3000, Hq=1, Hkv=1, Cq=300, Ck=1030, block=3000)),
    # one full minibatch and a ragged one; fewer rows than a tile of centroids
    "fp32_tiny": ("cfg1", dict(N=96, Cq=3, Ck=40, block=48)),
    "bf16_single_minibatch": ("cfg2", dict(N=40, Hq=1, Hkv=1, Cq=2, Ck=7, block=40)),
}


def _sides(w, d, p):
    Q, K = dev(d["Q"], p), dev(d["K"], p)
    return ((0, Q, w.Hq, w.Cq, d["q_init_idx"]), (1, K, w.Hkv, w.Ck, d["k_init_idx"]))


def _check_side(oracle, p, side, X, H, Cn, init, what):
    cent, sa, cnt = mb.muse_kmeans_stream(p, side, X, init.cuda())
    torch.cuda.synchronize()
    for h in range(H):
        got_a = sa[0, h].cpu().numpy()
        assert (got_a >= 0).all() and (got_a < Cn).all(), what
        o = oracle.kmeans_stream(f64(X[0, h]), Cn, init[0, h].numpy(), forced=got_a)
        worst = float(o["regret"].max())
        assert worst <= MARGIN, f"{what} head {h}: an assignment is {worst:.2e} (relative) from the nearest centroid"
        np.testing.assert_array_equal(cnt[0, h].cpu().numpy(), o["c"].astype(np.float32), err_msg=f"{what} head {h}: counts")
        np.testing.assert_array_equal(cent[0, h].cpu().numpy(), o["cent"].astype(np.float32),
                                      err_msg=f"{what} head {h}: centroids")
        # the oracle left alone takes the same assignments wherever its own margin is safe, until the first
        # row where the two part (after that the centroids differ and nothing can be compared)
        free = oracle.kmeans_stream(f64(X[0, h]), Cn, init[0, h].numpy())
        diff = np.flatnonzero(free["assign"] != got_a)
        if diff.size:
            assert free["margin"][diff[0]] <= MARGIN, f"{what} head {h}: first difference at row {diff[0]} is not a near-tie"
    return cent, sa, cnt


@pytest.mark.parametrize("name", list(CASES))
def test_stream_pass_teacher_forced(oracle, name):
    base, kw = CASES[name]
    w = small(base, **kw)
    d = generate(w)
    p = mb.params_for(w)
    for side, X, H, Cn, init in _sides(w, d, p):
        _check_side(oracle, p, side, X, H, Cn, init, f"{name} side {side}")


def test_cluster_with_streaming_flag(oracle):
    """muse_cluster with MUSE_FLAG_STREAMING_KMEANS: the centroids of the pass, then the usual final assignment."""
    w = small("cfg2", N=4096, Hq=2, Hkv=2, Cq=48, Ck=200, block=512)
    d = generate(w)
    p = mb.params_for(w, flags=mb.FLAG_STREAMING_KMEANS)
    Q, K = dev(d["Q"], p), dev(d["K"], p)
    qi, ki = d["q_init_idx"].cuda(), d["k_init_idx"].cuda()
    qc, qa, kc, ka = mb.muse_cluster(p, Q, K, qi, ki)
    again = mb.muse_cluster(p, Q, K, qi, ki)
    for x, y in zip((qc, qa, kc, ka), again):
        assert torch.equal(x, y)
    for side, X, H, Cn, cent, asg, init in ((0, Q, w.Hq, w.Cq, qc, qa, qi), (1, K, w.Hkv, w.Ck, kc, ka, ki)):
        alone, _, _ = mb.muse_kmeans_stream(p, side, X, init)
        assert torch.equal(alone, cent)
        for h in range(H):
            chk = oracle.kmeans(f64(X[0, h]), Cn, 0, cent0=cent[0, h].cpu().double().numpy(), round_mode=1)
            safe = chk["margin"] > MARGIN
            assert safe.mean() > 0.99
            np.testing.assert_array_equal(asg[0, h].cpu().numpy()[safe], chk["assign"][safe])
    # the Lloyd iteration count plays no role
    p5 = dataclasses.replace(p, kmeans_iters=5)
    other = mb.muse_cluster(p5, Q, K, qi, ki)
    assert torch.equal(other[0], qc) and torch.equal(other[3], ka)


def test_stream_pass_starts_from_given_centroids(oracle):
    """init_idx == NULL: the totals start at the centroid buffer.  Starting from the rows the initialisation
    would pick gives the same run (they are binary16 values already)."""
    w = small("cfg2", N=1024, Hq=1, Hkv=1, Cq=8, Ck=24, block=1024)
    d = generate(w)
    p = mb.params_for(w)
    K = dev(d["K"], p)
    ki = d["k_init_idx"]
    a = mb.muse_kmeans_stream(p, 1, K, ki.cuda())
    c0 = K[0, 0][ki[0, 0].long().cuda()].float().reshape(1, 1, w.Ck, w.D).contiguous()
    b = mb.muse_kmeans_stream(p, 1, K, None, centroids=c0)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_stream_pass_full_size_one_head(oracle):
    """The launch configuration the benchmark times (cfg3: N = 65536, 1024 key clusters), one head replayed by
    the oracle along the library's assignments."""
    w = dataclasses.replace(CONFIGS["cfg3"], Hq=1, Hkv=1)
    d = generate(w)
    p = mb.params_for(w)
    K = dev(d["K"], p)
    _check_side(oracle, p, 1, K, 1, w.Ck, d["k_init_idx"], "cfg3 keys")


# ---------------------------------------------------------------------------
# balanced assignment (App. C "Balanced Assignment", MUSE_FLAG_BALANCED_ASSIGN)
# ---------------------------------------------------------------------------
BALANCED = {
    # name: (base, overrides, extra flags); cap = floor(4 block / C)
    "bf16_lloyd": ("cfg2", dict(N=4096, Hq=2, Hkv=2, Cq=48, Ck=200, block=512, kmeans_iters=3), 0),
    "bf16_streaming": ("cfg2", dict(N=4096, Hq=2, Hkv=2, Cq=48, Ck=200, block=512), mb.FLAG_STREAMING_KMEANS),
    "bf16_tight": ("cfg4", dict(N=2048, Hq=2, Hkv=1, Cq=64, Ck=256, block=256, kmeans_iters=1), 0),   # cap 16 and 4
    "fp32_ragged": ("cfg1", dict(N=1000, Cq=5, Ck=37, block=125, kmeans_iters=2), 0),
    "bf16_d128": ("cfg5", dict(N=2080, Hq=2, Hkv=1, Cq=40, Ck=130, block=260, kmeans_iters=1), mb.FLAG_STREAMING_KMEANS),
    # the cap leaves exactly one place per row (cap 1 with as many clusters as rows in a block would; here cap 2, 4)
    "fp32_full_house": ("cfg1", dict(N=256, Cq=64, Ck=32, block=32, kmeans_iters=1), 0),
}


@pytest.mark.parametrize("name", list(BALANCED))
def test_balanced_assignment(oracle, name):
    """The library's capped assignment replayed by the oracle along the library's own choices: nothing breaks the
    rule, every displaced row sits within MARGIN of the best centroid that had room; and the oracle left free
    gives the same assignment when no decision of either phase is a near-tie."""
    base, kw, extra = BALANCED[name]
    w = small(base, **kw)
    d = generate(w)
    p = mb.params_for(w, flags=mb.FLAG_BALANCED_ASSIGN | extra)
    p_plain = mb.params_for(w, flags=extra)
    Q, K = dev(d["Q"], p), dev(d["K"], p)
    qi, ki = d["q_init_idx"].cuda(), d["k_init_idx"].cuda()
    qc, qa, kc, ka = mb.muse_cluster(p, Q, K, qi, ki)
    qc0, qa0, kc0, ka0 = mb.muse_cluster(p_plain, Q, K, qi, ki)
    assert torch.equal(qc, qc0) and torch.equal(kc, kc0)   # the cap touches the assignment only
    rm = 1 if w.dtype == "bf16" else 0
    displaced = 0
    for X, cent, asg, plain, H, Cn in ((Q, qc, qa, qa0, w.Hq, w.Cq), (K, kc, ka, ka0, w.Hkv, w.Ck)):
        cap = 4 * w.Bs // Cn
        for h in range(H):
            got = asg[0, h].cpu().numpy()
            sizes = np.stack([np.bincount(got[b * w.Bs:(b + 1) * w.Bs], minlength=Cn) for b in range(w.N // w.Bs)])
            assert sizes.max() <= cap, f"{name}: a cluster holds {sizes.max()} rows of a block, cap {cap}"
            displaced += int((got != plain[0, h].cpu().numpy()).sum())
            Xh, ch = f64(X[0, h]), cent[0, h].cpu().double().numpy()
            rep = oracle.balanced_assign(Xh, ch, w.Bs, cap, round_mode=rm, forced=got, tol=MARGIN)
            assert rep["broken"] == 0, f"{name} head {h}: {rep['broken']} rows break the rule"
            assert rep["regret"] <= MARGIN, f"{name} head {h}: a displaced row is {rep['regret']:.2e} from the best centroid with room"
            free = oracle.balanced_assign(Xh, ch, w.Bs, cap, round_mode=rm)["assign"]
            if oracle.kmeans(Xh, Cn, 0, cent0=ch, round_mode=rm)["margin"].min() > MARGIN:
                diff = np.flatnonzero(free != got)
                assert diff.size == 0, f"{name} head {h}: differs from the free oracle at rows {diff[:5]}"
    if name in ("bf16_tight", "bf16_streaming"):
        assert displaced > 0, "the case was meant to make the cap bind"


def test_balanced_assignment_rejects_a_cap_without_room():
    w = small("cfg2", N=1024, Hq=1, Hkv=1, Cq=2048 // 2, Ck=8, block=128)   # cap = floor(512 / 1024) = 0
    d = generate(w)
    p = mb.params_for(w, flags=mb.FLAG_BALANCED_ASSIGN)
    with pytest.raises(mb.MuseError, match="unsupported"):
        mb.muse_cluster(p, dev(d["Q"], p), None, d["q_init_idx"].cuda(), None)


def test_paper_clustering_full_size_one_head(oracle):
    """Streaming pass + balanced assignment at the benchmark's shape (cfg3 keys: N = 65536, 1024 clusters, blocks
    of 8192, cap 32), one head: the cap holds and the oracle's replay finds nothing wrong."""
    w = dataclasses.replace(CONFIGS["cfg3"], Hq=1, Hkv=1)
    d = generate(w)
    p = mb.params_for(w, flags=mb.FLAG_STREAMING_KMEANS | mb.FLAG_BALANCED_ASSIGN)
    K = dev(d["K"], p)
    _, _, kc, ka = mb.muse_cluster(p, None, K, None, d["k_init_idx"].cuda())
    got = ka[0, 0].cpu().numpy()
    cap = 4 * w.Bs // w.Ck
    sizes = np.stack([np.bincount(got[b * w.Bs:(b + 1) * w.Bs], minlength=w.Ck) for b in range(w.N // w.Bs)])
    assert sizes.max() <= cap
    rep = oracle.balanced_assign(f64(K[0, 0]), kc[0, 0].cpu().double().numpy(), w.Bs, cap, round_mode=1, forced=got, tol=MARGIN)
    assert rep["broken"] == 0 and rep["regret"] <= MARGIN, rep
