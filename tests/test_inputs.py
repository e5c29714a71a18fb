"""Host-side input recipe: the App. C initialisation rule lives in the shared generator module."""
import torch

from paper_2509_10406_amd.inputs import CONFIGS, generate, init_indices, small


def test_init_indices_follow_the_shuffle_and_stride_rule():
    """App. C "Centroid Computation", step 1: shuffle the positions with a fixed seed, then take every
    floor(N/C)-th one.  Re-drawn here from the same seed with the library permutation routine."""
    for N, C in ((64, 8), (100, 7), (4096, 1024), (50, 50)):
        g = torch.Generator().manual_seed(11)
        idx = init_indices(g, 2, 3, N, C)
        g2 = torch.Generator().manual_seed(11)
        for b in range(2):
            for h in range(3):
                perm = torch.randperm(N, generator=g2)
                want = perm[:: N // C][:C].to(torch.int32)
                assert torch.equal(idx[b, h], want)
                assert len(set(idx[b, h].tolist())) == C            # distinct rows -> distinct start centroids
                assert 0 <= int(idx[b, h].min()) and int(idx[b, h].max()) < N
    assert idx.dtype == torch.int32


def test_generators_are_seeded_and_storage_rounded():
    w = small("cfg2", N=256, Hq=2, Hkv=1, Cq=4, Ck=8)
    a, b = generate(w, need_dO=True), generate(w, need_dO=True)
    for k in a:
        assert torch.equal(a[k], b[k]), k
    for k in ("Q", "K", "V", "dO"):   # values are exactly representable in the storage type
        assert torch.equal(a[k], a[k].to(torch.bfloat16).to(torch.float32))
    assert a["Q"].shape == (1, 2, 256, 64) and a["K"].shape == (1, 1, 256, 64)
    assert set(CONFIGS) >= {"cfg1", "cfg2", "cfg3", "cfg4", "cfg5"}
