"""exact_attn_bwd_static (the entry point for callers that cannot allocate) against exact_attn_bwd, through
the C ABI: two calls in a row on the library's static scratch, the second with a smaller input."""
import dataclasses

import pytest
import torch

from paper_2509_10406_amd import binding as mb
from paper_2509_10406_amd.inputs import generate, small

pytestmark = pytest.mark.gpu


def _case(N, Hq, Hkv, D, grad_dtype, seed):
    w = small("cfg4" if D == 64 else "cfg5", N=N, Hq=Hq, Hkv=Hkv, seed=seed)
    d = generate(w, need_dO=True)
    p = dataclasses.replace(mb.params_for(w), grad_dtype=grad_dtype)
    Q, K, V, dO = (d[x].to(p.torch_dtype).cuda().contiguous() for x in ("Q", "K", "V", "dO"))
    return p, Q, K, V, dO


def _grads(p, Q, K):
    t = p.torch_grad_dtype
    return tuple(torch.full(x.shape, float("nan"), dtype=t, device="cuda") for x in (Q, K, K))


@pytest.mark.parametrize("grad_dtype", [mb.BF16, mb.FP32])
def test_static_scratch_matches_workspace_entry_point(grad_dtype):
    # the second input is smaller: what the first call left in the scratch must not leak into it
    for N, Hq, Hkv, D, seed in ((2048, 4, 2, 64, 5), (640, 2, 1, 128, 6)):
        p, Q, K, V, dO = _case(N, Hq, Hkv, D, grad_dtype, seed)
        O, LSE = mb.exact_attn_fwd(p, Q, K, V)
        want = mb.exact_attn_bwd(p, Q, K, V, O, LSE, dO)
        out = _grads(p, Q, K)
        torch.cuda.synchronize()
        before = torch.cuda.memory_stats()["allocation.all.allocated"]   # allocations ever made through torch
        got = mb.exact_attn_bwd_static(p, Q, K, V, O, LSE, dO, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats()["allocation.all.allocated"] == before
        for a, b, name in zip(got, want, ("dQ", "dK", "dV")):
            assert torch.isfinite(a.float()).all(), name
            assert torch.equal(a, b), f"{name}: N={N} differs from exact_attn_bwd by {(a.float() - b.float()).abs().max().item():.3e}"


def test_static_scratch_rejects_oversized_input():
    p = mb.Params(1, 16, 16, 65536, 64, grad_dtype=mb.BF16)   # 3 x 268 MB of fp32 accumulators
    Q = torch.zeros(1, dtype=torch.bfloat16, device="cuda")    # never read: the size check comes first
    with pytest.raises(mb.MuseError, match="scratch"):
        mb.exact_attn_bwd_static(p, Q, Q, Q, Q, torch.zeros(1, device="cuda"), Q, (Q, Q, Q))
