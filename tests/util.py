"""Shared helpers of the GPU parity tests (no method arithmetic here)."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

from paper_2509_10406_amd import binding as mb

BF16_ABS = 2e-2   # bf16: max absolute error of outputs and of gradients taken as fp32 outputs
FP32_REL = 1e-4   # fp32: max|a-b| / max|b| per tensor
ERRORS = []       # (what, max abs err, max|want|) of every comparison, listed at the end of the session


def dev(x: torch.Tensor, p: "mb.Params"):
    """Host float32 tensor holding storage-rounded values -> device tensor of the storage type."""
    return x.to(p.torch_dtype).cuda().contiguous()


def f64(x: torch.Tensor) -> np.ndarray:
    return x.detach().to(torch.float32).cpu().double().numpy()


def max_rel(a: np.ndarray, b: np.ndarray) -> float:
    """max|a-b| / max|b| (the normalisation used for the fp32 tolerance)."""
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


def max_abs(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.abs(a - b).max())


def bf16_grad_bound(want_max: float) -> float:
    """Bound on the max absolute error of a gradient tensor of a bf16 run (the library's fp32 output): 2e-2, or
    one bf16 unit in the last place (2^-8 relative) of the tensor's largest entry where that is more.  The
    probabilities and their gradients enter the matrix cores rounded to bf16, so an entry that is essentially one
    product (a peaked softmax row) carries that rounding whatever the accumulator's precision; at max|g| <= 5.1
    the bound is the plain 2e-2."""
    return max(BF16_ABS, want_max / 256.0)


def assert_close(got: np.ndarray, want: np.ndarray, p: "mb.Params", what: str, grad: bool = False):
    """fp32: <= 1e-4 max relative error per tensor.  bf16: <= 2e-2 max ABSOLUTE error for O and LSE; gradients
    <= bf16_grad_bound (2e-2 unless the tensor's entries exceed 5.1).  Every comparison is recorded with its
    absolute error and max|want| and listed at the end of the session."""
    e = max_abs(got, want) if got.size else 0.0
    mx = float(np.abs(want).max()) if want.size else 0.0
    ERRORS.append((what, e, mx))
    if p.dtype == mb.FP32:
        r = max_rel(got, want) if got.size else 0.0
        assert r <= FP32_REL, f"{what}: max rel err {r:.3e} > {FP32_REL}"
    else:
        bound = bf16_grad_bound(mx) if grad else BF16_ABS
        assert e <= bound, f"{what}: max abs err {e:.3e} > {bound:.3e} (max|want| {mx:.3g})"


def segment_sizes(assign: np.ndarray, Bs: int, C: int) -> np.ndarray:
    """[nb, C] number of rows of every (spatial block, cluster) segment."""
    N = assign.shape[0]
    return np.bincount((np.arange(N) // Bs) * C + assign, minlength=(N // Bs) * C).reshape(N // Bs, C)


def oracle_head(orc, op, q, k, v, g, qc, aq, ak, sel, threads=8, rows=None, with_bwd=True):
    """The oracle on one (batch, head) with the selections `sel` = (selc, selb) given, split over threads by
    query cluster (the oracle builds the summaries of the query clusters it meets, and its gradients are sums
    over the listed rows, so the pieces add up).  Returns dict(free=..., forced=..., grads=(dQ, dK, dV) | None):
    `free` holds the oracle's own selections and their margins, `forced` O / LSE / slack at the given ones."""
    N = q.shape[0]
    rows = np.arange(N, dtype=np.int32) if rows is None else np.asarray(rows, dtype=np.int32)
    order = np.argsort(aq[rows], kind="stable")
    # whole query clusters per piece, pieces of about equal size
    cuts = [0]
    target = max(1, len(rows) // max(1, threads))
    srt = aq[rows][order]
    for t in range(1, len(rows)):
        if srt[t] != srt[t - 1] and t - cuts[-1] >= target:
            cuts.append(t)
    cuts.append(len(rows))
    pieces = [np.sort(rows[order[a:b]]).astype(np.int32) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]

    def run(rs):
        free = orc.muse_fwd(op, q, k, v, qc, aq, ak, rows=rs)
        forced = orc.muse_fwd(op, q, k, v, qc, aq, ak, rows=rs, sel=sel)
        gr = None
        if with_bwd:
            gr = orc.muse_bwd(op, q, k, v, qc, aq, ak, forced["O"], forced["LSE"], g, sel[0], sel[1], rows=rs)
        return rs, free, forced, gr

    with ThreadPoolExecutor(max(1, threads)) as ex:
        out = list(ex.map(run, pieces))
    free = {x: out[0][1][x].copy() for x in ("selc", "selb", "margin_c", "margin_b", "mass")}
    forced = {x: out[0][2][x].copy() for x in ("O", "LSE", "margin_c", "margin_b")}
    grads = [x.copy() for x in out[0][3]] if with_bwd else None
    for rs, fr, fo, gr in out[1:]:
        for x in free:
            free[x][rs] = fr[x][rs]
        for x in forced:
            forced[x][rs] = fo[x][rs]
        if with_bwd:
            grads[0][rs] = gr[0][rs]
            grads[1] += gr[1]
            grads[2] += gr[2]
    return dict(free=free, forced=forced, grads=grads, rows=rows)


def blocks_by_cluster(selc: np.ndarray, selb: np.ndarray) -> np.ndarray:
    """[n, r, k2e] block sets re-ordered so that slots are sorted by cluster id and blocks inside a slot are
    sorted: two exports with the same (cluster -> block set) map give the same array whatever their slot order."""
    o = np.argsort(selc, axis=1, kind="stable")
    sb = np.take_along_axis(selb, o[:, :, None], axis=1)
    return np.sort(sb, axis=-1)
