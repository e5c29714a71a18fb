"""Shared helpers of the GPU parity tests (no method arithmetic here)."""
import numpy as np
import torch

from paper_2509_10406_amd import binding as mb


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


def assert_close(got: np.ndarray, want: np.ndarray, p: "mb.Params", what: str, grad: bool = False):
    """fp32: <= 1e-4 max relative error; bf16: <= 2e-2 max absolute error (gradients are compared as fp32
    outputs of the library, normalised by max|want| when that exceeds 1, because their scale is set by dO)."""
    if p.dtype == mb.FP32:
        e = max_rel(got, want)
        assert e <= 1e-4, f"{what}: max rel err {e:.3e} > 1e-4"
    else:
        e = max_abs(got, want)
        if grad:
            e /= max(1.0, float(np.abs(want).max()))
        assert e <= 2e-2, f"{what}: max abs err {e:.3e} > 2e-2"
