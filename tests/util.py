"""Shared helpers for the GPU parity tests (data movement and tolerances only)."""
import numpy as np
import torch

from paper_2407_18121_amd import synthetic as syn

ATOL = {"f32": 1e-4, "bf16": 2e-2}  # max-abs bars for floating-point outputs


def to_dev(x_f32: np.ndarray, dtype: str) -> torch.Tensor:
    """fp32 numpy array (values exact in `dtype`) -> CUDA tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32)).cuda()
    return t if dtype == "f32" else t.to(torch.bfloat16)


def to_host(t: torch.Tensor) -> np.ndarray:
    """CUDA tensor -> float64 numpy (exact)."""
    return t.detach().float().cpu().numpy().astype(np.float64)


def torch_dtype(dtype: str):
    return torch.float32 if dtype == "f32" else torch.bfloat16


def quantize(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an fp64/fp32 array to the storage type; returns fp32 holding exact values."""
    return syn.round_to_dtype(np.asarray(x, dtype=np.float32), dtype)


def assert_close(got: np.ndarray, ref: np.ndarray, dtype: str, what: str, stored: bool = False):
    """max-abs bar; `stored` = the value is a bf16 rounding of a possibly large number, for which
    the bf16 grid itself is coarser than the bar above |x| = 8 (half-spacing 2^-8 |x| at most)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    tol = np.full(ref.shape, ATOL[dtype])
    if stored and dtype == "bf16":
        tol = np.maximum(tol, np.abs(ref) * 2.0 ** -8)
    err = np.abs(got - ref)
    bad = err > tol
    assert not bad.any(), (f"{what}: {bad.sum()} of {bad.size} beyond tolerance; max err {err.max():.3e} "
                           f"at {np.unravel_index(err.argmax(), err.shape)}")
