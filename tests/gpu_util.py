"""Harness helpers for the GPU parity tests (plumbing only: conversions and comparison metrics)."""
import numpy as np
import torch

DEV = "cuda:0"


def bf16_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


def f32_dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV)


def to_dev(x: np.ndarray) -> torch.Tensor:
    if x.dtype == np.uint16:
        return bf16_dev(x)
    if x.dtype == np.int32:
        return torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return f32_dev(x)


def host(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def assert_norms_close(x, ref, tol, what=""):
    """Per-example squared norms: positive, no cancellation -> element-wise relative bound."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(x - ref) / np.maximum(np.abs(ref), 1e-300)
    assert np.all(err <= tol), f"{what}: max rel err {err.max():.3e} > {tol:.1e} at {err.argmax()}"
    return float(err.max())


def assert_sums_close(x, ref, tol, what=""):
    """Signed sums: relative error in the 2-norm of the tensor, and element-wise against |ref| + rms(ref)."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert x.shape == ref.shape, f"{what}: shape {x.shape} vs {ref.shape}"
    nref = np.linalg.norm(ref)
    if nref == 0:
        assert np.all(x == 0), f"{what}: expected exact zeros"
        return 0.0
    rel = np.linalg.norm(x - ref) / nref
    assert rel <= tol, f"{what}: ||x-ref||/||ref|| = {rel:.3e} > {tol:.1e}"
    rms = nref / np.sqrt(ref.size)
    bad = np.abs(x - ref) > tol * (np.abs(ref) + rms)
    assert not bad.any(), f"{what}: {bad.sum()} entries off, worst {np.abs(x - ref).max():.3e} (rms {rms:.3e})"
    return float(rel)
