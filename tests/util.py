"""Shared helpers for the tests (no arithmetic of the method)."""
import numpy as np


def per_token_errors(got: np.ndarray, ref: np.ndarray):
    """Per row: max|got-ref| / max|ref| and the cosine similarity."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    num = np.abs(got - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    rel = num / np.maximum(den, 1e-30)
    cos = (got * ref).sum(1) / np.maximum(np.linalg.norm(got, axis=1) * np.linalg.norm(ref, axis=1), 1e-30)
    return rel, cos


def assert_tokens_close(got, ref, rel_tol, cos_tol, what=""):
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    if got.shape[0] == 0:
        return
    rel, cos = per_token_errors(got, ref)
    assert rel.max() <= rel_tol, f"{what}: max per-token relative error {rel.max():.3e} > {rel_tol} (row {rel.argmax()})"
    assert cos.min() >= cos_tol, f"{what}: min cosine {cos.min():.6f} < {cos_tol} (row {cos.argmin()})"


def bf16_grid(x: np.ndarray) -> np.ndarray:
    """Snap test inputs to bf16-representable values (data preparation only)."""
    import workloads
    return workloads.snap_to_bf16_grid(np.asarray(x, np.float32))
