"""Shared helpers of the parity tests (error norms, top-k equivalence)."""
import numpy as np
import torch

# spec tolerances: fp32 I/O 1e-4 relative, bf16 I/O with fp32 accumulation 2e-2
TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}


def rel_errors(got, ref):
    """(max-abs error / max-abs ref, relative Frobenius error) in float64."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, 0.0
    denom_max = max(np.abs(ref).max(), 1e-300)
    denom_fro = max(np.sqrt((ref ** 2).sum()), 1e-300)
    assert np.isfinite(got).all(), "non-finite values in the device result"
    return np.abs(got - ref).max() / denom_max, np.sqrt(((got - ref) ** 2).sum()) / denom_fro


def assert_close(got, ref, tol, what=""):
    emax, efro = rel_errors(got, ref)
    assert emax <= tol and efro <= tol, "%s: max-rel %.3e, fro-rel %.3e > tol %.1e" % (what, emax, efro, tol)
    return emax, efro


def assert_topk_equivalent(idx_dev, scores_ref, K, tol, band_of_max=False):
    """The device selection may differ from the oracle's only in elements whose oracle score
    lies within tol * (K-th score) of the K-th score; what is unique must match exactly.
    band_of_max: the band is tol * (largest score) instead -- for scores that span hundreds of
    orders of magnitude (the decayed Mamba score), where the K-th score is far below what fp32
    resolves and the score tolerance itself is relative to the largest score."""
    import oracle
    idx_dev = np.asarray(idx_dev)
    N = scores_ref.shape[0]
    assert idx_dev.shape == (K,)
    assert (idx_dev >= 0).all() and (idx_dev < N).all()
    assert (np.diff(idx_dev) > 0).all(), "indices must be strictly ascending"
    want = oracle.select_topk(scores_ref, K)
    kth = np.sort(scores_ref)[::-1][K - 1]
    band = tol * max(abs(scores_ref.max() if band_of_max else kth), 1e-300)
    only_dev = np.setdiff1d(idx_dev, want)
    only_ref = np.setdiff1d(want, idx_dev)
    assert only_dev.size == only_ref.size
    assert (np.abs(scores_ref[only_dev] - kth) <= band).all(), "device kept a token clearly below the K-th score"
    assert (np.abs(scores_ref[only_ref] - kth) <= band).all(), "device dropped a token clearly above the K-th score"
    return only_dev.size
