"""Shared helpers of the parity tests (error norms, top-k equivalence)."""
import numpy as np
import torch

# spec tolerances: fp32 I/O 1e-4 relative, bf16 I/O with fp32 accumulation 2e-2
TOL = {torch.float32: 1e-4, torch.bfloat16: 2e-2}

# A unit (a head, a query row of a head, a token's score) whose largest reference magnitude is
# below this fraction of the tensor's largest one is measured against that floor instead of
# against itself: below it the result is rounding noise of the larger units' arithmetic.
UNIT_FLOOR = 1e-4


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


def unit_error(got, ref, unit_axes):
    """Largest, over the units, of max|got - ref| / max|ref| taken inside one unit.  `unit_axes`
    are the axes whose index names a unit (e.g. (1,) for the heads of y [T, H, P]; (0, 1) for the
    (query row, head) pairs of o [T, Hq, d]; (0,) for the tokens of a score vector): a unit that
    is small beside the rest of the tensor cannot hide behind the tensor-wide maximum.  Returns
    (worst ratio, index of the worst unit)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0, None
    unit_axes = tuple(a % ref.ndim for a in unit_axes)
    inner = tuple(a for a in range(ref.ndim) if a not in unit_axes)
    err = np.abs(got - ref)
    mag = np.abs(ref)
    if inner:
        err, mag = err.max(axis=inner), mag.max(axis=inner)
    denom = np.maximum(mag, max(UNIT_FLOOR * np.abs(ref).max(), 1e-300))
    ratio = err / denom
    worst = np.unravel_index(np.argmax(ratio), ratio.shape)
    return float(ratio[worst]), tuple(int(i) for i in worst)


def assert_close(got, ref, tol, what="", units=None):
    """Tensor-wide max and Frobenius relative errors within tol and, when `units` (a tuple of
    axes) is given, the same max-norm bound inside every unit."""
    emax, efro = rel_errors(got, ref)
    assert emax <= tol and efro <= tol, "%s: max-rel %.3e, fro-rel %.3e > tol %.1e" % (what, emax, efro, tol)
    if units is not None:
        eu, where = unit_error(got, ref, units)
        assert eu <= tol, "%s: unit %s is off by %.3e of its own largest value > tol %.1e" % (what, where, eu, tol)
    return emax, efro


def assert_topk_equivalent(idx_dev, scores_ref, K, tol, floor=0.0):
    """The device selection may differ from the oracle's only in elements whose oracle score lies
    within tol * (K-th score) of the K-th score; what is unique must match exactly.
    floor > 0: magnitudes below it are not resolved by the device's fp32 arithmetic (the decayed
    Mamba score spans hundreds of orders of magnitude).  The band is then tol * max(K-th score,
    floor); every token clearly above it must still be kept, and when the K-th score itself lies
    below the floor the remaining places may go to any tokens below it."""
    import oracle
    idx_dev = np.asarray(idx_dev)
    N = scores_ref.shape[0]
    assert idx_dev.shape == (K,)
    assert (idx_dev >= 0).all() and (idx_dev < N).all()
    assert (np.diff(idx_dev) > 0).all(), "indices must be strictly ascending"
    want = oracle.select_topk(scores_ref, K)
    kth = np.sort(scores_ref)[::-1][K - 1]
    eff = max(abs(kth), floor, 1e-300)
    band = tol * eff
    only_dev = np.setdiff1d(idx_dev, want)
    only_ref = np.setdiff1d(want, idx_dev)
    assert only_dev.size == only_ref.size
    assert (scores_ref[only_ref] <= eff + band).all(), "device dropped a token clearly above the K-th score"
    if abs(kth) >= floor:
        assert (scores_ref[only_dev] >= kth - band).all(), "device kept a token clearly below the K-th score"
    return only_dev.size
