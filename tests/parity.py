"""Shared helpers of the GPU parity tests: error measure and host<->device glue."""
import numpy as np

TOL = {np.dtype(np.float64): 1e-12, np.dtype(np.float32): 1e-5}


def to_gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t):
    return t.detach().cpu().numpy()


def rel_err(got, want, scale):
    """max_j |got_j - want_j| / max(|want_j|, scale_j): the error relative to the
    magnitude of what was summed into element j (the two sides add the same terms in
    a different order, so the rounding error scales with sum |terms|, not with the
    possibly cancelled result)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = np.maximum(np.abs(want), scale)
    diff = np.abs(got - want)
    bad = ~np.isfinite(got)
    if bad.any():
        return np.inf
    nz = den > 0
    out = 0.0
    if nz.any():
        out = float(np.max(diff[nz] / den[nz]))
    if (~nz).any() and np.max(diff[~nz]) > 0:
        return np.inf
    return out


def norm_err(got, want):
    """The plain measure max|got - want| / max|want| over the whole array."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    den = float(np.max(np.abs(want))) if want.size else 0.0
    num = float(np.max(np.abs(got - want))) if want.size else 0.0
    return num / den if den > 0 else (0.0 if num == 0 else np.inf)


def assert_close(got, want, scale, dtype, what=""):
    err = rel_err(got, want, scale)
    tol = TOL[np.dtype(dtype)]
    assert err <= tol, "%s: max relative error %.3e > %.1e" % (what, err, tol)
    plain = norm_err(got, want)
    assert plain <= tol, "%s: max|g-o|/max|o| = %.3e > %.1e" % (what, plain, tol)
    return err
