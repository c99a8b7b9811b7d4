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


def wave_primal_scale(u, u_prev, c, radius):
    """sum of the magnitudes of the terms of r[i] = 2u[i] - u_prev[i] + c[i] sum_o w_o u[i+o]: the
    scale against which a differently ordered evaluation of the primal is compared."""
    import scipy.ndimage as ndi
    from jacobians import star_weights
    u = np.abs(np.asarray(u, dtype=np.float64))
    w = np.abs(star_weights(radius))
    nd = u.ndim
    k = np.zeros((2 * radius + 1,) * nd)
    k[(radius,) * nd] = nd * w[0]
    for axis in range(nd):
        for o in range(1, radius + 1):
            for sgn in (-1, 1):
                pos = [radius] * nd
                pos[axis] += sgn * o
                k[tuple(pos)] = w[o]
    star = ndi.correlate(u, k, mode="constant")
    return 2.0 * u + np.abs(np.asarray(u_prev, dtype=np.float64)) + np.abs(np.asarray(c, dtype=np.float64)) * star
