"""Pins of the oracle for dense 3^d box stencils with arbitrary weights (the stencils
behind the loop-nest counts 5 / 25 / 125 of paper Section 3.3.4)."""
import numpy as np
import pytest
import scipy.ndimage as ndi

import inputs
import oracle
from jacobians import interior_mask


def _w(ndim, seed):
    return inputs.uniform(seed, "aux", (3,) * ndim, -2.0, 2.0)


def _fields(shape, seed):
    return (inputs.uniform(seed, "u", shape, -1, 1), inputs.uniform(seed, "c", shape, 0.5, 1.5),
            inputs.uniform(seed, "r_bar", shape, -1, 1), inputs.uniform(seed, "u_bar", shape, -1, 1))


@pytest.mark.parametrize("shape", [(17,), (9, 11), (6, 7, 8), (3, 3, 3), (3, 9), (3,)])
def test_primal_is_a_library_correlation_times_c(shape):
    ndim = len(shape)
    w = _w(ndim, 1)
    u, c, _, _ = _fields(shape, 2)
    want = c * ndi.correlate(u, w, mode="constant", cval=0.0)
    r0 = inputs.uniform(3, "u_prev", shape, -1, 1)
    got = oracle.box_primal(w, u, c, r_init=r0)
    m = interior_mask(shape, 1)
    assert np.allclose(got[m], want[m], rtol=1e-13, atol=1e-14)
    assert np.array_equal(got[~m], r0[~m])


@pytest.mark.parametrize("shape", [(3,), (4,), (5,), (12,), (3, 3), (3, 7), (6, 5), (3, 3, 3), (4, 3, 5), (5, 6, 7)])
def test_adjoint_equals_dense_JT_from_primal_unit_vectors(shape):
    ndim = len(shape)
    w = _w(ndim, 4)
    _, c, rb, ub = _fields(shape, 5)
    N = int(np.prod(shape))
    J = np.zeros((N, N))
    for k in range(N):
        e = np.zeros(N)
        e[k] = 1.0
        J[:, k] = oracle.box_primal(w, e.reshape(shape), c).ravel()
    m = interior_mask(shape, 1).ravel()
    got, sc = oracle.box_adjoint(w, c, rb, ub, want_scale=True)
    assert np.allclose(got.ravel(), ub.ravel() + J.T @ np.where(m, rb.ravel(), 0.0), rtol=1e-13, atol=1e-14)
    assert np.allclose(sc.ravel(), np.abs(J).T @ np.where(m, np.abs(rb.ravel()), 0.0), rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("ndim", [1, 2, 3])
def test_core_of_the_adjoint_is_the_mirrored_stencil_applied_to_c_r_bar(ndim):
    """Index shifting (Section 3.3.2): on the core the adjoint gathers w[-o] * (c r_bar)[j+o],
    i.e. a correlation with the point-mirrored weight table."""
    shape = tuple(8 + k for k in range(ndim))
    w = _w(ndim, 6)
    _, c, rb, _ = _fields(shape, 7)
    got, _ = oracle.box_adjoint(w, c, rb, np.zeros(shape))
    mirrored = w[(slice(None, None, -1),) * ndim]
    want = ndi.correlate(c * rb, mirrored, mode="constant", cval=0.0)
    core = interior_mask(shape, 2)
    assert core.sum() > 0
    assert np.allclose(got[core], want[core], rtol=1e-13, atol=1e-14)


def test_one_dimensional_case_is_the_papers_worked_example():
    n = 20
    w = np.array([2.0, -3.0, 4.0])
    _, c, rb, ub = _fields((n + 1,), 8)
    got, _ = oracle.box_adjoint(w, c, rb, ub)
    want = oracle.lin3_adjoint(c, rb, ub, 1, n - 1, 2.0, -3.0, 4.0)   # pinned to the paper's printed statements
    assert np.array_equal(got, want)


def test_values_outside_the_interior_are_never_read():
    shape = (5, 6, 7)
    w = _w(3, 9)
    _, c, rb, ub = _fields(shape, 10)
    m = interior_mask(shape, 1)
    a, _ = oracle.box_adjoint(w, c, rb, ub)
    b, _ = oracle.box_adjoint(w, np.where(m, c, np.nan), np.where(m, rb, np.nan), ub)
    assert np.array_equal(a, b)
