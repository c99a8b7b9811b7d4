"""Pins of the CPU oracle for the 1-D upwinded Burgers stencil (paper Section 4.2).

The primal is tied to closed forms and to the paper's printed primal listing; the
tangent to central finite differences of the primal; the scatter adjoint to the
tangent (dot-product test, dense J^T by a library mat-vec), to the paper's
printed gather core loop, and to what reverse mode fixes at the two ends."""
import numpy as np
import pytest

import inputs
import oracle

C, D = 0.1, 0.05


def _u(n, seed=0):
    return inputs.burgers_inputs(n, seed=seed, waves=3)


# ------------------------------------------------------------------- primal
def test_primal_closed_forms():
    n = 40
    i = np.arange(n, dtype=float)
    # constant state is a fixed point
    r = oracle.burgers_primal(np.full(n, 0.3), C, D)
    assert np.allclose(r[1:-1], 0.3, rtol=0, atol=1e-16) and r[0] == 0 and r[-1] == 0
    # positive linear profile: backward difference, no diffusion:  r = u - C u b
    a, b = 0.2, 0.01
    u = a + b * i
    r = oracle.burgers_primal(u, C, D)
    assert np.allclose(r[1:-1], (u - C * u * b)[1:-1], rtol=1e-13)
    # negative linear profile: forward difference, same closed form
    u = -a - b * i
    r = oracle.burgers_primal(u, C, D)
    assert np.allclose(r[1:-1], (u - C * u * (-b))[1:-1], rtol=1e-13)
    # quadratic positive profile: r = u - C u (u_i-u_{i-1}) + 2 D k
    k = 1e-3
    u = 0.1 + k * i * i
    r = oracle.burgers_primal(u, C, D)
    want = u - C * u * (k * (2 * i - 1)) + D * 2 * k
    assert np.allclose(r[1:-1], want[1:-1], rtol=1e-12)


def test_primal_reflection_symmetry():
    """x -> -x, u -> -u maps the equation to itself; upwinding respects it."""
    d = _u(257, seed=2)
    u = d["u"]
    r = oracle.burgers_primal(u, C, D)
    r2 = oracle.burgers_primal(-u[::-1].copy(), C, D)
    assert np.allclose(r2, -r[::-1], rtol=1e-14, atol=1e-16)


def test_primal_matches_the_papers_printed_listing():
    """Section 4.2 figure, 'Stencil Primal' (written there with fmin/fmax)."""
    d = _u(300, seed=3)
    u = d["u"]
    um, u0, up = u[:-2], u[1:-1], u[2:]
    want = (-C * ((-u0 + up) * np.fmin(0, u0) + (u0 - um) * np.fmax(0, u0))
            + D * (-2.0 * u0 + um + up) + u0)
    r0 = inputs.uniform(4, "aux", (300,), -1, 1)
    got = oracle.burgers_primal(u, C, D, r_init=r0)
    assert np.allclose(got[1:-1], want, rtol=1e-14, atol=1e-16)
    assert got[0] == r0[0] and got[-1] == r0[-1]


# ------------------------------------------------------------------- tangent
def test_tangent_matches_central_differences_away_from_kinks():
    d = _u(2000, seed=5)
    u = d["u"].copy()
    h = 1e-6
    u[np.abs(u) < 1e-3] = 0.01                       # stay clear of the kink at u = 0
    ud = inputs.uniform(5, "u_dot", u.shape, -1, 1)
    fd = (oracle.burgers_primal(u + h * ud, C, D) - oracle.burgers_primal(u - h * ud, C, D)) / (2 * h)
    td = oracle.burgers_tangent(u, ud, C, D)
    assert np.allclose(fd, td, rtol=0, atol=5e-10)
    assert np.abs(td).max() > 0.5


# ------------------------------------------------------------------- adjoint
def test_dot_product_identity():
    d = _u(3001, seed=6)
    ud = inputs.uniform(6, "u_dot", d["u"].shape, -1, 1)
    rd = oracle.burgers_tangent(d["u"], ud, C, D)
    ub, _ = oracle.burgers_adjoint(d["u"], d["r_bar"], np.zeros_like(ud), C, D)
    lhs = np.sum(rd[1:-1] * d["r_bar"][1:-1])
    rhs = np.sum(ud * ub)
    assert abs(lhs - rhs) < 1e-13 * np.sum(np.abs(rd * d["r_bar"]))


@pytest.mark.parametrize("n", [3, 4, 5, 6, 7, 12, 33])
def test_adjoint_equals_dense_JT(n):
    """J by the tangent on unit vectors (pinned to the primal by finite differences
    above); J^T r_bar by a dense library mat-vec.  n = 3..6 have an empty core."""
    d = _u(n, seed=n)
    J = np.zeros((n, n))
    for k in range(n):
        e = np.zeros(n)
        e[k] = 1.0
        J[:, k] = oracle.burgers_tangent(d["u"], e, C, D)
    rb = d["r_bar"].copy()
    rb[0] = rb[-1] = 0.0
    ub, sc = oracle.burgers_adjoint(d["u"], d["r_bar"], d["u_bar"], C, D, want_scale=True)
    assert np.allclose(ub, d["u_bar"] + J.T @ rb, rtol=1e-13, atol=1e-15)
    assert np.allclose(sc, np.abs(J).T @ np.abs(rb), rtol=1e-13, atol=1e-15)


def _partials(um, u0, up):
    """Partial derivatives of one Burgers iteration with respect to its three reads, from the
    upwind formula of Section 4.2; d max(a,0)/da = d min(a,0)/da = 1 at a == 0 (the convention of
    the paper's generated adjoint)."""
    pos, neg = np.maximum(u0, 0.0), np.minimum(u0, 0.0)
    ipos, ineg = (u0 >= 0).astype(float), (u0 <= 0).astype(float)
    g_left = C * pos + D
    g_right = -C * neg + D
    g_centre = 1.0 - 2.0 * D - C * (ipos * (u0 - um) + pos + ineg * (up - u0) - neg)
    return g_left, g_centre, g_right


def test_adjoint_core_is_the_three_shifted_partials_gathered():
    """On the core [2, n-3] every u_bar[j] receives the left-read partial of iteration j+1, the
    centre partial of iteration j and the right-read partial of iteration j-1 (Section 4.2's
    adjoint, Section 3.3.2's index shifting), here as whole-array expressions; a few u are set to
    exactly 0 so that the convention at the kink is covered as well."""
    n = 500
    d = _u(n, seed=8)
    u = d["u"].copy()
    u[[10, 11, 200, 201, 202, 350]] = 0.0
    rb, ub_in = d["r_bar"], d["u_bar"]
    gl, gc, gr = _partials(u[:-2], u[1:-1], u[2:])          # of iterations 1 .. n-2 (array index i-1)
    j = np.arange(2, n - 2)
    want = ub_in[j] + gl[j] * rb[j + 1] + gc[j - 1] * rb[j] + gr[j - 2] * rb[j - 1]
    got, _ = oracle.burgers_adjoint(u, rb, ub_in, C, D)
    assert np.allclose(got[2:n - 2], want, rtol=1e-13, atol=1e-15)


def test_adjoint_end_points_receive_only_the_terms_whose_primal_iteration_exists():
    """j = 0 is read only by iteration 1 (its left read), j = n-1 only by iteration
    n-2 (its right read); j = 1 and j = n-2 miss one term each (Section 3.2)."""
    n = 64
    d = _u(n, seed=9)
    u, rb = d["u"], d["r_bar"]
    got, _ = oracle.burgers_adjoint(u, rb, np.zeros(n), C, D)
    assert np.isclose(got[0], (C * max(u[1], 0.0) + D) * rb[1], rtol=1e-14)
    assert np.isclose(got[n - 1], (-C * min(u[n - 2], 0.0) + D) * rb[n - 2], rtol=1e-14)
    # NaN outside the primal interior of r_bar must not matter
    rp = rb.copy()
    rp[0] = rp[-1] = np.nan
    got2, _ = oracle.burgers_adjoint(u, rp, np.zeros(n), C, D)
    assert np.array_equal(got, got2)


def test_conservation_sum():
    """sum_j (J^T r_bar)_j = sum_i r_bar_i * (row sum of J_i); the diffusion part has
    zero row sum, the convection part leaves  -C*([u>=0](u_i-u_{i-1}) + [u<=0](u_{i+1}-u_i))."""
    d = _u(5000, seed=11)
    u, rb = d["u"], d["r_bar"]
    got, sc = oracle.burgers_adjoint(u, rb, np.zeros_like(u), C, D, want_scale=True)
    um, u0, up = u[:-2], u[1:-1], u[2:]
    rows = 1.0 - C * ((u0 >= 0) * (u0 - um) + (u0 <= 0) * (up - u0))
    assert abs(got.sum() - np.sum(rows * rb[1:-1])) < 1e-13 * sc.sum()


def test_bad_arguments_are_rejected():
    with pytest.raises(ValueError):
        oracle.burgers_adjoint(np.zeros(2), np.zeros(2), np.zeros(2), C, D)
