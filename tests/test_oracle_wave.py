"""Pins of the CPU oracle for the linear wave stencil (1-D, 2-D, 3-D; radius 1..4).

None of these tests compares the oracle with itself: each ties it to the
mathematics (polynomial exactness, conservation, zero rows), to a library routine
(scipy.ndimage.correlate, scipy.sparse Kronecker assembly + mat-vec, dense
mat-vec), or to a listing the paper prints (Section 4.1, the figure with the
primal, the gather adjoint and the scatter adjoint of the 3-D wave step)."""
import itertools

import numpy as np
import pytest
import scipy.ndimage as ndi

import inputs
import oracle
from jacobians import STAR, interior_mask, star_weights, wave_jacobians

SHAPES = {1: [(23,)], 2: [(13, 17)], 3: [(11, 12, 13)]}


def _fields(shape, seed=0, c_mode="iid"):
    return inputs.wave_inputs(shape, 0.01, 0.25, seed=seed, c_mode=c_mode)


def _shapes_for(radius):
    out = []
    for nd in (1, 2, 3):
        base = 4 * radius + 3
        out.append(tuple(base + k for k in range(nd)))
    return out


# ----------------------------------------------------------------- the weights
@pytest.mark.parametrize("radius", [1, 2, 3, 4])
def test_weights_are_the_textbook_rationals(radius):
    w = oracle.star_weights(radius)
    assert np.array_equal(w, star_weights(radius))
    full = [STAR[radius][abs(k)] for k in range(-radius, radius + 1)]
    assert sum(full) == 0
    assert sum(f * k * k for f, k in zip(full, range(-radius, radius + 1))) == 2
    for p in range(4, 2 * radius + 1, 2):          # higher even moments vanish
        assert sum(f * k ** p for f, k in zip(full, range(-radius, radius + 1))) == 0


@pytest.mark.parametrize("radius", [1, 2, 3, 4])
def test_primal_laplacian_is_exact_on_polynomials(radius):
    """With c = 1, u_prev = 0:  r - 2u = Lap(u); a radius-R star differentiates
    polynomials of degree <= 2R+1 exactly."""
    n = 4 * radius + 4
    z, y, x = np.meshgrid(np.arange(n, dtype=float), np.arange(n + 1, dtype=float),
                          np.arange(n + 2, dtype=float), indexing="ij")
    z, y, x = z / 8.0, y / 8.0, x / 8.0          # spacing 1/8: scale Lap by 64
    px, py, pz = 2 * radius + 1, 2 * radius, 2
    u = x ** px + 3.0 * y ** py - 0.5 * z ** pz + x * y * z
    lap_exact = (px * (px - 1) * x ** (px - 2) + 3.0 * py * (py - 1) * y ** (py - 2) - 0.5 * 2.0)
    r = oracle.wave_primal(u, np.zeros_like(u), np.ones_like(u), radius)
    m = interior_mask(u.shape, radius)
    got = (r - 2.0 * u)[m] * 64.0
    assert np.allclose(got, lap_exact[m], rtol=1e-10, atol=1e-9)
    assert np.all(r[~m] == 0.0)


# ------------------------------------------------- primal against library routine
@pytest.mark.parametrize("radius", [1, 2, 3, 4])
@pytest.mark.parametrize("ndim", [1, 2, 3])
def test_primal_matches_ndimage_correlate(radius, ndim):
    shape = _shapes_for(radius)[ndim - 1]
    d = _fields(shape, seed=radius)
    w = star_weights(radius)
    kern = np.zeros((2 * radius + 1,) * ndim)
    centre = (radius,) * ndim
    kern[centre] = ndim * w[0]
    for ax in range(ndim):
        for k in range(1, radius + 1):
            for s in (-k, k):
                idx = list(centre)
                idx[ax] += s
                kern[tuple(idx)] = w[k]
    lap = ndi.correlate(d["u"], kern, mode="constant", cval=0.0)
    want = 2.0 * d["u"] - d["u_prev"] + d["c"] * lap
    m = interior_mask(shape, radius)
    r0 = inputs.uniform(5, "aux", shape, -1, 1)
    got = oracle.wave_primal(d["u"], d["u_prev"], d["c"], radius, r_init=r0)
    assert np.allclose(got[m], want[m], rtol=1e-13, atol=1e-14)
    assert np.array_equal(got[~m], r0[~m])           # r outside I is left alone


def test_primal_matches_the_papers_printed_listing():
    """Section 4.1 figure, 'Stencil primal': D*(-6u1 + six neighbours)*c + 2u1 - u2 on
    [1,n-2]^3 (D folded into c)."""
    n = 9
    d = _fields((n, n, n), seed=3)
    u1, u2, c = d["u"], d["u_prev"], d["c"]
    s = slice(1, n - 1)
    want = ((-6 * u1[s, s, s] + u1[s, s, 0:n - 2] + u1[s, s, 2:n] + u1[s, 0:n - 2, s]
             + u1[s, 2:n, s] + u1[0:n - 2, s, s] + u1[2:n, s, s]) * c[s, s, s]
            + 2.0 * u1[s, s, s] - u2[s, s, s])
    got = oracle.wave_primal(u1, u2, c, 1)
    assert np.allclose(got[s, s, s], want, rtol=1e-13, atol=1e-14)


# ----------------------------------------------------- adjoint: dot-product test
@pytest.mark.parametrize("radius", [1, 2, 3, 4])
@pytest.mark.parametrize("ndim", [1, 2, 3])
def test_dot_product_identity(radius, ndim):
    shape = _shapes_for(radius)[ndim - 1]
    d = _fields(shape, seed=10 + radius)
    ud = inputs.uniform(1, "u_dot", shape, -1, 1)
    upd = inputs.uniform(1, "u_prev_dot", shape, -1, 1)
    rd = oracle.wave_tangent(d["c"], ud, upd, radius)
    zero = np.zeros(shape)
    ub, upb, _ = oracle.wave_adjoint(d["c"], d["r_bar"], zero, radius, u_prev_bar=zero)
    m = interior_mask(shape, radius)
    lhs = np.sum(rd[m] * d["r_bar"][m])
    rhs = np.sum(ud * ub) + np.sum(upd * upb)
    assert abs(lhs - rhs) <= 1e-13 * (np.sum(np.abs(rd[m] * d["r_bar"][m])) + 1.0)


@pytest.mark.parametrize("radius", [1, 4])
@pytest.mark.parametrize("ndim", [1, 2, 3])
def test_tangent_matches_central_differences_of_the_primal(radius, ndim):
    shape = _shapes_for(radius)[ndim - 1]
    d = _fields(shape, seed=20 + radius)
    ud = inputs.uniform(2, "u_dot", shape, -1, 1)
    upd = inputs.uniform(2, "u_prev_dot", shape, -1, 1)
    h = 2.0 ** -10                                   # power of two; the map is linear
    fp = oracle.wave_primal(d["u"] + h * ud, d["u_prev"] + h * upd, d["c"], radius)
    fm = oracle.wave_primal(d["u"] - h * ud, d["u_prev"] - h * upd, d["c"], radius)
    fd = (fp - fm) / (2 * h)
    rd = oracle.wave_tangent(d["c"], ud, upd, radius)
    assert np.allclose(fd, rd, rtol=0, atol=1e-11)


# --------------------------------- adjoint: assembled Jacobian, library mat-vec
@pytest.mark.parametrize("shape,radius", [((9,), 1), ((7, 8), 1), ((5, 6, 7), 1), ((9, 10, 11), 4),
                                          ((12, 11), 2)])
def test_adjoint_equals_dense_JT_from_primal_unit_vectors(shape, radius):
    """Column k of J is the primal applied to the k-th unit vector (the stencil is
    linear); J^T r_bar is a dense library mat-vec."""
    d = _fields(shape, seed=31)
    N = int(np.prod(shape))
    zero = np.zeros(shape)
    Ju = np.zeros((N, N))
    Jp = np.zeros((N, N))
    for k in range(N):
        e = np.zeros(N)
        e[k] = 1.0
        Ju[:, k] = oracle.wave_primal(e.reshape(shape), zero, d["c"], radius).ravel()
        Jp[:, k] = oracle.wave_primal(zero, e.reshape(shape), d["c"], radius).ravel()
    m = interior_mask(shape, radius).ravel()
    rb = np.where(m, d["r_bar"].ravel(), 0.0)
    want_u = d["u_bar"].ravel() + Ju.T @ rb
    want_p = d["u_prev_bar"].ravel() + Jp.T @ rb
    ub, upb, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius, u_prev_bar=d["u_prev_bar"])
    assert np.allclose(ub.ravel(), want_u, rtol=1e-13, atol=1e-14)
    assert np.allclose(upb.ravel(), want_p, rtol=1e-13, atol=1e-14)


def _brute_force_shapes():
    out = []
    for radius in (1, 2, 3, 4):
        lo, hi = 2 * radius + 1, 4 * radius + 3
        out += [((n,), radius) for n in range(lo, hi + 1)]
    for ny, nx in itertools.product(range(3, 8), repeat=2):
        out.append(((ny, nx), 1))
    for nz, ny, nx in itertools.product((3, 4, 5, 7), repeat=3):
        out.append(((nz, ny, nx), 1))
    sizes4 = (9, 10, 13, 16, 17, 19)
    for ny, nx in itertools.product(sizes4, repeat=2):
        out.append(((ny, nx), 4))
    for nz, ny, nx in [(9, 9, 9), (9, 17, 10), (16, 9, 19), (17, 17, 17), (19, 10, 13), (10, 19, 16),
                       (13, 13, 9), (19, 19, 19)]:
        out.append(((nz, ny, nx), 4))
    return out


def test_adjoint_equals_sparse_kronecker_JT_on_all_small_sizes():
    """Every size from 'interior is one cell' (2R+1) to 'core is three cells' (4R+3),
    including all sizes whose core is empty.  J is assembled from banded Toeplitz
    blocks with scipy.sparse.kron, independently of the oracle."""
    for shape, radius in _brute_force_shapes():
        d = _fields(shape, seed=sum(shape) + radius)
        ju, jp = wave_jacobians(d["c"], radius)
        want_u = d["u_bar"].ravel() + ju.T @ d["r_bar"].ravel()
        want_p = d["u_prev_bar"].ravel() + jp.T @ d["r_bar"].ravel()
        ub, upb, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius,
                                         u_prev_bar=d["u_prev_bar"])
        assert np.allclose(ub.ravel(), want_u, rtol=1e-13, atol=1e-14), (shape, radius)
        assert np.allclose(upb.ravel(), want_p, rtol=1e-13, atol=1e-14), (shape, radius)


# ----------------------------------------------- adjoint: the paper's own listings
def test_adjoint_core_matches_the_papers_printed_gather_loop():
    """Section 4.1 figure, 'PerforAD stencil adjoint': on [2,n-3]^3 the update of
    u_1_b gathers c*u_b from the six neighbours plus (-6c+2)*u_b at the centre, and
    u_2_b receives -u_b."""
    n = 10
    d = _fields((n, n, n), seed=41)
    c, rb = d["c"], d["r_bar"]
    q = c * rb
    s = slice(2, n - 2)
    lo, hi = slice(1, n - 3), slice(3, n - 1)
    want = (d["u_bar"][s, s, s] + q[s, s, hi] + q[s, hi, s] + q[hi, s, s]
            + (-6 * c[s, s, s] + 2.0) * rb[s, s, s] + q[lo, s, s] + q[s, lo, s] + q[s, s, lo])
    ub, upb, _ = oracle.wave_adjoint(c, rb, d["u_bar"], 1, u_prev_bar=d["u_prev_bar"])
    assert np.allclose(ub[s, s, s], want, rtol=1e-13, atol=1e-14)
    assert np.allclose(upb[s, s, s], d["u_prev_bar"][s, s, s] - rb[s, s, s], rtol=0, atol=1e-15)


def test_adjoint_on_the_whole_grid_is_a_sum_of_shifted_copies_of_c_times_r_bar():
    """Section 4.1's conventional adjoint sends t = c*r_bar of every interior point to its six
    neighbours and 2 r_bar - 6 t to the point itself.  Over the whole grid, boundary layers
    included, that is: the interior block of t added at the six shifted positions.  Written with
    whole-array slices, in no particular order (the result is order-independent up to rounding)."""
    n = 7
    d = _fields((n, n, n), seed=43)
    c, rb = d["c"], d["r_bar"]
    s = slice(1, n - 1)
    t = (c * rb)[s, s, s]
    want = d["u_bar"].copy()
    want[s, s, s] += 2.0 * rb[s, s, s] - 6.0 * t
    for axis in range(3):
        for shift in (-1, 1):
            idx = [s, s, s]
            idx[axis] = slice(1 + shift, n - 1 + shift)
            want[tuple(idx)] += t
    wantp = d["u_prev_bar"].copy()
    wantp[s, s, s] -= rb[s, s, s]
    ub, upb, _ = oracle.wave_adjoint(c, rb, d["u_bar"], 1, u_prev_bar=d["u_prev_bar"])
    assert np.allclose(ub, want, rtol=1e-13, atol=1e-14)
    assert np.allclose(upb, wantp, rtol=0, atol=1e-15)


# ---------------------------------------------------- adjoint: special cases, invariants
@pytest.mark.parametrize("radius", [1, 4])
@pytest.mark.parametrize("ndim", [1, 2, 3])
def test_constant_c_makes_the_core_operator_self_adjoint(radius, ndim):
    """Symmetric data flow: with c constant, on the core the adjoint update equals
    the primal operator applied to r_bar, i.e. 2 r_bar + c Lap(r_bar)."""
    shape = tuple(4 * radius + 4 + k for k in range(ndim))
    d = _fields(shape, seed=50)
    c0 = 0.07
    c = np.full(shape, c0)
    ub, _, _ = oracle.wave_adjoint(c, d["r_bar"], np.zeros(shape), radius)
    prim = oracle.wave_primal(d["r_bar"], np.zeros(shape), c, radius)
    core = interior_mask(shape, 2 * radius)
    assert core.sum() > 0
    assert np.allclose(ub[core], prim[core], rtol=1e-13, atol=1e-14)


@pytest.mark.parametrize("radius", [1, 2, 4])
@pytest.mark.parametrize("ndim", [1, 2, 3])
def test_conservation_sum(radius, ndim):
    """sum_j (J^T r_bar)_j = sum_i r_bar_i * (row sum of J) = 2 sum_{i in I} r_bar_i,
    because the Laplacian weights sum to zero."""
    shape = tuple(3 * radius + 2 + k for k in range(ndim))
    d = _fields(shape, seed=60)
    ub, _, sc = oracle.wave_adjoint(d["c"], d["r_bar"], np.zeros(shape), radius, want_scale=True)
    m = interior_mask(shape, radius)
    assert abs(ub.sum() - 2.0 * d["r_bar"][m].sum()) < 1e-12 * sc.sum()


@pytest.mark.parametrize("radius", [1, 4])
def test_rows_without_contribution_stay_untouched_and_outside_values_are_never_read(radius):
    """A star reaches index j only if at most one coordinate of j lies outside the
    primal interior; r_bar and c outside the interior are never read (NaN there
    must not propagate)."""
    shape = (3 * radius + 3, 3 * radius + 2, 3 * radius + 4)
    d = _fields(shape, seed=70)
    m = interior_mask(shape, radius)
    outside_count = np.zeros(shape, dtype=int)
    for ax, n in enumerate(shape):
        idx = np.arange(n)
        out = (idx < radius) | (idx > n - 1 - radius)
        outside_count += out.reshape([-1 if a == ax else 1 for a in range(3)])
    ub, upb, sc = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius,
                                      u_prev_bar=d["u_prev_bar"], want_scale=True)
    untouched = outside_count >= 2
    assert np.array_equal(ub[untouched], d["u_bar"][untouched])
    assert np.all(sc[untouched] == 0)
    assert np.all(sc[~untouched] > 0)
    assert np.array_equal(upb[~m], d["u_prev_bar"][~m])
    cp, rp = d["c"].copy(), d["r_bar"].copy()
    cp[~m] = np.nan
    rp[~m] = np.nan
    ub2, upb2, _ = oracle.wave_adjoint(cp, rp, d["u_bar"], radius, u_prev_bar=d["u_prev_bar"])
    assert np.array_equal(ub2, ub) and np.array_equal(upb2, upb)


def test_scale_bounds_the_update_and_optional_output_does_not_change_u_bar():
    shape = (10, 11, 12)
    d = _fields(shape, seed=80)
    ub, _, sc = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 4, want_scale=True)
    ub2, upb2, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 4, u_prev_bar=d["u_prev_bar"])
    assert np.array_equal(ub, ub2)
    assert np.all(np.abs(ub - d["u_bar"]) <= sc + 1e-14 * (np.abs(d["u_bar"]) + sc))
    # the scale is the adjoint of the same stencil with every factor replaced by its magnitude
    ju, _ = wave_jacobians(d["c"], 4)
    assert np.allclose(sc.ravel(), abs(ju).T @ np.abs(d["r_bar"].ravel()), rtol=1e-13)


def test_inputs_are_not_modified_and_fp32_inputs_are_widened():
    shape = (9, 9, 9)
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=1, dtype=np.float32)
    keep = {k: v.copy() for k, v in d.items()}
    ub, _, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 4)
    assert ub.dtype == np.float64
    for k in d:
        assert np.array_equal(d[k], keep[k])
    ub64, _, _ = oracle.wave_adjoint(d["c"].astype(np.float64), d["r_bar"].astype(np.float64),
                                     d["u_bar"].astype(np.float64), 4)
    assert np.array_equal(ub, ub64)


def test_bad_arguments_are_rejected():
    z = np.zeros((8, 9, 9))
    with pytest.raises(ValueError):
        oracle.wave_adjoint(z, z, z, 4)          # nz = 8 < 2R+1
    with pytest.raises(ValueError):
        oracle.wave_adjoint(np.zeros((9, 9, 9)), np.zeros((9, 9, 9)), np.zeros((9, 9, 9)), 5)


@pytest.mark.parametrize("radius,shape", [(4, (13, 17, 21)), (4, (9, 9, 9)), (4, (20, 11, 30)), (1, (3, 3, 3)), (1, (5, 6, 7))])
def test_scatter_order_emulation_equals_the_sequential_scatter_bit_for_bit(radius, shape):
    """The whole-array formulation of the scatter's summation order (tests/scatter_order.py)
    must reproduce the oracle's sequential loop exactly, signs of zeros included; it then
    serves as the fp32 reference of the library's scatter-order mode (Section 3.5)."""
    from scatter_order import wave3d_adjoint_scatter_order
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=radius + shape[0], c_mode="iid")
    d["u_bar"][1, 1, :] = -0.0
    want = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius)[0]
    got = wave3d_adjoint_scatter_order(d["c"], d["r_bar"], d["u_bar"], radius)
    assert np.array_equal(got.view(np.int64), want.view(np.int64))
