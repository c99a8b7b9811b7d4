"""Pins of the oracle's star-shaped loop with a caller-supplied body in one to three
dimensions (paper Section 3.3.1: uninterpreted loop body and derivative functions; its example
is two-dimensional).  The generic primal / scatter-adjoint loops are checked against the
oracle's separately pinned wave, free-weight star and three-point routines, against
whole-array numpy formulations of the paper's 2-D example, and against finite differences
and the dot-product identity for a nonlinear body."""
import os
import sys

import numpy as np
import pytest

import inputs
import oracle

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "functor_example"))
import star_bodies  # noqa: E402


def _fields(shape, seed):
    mk = lambda name, lo, hi: inputs.uniform(seed, name, shape, lo, hi)
    return mk("u", -1, 1), mk("c", 0.01, 0.2), mk("r_bar", -1, 1), mk("u_bar", -1, 1)


@pytest.mark.parametrize("shape,R", [((9,), 1), ((12,), 4), ((7, 9), 1), ((11, 13), 2), ((5, 6, 7), 1),
                                     ((9, 10, 11), 2), ((9, 9, 10), 4)])
def test_linear_wave_body_equals_the_wave_oracle(shape, R):
    u, c, rb, ub = _fields(shape, 3)
    f, df = star_bodies.lin_wave(list(oracle.star_weights(R)))
    r = oracle.starfn_primal(f, u, c, R)
    want = oracle.wave_primal(u, np.zeros_like(u), c, R)
    assert np.allclose(r, want, rtol=1e-14, atol=1e-15)
    got = oracle.starfn_adjoint(df, u, c, rb, ub, R)
    assert np.allclose(got, oracle.wave_adjoint(c, rb, ub, R)[0], rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("R", [1, 2, 3])
def test_free_weight_body_equals_the_star_oracle_and_mirrors_offsets(R):
    shape = (2 * R + 3, 2 * R + 4, 2 * R + 6)
    u, c, rb, ub = _fields(shape, 5)
    w = list(inputs.uniform(7, "aux", (1 + 6 * R,), -1, 1))          # asymmetric on purpose
    r = oracle.starfn_primal(lambda v, p: p * sum(a * b for a, b in zip(w, v)), u, c, R)
    assert np.allclose(r, oracle.star3d_primal(w, u, c, R), rtol=1e-14, atol=1e-15)
    got = oracle.starfn_adjoint(lambda v, p: [p * a for a in w], u, c, rb, ub, R)
    assert np.allclose(got, oracle.star3d_adjoint(w, c, rb, ub, R)[0], rtol=1e-14, atol=1e-15)


def test_one_dimensional_case_equals_the_three_point_callback_loop():
    n = 40
    u, c, rb, ub = _fields((n,), 9)
    f3 = lambda um, u0, up, p: u0 * up - p * um * um
    d3 = lambda um, u0, up, p: (-2.0 * p * um, up, u0)
    r = oracle.starfn_primal(lambda v, p: f3(v[1], v[0], v[2], p), u, c, 1)
    assert np.array_equal(r, oracle.stencil1d_primal(f3, u, c))
    got = oracle.starfn_adjoint(lambda v, p: (lambda d: [d[1], d[0], d[2]])(d3(v[1], v[0], v[2], p)), u, c, rb, ub, 1)
    assert np.allclose(got, oracle.stencil1d_adjoint(d3, u, c, rb, ub), rtol=1e-15, atol=1e-16)


def test_the_papers_two_dimensional_example_against_shifted_whole_array_sums():
    # r[y, x] = a b + p a,  a = u[y, x-1], b = u[y-1, x]  on I = [1, n-2]^2
    ny, nx = 8, 11
    u, p, rb, ub = _fields((ny, nx), 11)
    r = oracle.starfn_primal(star_bodies.pair_product_f, u, p, 1)
    a, b = u[1:-1, 0:-2], u[0:-2, 1:-1]
    want = np.zeros_like(u)
    want[1:-1, 1:-1] = a * b + p[1:-1, 1:-1] * a
    assert np.allclose(r, want, rtol=1e-15, atol=1e-16)
    got = oracle.starfn_adjoint(star_bodies.pair_product_df, u, p, rb, ub, 1)
    wantb = ub.copy()
    wantb[1:-1, 0:-2] += (b + p[1:-1, 1:-1]) * rb[1:-1, 1:-1]      # df/da lands on u_bar[y, x-1]
    wantb[0:-2, 1:-1] += a * rb[1:-1, 1:-1]                        # df/db lands on u_bar[y-1, x]
    assert np.allclose(got, wantb, rtol=1e-14, atol=1e-15)
    # rows and columns no iteration reads stay untouched
    assert np.array_equal(got[-1, :], ub[-1, :]) and np.array_equal(got[:, -1], ub[:, -1])


@pytest.mark.parametrize("shape", [(6, 7), (5, 6, 7)])
def test_nonlinear_body_adjoint_against_central_differences_and_dot_product(shape):
    u, p, rb, ub = _fields(shape, 13)
    du = inputs.uniform(17, "u_dot", shape, -1, 1)
    f, df = star_bodies.soft_wave_f, star_bodies.soft_wave_df
    h = 1e-6
    jdu = (oracle.starfn_primal(f, u + h * du, p, 1) - oracle.starfn_primal(f, u - h * du, p, 1)) / (2 * h)
    jt_rb = oracle.starfn_adjoint(df, u, p, rb, np.zeros_like(u), 1)
    lhs, rhs = float(np.sum(jdu * rb)), float(np.sum(jt_rb * du))
    assert abs(lhs - rhs) <= 1e-8 * max(1.0, abs(lhs))
    # accumulation: the incoming u_bar is added to, not overwritten
    assert np.allclose(oracle.starfn_adjoint(df, u, p, rb, ub, 1), ub + jt_rb, rtol=1e-14, atol=1e-15)


def test_values_outside_the_iteration_space_are_never_used():
    shape = (5, 6, 7)
    u, p, rb, ub = _fields(shape, 19)
    rb2, p2 = rb.copy(), p.copy()
    m = np.zeros(shape, dtype=bool)
    m[1:-1, 1:-1, 1:-1] = True
    rb2[~m] = np.nan
    p2[~m] = np.nan
    got = oracle.starfn_adjoint(star_bodies.soft_wave_df, u, p2, rb2, ub, 1)
    assert np.array_equal(got, oracle.starfn_adjoint(star_bodies.soft_wave_df, u, p, rb, ub, 1))
