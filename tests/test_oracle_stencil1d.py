"""Pins of the oracle's three-point loop with a caller-supplied body (paper Section 3.3.1,
uninterpreted loop-body function): the generic primal / scatter-adjoint loops against the
oracle's own, separately pinned Burgers and weighted three-point routines, and the example
body of tests/functor_example against finite differences of itself."""
import math
import os
import sys

import numpy as np
import pytest

import inputs
import oracle

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "functor_example"))
import sine_flux  # noqa: E402

C, D = 0.1, 0.05


def _pos(a):
    return a if a > 0.0 else 0.0


def _neg(a):
    return a if a < 0.0 else 0.0


def burgers_f(um, u0, up, p):
    return u0 - C * (_pos(u0) * (u0 - um) + _neg(u0) * (up - u0)) + D * (um - 2.0 * u0 + up)


def burgers_df(um, u0, up, p):
    dpos = 1.0 if u0 >= 0.0 else 0.0
    dneg = 1.0 if -u0 >= 0.0 else 0.0
    return (C * _pos(u0) + D,
            1.0 - C * (dpos * (u0 - um) + _pos(u0) + dneg * (up - u0) - _neg(u0)) - 2.0 * D,
            -C * _neg(u0) + D)


@pytest.mark.parametrize("n", [3, 4, 5, 64, 1000])
def test_generic_loop_with_the_burgers_body_equals_the_burgers_oracle(n):
    d = inputs.burgers_inputs(n, seed=n)
    r = oracle.stencil1d_primal(burgers_f, d["u"])
    assert np.allclose(r, oracle.burgers_primal(d["u"], C, D), rtol=1e-15, atol=1e-16)
    got = oracle.stencil1d_adjoint(burgers_df, d["u"], None, d["r_bar"], d["u_bar"])
    want = oracle.burgers_adjoint(d["u"], d["r_bar"], d["u_bar"], C, D)[0]
    assert np.allclose(got, want, rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("n", [3, 7, 200])
def test_generic_loop_with_a_weighted_linear_body_equals_the_worked_example(n):
    wm, w0, wp = 2.0, -3.0, 4.0
    c = inputs.uniform(n, "c", (n,), 0.5, 1.5)
    u = inputs.uniform(n, "u", (n,), -1, 1)
    rb = inputs.uniform(n, "r_bar", (n,), -1, 1)
    ub = inputs.uniform(n, "u_bar", (n,), -1, 1)
    r = oracle.stencil1d_primal(lambda um, u0, up, p: p * (wm * um + w0 * u0 + wp * up), u, c)
    assert np.allclose(r, oracle.lin3_primal(c, u, 1, n - 2, wm, w0, wp), rtol=1e-15, atol=1e-16)
    got = oracle.stencil1d_adjoint(lambda um, u0, up, p: (p * wm, p * w0, p * wp), u, c, rb, ub)
    assert np.allclose(got, oracle.lin3_adjoint(c, rb, ub, 1, n - 2, wm, w0, wp), rtol=1e-14, atol=1e-15)


def test_untouched_ends_and_scale():
    n = 50
    u = inputs.uniform(1, "u", (n,), -1, 1)
    r0 = np.full(n, 7.0)
    r = oracle.stencil1d_primal(sine_flux.f, u, np.ones(n), r_init=r0)
    assert r[0] == 7.0 and r[-1] == 7.0 and not np.any(r[1:-1] == 7.0)
    rb = np.zeros(n); rb[0] = rb[-1] = np.nan          # outside I: never read
    ub, scale = oracle.stencil1d_adjoint(sine_flux.df, u, np.ones(n), rb, np.zeros(n), want_scale=True)
    assert np.all(ub == 0.0) and np.all(scale == 0.0)


def test_example_body_partials_match_central_differences_of_the_body():
    h = 1e-6
    for k in range(200):
        um, u0, up = (float(v) for v in inputs.uniform(k, "u", (3,), -2, 2))
        p = float(inputs.uniform(k, "c", (1,), 0.2, 1.5)[0])
        dm, d0, dp = sine_flux.df(um, u0, up, p)
        fd = ((sine_flux.f(um + h, u0, up, p) - sine_flux.f(um - h, u0, up, p)) / (2 * h),
              (sine_flux.f(um, u0 + h, up, p) - sine_flux.f(um, u0 - h, up, p)) / (2 * h),
              (sine_flux.f(um, u0, up + h, p) - sine_flux.f(um, u0, up - h, p)) / (2 * h))
        assert np.allclose((dm, d0, dp), fd, rtol=1e-7, atol=1e-8)


def test_example_adjoint_is_the_transposed_jacobian_of_the_example_primal():
    n = 40
    u = inputs.uniform(5, "u", (n,), -1.5, 1.5)
    p = inputs.uniform(5, "c", (n,), 0.2, 1.5)
    rb = inputs.uniform(5, "r_bar", (n,), -1, 1)
    ub0 = inputs.uniform(5, "u_bar", (n,), -1, 1)
    h = 1e-6
    J = np.zeros((n, n))
    for k in range(n):
        e = np.zeros(n); e[k] = h
        J[:, k] = (oracle.stencil1d_primal(sine_flux.f, u + e, p) - oracle.stencil1d_primal(sine_flux.f, u - e, p)) / (2 * h)
    rb_in = rb.copy(); rb_in[0] = rb_in[-1] = 0.0       # rows 0 and n-1 of J are zero anyway
    want = ub0 + J.T @ rb_in
    got = oracle.stencil1d_adjoint(sine_flux.df, u, p, rb, ub0)
    assert np.allclose(got, want, rtol=1e-7, atol=1e-8)
    assert math.isfinite(got.sum())
