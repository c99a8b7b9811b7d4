"""Randomised property checks of the oracle (hypothesis): identities that hold for every
shape, radius and field, so that a mistake which happens to cancel on the hand-picked
cases of the other test files still has to survive many drawn ones."""
import numpy as np
import scipy.ndimage as ndi
from hypothesis import given, settings, strategies as st

import inputs
import oracle
from jacobians import interior_mask

PROFILE = dict(max_examples=40, deadline=None, derandomize=True)


@st.composite
def wave_case(draw):
    ndim = draw(st.integers(1, 3))
    radius = draw(st.integers(1, 4))
    shape = tuple(draw(st.integers(2 * radius + 1, 2 * radius + 7)) for _ in range(ndim))
    seed = draw(st.integers(0, 10 ** 6))
    return radius, shape, seed


@settings(**PROFILE)
@given(wave_case())
def test_wave_dot_product_identity_and_linearity(case):
    radius, shape, seed = case
    d = inputs.wave_inputs(shape, 0.01, 0.3, seed=seed, c_mode="iid")
    z = np.zeros(shape)
    u_dot, p_dot = d["u"], d["u_prev"]
    r_dot = oracle.wave_tangent(d["c"], u_dot, p_dot, radius)
    ub, pb, _ = oracle.wave_adjoint(d["c"], d["r_bar"], z, radius, u_prev_bar=z)
    m = interior_mask(shape, radius)
    lhs = float(np.sum(r_dot[m] * d["r_bar"][m]))
    rhs = float(np.sum(u_dot * ub) + np.sum(p_dot * pb))
    scale = float(np.sum(np.abs(u_dot * ub)) + np.sum(np.abs(p_dot * pb))) + 1e-300
    assert abs(lhs - rhs) <= 1e-13 * scale
    # accumulate semantics and linearity in r_bar
    ub2, _, _ = oracle.wave_adjoint(d["c"], 3.0 * d["r_bar"], d["u_bar"], radius)
    assert np.allclose(ub2, d["u_bar"] + 3.0 * ub, rtol=1e-13, atol=1e-14)
    # nothing outside the interior of r_bar or c is ever read
    poisoned_r = np.where(m, d["r_bar"], np.nan)
    poisoned_c = np.where(m, d["c"], np.nan)
    ub3, _, _ = oracle.wave_adjoint(poisoned_c, poisoned_r, z, radius)
    assert np.array_equal(ub3, ub)


@st.composite
def box_case(draw):
    ndim = draw(st.integers(1, 3))
    shape = tuple(draw(st.integers(3, 9)) for _ in range(ndim))
    seed = draw(st.integers(0, 10 ** 6))
    return shape, seed


@settings(**PROFILE)
@given(box_case())
def test_box_adjoint_is_the_transpose_of_the_box_primal(case):
    shape, seed = case
    ndim = len(shape)
    w = inputs.uniform(seed, "aux", (3,) * ndim, -2.0, 2.0)
    c = inputs.uniform(seed, "c", shape, 0.5, 1.5)
    u = inputs.uniform(seed, "u", shape, -1, 1)
    rb = inputs.uniform(seed, "r_bar", shape, -1, 1)
    m = interior_mask(shape, 1)
    r = oracle.box_primal(w, u, c)
    # the primal is a correlation with the weight table, scaled by c, on the interior
    assert np.allclose(r[m], (c * ndi.correlate(u, w, mode="constant"))[m], rtol=1e-13, atol=1e-14)
    ub = oracle.box_adjoint(w, c, rb, np.zeros(shape))[0]
    lhs = float(np.sum(r[m] * rb[m]))
    rhs = float(np.sum(u * ub))
    assert abs(lhs - rhs) <= 1e-13 * (float(np.sum(np.abs(u * ub))) + 1e-300)


@settings(**PROFILE)
@given(st.integers(3, 40), st.integers(0, 10 ** 6), st.floats(0.0, 0.4), st.floats(0.0, 0.3))
def test_burgers_dot_product_identity(n, seed, C, D):
    d = inputs.burgers_inputs(n, seed=seed)
    u_dot = inputs.uniform(seed, "u_prev", (n,), -1, 1)
    r_dot = oracle.burgers_tangent(d["u"], u_dot, C, D)
    ub, _ = oracle.burgers_adjoint(d["u"], d["r_bar"], np.zeros(n), C, D)
    lhs = float(np.sum(r_dot[1:-1] * d["r_bar"][1:-1]))
    rhs = float(np.sum(u_dot * ub))
    assert abs(lhs - rhs) <= 1e-13 * (float(np.sum(np.abs(u_dot * ub))) + 1e-300)
