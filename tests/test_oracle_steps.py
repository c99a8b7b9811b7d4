"""Pins of the oracle's reverse sweep over a time loop of wave steps.

The sweep is tied to (i) the forward time loop built from the (already pinned) tangent
step through the dot-product identity, (ii) products of independently assembled
sparse Jacobians, (iii) the single-step adjoint for nsteps = 1, and (iv) the fact that a
buffer recycled for an older state must start from zero."""
import numpy as np
import pytest

import inputs
import oracle
from jacobians import interior_mask, wave_jacobians


def _lams(shape, seed):
    return [inputs.uniform(seed, name, shape, -1, 1) for name in ("r_bar", "u_bar", "u_prev_bar")]


def _forward_tangent(c, ud_prev, ud_cur, radius, nsteps):
    """u_dot^{k+1} = J_u u_dot^k + J_p u_dot^{k-1} on I, zero outside I (cells outside I of
    a new state are inputs with zero tangent)."""
    prev, cur = ud_prev, ud_cur
    for _ in range(nsteps):
        prev, cur = cur, oracle.wave_tangent(c, cur, prev, radius)
    return prev, cur


@pytest.mark.parametrize("shape,radius,nsteps", [((23,), 1, 5), ((9, 11), 1, 4), ((7, 8, 9), 1, 3),
                                                 ((10, 11, 12), 4, 1), ((10, 11, 12), 4, 2), ((10, 11, 12), 4, 7)])
def test_dot_product_identity_over_the_time_loop(shape, radius, nsteps):
    c = inputs.uniform(1, "c", shape, 0.01, 0.1)
    ud0 = inputs.uniform(2, "u_prev_dot", shape, -1, 1)
    ud1 = inputs.uniform(2, "u_dot", shape, -1, 1)
    lamT, lamTm1, lamTm2 = _lams(shape, 3)
    zero = np.zeros(shape)
    # objective: <lamT, u^{K+1}> + <lamTm1, u^K>; no direct dependence on older states
    prev, cur = _forward_tangent(c, ud0, ud1, radius, nsteps)
    lhs = np.sum(lamT * cur) + np.sum(lamTm1 * prev)
    bufs = oracle.wave_adjoint_steps(c, lamT, lamTm1, zero, radius, nsteps)
    new, old = bufs[nsteps % 3], bufs[(nsteps + 1) % 3]
    rhs = np.sum(new * ud1) + np.sum(old * ud0)
    scale = np.sum(np.abs(lamT * cur)) + np.sum(np.abs(lamTm1 * prev)) + 1.0
    assert abs(lhs - rhs) <= 1e-12 * scale


@pytest.mark.parametrize("shape,radius,nsteps", [((9, 11), 1, 5), ((10, 9, 11), 4, 4)])
def test_sweep_equals_products_of_assembled_jacobians(shape, radius, nsteps):
    c = inputs.uniform(4, "c", shape, 0.01, 0.1)
    ju, jp = wave_jacobians(c, radius)
    lam = [x.ravel().copy() for x in _lams(shape, 5)]       # lam^{K+1}, lam^K, lam^{K-1}
    a, b, p = lam
    for s in range(nsteps):
        if s > 0:
            p = np.zeros_like(p)
        b = b + ju.T @ a
        p = p + jp.T @ a
        a, b, p = b, p, a
    bufs = oracle.wave_adjoint_steps(c, *_lams(shape, 5), radius, nsteps)
    assert np.allclose(bufs[nsteps % 3].ravel(), a, rtol=1e-12, atol=1e-13)
    assert np.allclose(bufs[(nsteps + 1) % 3].ravel(), b, rtol=1e-12, atol=1e-13)


def test_one_step_is_the_single_step_adjoint_and_zero_steps_do_nothing():
    shape, radius = (9, 10, 11), 4
    c = inputs.uniform(6, "c", shape, 0.01, 0.1)
    l0, l1, l2 = _lams(shape, 7)
    same = oracle.wave_adjoint_steps(c, l0, l1, l2, radius, 0)
    assert all(np.array_equal(x, y) for x, y in zip(same, (l0, l1, l2)))
    one = oracle.wave_adjoint_steps(c, l0, l1, l2, radius, 1)
    ub, upb, _ = oracle.wave_adjoint(c, l0, l1, radius, u_prev_bar=l2)
    assert np.array_equal(one[0], l0) and np.array_equal(one[1], ub) and np.array_equal(one[2], upb)


def test_recycled_buffer_starts_from_zero():
    """After two steps the buffer that first held lam^{K+1} stands for lam^{K-2}: it holds
    -lam^K(updated) on I and zero outside I, whatever it held before."""
    shape, radius = (9, 10, 11), 1
    c = inputs.uniform(8, "c", shape, 0.01, 0.1)
    l0, l1, l2 = _lams(shape, 9)
    two = oracle.wave_adjoint_steps(c, l0, l1, l2, radius, 2)
    one = oracle.wave_adjoint_steps(c, l0, l1, l2, radius, 1)
    m = interior_mask(shape, radius)
    assert np.array_equal(two[0][~m], np.zeros(shape)[~m])
    assert np.array_equal(two[0][m], -one[1][m])
