"""Pins of the oracle's Burgers time loop (forward sweep storing all states, reverse sweep
over them): chain rule over the steps (paper Sections 3.1, 4.2) checked against products of
Jacobians, the tangent loop, and finite differences of the whole nonlinear solve."""
import numpy as np
import pytest

import inputs
import oracle

C, D = 0.1, 0.05


def _states(n, nsteps, seed):
    st = np.empty((nsteps + 1, n))
    st[0] = inputs.burgers_inputs(n, seed=seed)["u"]
    for t in range(1, nsteps + 1):                       # boundary data of the later states
        st[t] = inputs.uniform(seed + t, "u_prev", (n,), -0.5, 0.5)
    return st


def _jacobian(u):
    n = u.size
    J = np.zeros((n, n))
    for k in range(n):
        e = np.zeros(n); e[k] = 1.0
        J[:, k] = oracle.burgers_tangent(u, e, C, D)
    return J                                              # rows 0 and n-1 are zero


@pytest.mark.parametrize("n,nsteps", [(12, 1), (12, 4), (30, 7), (3, 3)])
def test_reverse_sweep_equals_the_product_of_transposed_step_jacobians(n, nsteps):
    st = oracle.burgers_primal_steps(_states(n, nsteps, n), nsteps, C, D)
    lam_last = inputs.uniform(n, "r_bar", (n,), -1, 1)
    seed_prev = inputs.uniform(n, "u_bar", (n,), -1, 1)
    a, b = oracle.burgers_adjoint_steps(st, nsteps, nsteps, lam_last, seed_prev, C, D)
    got = (a, b)[nsteps % 2]
    lam = lam_last.copy()
    for s in range(nsteps):
        t = nsteps - 1 - s
        lam = _jacobian(st[t]).T @ lam + (seed_prev if s == 0 else 0.0)
    assert np.allclose(got, lam, rtol=1e-13, atol=1e-14)


def test_forward_sweep_is_the_repeated_single_step_and_keeps_boundary_data():
    n, nsteps = 50, 5
    st0 = _states(n, nsteps, 3)
    st = oracle.burgers_primal_steps(st0, nsteps, C, D)
    assert np.array_equal(st[:, 0], st0[:, 0]) and np.array_equal(st[:, -1], st0[:, -1])
    assert np.array_equal(st[0], st0[0])
    for t in range(nsteps):
        want = oracle.burgers_primal(st[t], C, D, r_init=st0[t + 1])
        assert np.array_equal(st[t + 1], want)


def test_gradient_of_the_whole_solve_matches_central_differences():
    n, nsteps = 24, 6
    st0 = _states(n, nsteps, 9)
    w = inputs.uniform(1, "r_bar", (n,), -1, 1)

    def objective(u0):
        s = st0.copy(); s[0] = u0
        return float(np.dot(w[1:-1], oracle.burgers_primal_steps(s, nsteps, C, D)[nsteps][1:-1]))

    st = oracle.burgers_primal_steps(st0, nsteps, C, D)
    a, b = oracle.burgers_adjoint_steps(st, nsteps, nsteps, w, np.zeros(n), C, D)
    grad = (a, b)[nsteps % 2]
    h = 1e-6
    for k in (0, 1, 2, 7, 11, 12, n - 2, n - 1):
        e = np.zeros(n); e[k] = h
        fd = (objective(st0[0] + e) - objective(st0[0] - e)) / (2 * h)
        assert abs(fd - grad[k]) <= 1e-7 * max(1.0, abs(fd)), (k, fd, grad[k])


def test_partial_sweeps_compose_and_zero_steps_do_nothing():
    n, K = 40, 6
    st = oracle.burgers_primal_steps(_states(n, K, 4), K, C, D)
    lam = inputs.uniform(4, "r_bar", (n,), -1, 1)
    z = np.zeros(n)
    a0, b0 = oracle.burgers_adjoint_steps(st, K, 0, lam, z, C, D)
    assert np.array_equal(a0, lam) and np.array_equal(b0, z)
    full = oracle.burgers_adjoint_steps(st, K, K, lam, z, C, D)[K % 2]
    first = oracle.burgers_adjoint_steps(st, K, 2, lam, z, C, D)[0]       # adjoint of u^{K-2}
    rest = oracle.burgers_adjoint_steps(st, K - 2, K - 2, first, z, C, D)[(K - 2) % 2]
    assert np.allclose(full, rest, rtol=1e-14, atol=1e-15)
    one = oracle.burgers_adjoint_steps(st, K, 1, lam, z, C, D)[1]
    assert np.array_equal(one, oracle.burgers_adjoint(st[K - 1], lam, z, C, D)[0])
    with pytest.raises(ValueError):
        oracle.burgers_adjoint_steps(st, 2, 3, lam, z, C, D)
