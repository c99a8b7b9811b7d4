"""The paper's 1-D worked example (Section 3.2): asymmetric weights (2,-3,4), variable
c, iteration space [1,n-1] on arrays of length n+1.  The scatter oracle must give
what the paper's remainder statements and merged core loop give (derived here from the
weight table and checked against the facts the section states about them); the
asymmetric weights catch a mirrored-offset mistake that a symmetric Laplacian hides."""
import os

import numpy as np
import pytest

import inputs
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "example1d_adjoint_statements.txt")
W = (2.0, -3.0, 4.0)


def _facts():
    out = {}
    with open(GOLDEN) as fh:
        for ln in fh:
            if ln.strip() and not ln.startswith("#"):
                key, *vals = ln.split()
                out[key] = vals
    return out


def _statements(n):
    """Every update ub[target] += w * c[source] * rb[source] of the adjoint, derived from the
    primal's weight table: iteration i in [1, n-1] reads u[i-1], u[i], u[i+1] with W."""
    return [(i + o, w, i) for i in range(1, n) for o, w in zip((-1, 0, 1), W)]


def _split_adjoint(n, c, rb, ub):
    """The statements regrouped by target as Section 3.2 does: those whose target has all three
    sources form the core loop, the others remain single statements."""
    ub = ub.copy()
    st = _statements(n)
    by_target = {}
    for t, w, s_ in st:
        by_target.setdefault(t, []).append((w, s_))
    core = sorted(t for t, lst in by_target.items() if len(lst) == 3)
    rest = sorted(t for t, lst in by_target.items() if len(lst) < 3 for _ in lst)
    for t, lst in by_target.items():
        for w, s_ in lst:
            ub[t] += w * c[s_] * rb[s_]
    return ub, core, rest, by_target


def _fields(n, seed):
    c = inputs.uniform(seed, "c", (n + 1,), 0.5, 1.5)
    rb = inputs.uniform(seed, "r_bar", (n + 1,), -1, 1)
    ub = inputs.uniform(seed, "u_bar", (n + 1,), -1, 1)
    return c, rb, ub


@pytest.mark.parametrize("n", [4, 5, 6, 17, 100])
def test_scatter_oracle_equals_the_printed_remainder_and_core(n):
    c, rb, ub = _fields(n, n)
    got = oracle.lin3_adjoint(c, rb, ub, 1, n - 1, *W)
    want, core, rest, by_target = _split_adjoint(n, c, rb, ub)
    assert np.allclose(got, want, rtol=1e-14, atol=1e-15)
    # the split has the structure the paper states
    facts = _facts()
    env = {"n": n}
    lo, hi = (eval(v, env) for v in facts["core_bounds"])
    assert core == list(range(lo, hi + 1))
    assert rest == sorted(eval(v, env) for v in facts["remainder_targets"])
    want_factors = [float(v) for v in facts["core_factors_at_j-1_j_j+1"]]
    for j in core:
        assert [w for w, s_ in sorted(by_target[j], key=lambda ws: ws[1])] == want_factors


def test_weights_swap_sides_between_primal_and_adjoint():
    """Section 3.2 ends by noting that the factors 4 and 2 trade places: with c = 1 the
    primal reads (2,-3,4) at (i-1,i,i+1), the core adjoint reads (4,-3,2)."""
    n = 12
    ones = np.ones(n + 1)
    e = np.zeros(n + 1)
    e[6] = 1.0
    r = oracle.lin3_primal(ones, e, 1, n - 1, *W)          # column 6 of J
    assert (r[5], r[6], r[7]) == (4.0, -3.0, 2.0)           # u[6] is i+1 for i=5, i-1 for i=7
    ub = oracle.lin3_adjoint(ones, e, np.zeros(n + 1), 1, n - 1, *W)   # row 6 of J, scattered
    assert (ub[5], ub[6], ub[7]) == (2.0, -3.0, 4.0)


@pytest.mark.parametrize("n", [3, 4, 9])
def test_adjoint_equals_dense_JT(n):
    c, rb, ub = _fields(n, 30 + n)
    J = np.zeros((n + 1, n + 1))
    for k in range(n + 1):
        e = np.zeros(n + 1)
        e[k] = 1.0
        J[:, k] = oracle.lin3_primal(c, e, 1, n - 1, *W)
    rbm = rb.copy()
    rbm[0] = rbm[n] = 0.0
    got = oracle.lin3_adjoint(c, rb, ub, 1, n - 1, *W)
    assert np.allclose(got, ub + J.T @ rbm, rtol=1e-14, atol=1e-15)


def test_primal_value():
    n = 8
    c, _, _ = _fields(n, 1)
    u = inputs.uniform(1, "u", (n + 1,), -1, 1)
    r = oracle.lin3_primal(c, u, 1, n - 1, *W)
    for i in range(1, n):
        assert np.isclose(r[i], c[i] * (2.0 * u[i - 1] - 3.0 * u[i] + 4 * u[i + 1]), rtol=1e-15)
    assert r[0] == 0 and r[n] == 0


def test_wave1d_is_the_symmetric_instance():
    """The 1-D wave config r = 2u - u_prev + c(u[i-1]-2u[i]+u[i+1]) differs from the
    3-point example only by the 2u - u_prev part: its adjoint is the lin3 adjoint with
    weights (1,-2,1) plus 2 r_bar on the interior."""
    n = 50
    d = inputs.wave_inputs((n,), 0.01, 0.25, seed=4)
    ub, _, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1)
    want = oracle.lin3_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, n - 2, 1.0, -2.0, 1.0)
    want[1:n - 1] += 2.0 * d["r_bar"][1:n - 1]
    assert np.allclose(ub, want, rtol=1e-14, atol=1e-15)
