"""Independent constructions of the stencil Jacobians from library routines
(fractions, scipy.sparse.diags / kron).  Nothing here calls the oracle or the
HIP library; the tests use these matrices to pin the oracle (and, transposed by a
library mat-vec, as a second opinion on the adjoint)."""
from fractions import Fraction

import numpy as np
import scipy.sparse as sp

# central second-derivative weights on a unit grid, from the textbook tables
STAR = {
    1: [Fraction(-2), Fraction(1)],
    2: [Fraction(-5, 2), Fraction(4, 3), Fraction(-1, 12)],
    3: [Fraction(-49, 18), Fraction(3, 2), Fraction(-3, 20), Fraction(1, 90)],
    4: [Fraction(-205, 72), Fraction(8, 5), Fraction(-1, 5), Fraction(8, 315), Fraction(-1, 560)],
}


def star_weights(radius):
    return np.array([float(w) for w in STAR[radius]])


def second_difference_matrix(n, radius):
    """n x n banded Toeplitz matrix of the 1-D star (rows near the ends are
    truncated; they are masked out by the interior selector later)."""
    w = star_weights(radius)
    diags = [np.full(n - abs(k), w[abs(k)]) for k in range(-radius, radius + 1) if n - abs(k) > 0]
    offs = [k for k in range(-radius, radius + 1) if n - abs(k) > 0]
    return sp.diags(diags, offs, shape=(n, n), format="csr")


def interior_mask(shape, radius):
    m = np.ones(shape, dtype=bool)
    for ax, n in enumerate(shape):
        idx = np.arange(n)
        ok = (idx >= radius) & (idx <= n - 1 - radius)
        m &= ok.reshape([-1 if a == ax else 1 for a in range(len(shape))])
    return m


def wave_jacobians(c, radius):
    """(J_u, J_uprev) of r = 2u - u_prev + c*Lap_w(u) restricted to rows in the
    primal interior (all other rows zero).  c has shape slowest-axis-first."""
    shape = c.shape
    N = c.size
    lap = sp.csr_matrix((N, N))
    for ax, n in enumerate(shape):
        mats = [sp.identity(m, format="csr") for m in shape]
        mats[ax] = second_difference_matrix(n, radius)
        term = mats[0]
        for m in mats[1:]:
            term = sp.kron(term, m, format="csr")
        lap = lap + term
    sel = sp.diags(interior_mask(shape, radius).ravel().astype(np.float64))
    ju = sel @ (2.0 * sp.identity(N) + sp.diags(c.ravel()) @ lap)
    jp = -sel
    return ju.tocsr(), jp.tocsr()
