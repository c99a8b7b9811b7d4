"""Pins of the oracle's general 3-D star stencil (free weight per read offset): library
correlation / convolution with the star-shaped kernel, the already pinned wave and box
oracles as special cases, and the dot-product identity."""
import numpy as np
import pytest
import scipy.ndimage as ndi

import inputs
import oracle
from jacobians import interior_mask, star_weights


def _table(radius, seed):
    return inputs.uniform(seed, "aux", (1 + 6 * radius,), -2.0, 2.0)


def _kernel(w, radius):
    """Correlation kernel k[oz+R, oy+R, ox+R] of the star with table w (arrays are (z, y, x))."""
    k = np.zeros((2 * radius + 1,) * 3)
    k[radius, radius, radius] = w[0]
    for d, axis in enumerate((2, 1, 0)):                 # x, y, z -> numpy axes
        for idx, o in enumerate(list(range(-radius, 0)) + list(range(1, radius + 1))):
            pos = [radius] * 3
            pos[axis] += o
            k[tuple(pos)] = w[1 + d * 2 * radius + idx]
    return k


@pytest.mark.parametrize("radius,shape", [(1, (3, 3, 3)), (1, (5, 6, 7)), (2, (6, 7, 9)), (3, (8, 9, 11)), (4, (9, 9, 9)),
                                          (4, (11, 13, 12))])
def test_primal_is_a_correlation_and_adjoint_a_convolution_with_the_star_kernel(radius, shape):
    w = _table(radius, sum(shape))
    u = inputs.uniform(1, "u", shape, -1, 1)
    c = inputs.uniform(1, "c", shape, 0.5, 1.5)
    rb = inputs.uniform(1, "r_bar", shape, -1, 1)
    ub = inputs.uniform(1, "u_bar", shape, -1, 1)
    m = interior_mask(shape, radius)
    k = _kernel(w, radius)
    r0 = np.full(shape, 9.0)
    r = oracle.star3d_primal(w, u, c, radius, r_init=r0)
    assert np.array_equal(r[~m], r0[~m])
    assert np.allclose(r[m], (c * ndi.correlate(u, k, mode="constant"))[m], rtol=1e-13, atol=1e-13)
    # adjoint: the transposed operator is the convolution (point-mirrored kernel) of q = c*r_bar on I
    q = np.where(m, c * rb, 0.0)
    got, scale = oracle.star3d_adjoint(w, np.where(m, c, np.nan), np.where(m, rb, np.nan), ub, radius, want_scale=True)
    assert np.allclose(got, ub + ndi.convolve(q, k, mode="constant"), rtol=1e-13, atol=1e-13)
    assert np.allclose(scale, ndi.convolve(np.abs(q), np.abs(k), mode="constant"), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("radius", [1, 2, 3, 4])
def test_symmetric_laplacian_weights_give_the_wave_adjoint_without_its_2_r_bar_term(radius):
    shape = (2 * radius + 4, 2 * radius + 3, 2 * radius + 6)
    sw = star_weights(radius)
    axis = [sw[abs(o)] for o in list(range(-radius, 0)) + list(range(1, radius + 1))]
    w = np.array([3 * sw[0]] + axis * 3)
    d = inputs.wave_inputs(shape, 0.01, 0.3, seed=radius, c_mode="iid")
    m = interior_mask(shape, radius)
    wave, _, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius)
    star, _ = oracle.star3d_adjoint(w, d["c"], d["r_bar"], d["u_bar"], radius)
    assert np.allclose(star, wave - np.where(m, 2.0 * d["r_bar"], 0.0), rtol=1e-13, atol=1e-14)
    prim = oracle.star3d_primal(w, d["u"], d["c"], radius)
    wavep = oracle.wave_primal(d["u"], d["u_prev"], d["c"], radius)
    assert np.allclose(prim[m], (wavep - 2 * d["u"] + d["u_prev"])[m], rtol=1e-12, atol=1e-13)


def test_radius_one_equals_the_box_oracle_with_axis_entries_only():
    shape = (6, 7, 8)
    w = _table(1, 3)                                     # centre, x-, x+, y-, y+, z-, z+
    box = np.zeros((3, 3, 3))
    box[1, 1, 1] = w[0]
    box[1, 1, 0], box[1, 1, 2] = w[1], w[2]
    box[1, 0, 1], box[1, 2, 1] = w[3], w[4]
    box[0, 1, 1], box[2, 1, 1] = w[5], w[6]
    c = inputs.uniform(2, "c", shape, 0.5, 1.5)
    rb = inputs.uniform(2, "r_bar", shape, -1, 1)
    ub = inputs.uniform(2, "u_bar", shape, -1, 1)
    u = inputs.uniform(2, "u", shape, -1, 1)
    assert np.allclose(oracle.star3d_adjoint(w, c, rb, ub, 1)[0], oracle.box_adjoint(box, c, rb, ub)[0], rtol=1e-14, atol=1e-15)
    assert np.allclose(oracle.star3d_primal(w, u, c, 1), oracle.box_primal(box, u, c), rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("radius", [1, 4])
def test_dot_product_identity(radius):
    shape = (2 * radius + 5, 2 * radius + 2, 2 * radius + 7)
    w = _table(radius, 11)
    u = inputs.uniform(4, "u", shape, -1, 1)
    c = inputs.uniform(4, "c", shape, 0.5, 1.5)
    rb = inputs.uniform(4, "r_bar", shape, -1, 1)
    m = interior_mask(shape, radius)
    lhs = float(np.sum(oracle.star3d_primal(w, u, c, radius)[m] * rb[m]))
    ub, _ = oracle.star3d_adjoint(w, c, rb, np.zeros(shape), radius)
    rhs = float(np.sum(u * ub))
    assert abs(lhs - rhs) <= 1e-13 * float(np.sum(np.abs(u * ub)))
