"""GPU parity of the dense 3^d box stencils with asymmetric weights (sadj_primal_box,
sadj_adjoint_box) against the CPU oracle."""
import numpy as np
import pytest
import scipy.ndimage as ndi

import inputs
import oracle
from jacobians import interior_mask
from parity import assert_close, to_gpu, to_host

pytestmark = pytest.mark.gpu

SHAPES = [(3,), (4,), (65,), (127,), (128,), (129,), (1000,), (100003,),
          (3, 3), (3, 200), (200, 3), (67, 131), (130, 256), (70, 1030), (300, 301),
          (3, 3, 3), (4, 5, 7), (21, 37, 150), (9, 70, 130), (40, 33, 64), (70, 18, 65),
          (24, 400, 610),        # left-over tiles cut finer along z than the rest
          (6, 20, 1000), (9, 40, 500), (5, 33, 250)]   # rows not cache-line multiples: 256 x 16 tiles


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    return lib


@pytest.fixture(params=[0, 1], ids=["handwritten", "functor"])
def path1d(sadj, request):
    """The 1-D case runs through its own kernel and through the generic three-point functor
    kernel (include/sadj_stencil1d.hpp, a linear functor with a passive coefficient)."""
    sadj.set_option("stencil1d.functor", request.param)
    yield request.param
    sadj.set_option("stencil1d.functor", 0)


def _weights(ndim, seed):
    return inputs.uniform(seed, "aux", (3,) * ndim, -2.0, 2.0)


# the functor path exists in 1-D only
CASES = [(s, 0) for s in SHAPES] + [(s, 1) for s in SHAPES if len(s) == 1]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape,functor", CASES)
def test_box_adjoint_and_primal(sadj, shape, functor, dtype):
    import torch
    ndim = len(shape)
    sadj.set_option("stencil1d.functor", functor)
    try:
        _box_case(sadj, shape, dtype, ndim, torch)
        if ndim == 2:                                   # the strip march as well as the default tile form
            sadj.set_option("wave2d.variant", 1)
            _box_case(sadj, shape, dtype, ndim, torch)
    finally:
        sadj.set_option("stencil1d.functor", 0)
        sadj.set_option("wave2d.variant", 0)


def _box_case(sadj, shape, dtype, ndim, torch):
    w = _weights(ndim, sum(shape))
    wq = w.astype(dtype).astype(np.float64)            # the library converts the weights to dtype
    u = inputs.uniform(1, "u", shape, -1, 1).astype(dtype)
    c = inputs.uniform(1, "c", shape, 0.5, 1.5).astype(dtype)
    rb = inputs.uniform(1, "r_bar", shape, -1, 1).astype(dtype)
    ub = inputs.uniform(1, "u_bar", shape, -1, 1).astype(dtype)
    m = interior_mask(shape, 1)
    # adjoint, with NaN outside the interior of c and r_bar: they must never be used
    cg = to_gpu(np.where(m, c, np.nan).astype(dtype))
    rg = to_gpu(np.where(m, rb, np.nan).astype(dtype))
    ug = to_gpu(ub)
    sadj.sadj_adjoint_box(w, cg, rg, ug)
    torch.cuda.synchronize()
    want, scale = oracle.box_adjoint(wq, c, rb, ub, want_scale=True)
    assert_close(to_host(ug), want, scale + np.abs(ub.astype(np.float64)), dtype, "box adjoint %s" % (shape,))
    # primal
    r0 = inputs.uniform(2, "u_prev", shape, -1, 1).astype(dtype)
    r = to_gpu(r0)
    sadj.sadj_primal_box(w, to_gpu(u), to_gpu(c), r)
    torch.cuda.synchronize()
    wantr = oracle.box_primal(wq, u, c, r_init=r0)
    got = to_host(r)
    assert np.array_equal(got[~m], r0[~m])
    sc = np.abs(c.astype(np.float64)) * ndi.correlate(np.abs(u.astype(np.float64)), np.abs(wq), mode="constant")
    assert_close(got[m], wantr[m], sc[m], dtype, "box primal %s" % (shape,))


def test_the_papers_one_dimensional_example(sadj, path1d):
    """Weights (2,-3,4) on [1, n-1] of arrays of length n+1 (Section 3.2)."""
    import torch
    n = 4096
    w = [2.0, -3.0, 4.0]
    c = inputs.uniform(3, "c", (n + 1,), 0.5, 1.5)
    rb = inputs.uniform(3, "r_bar", (n + 1,), -1, 1)
    ub = inputs.uniform(3, "u_bar", (n + 1,), -1, 1)
    ug = to_gpu(ub)
    sadj.sadj_adjoint_box(w, to_gpu(c), to_gpu(rb), ug)
    torch.cuda.synchronize()
    want = oracle.lin3_adjoint(c, rb, ub, 1, n - 1, 2.0, -3.0, 4.0)
    got = to_host(ug)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-14)
    # the outer weights trade places: a unit r_bar at i spreads 2, -3, 4 to i-1, i, i+1
    e = np.zeros(n + 1); e[100] = 1.0
    ug = to_gpu(np.zeros(n + 1))
    sadj.sadj_adjoint_box(w, to_gpu(np.ones(n + 1)), to_gpu(e), ug)
    got = to_host(ug)
    assert (got[99], got[100], got[101]) == (2.0, -3.0, 4.0)


def test_box_full_size_3d(sadj):
    import torch
    shape = (256, 256, 512)
    w = _weights(3, 11)
    c = inputs.uniform(4, "c", shape, 0.5, 1.5)
    rb = inputs.uniform(4, "r_bar", shape, -1, 1)
    ub = inputs.uniform(4, "u_bar", shape, -1, 1)
    ug = to_gpu(ub)
    sadj.sadj_adjoint_box(w, to_gpu(c), to_gpu(rb), ug)
    torch.cuda.synchronize()
    want, scale = oracle.box_adjoint(w, c, rb, ub, want_scale=True)
    assert_close(to_host(ug), want, scale + np.abs(ub), np.float64, "box 3-D 256x256x512")


@pytest.mark.parametrize("case", range(16))
def test_box_on_drawn_shapes(sadj, case):
    """Dimension, shape, dtype and z-chunk drawn from a seeded generator."""
    import torch
    rng = np.random.default_rng(500 + case)
    ndim = int(rng.integers(2, 4))
    dtype = [np.float64, np.float32][int(rng.integers(0, 2))]
    shape = tuple(int(rng.integers(3, hi)) for hi in ((60, 400) if ndim == 2 else (40, 90, 260)))
    zchunk = int(rng.choice([0, 0, 6, 17]))
    sadj.set_option("wave3d.zchunk", zchunk)
    sadj.set_option("wave2d.variant", int(rng.integers(0, 2)))
    try:
        _box_case(sadj, shape, dtype, ndim, torch)
    finally:
        sadj.set_option("wave3d.zchunk", 0)
        sadj.set_option("wave2d.variant", 0)
