"""GPU parity of the 3-D star stencils with arbitrary (asymmetric) weights
(sadj_primal_star3d, sadj_adjoint_star3d) against the CPU oracle."""
import numpy as np
import pytest

import inputs
import oracle
from jacobians import interior_mask
from parity import assert_close, to_gpu, to_host

pytestmark = pytest.mark.gpu

CASES = [(1, (3, 3, 3)), (1, (4, 5, 7)), (1, (21, 37, 150)), (1, (70, 18, 65)),
         (2, (5, 5, 5)), (2, (33, 45, 150)), (3, (7, 7, 7)), (3, (30, 41, 136)),
         (4, (9, 9, 9)), (4, (16, 17, 19)), (4, (37, 45, 150)), (4, (40, 16, 200)), (4, (70, 20, 129)),
         # left-over tiles cut finer than the rest (two groups of workgroups)
         (1, (24, 400, 610)), (2, (64, 130, 1150)),
         # rows not cache-line multiples: tiles of 16 rows with long rows
         (1, (6, 20, 1000)), (1, (9, 40, 500)), (1, (5, 33, 250)),
         (4, (20, 37, 250)), (2, (9, 40, 500)), (3, (12, 20, 1000))]


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    yield lib
    lib.set_option("wave3d.zchunk", 0)


def _table(radius, seed):
    return inputs.uniform(seed, "aux", (1 + 6 * radius,), -2.0, 2.0)


def _abs_star(w, radius, a):
    """sum_o |w_o| |a[i+o]| on the whole grid (zero outside): scale of the primal's sum."""
    import scipy.ndimage as ndi
    k = np.zeros((2 * radius + 1,) * 3)
    k[radius, radius, radius] = abs(w[0])
    for d, axis in enumerate((2, 1, 0)):
        for idx, o in enumerate(list(range(-radius, 0)) + list(range(1, radius + 1))):
            pos = [radius] * 3
            pos[axis] += o
            k[tuple(pos)] = abs(w[1 + d * 2 * radius + idx])
    return ndi.correlate(np.abs(a), k, mode="constant")


@pytest.fixture(params=[0, 1], ids=["handwritten", "functor"])
def star_path(request, sadj):
    """Radius-1 calls also run through the generic functor kernels of
    include/sadj_stencil_star.hpp (a linear 7-point functor with a passive coefficient); both
    paths must meet the same bar.  Other radii and shapes that rule out 16-byte accesses fall
    back to the hand-written kernel."""
    sadj.set_option("star3d.functor", request.param)
    yield request.param
    sadj.set_option("star3d.functor", 0)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius,shape", CASES)
def test_star_adjoint_and_primal(sadj, star_path, radius, shape, dtype):
    import torch
    if star_path == 1 and radius != 1:
        pytest.skip("the functor path exists for radius 1")
    w = _table(radius, sum(shape))
    wq = w.astype(dtype).astype(np.float64)             # the library converts the weights to dtype
    u = inputs.uniform(1, "u", shape, -1, 1).astype(dtype)
    c = inputs.uniform(1, "c", shape, 0.5, 1.5).astype(dtype)
    rb = inputs.uniform(1, "r_bar", shape, -1, 1).astype(dtype)
    ub = inputs.uniform(1, "u_bar", shape, -1, 1).astype(dtype)
    m = interior_mask(shape, radius)
    for zchunk in (0, 9):
        sadj.set_option("wave3d.zchunk", zchunk)
        ug = to_gpu(ub)
        sadj.sadj_adjoint_star3d(radius, w, to_gpu(np.where(m, c, np.nan).astype(dtype)),
                                 to_gpu(np.where(m, rb, np.nan).astype(dtype)), ug)
        torch.cuda.synchronize()
        want, scale = oracle.star3d_adjoint(wq, c, rb, ub, radius, want_scale=True)
        assert_close(to_host(ug), want, scale + np.abs(ub.astype(np.float64)), dtype,
                     "star adjoint R=%d %s zchunk=%d" % (radius, shape, zchunk))
        r0 = inputs.uniform(2, "u_prev", shape, -1, 1).astype(dtype)
        r = to_gpu(r0)
        sadj.sadj_primal_star3d(radius, w, to_gpu(u), to_gpu(c), r)
        torch.cuda.synchronize()
        got = to_host(r)
        wantr = oracle.star3d_primal(wq, u, c, radius, r_init=r0)
        assert np.array_equal(got[~m], r0[~m])
        sc = np.abs(c.astype(np.float64)) * _abs_star(wq, radius, u.astype(np.float64))
        assert_close(got[m], wantr[m], sc[m], dtype, "star primal R=%d %s" % (radius, shape))
    sadj.set_option("wave3d.zchunk", 0)


def test_symmetric_weights_reproduce_the_wave_kernel_up_to_its_2_r_bar_term(sadj):
    """Same stencil through two kernels: the general star with the Laplacian table and the
    wave kernel with its built-in weights."""
    import torch
    from jacobians import star_weights
    radius, shape = 4, (30, 50, 140)
    sw = star_weights(radius)
    axis = [sw[abs(o)] for o in list(range(-radius, 0)) + list(range(1, radius + 1))]
    w = [3 * sw[0]] + axis * 3
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=8, c_mode="iid")
    m = interior_mask(shape, radius)
    c, rb = to_gpu(d["c"]), to_gpu(d["r_bar"])
    a, b = to_gpu(d["u_bar"]), to_gpu(d["u_bar"])
    sadj.sadj_adjoint_star3d(radius, w, c, rb, a)
    sadj.sadj_adjoint_wave3d(radius, c, rb, b)
    torch.cuda.synchronize()
    diff = to_host(b) - to_host(a)
    assert np.allclose(diff, np.where(m, 2.0 * d["r_bar"], 0.0), rtol=0, atol=1e-13)


def test_star_full_size(sadj):
    """512^3, radius 4, fp64, an upwind-biased (asymmetric) table."""
    import torch
    radius, shape = 4, (512, 512, 512)
    w = _table(radius, 77)
    d = inputs.config_inputs("wave3d_r4", fields=("c", "r_bar", "u_bar"))
    ug = to_gpu(d["u_bar"])
    sadj.sadj_adjoint_star3d(radius, w, to_gpu(d["c"]), to_gpu(d["r_bar"]), ug)
    torch.cuda.synchronize()
    want, scale = oracle.star3d_adjoint(w, d["c"], d["r_bar"], d["u_bar"], radius, want_scale=True)
    assert_close(to_host(ug), want, scale + np.abs(d["u_bar"]), np.float64, "star 512^3 R=4")


def test_star_argument_errors(sadj):
    import paper_1907_02818_amd as lib
    import torch
    t = [torch.zeros(12, 12, 12, dtype=torch.float64, device="cuda") for _ in range(3)]
    with pytest.raises(ValueError):
        sadj.sadj_adjoint_star3d(4, [1.0] * 7, *t)          # table too short for the radius
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_star3d(4, [1.0] * 25, t[0], t[1], t[0])
    assert e.value.status == 3
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_star3d(5, [1.0] * 31, *t)
    assert e.value.status == 4
