"""GPU parity of sadj_adjoint_wave3d_steps_fused (reverse sweep of a time loop of wave steps,
two steps per pass where the kernel exists) against the CPU oracle."""
import numpy as np
import pytest

import inputs
import oracle
from parity import TOL, to_gpu, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    return lib


def _lams(shape, seed, dtype):
    return [inputs.uniform(seed, name, shape, -1, 1).astype(dtype) for name in ("r_bar", "u_bar", "u_prev_bar")]


def _dyadic(x, denom, lo, hi):
    """Round to multiples of 1/denom in [lo, hi]: sums and products of a few such numbers are exact."""
    return np.clip(np.round(x * denom) / denom, lo, hi)


def _run_fused(sadj, radius, nsteps, c, lams, dtype, poison=None):
    import torch
    g = [to_gpu(x.astype(dtype)) for x in lams]
    work = torch.full_like(g[0], float("nan") if poison is None else poison)
    sadj.sadj_adjoint_wave3d_steps_fused(radius, nsteps, to_gpu(c.astype(dtype)), *g, work)
    torch.cuda.synchronize()
    return [to_host(t) for t in g]


SHAPES = [(21, 37, 150), (3, 3, 4), (3, 5, 8), (4, 33, 66), (5, 64, 128), (9, 70, 130), (40, 35, 262), (150, 40, 20),
          (7, 31, 258), (6, 96, 64), (33, 3, 1000)]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("nsteps", [0, 1, 2, 3, 5, 6, 7])
def test_fused_sweep_is_exact_on_dyadic_data(sadj, shape, nsteps):
    """With c a multiple of 1/4 and adjoints small integers every product and sum of up to seven
    steps is exact in fp64, so the order of the additions does not matter and the GPU must
    return the oracle's numbers bit for bit, at every element of the two live buffers."""
    c = _dyadic(inputs.uniform(3, "c", shape, 0, 1), 4, 0.0, 1.0)
    lams = [_dyadic(4 * x, 1, -4, 4) for x in _lams(shape, 11 + nsteps, np.float64)]
    want = oracle.wave_adjoint_steps(c, *lams, 1, nsteps)
    assert max(np.max(np.abs(w)) for w in want) < 2.0 ** 40       # far from where fp64 would round
    got = _run_fused(sadj, 1, nsteps, c, lams, np.float64)
    live = [nsteps % 3, (nsteps + 1) % 3] if nsteps > 0 else [0, 1, 2]
    for k in live:
        assert np.array_equal(got[k], want[k]), "buffer %d after %d steps, shape %s: %d cells differ" % (
            k, nsteps, shape, int(np.sum(got[k] != want[k])))


@pytest.mark.parametrize("zchunk", [1, 2, 3, 8, 37])
@pytest.mark.parametrize("shape,nsteps", [((2500, 9, 20), 7), ((64, 300, 2100), 5), ((23, 40, 66), 6)])
def test_fused_sweep_is_exact_for_any_cut_along_z(sadj, shape, nsteps, zchunk):
    """Tall grids cut into hundreds of z-chunks, chunks shorter than the pipeline of the two-stage
    march, planes wide enough for the banded tile numbering: same bits as the oracle (dyadic data)."""
    c = _dyadic(inputs.uniform(1, "c", shape, 0, 1), 4, 0.0, 1.0)
    lams = [_dyadic(4 * x, 1, -4, 4) for x in _lams(shape, 2, np.float64)]
    want = oracle.wave_adjoint_steps(c, *lams, 1, nsteps)
    sadj.set_option("wave3d.zchunk", zchunk)
    try:
        got = _run_fused(sadj, 1, nsteps, c, lams, np.float64)
    finally:
        sadj.set_option("wave3d.zchunk", 0)
    for k in (nsteps % 3, (nsteps + 1) % 3):
        assert np.array_equal(got[k], want[k])


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape,nsteps", [((21, 37, 150), 5), ((21, 37, 150), 12), ((40, 35, 264), 8), ((9, 70, 132), 13),
                                          ((3, 3, 4), 9), ((6, 33, 1000), 6)])
def test_fused_sweep_matches_the_oracle(sadj, shape, nsteps, dtype):
    """Seeded real-valued inputs: the live buffers against the oracle's sweep, and element by
    element against the single-step sweep of the library within the rounding of the terms."""
    import torch
    c = inputs.uniform(1, "c", shape, 0.01, 0.1).astype(dtype)
    lams = _lams(shape, 2 + nsteps, dtype)
    want = oracle.wave_adjoint_steps(c, *lams, 1, nsteps)
    got = _run_fused(sadj, 1, nsteps, c, lams, dtype)
    plain = [to_gpu(x) for x in lams]
    sadj.sadj_adjoint_wave3d_steps(1, nsteps, to_gpu(c), *plain)
    torch.cuda.synchronize()
    tol = TOL[np.dtype(dtype)]
    for k in (nsteps % 3, (nsteps + 1) % 3):
        g = got[k].astype(np.float64)
        assert np.isfinite(g).all()
        top = max(np.max(np.abs(want[k])), 1e-300)
        assert np.max(np.abs(g - want[k])) / top <= tol * nsteps
        # against the unfused kernels: same terms, other order; each element within the rounding of
        # the largest magnitudes that entered it (its own neighbourhood's, bounded by the array's)
        p = to_host(plain[k]).astype(np.float64)
        assert np.max(np.abs(g - p)) / top <= tol * nsteps


def test_values_outside_the_iteration_space_do_not_leak(sadj):
    """c is never read outside I, and adjoints outside I are never multiplied into anything:
    NaN planted there must not reach a cell that the oracle computes as finite."""
    shape, nsteps = (12, 40, 70), 6
    c = inputs.uniform(1, "c", shape, 0.01, 0.1)
    lams = _lams(shape, 4, np.float64)
    inside = np.zeros(shape, dtype=bool)
    inside[1:-1, 1:-1, 1:-1] = True
    want = oracle.wave_adjoint_steps(c, *lams, 1, nsteps)
    cp = c.copy()
    cp[~inside] = np.nan
    lp = [x.copy() for x in lams]
    lp[0][~inside] = np.nan                      # lam0 is only ever used as r_bar: read on I only
    got = _run_fused(sadj, 1, nsteps, cp, lp, np.float64)
    for k in (nsteps % 3, (nsteps + 1) % 3):
        assert np.isfinite(got[k]).all()
        assert np.max(np.abs(got[k] - want[k])) <= 1e-12 * max(np.max(np.abs(want[k])), 1.0) * nsteps


@pytest.mark.parametrize("radius,shape,nsteps", [(4, (37, 45, 150), 5), (2, (20, 33, 70), 4), (1, (9, 21, 151), 7)])
def test_where_pairs_cannot_be_fused_the_single_steps_run(sadj, radius, shape, nsteps):
    """Other radii and rows of odd length take the single-step kernels: same bits as the plain sweep."""
    import torch
    c = inputs.uniform(1, "c", shape, 0.01, 0.1)
    lams = _lams(shape, 9, np.float64)
    got = _run_fused(sadj, radius, nsteps, c, lams, np.float64)
    plain = [to_gpu(x) for x in lams]
    sadj.sadj_adjoint_wave3d_steps(radius, nsteps, to_gpu(c), *plain)
    torch.cuda.synchronize()
    for k in (nsteps % 3, (nsteps + 1) % 3):
        assert np.array_equal(got[k], to_host(plain[k]))


def test_option_switches_fusion_off(sadj):
    import torch
    shape, nsteps = (21, 37, 150), 7
    c = inputs.uniform(1, "c", shape, 0.01, 0.1)
    lams = _lams(shape, 9, np.float64)
    sadj.set_option("wave3d.fuse", 1)
    try:
        got = _run_fused(sadj, 1, nsteps, c, lams, np.float64)
    finally:
        sadj.set_option("wave3d.fuse", 0)
    plain = [to_gpu(x) for x in lams]
    sadj.sadj_adjoint_wave3d_steps(1, nsteps, to_gpu(c), *plain)
    torch.cuda.synchronize()
    for k in (nsteps % 3, (nsteps + 1) % 3):
        assert np.array_equal(got[k], to_host(plain[k]))


def test_fused_argument_errors(sadj):
    import torch
    t = [torch.zeros(16, 16, 16, dtype=torch.float64, device="cuda") for _ in range(5)]
    with pytest.raises(sadj.SadjError) as e:
        sadj.sadj_adjoint_wave3d_steps_fused(1, 2, t[0], t[1], t[2], t[3], t[3])     # work overlaps lam2
    assert e.value.status == 3
    with pytest.raises(sadj.SadjError) as e:
        sadj.sadj_adjoint_wave3d_steps_fused(1, 2, t[0], t[1], t[2], t[3], t[0])     # work overlaps c
    assert e.value.status == 3
    with pytest.raises(sadj.SadjError) as e:
        sadj.sadj_adjoint_wave3d_steps_fused(1, -1, *t)
    assert e.value.status == 2
    with pytest.raises(sadj.SadjError) as e:
        sadj.sadj_adjoint_wave3d_steps_fused(5, 1, *t)
    assert e.value.status == 4


def test_full_size_sweep_on_sampled_planes(sadj):
    """512^3 fp64, the launch configuration the benchmark times: 7 steps on dyadic data (exact),
    compared with the oracle on slabs around sampled planes.  The oracle treats the cut ends of a
    slab as grid boundaries; that error travels one plane per step, so planes more than nsteps + 1
    planes away from a cut end are those of the full grid."""
    import torch
    n, nsteps = 512, 7
    shape = (n, n, n)
    c = to_gpu(_dyadic(inputs.uniform(3, "c", shape, 0, 1), 4, 0.0, 1.0))
    lams = [to_gpu(_dyadic(4 * x, 1, -4, 4)) for x in _lams(shape, 21, np.float64)]
    g = [x.clone() for x in lams]
    work = torch.empty_like(c)
    sadj.sadj_adjoint_wave3d_steps_fused(1, nsteps, c, *g, work)
    torch.cuda.synchronize()
    for z0, z1 in [(0, 6), (250, 262), (506, 512)]:
        lo, hi = max(0, z0 - nsteps - 2), min(n, z1 + nsteps + 2)
        cs = to_host(c[lo:hi])
        ls = [to_host(x[lo:hi]) for x in lams]
        want = oracle.wave_adjoint_steps(cs, *ls, 1, nsteps)
        for k in (nsteps % 3, (nsteps + 1) % 3):
            got = to_host(g[k][z0:z1])
            w = want[k][z0 - lo:z1 - lo]
            assert np.array_equal(got, w), "planes %d..%d buffer %d: %d cells differ" % (z0, z1, k, int(np.sum(got != w)))


def test_fused_sweep_can_be_captured_in_a_hip_graph(sadj):
    """The sweep only enqueues kernels (no allocation, no memset, no synchronisation): recorded
    into a HIP graph, every replay on fresh inputs reproduces the eager result bit for bit."""
    import torch
    shape, nsteps = (21, 37, 150), 9
    c = to_gpu(inputs.uniform(1, "c", shape, 0.01, 0.1))
    lams = _lams(shape, 5, np.float64)
    eager = [to_gpu(x) for x in lams]
    sadj.sadj_adjoint_wave3d_steps_fused(1, nsteps, c, *eager, torch.zeros_like(c))
    torch.cuda.synchronize()
    want = [to_host(t) for t in eager]
    static = [to_gpu(x) for x in lams]
    work = torch.zeros_like(c)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sadj.sadj_adjoint_wave3d_steps_fused(1, nsteps, c, *static, work)          # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    for t, src in zip(static, lams):
        t.copy_(torch.from_numpy(src))
    with torch.cuda.graph(graph):
        sadj.sadj_adjoint_wave3d_steps_fused(1, nsteps, c, *static, work)
    for replay in range(3):
        for t, src in zip(static, lams):
            t.copy_(torch.from_numpy(src))
        other = torch.ones(1000, device="cuda").sum()          # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in (nsteps % 3, (nsteps + 1) % 3):
            assert np.array_equal(to_host(static[k]), want[k]), "replay %d buffer %d" % (replay, k)
        assert float(other) == 1000.0
