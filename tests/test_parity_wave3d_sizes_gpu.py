"""GPU parity of the 3-D wave adjoint at the grid sizes where its launch takes other paths than
at 512^3: rows that are not cache-line multiples (wide tiles), several rounds of workgroups,
left-over tiles cut finer than the rest (two groups of workgroups), and the u_prev_bar form at
its own tile shape.  The oracle runs on slabs of planes; a slab is a grid of its own, so its
planes from 2R to S-2R-1 (all their sources lie in the slab's interior) -- and, at the bottom /
top of the grid, also its first / last planes -- equal those of the full problem.  A closed-form
sum over the whole grid checks that nothing else was left out or written twice."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import inputs
import oracle
from parity import assert_close, to_host

pytestmark = pytest.mark.gpu

RANGES = {"c": (0.01, 0.1), "r_bar": (-1.0, 1.0), "u_bar": (-1.0, 1.0), "u_prev_bar": (-1.0, 1.0)}


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    return lib


def _device_field(seed, name, shape, chunk=25):
    """The array inputs.uniform(seed, name, shape, lo, hi) on the GPU, generated in chunks of planes."""
    import torch
    lo, hi = RANGES[name]
    out = torch.empty(shape, dtype=torch.float64, device="cuda")
    starts = list(range(0, shape[0], chunk))
    with ThreadPoolExecutor(max_workers=8) as pool:
        parts = pool.map(lambda z0: (z0, inputs.uniform_planes(seed, name, shape, lo, hi, z0, min(chunk, shape[0] - z0))), starts)
        for z0, a in parts:
            out[z0:z0 + a.shape[0]].copy_(torch.from_numpy(a))
    return out


def _slab(seed, name, shape, z0, S):
    lo, hi = RANGES[name]
    return inputs.uniform_planes(seed, name, shape, lo, hi, z0, S)


def _check_on_slabs(sadj, radius, shape, with_prev, slab_starts, seed):
    import torch
    nz = shape[0]
    c, rb, ub = (_device_field(seed, k, shape) for k in ("c", "r_bar", "u_bar"))
    up = _device_field(seed, "u_prev_bar", shape) if with_prev else None
    sum_rb_I = float(rb[radius:nz - radius, radius:shape[1] - radius, radius:shape[2] - radius].sum())
    sum_ub0 = float(ub.sum())
    sum_up0 = float(up.sum()) if with_prev else 0.0
    sadj.sadj_adjoint_wave3d(radius, c, rb, ub, up)
    torch.cuda.synchronize()
    S = 6 * radius + 2 if radius > 1 else 12
    for z0 in slab_starts:
        z0 = max(0, min(z0, nz - S))
        lo = 0 if z0 == 0 else 2 * radius
        hi = S if z0 + S == nz else S - 2 * radius
        cs, rs, us = (_slab(seed, k, shape, z0, S) for k in ("c", "r_bar", "u_bar"))
        ps = _slab(seed, "u_prev_bar", shape, z0, S) if with_prev else None
        want, wantp, scale = oracle.wave_adjoint(cs, rs, us, radius, u_prev_bar=ps, want_scale=True)
        got = to_host(ub[z0:z0 + S])
        assert_close(got[lo:hi], want[lo:hi], (scale + np.abs(us))[lo:hi], np.float64,
                     "u_bar planes %d..%d of %s r=%d" % (z0 + lo, z0 + hi - 1, shape, radius))
        if with_prev:
            gotp = to_host(up[z0:z0 + S])
            # u_prev_bar[j] -= r_bar[j] on I: a plane depends on its own plane only
            assert_close(gotp[lo:hi], wantp[lo:hi], (np.abs(ps) + np.abs(rs))[lo:hi], np.float64, "u_prev_bar planes from %d" % z0)
    # conservation: the Laplacian weights sum to zero, so sum(delta u_bar) = 2 sum_I r_bar; sum(delta u_prev_bar) = -sum_I r_bar
    absdelta = 30.0 * abs(sum_rb_I) + float(ub.abs().sum()) * 1e-3
    assert abs((float(ub.sum()) - sum_ub0) - 2.0 * sum_rb_I) <= 1e-9 * absdelta
    if with_prev:
        assert abs((float(up.sum()) - sum_up0) + sum_rb_I) <= 1e-9 * absdelta


def test_paper_size_7_point_star_with_u_prev_bar_1000_cubed(sadj):
    """The paper's own wave experiment (Section 4.1): 7-point star, 1000^3, both adjoint outputs.
    Rows of 8000 bytes: wide tiles, several rounds of workgroups."""
    _check_on_slabs(sadj, 1, (1000, 1000, 1000), True, [0, 120, 497, 744, 988], seed=41)


def test_radius_4_at_1000_cubed(sadj):
    _check_on_slabs(sadj, 4, (1000, 1000, 1000), False, [0, 240, 487, 974], seed=42)


def test_radius_4_at_768_cubed_where_left_over_tiles_are_cut_finer(sadj):
    """288 tiles for 256 compute units: 256 tiles march all planes, 32 are cut into chunks of 96;
    slabs straddle chunk ends (96, 384, 672) and the grid's ends."""
    info, _ = sadj.sadj_describe_wave3d_plan(1, 4, 768, 768, 768, with_tiles=False)
    assert info["tiles_a"] > 0, "this size is meant to take the two-group plan"
    _check_on_slabs(sadj, 4, (768, 768, 768), False, [0, 83, 371, 659, 742], seed=43)


def test_radius_4_with_u_prev_bar_full_size_every_element(sadj):
    """512^3, radius 4, fp64, both outputs (the form the paper differentiates, at the benchmark's
    radius): every element against the oracle."""
    import torch
    shape = (512, 512, 512)
    d = inputs.config_inputs("wave3d_r4", shape=shape, fields=("c", "r_bar", "u_bar", "u_prev_bar"))
    c, rb, ub, up = (torch.from_numpy(d[k]).cuda() for k in ("c", "r_bar", "u_bar", "u_prev_bar"))
    sadj.sadj_adjoint_wave3d(4, c, rb, ub, up)
    torch.cuda.synchronize()
    want, wantp, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 4, u_prev_bar=d["u_prev_bar"], want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]), np.float64, "u_bar 512^3 r=4 with u_prev_bar")
    assert_close(to_host(up), wantp, np.abs(d["u_prev_bar"]) + np.abs(d["r_bar"]), np.float64, "u_prev_bar 512^3 r=4")
