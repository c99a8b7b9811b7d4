"""GPU parity: sadj_adjoint_wave3d / sadj_primal_wave3d against the CPU oracle,
element by element, on the same seeded inputs (called through the C ABI binding)."""
import numpy as np
import pytest
import scipy.ndimage as ndi

import inputs
import oracle
from jacobians import interior_mask, star_weights
from parity import assert_close, to_gpu, to_host

pytestmark = pytest.mark.gpu

SMALL = [
    # (radius, (nz, ny, nx)) -- several tiles + ragged tails; sizes with an empty core
    (4, (37, 45, 150)), (4, (9, 9, 9)), (4, (16, 17, 19)), (4, (17, 40, 70)), (4, (40, 16, 200)),
    (4, (21, 33, 64)), (4, (70, 20, 129)),
    (1, (3, 3, 3)), (1, (4, 5, 7)), (1, (21, 37, 150)), (1, (70, 18, 65)), (1, (5, 64, 128)),
    (2, (5, 5, 5)), (2, (9, 11, 70)), (2, (33, 45, 150)), (3, (7, 7, 7)), (3, (13, 15, 17)), (3, (30, 41, 136)),
    (4, (3000, 9, 20)), (1, (5000, 5, 9)),      # one tile, hundreds of z-chunks
    (4, (12, 300, 2100)), (2, (9, 270, 4100)),  # 32 and more tiles per row: tiles numbered in bands of 8 rows
]


def _run_adjoint(sadj, d, radius, with_prev):
    c, rb = to_gpu(d["c"]), to_gpu(d["r_bar"])
    ub = to_gpu(d["u_bar"])
    upb = to_gpu(d["u_prev_bar"]) if with_prev else None
    sadj.sadj_adjoint_wave3d(radius, c, rb, ub, upb)
    import torch
    torch.cuda.synchronize()
    return to_host(ub), (to_host(upb) if with_prev else None)


def _check_adjoint(sadj, d, radius, dtype, with_prev, what):
    got_u, got_p = _run_adjoint(sadj, d, radius, with_prev)
    want_u, want_p, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius,
                                                u_prev_bar=d["u_prev_bar"] if with_prev else None,
                                                want_scale=True)
    scale = scale + np.abs(d["u_bar"].astype(np.float64))
    e = assert_close(got_u, want_u, scale, dtype, what + " u_bar")
    if with_prev:
        sp = np.abs(d["u_prev_bar"].astype(np.float64)) + np.abs(d["r_bar"].astype(np.float64))
        assert_close(got_p, want_p, sp, dtype, what + " u_prev_bar")
        m = interior_mask(d["c"].shape, radius)
        assert np.array_equal(got_p[~m], d["u_prev_bar"][~m])
    return e


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    yield lib
    lib.set_option("wave3d.zchunk", 0)
    lib.set_option("wave3d.variant", 0)
    lib.set_option("wave3d.remainder", 0)
    lib.set_option("wave3d.order", 0)
    lib.set_option("wave3d.split", 0)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius,shape", SMALL)
def test_adjoint_small(sadj, radius, shape, dtype):
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=sum(shape), dtype=dtype, c_mode="iid")
    for zchunk in (0, 16, 7):
        sadj.set_option("wave3d.zchunk", zchunk)
        _check_adjoint(sadj, d, radius, dtype, with_prev=False,
                       what="R=%d %s zchunk=%d" % (radius, shape, zchunk))
    sadj.set_option("wave3d.zchunk", 0)
    _check_adjoint(sadj, d, radius, dtype, with_prev=True, what="R=%d %s with u_prev_bar" % (radius, shape))


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 5, 10, 11])
@pytest.mark.parametrize("radius", [1, 4])
def test_adjoint_tile_variants(sadj, radius, variant):
    sadj.set_option("wave3d.variant", variant)
    try:
        for shape, dtype in (((30, 75, 140), np.float64), ((23, 41, 270), np.float32), ((12, 70, 133), np.float32)):
            d = inputs.config_inputs("wave3d_r4", shape=shape, seed=variant, dtype=dtype)   # layered c, as benchmarked
            _check_adjoint(sadj, d, radius, dtype, with_prev=True, what="variant %d %s" % (variant, shape))
    finally:
        sadj.set_option("wave3d.variant", 0)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius", [1, 2, 3, 4])
def test_remainder_strategies_agree(sadj, radius, dtype):
    """Section 3.3.4 names several treatments of the remainder (disjoint nests, guarded
    statements, zero padding).  The library's three strategies must match the oracle and,
    since every cell sums the same terms in the same order, each other bit for bit."""
    for shape in ((30, 75, 140), (23, 41, 272), (12, 20, 64), (9, 9, 12)):
        d = inputs.wave_inputs(shape, 0.01, 0.1, seed=shape[1], dtype=dtype, c_mode="iid")
        ref, _ = _run_adjoint(sadj, d, radius, False)
        try:
            for strategy in (1, 2):
                sadj.set_option("wave3d.remainder", strategy)
                _check_adjoint(sadj, d, radius, dtype, with_prev=False,
                               what="remainder strategy %d R=%d %s" % (strategy, radius, shape))
                got, _ = _run_adjoint(sadj, d, radius, False)
                assert np.array_equal(got, ref), (strategy, shape)
        finally:
            sadj.set_option("wave3d.remainder", 0)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius,shape", [(4, (37, 45, 150)), (4, (9, 9, 9)), (4, (17, 40, 70)), (1, (3, 3, 3)),
                                          (1, (21, 37, 150)), (1, (70, 18, 65)), (2, (20, 30, 70)), (3, (7, 7, 7)),
                                          (3, (21, 30, 66))])
def test_atomic_scatter_contrast_kernel_matches_the_oracle(sadj, radius, shape, dtype):
    """The conventional scatter with atomic updates (Sections 1, 3.2, 4.1), kept as a
    baseline to compare the gather with; same result up to summation order."""
    import torch
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=11 + sum(shape), dtype=dtype, c_mode="iid")
    m = interior_mask(shape, radius)
    c = to_gpu(np.where(m, d["c"], np.nan).astype(dtype))
    rb = to_gpu(np.where(m, d["r_bar"], np.nan).astype(dtype))
    ub = to_gpu(d["u_bar"])
    sadj.sadj_adjoint_wave3d_atomic_scatter(radius, c, rb, ub)
    torch.cuda.synchronize()
    want, _, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius, want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"].astype(np.float64)), dtype,
                 "atomic scatter R=%d %s" % (radius, shape))


def _bits(a):
    return a.view(np.int64 if a.dtype == np.float64 else np.int32)


@pytest.mark.parametrize("radius,shape", SMALL + [(4, (30, 75, 140)), (1, (23, 41, 272))])
def test_scatter_order_mode_equals_the_sequential_scatter_bit_for_bit(sadj, radius, shape):
    """Section 3.5: a gather can respect a summation order the user chooses.  With
    "wave3d.order" = 1 the library adds the terms of each u_bar[j] in the order and with
    the rounding of the sequential scatter loop; in fp64 that loop is the oracle itself,
    in fp32 its whole-array formulation (pinned to the oracle in test_oracle_wave.py)."""
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=7 + sum(shape), c_mode="iid")
    d["u_bar"][0, 0, :] = -0.0                      # a cell without terms keeps even the sign of zero
    m = interior_mask(shape, radius)
    poisoned = dict(d, c=np.where(m, d["c"], np.nan), r_bar=np.where(m, d["r_bar"], np.nan))
    want_u, want_p, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius, u_prev_bar=d["u_prev_bar"])
    sadj.set_option("wave3d.order", 1)
    try:
        for zchunk in (0, 11):
            sadj.set_option("wave3d.zchunk", zchunk)
            for data in (d, poisoned):
                got_u, got_p = _run_adjoint(sadj, data, radius, True)
                assert np.array_equal(_bits(got_u), _bits(want_u)), (zchunk, "u_bar")
                assert np.array_equal(_bits(got_p), _bits(want_p)), (zchunk, "u_prev_bar")
            got_u, _ = _run_adjoint(sadj, d, radius, False)
            assert np.array_equal(_bits(got_u), _bits(want_u))
        sadj.set_option("wave3d.zchunk", 0)
        from scatter_order import wave3d_adjoint_scatter_order
        d32 = {k: v.astype(np.float32) for k, v in d.items()}
        got32, _ = _run_adjoint(sadj, d32, radius, False)
        want32 = wave3d_adjoint_scatter_order(d32["c"], d32["r_bar"], d32["u_bar"], radius)
        assert np.array_equal(_bits(got32), _bits(want32))
    finally:
        sadj.set_option("wave3d.order", 0)
        sadj.set_option("wave3d.zchunk", 0)


@pytest.mark.parametrize("xcdmap,band", [(1, 0), (2, 0), (3, 0), (1, 2), (2, 3), (1, 8)])
def test_tile_mappings_give_identical_results(sadj, xcdmap, band):
    """Which workgroup marches which tile is a scheduling choice; every mapping must be a
    bijection onto the tiles (each u_bar element written exactly once) for ragged tile
    grids and several z-chunks, hence bit-identical results and parity with the oracle."""
    try:
        for radius, shape, zchunk in ((4, (40, 150, 330), 9), (1, (33, 70, 200), 0), (4, (700, 40, 70), 0)):
            d = inputs.wave_inputs(shape, 0.01, 0.1, seed=shape[2], c_mode="iid")
            sadj.set_option("wave3d.zchunk", zchunk)
            sadj.set_option("wave3d.xcdmap", 0)
            sadj.set_option("wave3d.band", 0)
            ref, _ = _run_adjoint(sadj, d, radius, False)
            sadj.set_option("wave3d.xcdmap", xcdmap)
            sadj.set_option("wave3d.band", band)
            _check_adjoint(sadj, d, radius, np.float64, with_prev=True, what="xcdmap %d band %d %s" % (xcdmap, band, shape))
            got, _ = _run_adjoint(sadj, d, radius, False)
            assert np.array_equal(got, ref)
    finally:
        sadj.set_option("wave3d.xcdmap", 0)
        sadj.set_option("wave3d.band", 0)
        sadj.set_option("wave3d.zchunk", 0)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius,shape", [(4, (90, 70, 200)), (1, (64, 130, 140)), (2, (50, 40, 330))])
def test_cutting_and_placing_the_work_differently_changes_no_bit(sadj, radius, shape, dtype):
    """z-chunk length, finer cuts of left-over tiles and the LDS request that sets the number
    of workgroups per CU move work between workgroups; the arithmetic of a cell is the same
    instruction sequence whichever workgroup runs it, so adjoint and primal results are
    bit-identical under all of them."""
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=sum(shape), dtype=dtype, c_mode="iid")
    r0 = inputs.uniform(3, "aux", shape, -1, 1).astype(dtype)

    def run():
        ub, upb = _run_adjoint(sadj, d, radius, True)
        ub2, _ = _run_adjoint(sadj, d, radius, False)
        r = to_gpu(r0)
        sadj.sadj_primal_wave3d(radius, to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
        return ub, upb, ub2, to_host(r)

    ref = run()
    try:
        for opts in ({"wave3d.zchunk": 7}, {"wave3d.zchunk": 33}, {"wave3d.split": 1}, {"wave3d.ldspad": -1},
                     {"wave3d.zchunk": 16, "wave3d.xcdmap": 3, "wave3d.band": 2}):
            for k, v in opts.items():
                sadj.set_option(k, v)
            got = run()
            for k in opts:
                sadj.set_option(k, 0)
            for a, b in zip(got, ref):
                assert np.array_equal(a, b), opts
    finally:
        for k in ("wave3d.zchunk", "wave3d.split", "wave3d.ldspad", "wave3d.xcdmap", "wave3d.band"):
            sadj.set_option(k, 0)


@pytest.mark.parametrize("case", range(24))
def test_adjoint_and_primal_on_drawn_shapes_and_options(sadj, case):
    """Shapes, radius, dtype and scheduling options drawn from a seeded generator: ragged
    tiles in both directions, z-chunks that do not divide nz, every id mapping."""
    rng = np.random.default_rng(1000 + case)
    radius = int(rng.integers(1, 5))
    dtype = [np.float64, np.float32][int(rng.integers(0, 2))]
    lo = 2 * radius + 1
    shape = (int(rng.integers(lo, 90)), int(rng.integers(lo, 120)), int(rng.integers(lo, 300)))
    opts = {"wave3d.zchunk": int(rng.choice([0, 0, 5, 13, 40])), "wave3d.xcdmap": int(rng.integers(0, 4)),
            "wave3d.band": int(rng.choice([0, 0, 2, 5])), "wave3d.ldspad": int(rng.choice([0, -1]))}
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=case, dtype=dtype, c_mode="iid")
    try:
        for k, v in opts.items():
            sadj.set_option(k, v)
        what = "case %d R=%d %s %s %s" % (case, radius, shape, np.dtype(dtype).name, opts)
        _check_adjoint(sadj, d, radius, dtype, with_prev=bool(rng.integers(0, 2)), what=what)
        import torch
        r0 = inputs.uniform(case, "aux", shape, -1, 1).astype(dtype)
        r = to_gpu(r0)
        sadj.sadj_primal_wave3d(radius, to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
        torch.cuda.synchronize()
        got = to_host(r)
        want = oracle.wave_primal(d["u"], d["u_prev"], d["c"], radius, r_init=r0)
        m = interior_mask(shape, radius)
        assert np.array_equal(got[~m], r0[~m])
        assert_close(got[m], want[m], _primal_scale(d, radius)[m], dtype, what + " primal")
    finally:
        for k in opts:
            sadj.set_option(k, 0)


def test_remainder_strategy_declines_what_it_does_not_cover(sadj):
    import paper_1907_02818_amd as lib
    d = inputs.wave_inputs((12, 20, 64), 0.01, 0.1, seed=1)
    c, rb, ub, upb = (to_gpu(d[k]) for k in ("c", "r_bar", "u_bar", "u_prev_bar"))
    sadj.set_option("wave3d.remainder", 2)
    try:
        with pytest.raises(lib.SadjError) as e:
            sadj.sadj_adjoint_wave3d(4, c, rb, ub, upb)
        assert e.value.status == 4
        import torch
        torch.cuda.synchronize()
        assert np.array_equal(to_host(ub), d["u_bar"]) and np.array_equal(to_host(upb), d["u_prev_bar"])
    finally:
        sadj.set_option("wave3d.remainder", 0)


def test_adjoint_is_bitwise_reproducible_and_ignores_values_outside_the_interior(sadj):
    radius, shape = 4, (33, 50, 133)
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=5, c_mode="iid")
    a, _ = _run_adjoint(sadj, d, radius, False)
    b, _ = _run_adjoint(sadj, d, radius, False)
    assert np.array_equal(a, b)
    m = interior_mask(shape, radius)
    dp = dict(d)
    dp["c"] = np.where(m, d["c"], np.nan)
    dp["r_bar"] = np.where(m, d["r_bar"], np.nan)
    p, pp = _run_adjoint(sadj, dp, radius, True)
    assert np.isfinite(p).all() and np.isfinite(pp).all()
    assert np.array_equal(p, a)


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_odd_extent_and_unaligned_arrays_take_the_scalar_shape(sadj, dtype):
    """Shapes that move several cells per lane need nx to be a multiple of the vector
    length and vector-aligned arrays; otherwise the library must fall back by itself."""
    import torch
    radius = 4
    for shape, shift in (((19, 37, 131), 0), ((19, 37, 132), 1), ((12, 33, 130), 1)):
        d = inputs.wave_inputs(shape, 0.01, 0.1, seed=shift + shape[2], dtype=dtype)
        n = int(np.prod(shape))

        def dev(a):
            t = torch.empty(n + shift, dtype=torch.from_numpy(a).dtype, device="cuda")
            v = t[shift:].view(shape)          # starts `shift` elements into the allocation
            v.copy_(torch.from_numpy(a))
            return v
        c, rb, ub, upb = dev(d["c"]), dev(d["r_bar"]), dev(d["u_bar"]), dev(d["u_prev_bar"])
        sadj.sadj_adjoint_wave3d(radius, c, rb, ub, upb)
        r0 = inputs.uniform(3, "aux", shape, -1, 1).astype(dtype)
        r = dev(r0)
        sadj.sadj_primal_wave3d(radius, dev(d["u"]), dev(d["u_prev"]), c, r)
        torch.cuda.synchronize()
        want_u, want_p, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius,
                                                    u_prev_bar=d["u_prev_bar"], want_scale=True)
        assert_close(to_host(ub), want_u, scale + np.abs(d["u_bar"].astype(np.float64)), dtype, "fallback %s" % (shape,))
        assert_close(to_host(upb), want_p, np.abs(d["u_prev_bar"].astype(np.float64)) + np.abs(d["r_bar"].astype(np.float64)),
                     dtype, "fallback u_prev_bar")
        want_r = oracle.wave_primal(d["u"], d["u_prev"], d["c"], radius, r_init=r0)
        m = interior_mask(shape, radius)
        got_r = to_host(r)
        assert np.array_equal(got_r[~m], r0[~m])
        assert_close(got_r[m], want_r[m], _primal_scale(d, radius)[m], dtype, "fallback primal")


def test_adjoint_on_a_side_stream(sadj):
    import torch
    radius, shape = 4, (20, 40, 100)
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=9)
    c, rb, ub = to_gpu(d["c"]), to_gpu(d["r_bar"]), to_gpu(d["u_bar"])
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        sadj.sadj_adjoint_wave3d(radius, c, rb, ub)
    st.synchronize()
    want, _, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], radius, want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]), np.float64, "side stream")


def _primal_scale(d, radius):
    w = star_weights(radius)
    kern = np.zeros((2 * radius + 1,) * 3)
    kern[radius, radius, radius] = 3 * abs(w[0])
    for ax in range(3):
        for k in range(1, radius + 1):
            for s in (-k, k):
                idx = [radius] * 3
                idx[ax] += s
                kern[tuple(idx)] = abs(w[k])
    u = np.abs(d["u"].astype(np.float64))
    return 2 * u + np.abs(d["u_prev"].astype(np.float64)) + np.abs(d["c"].astype(np.float64)) * \
        ndi.correlate(u, kern, mode="constant")


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius,shape", SMALL)
def test_primal_small(sadj, radius, shape, dtype):
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=1 + sum(shape), dtype=dtype, c_mode="iid")
    r0 = inputs.uniform(3, "aux", shape, -1, 1).astype(dtype)
    r = to_gpu(r0)
    sadj.sadj_primal_wave3d(radius, to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
    got = to_host(r)
    want = oracle.wave_primal(d["u"], d["u_prev"], d["c"], radius, r_init=r0)
    m = interior_mask(shape, radius)
    assert np.array_equal(got[~m], r0[~m])                 # r outside I untouched
    assert_close(got[m], want[m], _primal_scale(d, radius)[m], dtype, "primal R=%d %s" % (radius, shape))


# rows that are not a multiple of the 128-byte cache line: the launcher takes tiles of 16 rows
# with long rows when they cover nx well (radius 1: 256 cells, fp32 adjoint 512; larger radii:
# 1 KB); 1002 is not a multiple of four, so the fp32 calls fall back to the one-cell shape there
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius,shape", [(1, (20, 37, 250)), (1, (9, 40, 500)), (1, (6, 20, 1000)), (1, (5, 17, 1002)),
                                          (1, (19, 33, 750)), (1, (40, 16, 1500)),
                                          (4, (20, 37, 250)), (2, (9, 40, 500)), (3, (12, 20, 1000)), (4, (11, 33, 1002)),
                                          (4, (30, 50, 750)), (2, (5, 5, 1250))])
def test_unaligned_rows_take_wide_tiles(sadj, radius, shape, dtype):
    nz, ny, nx = shape
    info, _ = sadj.sadj_describe_wave3d_plan(1 if dtype == np.float64 else 0, radius, nx, ny, nz, with_tiles=False)
    if dtype == np.float32 and nx % 4 != 0:
        # whole four-float vectors are not possible: the radius-1 shape with two cells per lane
        # (256 x 16) where it covers nx well, else the one-cell shape
        assert (info["tile_w"], info["tile_h"]) in (((256, 16), (64, 32)) if radius == 1 and nx % 2 == 0 else ((64, 32),))
    else:
        assert info["tile_h"] == 16
        assert info["tile_w"] in ((256, 512) if radius == 1 else (1024 // np.dtype(dtype).itemsize,))
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=sum(shape), dtype=dtype, c_mode="iid")
    for zchunk in (0, 5):
        sadj.set_option("wave3d.zchunk", zchunk)
        _check_adjoint(sadj, d, radius, dtype, with_prev=False, what="wide tiles R=%d %s zchunk=%d" % (radius, shape, zchunk))
    sadj.set_option("wave3d.zchunk", 0)
    _check_adjoint(sadj, d, radius, dtype, with_prev=True, what="wide tiles R=%d %s with u_prev_bar" % (radius, shape))
    r0 = inputs.uniform(3, "aux", shape, -1, 1).astype(dtype)
    r = to_gpu(r0)
    sadj.sadj_primal_wave3d(radius, to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
    got = to_host(r)
    want = oracle.wave_primal(d["u"], d["u_prev"], d["c"], radius, r_init=r0)
    m = interior_mask(shape, radius)
    assert np.array_equal(got[~m], r0[~m])
    assert_close(got[m], want[m], _primal_scale(d, radius)[m], dtype, "primal wide tiles R=%d %s" % (radius, shape))


# shapes whose x-y tiles do not fill whole rounds of the chip's compute units, so that the
# left-over tiles are cut into more z-chunks than the others (two groups of workgroups)
TWO_GROUP = [(np.float64, 4, (64, 580, 520)), (np.float64, 1, (24, 400, 610)), (np.float64, 2, (64, 70, 1856)),
             (np.float64, 3, (24, 610, 832)), (np.float32, 1, (24, 400, 1216))]


@pytest.mark.parametrize("dtype,radius,shape", TWO_GROUP)
def test_shapes_whose_left_over_tiles_are_cut_finer(sadj, dtype, radius, shape):
    nz, ny, nx = shape
    info, tiles = sadj.sadj_describe_wave3d_plan(1 if dtype == np.float64 else 0, radius, nx, ny, nz)
    if info["tiles_a"] == 0:
        pytest.skip("this device's compute-unit count does not leave tiles over at this shape")
    assert len({ze - zs for _, _, zs, ze in tiles}) >= 2
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=sum(shape), dtype=dtype, c_mode="iid")
    _check_adjoint(sadj, d, radius, dtype, with_prev=True, what="two groups R=%d %s" % (radius, shape))
    sadj.set_option("wave3d.split", 1)
    try:
        alike, _ = _run_adjoint(sadj, d, radius, False)
    finally:
        sadj.set_option("wave3d.split", 0)
    finer, _ = _run_adjoint(sadj, d, radius, False)
    assert np.array_equal(alike, finer)              # the cut along z does not change any value
    r0 = inputs.uniform(3, "aux", shape, -1, 1).astype(dtype)
    r = to_gpu(r0)
    sadj.sadj_primal_wave3d(radius, to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
    got = to_host(r)
    want = oracle.wave_primal(d["u"], d["u_prev"], d["c"], radius, r_init=r0)
    m = interior_mask(shape, radius)
    assert np.array_equal(got[~m], r0[~m])
    assert_close(got[m], want[m], _primal_scale(d, radius)[m], dtype, "primal two groups R=%d %s" % (radius, shape))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_adjoint_full_size_headline(sadj, dtype):
    """512^3, radius 4, default launch configuration (the one bench.py times), every
    element compared with the oracle."""
    d = inputs.config_inputs("wave3d_r4", dtype=dtype)
    e = _check_adjoint(sadj, d, 4, dtype, with_prev=False, what="512^3 R=4 %s" % np.dtype(dtype).name)
    print("512^3 R=4 %s max rel err %.3e" % (np.dtype(dtype).name, e))
    # closed form that holds at any size: the star weights sum to zero, so the increments of
    # u_bar add up to 2 * sum of r_bar over the primal interior (u_dot = 1 in the dot-product test)
    got, _ = _run_adjoint(sadj, d, 4, False)
    delta = got.astype(np.float64) - d["u_bar"].astype(np.float64)
    m = interior_mask(d["c"].shape, 4)
    want_sum = 2.0 * d["r_bar"].astype(np.float64)[m].sum()
    bound = (1e-12 if dtype == np.float64 else 1e-5) * np.abs(delta).sum()
    assert abs(delta.sum() - want_sum) <= bound, (delta.sum(), want_sum, bound)


def test_scatter_order_mode_full_size_is_bit_identical_to_the_sequential_scatter(sadj):
    """512^3, radius 4, fp64 with "wave3d.order" = 1: all 134 million elements equal the
    oracle's sequential scatter loop bit for bit (Section 3.5)."""
    d = inputs.config_inputs("wave3d_r4")
    want, _, _ = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 4)
    sadj.set_option("wave3d.order", 1)
    try:
        got, _ = _run_adjoint(sadj, d, 4, False)
    finally:
        sadj.set_option("wave3d.order", 0)
    assert np.array_equal(got.view(np.int64), want.view(np.int64))


def test_adjoint_full_size_r1(sadj):
    d = inputs.config_inputs("wave3d_r1")
    _check_adjoint(sadj, d, 1, np.float64, with_prev=True, what="512^3 R=1")


def test_arrays_beyond_4_gib_are_addressed_with_64_bits(sadj):
    """1024 x 1024 x 640 in fp64: every array holds 5.4 GB, so element offsets pass 2^32
    bytes and the dispatch takes two rounds of workgroups.  The oracle runs on three slabs
    of planes (bottom with the global boundary, one across the 4 GiB mark, top); a slab is
    a grid of its own, so its planes from 2R to S-2R-1 (all their sources lie in the slab's
    interior) -- and, at the bottom / top of the grid, also its first / last planes --
    equal those of the full problem."""
    import torch
    radius, shape = 4, (640, 1024, 1024)
    nz = shape[0]
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=21, c_mode="iid", fields=("c", "r_bar", "u_bar"))
    c, rb, ub = to_gpu(d["c"]), to_gpu(d["r_bar"]), to_gpu(d["u_bar"])
    sadj.sadj_adjoint_wave3d(radius, c, rb, ub)
    torch.cuda.synchronize()
    got = to_host(ub)
    del c, rb, ub
    plane_bytes = shape[1] * shape[2] * 8
    zmark = (1 << 32) // plane_bytes                       # the plane that contains byte offset 2^32
    S = 24
    for z0, lo, hi in ((0, 0, S - 2 * radius), (zmark - S // 2, 2 * radius, S - 2 * radius), (nz - S, 2 * radius, S)):
        sl = slice(z0, z0 + S)
        want, _, scale = oracle.wave_adjoint(d["c"][sl], d["r_bar"][sl], d["u_bar"][sl], radius, want_scale=True)
        scale = scale + np.abs(d["u_bar"][sl])
        assert_close(got[sl][lo:hi], want[lo:hi], scale[lo:hi], np.float64, "planes %d..%d" % (z0 + lo, z0 + hi - 1))
    # and nothing else was left untouched or written twice: the closed-form sum over the grid
    delta = got - d["u_bar"]
    m = interior_mask(shape, radius)
    want_sum = 2.0 * d["r_bar"][m].sum()
    assert abs(delta.sum() - want_sum) <= 1e-12 * np.abs(delta).sum()
