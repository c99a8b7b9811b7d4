"""GPU parity for the 1-D and 2-D stencils (wave 3-point, wave 5-point, Burgers):
HIP path through the C ABI binding vs the CPU oracle, element by element."""
import numpy as np
import pytest

import inputs
import oracle
from jacobians import interior_mask
from parity import wave_primal_scale, assert_close, to_gpu, to_host

pytestmark = pytest.mark.gpu

C, D = 0.1, 0.05


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    return lib


@pytest.fixture(params=[0, 1], ids=["handwritten", "functor"])
def path1d(sadj, request):
    """Burgers runs through its hand-written kernel and through the generic three-point
    functor kernel (include/sadj_stencil1d.hpp); both must meet the same bar."""
    sadj.set_option("stencil1d.functor", request.param)
    yield request.param
    sadj.set_option("stencil1d.functor", 0)


def _sync():
    import torch
    torch.cuda.synchronize()


# ---------------------------------------------------------------------- 1-D wave
N1D = [3, 4, 5, 7, 63, 64, 65, 127, 128, 129, 130, 131, 255, 256, 257, 258, 259, 260, 511, 1000,
       4096, 4097, 100003]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n", N1D)
def test_wave1d_adjoint_and_primal(sadj, n, dtype):
    d = inputs.wave_inputs((n,), 0.01, 0.25, seed=n, dtype=dtype)
    for with_prev in (False, True):
        ub = to_gpu(d["u_bar"])
        upb = to_gpu(d["u_prev_bar"]) if with_prev else None
        sadj.sadj_adjoint_wave1d(to_gpu(d["c"]), to_gpu(d["r_bar"]), ub, upb)
        _sync()
        want, wantp, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1,
                                                 u_prev_bar=d["u_prev_bar"] if with_prev else None,
                                                 want_scale=True)
        assert_close(to_host(ub), want, scale + np.abs(d["u_bar"].astype(np.float64)), dtype, "wave1d n=%d" % n)
        if with_prev:
            sp = np.abs(d["u_prev_bar"].astype(np.float64)) + np.abs(d["r_bar"].astype(np.float64))
            assert_close(to_host(upb), wantp, sp, dtype, "wave1d u_prev_bar n=%d" % n)
            assert to_host(upb)[0] == d["u_prev_bar"][0] and to_host(upb)[-1] == d["u_prev_bar"][-1]
    r0 = inputs.uniform(1, "aux", (n,), -1, 1).astype(dtype)
    r = to_gpu(r0)
    sadj.sadj_primal_wave1d(to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
    _sync()
    want = oracle.wave_primal(d["u"], d["u_prev"], d["c"], 1, r_init=r0)
    got = to_host(r)
    assert got[0] == r0[0] and got[-1] == r0[-1]
    u = np.abs(d["u"].astype(np.float64))
    sc = 2 * u + np.abs(d["u_prev"].astype(np.float64))
    sc[1:-1] += np.abs(d["c"].astype(np.float64))[1:-1] * (u[:-2] + 2 * u[1:-1] + u[2:])
    assert_close(got, want, sc, dtype, "wave1d primal n=%d" % n)


def test_wave1d_unaligned_pointers_and_nan_outside_interior(sadj):
    import torch
    n = 1001
    d = inputs.wave_inputs((n,), 0.01, 0.25, seed=2)
    d["c"][0] = d["c"][-1] = np.nan
    d["r_bar"][0] = d["r_bar"][-1] = np.nan
    # views that start 8 bytes into an allocation: not 16-byte aligned
    def off(a):
        t = torch.empty(n + 1, dtype=torch.float64, device="cuda")
        t[1:] = torch.from_numpy(a).cuda()
        return t[1:]
    ub = off(d["u_bar"])
    sadj.sadj_adjoint_wave1d(off(d["c"]), off(d["r_bar"]), ub)
    _sync()
    want, _, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, want_scale=True)
    assert np.isfinite(to_host(ub)).all()
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]), np.float64, "unaligned 1-D")


# ----------------------------------------------------------------------- Burgers
@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n", N1D + [1 << 20])
def test_burgers_adjoint_and_primal(sadj, path1d, n, dtype):
    d = inputs.burgers_inputs(n, seed=n, dtype=dtype)
    u = d["u"].copy()
    if n > 300:
        u[[5, 100, 101, 200]] = 0.0             # exact zeros: the kink convention
    ub = to_gpu(d["u_bar"])
    sadj.sadj_adjoint_burgers1d(C, D, to_gpu(u), to_gpu(d["r_bar"]), ub)
    _sync()
    Cd, Dd = (float(np.float32(C)), float(np.float32(D))) if dtype == np.float32 else (C, D)
    want, scale = oracle.burgers_adjoint(u, d["r_bar"], d["u_bar"], Cd, Dd, want_scale=True)
    # the centre partial is itself a cancelling sum of O(1) terms: add |r_bar| to the scale
    sc = scale + np.abs(d["u_bar"].astype(np.float64)) + np.abs(d["r_bar"].astype(np.float64))
    assert_close(to_host(ub), want, sc, dtype, "burgers adjoint n=%d" % n)
    r0 = inputs.uniform(1, "aux", (n,), -1, 1).astype(dtype)
    r = to_gpu(r0)
    sadj.sadj_primal_burgers1d(C, D, to_gpu(u), r)
    _sync()
    want = oracle.burgers_primal(u, Cd, Dd, r_init=r0)
    got = to_host(r)
    assert got[0] == r0[0] and got[-1] == r0[-1]
    assert_close(got, want, np.abs(want) + 1.0, dtype, "burgers primal n=%d" % n)


def test_burgers_nan_in_r_bar_outside_interior_and_reproducible(sadj, path1d):
    n = 5000
    d = inputs.burgers_inputs(n, seed=3)
    rb = d["r_bar"].copy()
    rb[0] = rb[-1] = np.nan
    outs = []
    for _ in range(2):
        ub = to_gpu(d["u_bar"])
        sadj.sadj_adjoint_burgers1d(C, D, to_gpu(d["u"]), to_gpu(rb), ub)
        _sync()
        outs.append(to_host(ub))
    assert np.isfinite(outs[0]).all()
    assert np.array_equal(outs[0], outs[1])


def test_burgers_full_size(sadj, path1d):
    n = 1 << 24
    d = inputs.config_inputs("burgers1d")
    ub = to_gpu(d["u_bar"])
    sadj.sadj_adjoint_burgers1d(C, D, to_gpu(d["u"]), to_gpu(d["r_bar"]), ub)
    _sync()
    want, scale = oracle.burgers_adjoint(d["u"], d["r_bar"], d["u_bar"], C, D, want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]) + np.abs(d["r_bar"]), np.float64,
                 "burgers n=2^24")


# ---------------------------------------------------------------------- 2-D wave
SHAPES2D = [(3, 3), (3, 200), (200, 3), (5, 7), (66, 130), (67, 131), (130, 256), (129, 258),
            (200, 513), (70, 1030), (300, 300)]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("shape", SHAPES2D)
def test_wave2d_adjoint_and_primal(sadj, shape, dtype):
    d = inputs.wave_inputs(shape, 0.01, 0.2, seed=sum(shape), dtype=dtype)
    m = interior_mask(shape, 1)
    for with_prev in (False, True):
        ub = to_gpu(d["u_bar"])
        upb = to_gpu(d["u_prev_bar"]) if with_prev else None
        sadj.sadj_adjoint_wave2d(to_gpu(d["c"]), to_gpu(d["r_bar"]), ub, upb)
        _sync()
        want, wantp, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1,
                                                 u_prev_bar=d["u_prev_bar"] if with_prev else None,
                                                 want_scale=True)
        assert_close(to_host(ub), want, scale + np.abs(d["u_bar"].astype(np.float64)), dtype,
                     "wave2d %s" % (shape,))
        if with_prev:
            sp = np.abs(d["u_prev_bar"].astype(np.float64)) + np.abs(d["r_bar"].astype(np.float64))
            assert_close(to_host(upb), wantp, sp, dtype, "wave2d u_prev_bar %s" % (shape,))
            assert np.array_equal(to_host(upb)[~m], d["u_prev_bar"][~m])
    r0 = inputs.uniform(1, "aux", shape, -1, 1).astype(dtype)
    r = to_gpu(r0)
    sadj.sadj_primal_wave2d(to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
    _sync()
    want = oracle.wave_primal(d["u"], d["u_prev"], d["c"], 1, r_init=r0)
    got = to_host(r)
    assert np.array_equal(got[~m], r0[~m])
    assert_close(got[m], want[m], wave_primal_scale(d["u"], d["u_prev"], d["c"], 1)[m], dtype, "wave2d primal %s" % (shape,))


@pytest.mark.parametrize("variant,ychunk", [(0, 0), (1, 0), (1, 5), (1, 16), (1, 33), (2, 0)])
def test_wave2d_variants(sadj, variant, ychunk):
    shape = (131, 523)
    d = inputs.wave_inputs(shape, 0.01, 0.2, seed=variant + ychunk)
    sadj.set_option("wave2d.variant", variant)
    sadj.set_option("wave2d.ychunk", ychunk)
    try:
        ub, upb = to_gpu(d["u_bar"]), to_gpu(d["u_prev_bar"])
        sadj.sadj_adjoint_wave2d(to_gpu(d["c"]), to_gpu(d["r_bar"]), ub, upb)
        _sync()
    finally:
        sadj.set_option("wave2d.variant", 0)
        sadj.set_option("wave2d.ychunk", 0)
    want, wantp, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, u_prev_bar=d["u_prev_bar"],
                                             want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]), np.float64, "wave2d variant %d" % variant)
    assert_close(to_host(upb), wantp, np.abs(d["u_prev_bar"]) + np.abs(d["r_bar"]), np.float64, "u_prev_bar")


def test_wave2d_nan_outside_interior_and_reproducible(sadj):
    shape = (150, 390)
    d = inputs.wave_inputs(shape, 0.01, 0.2, seed=4)
    m = interior_mask(shape, 1)
    c = np.where(m, d["c"], np.nan)
    rb = np.where(m, d["r_bar"], np.nan)
    outs = []
    for _ in range(2):
        ub = to_gpu(d["u_bar"])
        sadj.sadj_adjoint_wave2d(to_gpu(c), to_gpu(rb), ub)
        _sync()
        outs.append(to_host(ub))
    assert np.isfinite(outs[0]).all() and np.array_equal(outs[0], outs[1])
    want, _, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, want_scale=True)
    assert_close(outs[0], want, scale + np.abs(d["u_bar"]), np.float64, "wave2d NaN-poisoned")


def test_wave2d_full_size(sadj):
    """8192^2, every element, in the default (tile) form and in the strip-march form."""
    d = inputs.config_inputs("wave2d")
    want, _, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, want_scale=True)
    for variant in (0, 1):
        sadj.set_option("wave2d.variant", variant)
        try:
            ub = to_gpu(d["u_bar"])
            sadj.sadj_adjoint_wave2d(to_gpu(d["c"]), to_gpu(d["r_bar"]), ub)
            _sync()
        finally:
            sadj.set_option("wave2d.variant", 0)
        assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]), np.float64, "wave2d 8192^2 variant %d" % variant)


def test_wave2d_full_size_primal_and_both_adjoint_outputs(sadj):
    """8192^2 in the default (tile) form: the primal and the adjoint with u_prev_bar, every element."""
    d = inputs.config_inputs("wave2d")
    shape = d["c"].shape
    m = interior_mask(shape, 1)
    u_prev_bar0 = inputs.uniform(3, "u_prev_bar", shape, -1, 1)
    ub, upb = to_gpu(d["u_bar"]), to_gpu(u_prev_bar0)
    sadj.sadj_adjoint_wave2d(to_gpu(d["c"]), to_gpu(d["r_bar"]), ub, upb)
    _sync()
    want, wantp, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, u_prev_bar=u_prev_bar0, want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]), np.float64, "wave2d 8192^2 with u_prev_bar")
    assert_close(to_host(upb), wantp, np.abs(u_prev_bar0) + np.abs(d["r_bar"]), np.float64, "wave2d 8192^2 u_prev_bar")
    assert np.array_equal(to_host(upb)[~m], u_prev_bar0[~m])
    del ub, upb, want, wantp, scale
    u = inputs.uniform(4, "u", shape, -1, 1)
    u_prev = inputs.uniform(5, "u_prev", shape, -1, 1)
    r0 = inputs.uniform(6, "aux", shape, -1, 1)
    r = to_gpu(r0)
    sadj.sadj_primal_wave2d(to_gpu(u), to_gpu(u_prev), to_gpu(d["c"]), r)
    _sync()
    got = to_host(r)
    wantr = oracle.wave_primal(u, u_prev, d["c"], 1, r_init=r0)
    assert np.array_equal(got[~m], r0[~m])
    assert_close(got[m], wantr[m], wave_primal_scale(u, u_prev, d["c"], 1)[m], np.float64, "wave2d 8192^2 primal")


def test_wave2d_full_size_fp32(sadj):
    """8192^2 in fp32 (four cells per lane, 128-cell tiles), every element."""
    d = inputs.config_inputs("wave2d")
    c, rb, ub0 = (d[k].astype(np.float32) for k in ("c", "r_bar", "u_bar"))
    ub = to_gpu(ub0)
    sadj.sadj_adjoint_wave2d(to_gpu(c), to_gpu(rb), ub)
    _sync()
    want, _, scale = oracle.wave_adjoint(c, rb, ub0, 1, want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(ub0.astype(np.float64)), np.float32, "wave2d 8192^2 fp32")


# ------------------------------------------------------------------ graph capture
def test_calls_can_be_captured_in_a_hip_graph_and_replayed(sadj):
    """The entry points only enqueue kernels on the given stream (no allocation, no
    synchronisation, no memset), so a caller may record them into a HIP graph -- the way
    to run the launch-bound small sizes.  Every replay must reproduce the eager result."""
    import torch
    n, reps = 4096, 6
    d = inputs.config_inputs("wave1d")
    b = inputs.burgers_inputs(n, seed=2)
    c, rb = to_gpu(d["c"]), to_gpu(d["r_bar"])
    u, brb = to_gpu(b["u"]), to_gpu(b["r_bar"])
    shape3 = (20, 33, 64)
    w = inputs.wave_inputs(shape3, 0.01, 0.1, seed=4)
    c3, rb3 = to_gpu(w["c"]), to_gpu(w["r_bar"])

    def work(ub, bub, ub3):
        for _ in range(reps):
            sadj.sadj_adjoint_wave1d(c, rb, ub)
            sadj.sadj_adjoint_burgers1d(C, D, u, brb, bub)
        sadj.sadj_adjoint_wave3d(4, c3, rb3, ub3)

    def fresh():
        return to_gpu(d["u_bar"]), to_gpu(b["u_bar"]), to_gpu(w["u_bar"])

    eager = fresh()
    work(*eager)
    _sync()
    want = [to_host(t) for t in eager]

    static = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on the capture stream
        work(*static)
    torch.cuda.current_stream().wait_stream(side)
    _sync()
    graph = torch.cuda.CUDAGraph()
    for t, src in zip(static, fresh()):
        t.copy_(src)
    _sync()
    with torch.cuda.graph(graph):
        work(*static)
    for replay in range(3):
        for t, src in zip(static, fresh()):
            t.copy_(src)
        other = torch.ones(1000, device="cuda").sum()  # unrelated eager work between replays
        _sync()
        graph.replay()
        _sync()
        for got, ref in zip(static, want):
            assert np.array_equal(to_host(got), ref), "replay %d" % replay
        assert float(other) == 1000.0


@pytest.mark.parametrize("case", range(16))
def test_wave2d_on_drawn_shapes_and_options(sadj, case):
    rng = np.random.default_rng(700 + case)
    dtype = [np.float64, np.float32][int(rng.integers(0, 2))]
    shape = (int(rng.integers(3, 300)), int(rng.integers(3, 1200)))
    opts = {"wave2d.variant": int(rng.integers(0, 3)), "wave2d.ychunk": int(rng.choice([0, 0, 4, 9, 50]))}
    d = inputs.wave_inputs(shape, 0.01, 0.2, seed=case, dtype=dtype, c_mode="iid")
    m = interior_mask(shape, 1)
    try:
        for k, v in opts.items():
            sadj.set_option(k, v)
        ub, upb = to_gpu(d["u_bar"]), to_gpu(d["u_prev_bar"])
        sadj.sadj_adjoint_wave2d(to_gpu(np.where(m, d["c"], np.nan).astype(dtype)),
                                 to_gpu(np.where(m, d["r_bar"], np.nan).astype(dtype)), ub, upb)
        _sync()
        want_u, want_p, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, u_prev_bar=d["u_prev_bar"],
                                                    want_scale=True)
        what = "case %d %s %s %s" % (case, shape, np.dtype(dtype).name, opts)
        assert_close(to_host(ub), want_u, scale + np.abs(d["u_bar"].astype(np.float64)), dtype, what)
        assert_close(to_host(upb), want_p, np.abs(d["u_prev_bar"].astype(np.float64)) + np.abs(d["r_bar"].astype(np.float64)),
                     dtype, what + " u_prev_bar")
        r0 = inputs.uniform(case, "aux", shape, -1, 1).astype(dtype)
        r = to_gpu(r0)
        sadj.sadj_primal_wave2d(to_gpu(d["u"]), to_gpu(d["u_prev"]), to_gpu(d["c"]), r)
        _sync()
        got = to_host(r)
        want = oracle.wave_primal(d["u"], d["u_prev"], d["c"], 1, r_init=r0)
        assert np.array_equal(got[~m], r0[~m])
        assert_close(got[m], want[m], wave_primal_scale(d["u"], d["u_prev"], d["c"], 1)[m], dtype, what + " primal")
    finally:
        for k in opts:
            sadj.set_option(k, 0)


def test_wave2d_at_the_documented_plane_limit(sadj):
    """16384 x 16384 = 2^28 elements per array, the largest plane the library accepts
    (in-plane byte offsets are 32-bit): every element against the oracle."""
    shape = (16384, 16384)
    d = inputs.wave_inputs(shape, 0.01, 0.2, seed=31, c_mode="iid", fields=("c", "r_bar", "u_bar"))
    ub = to_gpu(d["u_bar"])
    sadj.sadj_adjoint_wave2d(to_gpu(d["c"]), to_gpu(d["r_bar"]), ub)
    _sync()
    want, _, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]), np.float64, "wave2d 16384^2")


def test_burgers_beyond_4_gib_per_array(sadj, path1d):
    """n = 2^29 + 3 doubles: element offsets pass 2^32 bytes in the 1-D kernels (64-bit
    indexing), with a ragged last segment; every element against the oracle."""
    n = (1 << 29) + 3
    d = inputs.burgers_inputs(n, seed=12)
    ub = to_gpu(d["u_bar"])
    sadj.sadj_adjoint_burgers1d(C, D, to_gpu(d["u"]), to_gpu(d["r_bar"]), ub)
    _sync()
    want, scale = oracle.burgers_adjoint(d["u"], d["r_bar"], d["u_bar"], C, D, want_scale=True)
    assert_close(to_host(ub), want, scale + np.abs(d["u_bar"]) + np.abs(d["r_bar"]), np.float64, "burgers n=2^29+3")
