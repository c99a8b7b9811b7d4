"""GPU parity of the functor hook in two and three dimensions (include/sadj_stencil_star.hpp)
on stencils that exist nowhere in the library: tests/functor_example/star_bodies.hip defines
only functors and is compiled against the public header alone.  Reference: the oracle's generic
star-shaped loop with the same bodies written separately in Python
(tests/functor_example/star_bodies.py), pinned in test_oracle_starfn.py; for the linear wave
body at full size, the wave oracle itself."""
import ctypes
import os
import sys

import numpy as np
import pytest

import inputs
import oracle
from parity import assert_close, to_gpu, to_host

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "functor_example"))
import star_bodies  # noqa: E402

pytestmark = pytest.mark.gpu

LIB = os.path.join(os.path.dirname(__file__), "functor_example", "libstar_bodies.so")
SOFT, PAIR, LIN = 0, 1, 2
BODIES = {SOFT: (star_bodies.soft_wave_f, star_bodies.soft_wave_df),
          PAIR: (star_bodies.pair_product_f, star_bodies.pair_product_df),
          LIN: star_bodies.lin_wave([-2.0, 1.0])}


@pytest.fixture(scope="module")
def example():
    import torch  # noqa: F401  (torch's HIP runtime must be the one in the process)
    assert os.path.exists(LIB), "build tests/functor_example/libstar_bodies.so first (__graft_entry__.build())"
    lib = ctypes.CDLL(LIB)
    lib.star_example.restype = ctypes.c_int
    return lib


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _p(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _call(lib, kind, adjoint, dtype, shape, u, p, rb, out):
    dims = list(shape[::-1]) + [1] * (3 - len(shape))
    return lib.star_example(kind, adjoint, int(dtype == np.float64), len(shape), dims[0], dims[1], dims[2],
                            _p(u), _p(p), _p(rb), _p(out), _stream())


def _fields(shape, seed, dtype):
    mk = lambda name, lo, hi: inputs.uniform(seed, name, shape, lo, hi).astype(dtype)
    return mk("u", -1, 1), mk("c", 0.02, 0.2), mk("r_bar", -1, 1), mk("u_bar", -1, 1)


def _outside_I(shape):
    m = np.ones(shape, dtype=bool)
    m[tuple(slice(1, -1) for _ in shape)] = False
    return m


# nx must be a multiple of 16 bytes' worth of elements (4 covers both dtypes); tiles are 64 (128) x 32:
# shapes below cover a single ragged tile, several tiles with ragged last ones, extents of 3 and 4
# (every cell in the remainder), and z extents shorter and longer than a chunk
SHAPES_2D = [(3, 4), (4, 8), (33, 68), (32, 128), (70, 260), (5, 1000)]
SHAPES_3D = [(3, 3, 4), (4, 5, 8), (7, 33, 68), (40, 34, 132), (19, 70, 72), (64, 32, 128)]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("kind,shape", [(SOFT, s) for s in SHAPES_2D + SHAPES_3D] + [(PAIR, s) for s in SHAPES_2D] +
                         [(LIN, s) for s in SHAPES_2D[2:4] + SHAPES_3D[2:4]])
def test_adjoint_and_primal_against_the_callback_oracle(example, kind, shape, dtype):
    import torch
    u, p, rb, ub = _fields(shape, 31 + len(shape), dtype)
    out_I = _outside_I(shape)
    rb_poison, p_poison = rb.copy(), p.copy()
    rb_poison[out_I] = np.nan                      # outside I: must never be used
    p_poison[out_I] = np.nan
    f, df = BODIES[kind]
    ug, pg, rg, bg = to_gpu(u), to_gpu(p_poison), to_gpu(rb_poison), to_gpu(ub)
    assert _call(example, kind, 1, dtype, shape, None if kind == LIN else ug, pg, rg, bg) == 0
    torch.cuda.synchronize()
    want, scale = oracle.starfn_adjoint(df, u, p, rb, ub, 1, want_scale=True)
    assert_close(to_host(bg), want, scale + np.abs(ub.astype(np.float64)), dtype, "adjoint kind %d %s" % (kind, shape))
    r0 = inputs.uniform(7, "aux", shape, -1, 1).astype(dtype)
    r = to_gpu(r0)
    assert _call(example, kind, 0, dtype, shape, ug, pg, None, r) == 0
    torch.cuda.synchronize()
    got = to_host(r)
    wantr = oracle.starfn_primal(f, u, p, 1, r_init=r0)
    assert np.array_equal(got[out_I], r0[out_I]), "primal wrote outside I"
    assert_close(got, wantr, np.abs(wantr) + 3.0, dtype, "primal kind %d %s" % (kind, shape))


def test_runs_repeat_bit_for_bit(example):
    import torch
    shape = (21, 70, 132)
    u, p, rb, ub = _fields(shape, 3, np.float64)
    outs = []
    for _ in range(2):
        ug, pg, rg, bg = to_gpu(u), to_gpu(p), to_gpu(rb), to_gpu(ub)
        assert _call(example, SOFT, 1, np.float64, shape, ug, pg, rg, bg) == 0
        torch.cuda.synchronize()
        outs.append(to_host(bg))
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_linear_wave_body_at_full_size_equals_the_wave_oracle(example, dtype):
    """512^3 through the functor kernels, every element against the wave oracle (u_bar part)."""
    import torch
    shape = (512, 512, 512)
    d = inputs.config_inputs("wave3d_r1", shape=shape, dtype=dtype, fields=("c", "r_bar", "u_bar"))
    cg, rg, bg = to_gpu(d["c"]), to_gpu(d["r_bar"]), to_gpu(d["u_bar"])
    assert _call(example, LIN, 1, dtype, shape, None, cg, rg, bg) == 0
    torch.cuda.synchronize()
    want, _, scale = oracle.wave_adjoint(d["c"], d["r_bar"], d["u_bar"], 1, want_scale=True)
    assert_close(to_host(bg), want, scale + np.abs(d["u_bar"].astype(np.float64)), dtype, "linear wave body 512^3")


def test_nonlinear_body_at_full_size_on_sampled_outputs(example):
    """soft_wave at 512^3: u_bar[j] recomputed for sampled j from the definition (the terms of the
    seven iterations that read u[j]), in the corners, on faces and in the interior."""
    import torch
    shape = (512, 512, 512)
    n = 512
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    ug = torch.rand(shape, generator=g, device="cuda", dtype=torch.float64) * 2 - 1
    pg = torch.rand(shape, generator=g, device="cuda", dtype=torch.float64) * 0.2 + 0.02
    rg = torch.rand(shape, generator=g, device="cuda", dtype=torch.float64) * 2 - 1
    b0 = torch.rand(shape, generator=g, device="cuda", dtype=torch.float64) * 2 - 1
    bg = b0.clone()
    assert _call(example, SOFT, 1, np.float64, shape, ug, pg, rg, bg) == 0
    torch.cuda.synchronize()
    u, p, rb = ug.cpu().numpy(), pg.cpu().numpy(), rg.cpu().numpy()
    rng = np.random.default_rng(1)
    pts = [tuple(rng.integers(0, n, 3)) for _ in range(300)]
    pts += [(0, 0, 0), (n - 1, n - 1, n - 1), (0, 5, 7), (1, 1, 1), (n - 2, 64, 63), (255, 0, 31), (31, 32, 64), (256, 31, 63)]
    offs = [(0, 0, 0), (0, 0, -1), (0, 0, 1), (0, -1, 0), (0, 1, 0), (-1, 0, 0), (1, 0, 0)]      # (dz, dy, dx) of read k
    got = bg.cpu().numpy()
    base = b0.cpu().numpy()
    for (z, y, x) in pts:
        want, mag = base[z, y, x], abs(base[z, y, x])
        for k, (dz, dy, dx) in enumerate(offs):
            iz, iy, ix = z - dz, y - dy, x - dx                     # the iteration whose read k is cell j
            if not (1 <= iz <= n - 2 and 1 <= iy <= n - 2 and 1 <= ix <= n - 2):
                continue
            v = [u[iz + a, iy + b, ix + c] for (a, b, c) in offs]
            t = star_bodies.soft_wave_df(v, p[iz, iy, ix])[k] * rb[iz, iy, ix]
            want += t
            mag += abs(t)
        assert abs(got[z, y, x] - want) <= 1e-12 * max(mag, abs(want)), (z, y, x)


def test_bad_arguments_are_refused(example):
    import torch
    t = torch.zeros((8, 8, 8), dtype=torch.float64, device="cuda")
    o = torch.zeros((8, 8, 8), dtype=torch.float64, device="cuda")
    assert _call(example, SOFT, 1, np.float64, (8, 8, 2), t, t, t, o) != 0          # nx = 2 < 3
    assert _call(example, SOFT, 1, np.float64, (8, 8, 7), t, t, t, o) != 0          # nx not a multiple of 2
    assert _call(example, SOFT, 1, np.float64, (8, 8, 8), t, None, t, o) != 0       # passive array missing
    torch.cuda.synchronize()
    assert float(o.abs().sum()) == 0.0
