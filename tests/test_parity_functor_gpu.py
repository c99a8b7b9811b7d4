"""GPU parity of the functor hook (include/sadj_stencil1d.hpp) on a stencil that exists
nowhere in the library: tests/functor_example/sine_flux.hip defines only a functor and is
compiled against the public header alone.  Reference: the oracle's generic three-point
loop with the same body written separately in Python (tests/functor_example/sine_flux.py),
pinned in test_oracle_stencil1d.py."""
import ctypes
import os
import sys

import numpy as np
import pytest

import inputs
import oracle
from parity import assert_close, to_gpu, to_host

sys.path.insert(0, os.path.join(os.path.dirname(__file__), "functor_example"))
import sine_flux  # noqa: E402

pytestmark = pytest.mark.gpu

LIB = os.path.join(os.path.dirname(__file__), "functor_example", "libsine_flux.so")


@pytest.fixture(scope="module")
def example():
    import torch  # noqa: F401  (torch's HIP runtime must be the one in the process)
    assert os.path.exists(LIB), "build tests/functor_example/libsine_flux.so first (__graft_entry__.build())"
    lib = ctypes.CDLL(LIB)
    for fn in (lib.sine_flux_primal, lib.sine_flux_adjoint):
        fn.restype = ctypes.c_int
    return lib


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _p(t):
    return ctypes.c_void_p(t.data_ptr())


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n", [3, 4, 5, 63, 64, 65, 127, 128, 129, 130, 255, 256, 257, 258, 259, 511, 1000, 4097, 30011])
def test_sine_flux_adjoint_and_primal(example, n, dtype):
    import torch
    u = inputs.uniform(n, "u", (n,), -1.5, 1.5).astype(dtype)
    p = inputs.uniform(n, "c", (n,), 0.2, 1.5).astype(dtype)
    rb = inputs.uniform(n, "r_bar", (n,), -1, 1).astype(dtype)
    ub = inputs.uniform(n, "u_bar", (n,), -1, 1).astype(dtype)
    rb_poison = rb.copy()
    rb_poison[0] = rb_poison[-1] = np.nan            # outside I: must not be used
    f64 = int(dtype == np.float64)
    ug, pg, rg, bg = to_gpu(u), to_gpu(p), to_gpu(rb_poison), to_gpu(ub)
    rc = example.sine_flux_adjoint(f64, ctypes.c_long(n), _p(ug), _p(pg), _p(rg), _p(bg), _stream())
    assert rc == 0
    torch.cuda.synchronize()
    want, scale = oracle.stencil1d_adjoint(sine_flux.df, u, p, rb, ub, want_scale=True)
    assert_close(to_host(bg), want, scale + np.abs(ub.astype(np.float64)), dtype, "sine-flux adjoint n=%d" % n)
    r0 = inputs.uniform(n, "aux", (n,), -1, 1).astype(dtype)
    r = to_gpu(r0)
    rc = example.sine_flux_primal(f64, ctypes.c_long(n), _p(ug), _p(pg), _p(r), _stream())
    assert rc == 0
    torch.cuda.synchronize()
    got = to_host(r)
    wantr = oracle.stencil1d_primal(sine_flux.f, u, p, r_init=r0)
    assert got[0] == r0[0] and got[-1] == r0[-1]
    assert_close(got, wantr, np.abs(wantr) + 3.0, dtype, "sine-flux primal n=%d" % n)


def test_unaligned_arrays_take_the_scalar_shape_and_runs_repeat_bit_for_bit(example):
    import torch
    n = 5003
    u = inputs.uniform(1, "u", (n,), -1.5, 1.5)
    p = inputs.uniform(1, "c", (n,), 0.2, 1.5)
    rb = inputs.uniform(1, "r_bar", (n,), -1, 1)
    ub = inputs.uniform(1, "u_bar", (n,), -1, 1)

    def shifted(a):
        t = torch.empty(n + 1, dtype=torch.float64, device="cuda")
        t[1:].copy_(torch.from_numpy(a))
        return t[1:]

    outs = []
    for mk in (shifted, to_gpu, to_gpu):
        ug, pg, rg, bg = mk(u), mk(p), mk(rb), mk(ub)
        assert example.sine_flux_adjoint(1, ctypes.c_long(n), _p(ug), _p(pg), _p(rg), _p(bg), _stream()) == 0
        torch.cuda.synchronize()
        outs.append(to_host(bg))
    want, scale = oracle.stencil1d_adjoint(sine_flux.df, u, p, rb, ub, want_scale=True)
    assert_close(outs[0], want, scale + np.abs(ub), np.float64, "unaligned")
    assert np.array_equal(outs[1], outs[2])


def test_bad_arguments_are_refused(example):
    import torch
    t = torch.zeros(8, dtype=torch.float64, device="cuda")
    o = torch.zeros(8, dtype=torch.float64, device="cuda")
    assert example.sine_flux_adjoint(1, ctypes.c_long(2), _p(t), _p(t), _p(t), _p(o), _stream()) != 0
    assert example.sine_flux_adjoint(1, ctypes.c_long(8), _p(t), ctypes.c_void_p(0), _p(t), _p(o), _stream()) != 0
    torch.cuda.synchronize()
    assert float(o.abs().sum()) == 0.0
