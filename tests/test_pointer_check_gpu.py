"""The optional pointer check (sadj_check_array, option "check.pointers") against real
allocations.  Only queries are made with bad arguments; every launch here has valid ones."""
import numpy as np
import pytest

import inputs
from parity import to_gpu, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    yield lib
    lib.set_option("check.pointers", 0)


def test_check_array_on_device_pinned_and_pageable_memory(sadj):
    import torch
    t = torch.zeros(1 << 20, dtype=torch.float64, device="cuda")
    assert sadj.sadj_check_array(t.data_ptr(), t.numel() * 8) == 0
    assert sadj.sadj_check_array(t.data_ptr() + 800, t.numel() * 8 - 800) == 0      # a view into it
    assert sadj.sadj_check_array(t.data_ptr(), 1 << 42) == 2                         # past any allocation
    pinned = torch.zeros(4096, dtype=torch.float64, pin_memory=True)
    assert sadj.sadj_check_array(pinned.data_ptr(), pinned.numel() * 8) == 0
    host = np.zeros(4096)
    assert sadj.sadj_check_array(host.ctypes.data, host.nbytes) == 5
    assert sadj.sadj_check_array(0, 8) == 1


def test_range_past_the_end_of_its_own_allocation(sadj):
    """A 64 MiB tensor gets an allocation of its own from torch's allocator (requests above
    10 MiB are not carved out of a shared block), so one element more does not fit."""
    import torch
    torch.cuda.empty_cache()                 # so that the request is served by a fresh allocation, not a cached larger block
    nbytes = 64 << 20
    t = torch.empty(nbytes // 8, dtype=torch.float64, device="cuda")
    assert sadj.sadj_check_array(t.data_ptr(), nbytes) == 0
    if sadj.sadj_check_array(t.data_ptr(), nbytes + 8) == 0:
        pytest.skip("this allocator configuration backs the tensor with a larger allocation")
    assert sadj.sadj_check_array(t.data_ptr(), nbytes + 8) == 2
    assert sadj.sadj_check_array(t.data_ptr() + 8, nbytes) == 2
    assert sadj.sadj_check_array(t.data_ptr() + 8, nbytes - 8) == 0


def test_results_do_not_depend_on_the_check(sadj):
    import torch
    shape = (20, 33, 70)
    d = inputs.wave_inputs(shape, 0.01, 0.1, seed=5, dtype=np.float64, c_mode="iid")
    out = []
    for on in (0, 1):
        sadj.set_option("check.pointers", on)
        ub, up = to_gpu(d["u_bar"]), to_gpu(d["u_prev_bar"])
        sadj.sadj_adjoint_wave3d(4, to_gpu(d["c"]), to_gpu(d["r_bar"]), ub, up)
        torch.cuda.synchronize()
        out.append((to_host(ub), to_host(up)))
    sadj.set_option("check.pointers", 0)
    assert np.array_equal(out[0][0], out[1][0]) and np.array_equal(out[0][1], out[1][1])


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n", [1, 2, 3, 5, 255, 256, 257, 1024, 4099, 1 << 20, (1 << 20) + 3])
@pytest.mark.parametrize("shape", [0, 1, 2])
def test_stream_probe_computes_out_plus_a_times_b(n, dtype, shape):
    """The streaming yardstick of the benchmark is a kernel like any other: out[i] += a[i]*b[i],
    every launch shape, sizes around the vector width and the workgroup's piece, ragged tails."""
    import torch
    import paper_1907_02818_amd as sadj
    from parity import to_gpu, to_host
    sadj.load()
    rng = np.random.default_rng(n)
    a, b, o = (rng.uniform(-1, 1, n).astype(dtype) for _ in range(3))
    og = to_gpu(o)
    sadj.sadj_stream_probe(shape, to_gpu(a), to_gpu(b), og)
    torch.cuda.synchronize()
    want = o.astype(np.float64) + a.astype(np.float64) * b.astype(np.float64)
    tol = 1e-15 if dtype == np.float64 else 1e-6
    assert np.max(np.abs(to_host(og) - want)) <= tol * 3.0
