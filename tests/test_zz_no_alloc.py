"""The entry point that allocates nothing (sadj_adjoint_burgers1d_ckpt_static: the checkpointed
Burgers reverse sweep with its scratch in a fixed device array of the library) against the
entry point that takes a workspace argument, through the C ABI: two calls in a row, the second
with a smaller input, results bit for bit; and the size limit."""
import numpy as np
import pytest

import inputs
from parity import to_gpu, to_host

pytestmark = pytest.mark.gpu

BC, BD = 0.1, 0.05


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    return lib


def _case(sadj, n, nsteps, every, dtype):
    import torch
    u0 = inputs.burgers_inputs(n, seed=n, dtype=dtype)["u"]
    rows = nsteps // every + 1
    ck = np.zeros((rows, n), dtype=dtype)
    ck[0] = u0
    ckg, work2 = to_gpu(ck), to_gpu(np.zeros((2, n), dtype=dtype))
    sadj.sadj_primal_burgers1d_ckpt(BC, BD, nsteps, every, ckg, work2)
    lam0 = inputs.uniform(n, "r_bar", (n,), -1, 1).astype(dtype)
    lam1 = inputs.uniform(n, "u_bar", (n,), -1, 1).astype(dtype)
    a0, a1 = to_gpu(lam0), to_gpu(lam1)
    wk = to_gpu(np.full(max(1, (every - 1) * n), np.nan, dtype=dtype))
    sadj.sadj_adjoint_burgers1d_ckpt(BC, BD, nsteps, every, ckg, wk, a0, a1)
    b0, b1 = to_gpu(lam0), to_gpu(lam1)
    sadj.sadj_adjoint_burgers1d_ckpt_static(BC, BD, nsteps, every, ckg, b0, b1)
    torch.cuda.synchronize()
    assert np.isfinite(to_host(b0)).all() and np.isfinite(to_host(b1)).all()
    assert np.array_equal(to_host(a0), to_host(b0)) and np.array_equal(to_host(a1), to_host(b1))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_two_calls_in_a_row_the_second_smaller(sadj, dtype):
    _case(sadj, 200003, 11, 4, dtype)
    _case(sadj, 4099, 7, 3, dtype)
    _case(sadj, 64, 5, 5, dtype)


def test_sizes_beyond_the_fixed_scratch_are_refused(sadj):
    import paper_1907_02818_amd as lib
    limit = sadj.sadj_static_scratch_bytes()
    assert limit == 64 << 20
    n = 1 << 20
    every = limit // (8 * n) + 2                         # (every-1)*n*8 bytes > limit
    ck = to_gpu(np.zeros((2, n)))
    a, b = to_gpu(np.zeros(n)), to_gpu(np.ones(n))
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_ckpt_static(BC, BD, every, every, ck, a, b)
    assert e.value.status == 2
    assert float(to_host(a).sum()) == 0.0 and float(to_host(b).sum()) == n      # nothing was enqueued
    # the largest size that fits is accepted
    every = limit // (8 * n) + 1
    sadj.sadj_adjoint_burgers1d_ckpt_static(BC, BD, 1, every, ck, a, b)
