"""GPU tests of the Burgers time loop with checkpoints (sadj_primal_burgers1d_ckpt,
sadj_adjoint_burgers1d_ckpt): the kept states and the reverse sweep's result must equal, bit for
bit, what the store-every-state calls produce from the same start, and the reverse sweep is
compared with the CPU oracle's sweep over the same states."""
import numpy as np
import pytest

import inputs
import oracle
from parity import assert_close, to_gpu, to_host

pytestmark = pytest.mark.gpu

BC, BD = 0.1, 0.05


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    return lib


def _full_history(sadj, u0, nsteps):
    """All states through the store-every-state call, boundary values held at those of u0."""
    import torch
    n = u0.shape[0]
    st = np.zeros((nsteps + 1, n), dtype=u0.dtype)
    st[0] = u0
    st[:, 0], st[:, -1] = u0[0], u0[-1]
    g = to_gpu(st)
    sadj.sadj_primal_burgers1d_steps(BC, BD, nsteps, g)
    torch.cuda.synchronize()
    return g


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n,nsteps,every", [(3, 1, 1), (64, 5, 1), (257, 7, 3), (1000, 12, 4), (1000, 12, 5),
                                            (4099, 9, 9), (4099, 9, 20), (100003, 10, 4), (515, 0, 3)])
def test_checkpointed_sweeps_equal_the_full_history_sweeps_bit_for_bit(sadj, n, nsteps, every, dtype):
    import torch
    Cd, Dd = (float(np.float32(BC)), float(np.float32(BD))) if dtype == np.float32 else (BC, BD)
    u0 = inputs.burgers_inputs(n, seed=n + every, dtype=dtype)["u"]
    full = _full_history(sadj, u0, nsteps)
    rows = nsteps // every + 1
    ck = np.full((rows, n), np.nan, dtype=dtype)
    ck[0] = u0
    ckg, work, fin = to_gpu(ck), to_gpu(np.full((2, n), np.nan, dtype=dtype)), to_gpu(np.zeros(n, dtype=dtype))
    sadj.sadj_primal_burgers1d_ckpt(BC, BD, nsteps, every, ckg, work, fin)
    torch.cuda.synchronize()
    full_h, ck_h = to_host(full), to_host(ckg)
    for j in range(rows):
        assert np.array_equal(ck_h[j], full_h[j * every]), "checkpoint %d" % j
    assert np.array_equal(to_host(fin), full_h[nsteps])

    lam0 = inputs.uniform(n, "r_bar", (n,), -1, 1).astype(dtype)
    lam1 = inputs.uniform(n, "u_bar", (n,), -1, 1).astype(dtype)
    a0, a1 = to_gpu(lam0), to_gpu(lam1)
    sadj.sadj_adjoint_burgers1d_steps(BC, BD, nsteps, nsteps, full, a0, a1)
    b0, b1 = to_gpu(lam0), to_gpu(lam1)
    wk = to_gpu(np.full(max(1, (every - 1) * n), np.nan, dtype=dtype)) if every > 1 else None
    sadj.sadj_adjoint_burgers1d_ckpt(BC, BD, nsteps, every, ckg, wk, b0, b1)
    torch.cuda.synchronize()
    res = nsteps % 2                      # the buffer that holds the result; the other holds consumed data
    assert np.array_equal(to_host((a0, a1)[res]), to_host((b0, b1)[res]))
    # and against the oracle's sweep over the same states
    w0, w1 = oracle.burgers_adjoint_steps(full_h, nsteps, nsteps, lam0, lam1, Cd, Dd)
    got, want = to_host((b0, b1)[nsteps % 2]), (w0, w1)[nsteps % 2]
    scale = np.abs(want) + np.abs(lam0.astype(np.float64)).max() * (1.5 ** nsteps)
    assert_close(got, want, scale, dtype, "checkpointed reverse sweep n=%d steps=%d every=%d" % (n, nsteps, every))


def test_checkpoint_argument_checks(sadj):
    import paper_1907_02818_amd as lib
    n = 100
    ck, work = to_gpu(np.zeros((4, n))), to_gpu(np.zeros((2, n)))
    a, b = to_gpu(np.zeros(n)), to_gpu(np.zeros(n))
    small = to_gpu(np.zeros(n))
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_ckpt(BC, BD, 9, 3, ck, small, a, b)        # work holds 1 row, 2 needed
    assert e.value.status == 2
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_ckpt(BC, BD, 9, 0, ck, small, a, b)        # every < 1
    assert e.value.status == 2
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_ckpt(BC, BD, 9, 3, ck, work, a, a)         # lam0 and lam1 overlap
    assert e.value.status == 3
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_ckpt(BC, BD, 9, 3, ck, ck[1:3], a, b)      # work inside the checkpoints
    assert e.value.status == 3
    with pytest.raises(ValueError):
        sadj.sadj_primal_burgers1d_ckpt(BC, BD, 20, 3, ck, work)               # too few checkpoint rows
