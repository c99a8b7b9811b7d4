"""GPU parity of sadj_adjoint_wave3d_steps (reverse sweep of a time loop of wave
steps) against the CPU oracle."""
import numpy as np
import pytest

import inputs
import oracle
from parity import TOL, assert_close, to_gpu, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sadj():
    import paper_1907_02818_amd as lib
    lib.load()
    return lib


def _lams(shape, seed, dtype):
    return [inputs.uniform(seed, name, shape, -1, 1).astype(dtype) for name in ("r_bar", "u_bar", "u_prev_bar")]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("radius,shape,nsteps", [(4, (37, 45, 150), 1), (4, (37, 45, 150), 2), (4, (37, 45, 150), 6),
                                                 (4, (12, 33, 131), 4), (1, (21, 37, 150), 5), (1, (3, 3, 3), 4),
                                                 (4, (9, 9, 9), 3), (4, (40, 70, 64), 0), (2, (20, 33, 70), 3),
                                                 (3, (15, 20, 66), 4),
                                                 (1, (9, 20, 250), 3), (4, (14, 20, 250), 3)])     # rows not line multiples: wide tiles
def test_steps_match_the_oracle(sadj, radius, shape, nsteps, dtype):
    """Element by element, step by step: the oracle's one-step scatter adjoint is applied to the
    GPU's own buffers after s steps and compared with the GPU's buffers after s+1 steps, each
    element against the magnitude of what was summed into it in that step.  The whole sweep
    is compared with the oracle's sweep as well."""
    import torch
    c = inputs.uniform(1, "c", shape, 0.01, 0.1).astype(dtype)
    lams = _lams(shape, 2 + nsteps, dtype)
    cg = to_gpu(c)

    def after(steps):
        g = [to_gpu(x) for x in lams]
        sadj.sadj_adjoint_wave3d_steps(radius, steps, cg, *g)
        torch.cuda.synchronize()
        return [to_host(t) for t in g]

    state = after(0)
    assert all(np.array_equal(x, y) for x, y in zip(state, lams))
    for s_ in range(nsteps):
        nxt = after(s_ + 1)
        a, b, p = state[s_ % 3], state[(s_ + 1) % 3], state[(s_ + 2) % 3]
        p_in = p if s_ == 0 else np.zeros_like(p)          # from the second step on the buffer is assigned
        wb, wp, scale = oracle.wave_adjoint(c, a, b, radius, u_prev_bar=p_in, want_scale=True)
        assert_close(nxt[(s_ + 1) % 3], wb, scale + np.abs(b.astype(np.float64)), dtype, "lam_b after step %d" % (s_ + 1))
        assert_close(nxt[(s_ + 2) % 3], wp, np.abs(p_in.astype(np.float64)) + np.abs(a.astype(np.float64)), dtype,
                     "lam_p after step %d" % (s_ + 1))
        state = nxt
    want = oracle.wave_adjoint_steps(c, *lams, radius, nsteps)
    live = [nsteps % 3, (nsteps + 1) % 3] if nsteps > 0 else [0, 1, 2]
    tol = TOL[np.dtype(dtype)]
    for k in live:
        got = state[k].astype(np.float64)
        assert np.isfinite(got).all()
        err = np.max(np.abs(got - want[k])) / max(np.max(np.abs(want[k])), 1e-300)
        assert err <= tol * max(1, nsteps), "buffer %d after %d steps: %.3e" % (k, nsteps, err)


def test_steps_equal_repeated_single_calls_bitwise(sadj):
    """The sweep is nothing but the single-step kernel with rotating buffers (the
    recycled buffer zeroed by the assign mode instead of by the caller)."""
    import torch
    radius, shape, nsteps = 4, (30, 40, 140), 4
    c = to_gpu(inputs.uniform(1, "c", shape, 0.01, 0.1))
    lams = _lams(shape, 5, np.float64)
    g = [to_gpu(x) for x in lams]
    sadj.sadj_adjoint_wave3d_steps(radius, nsteps, c, *g)
    h = [to_gpu(x) for x in lams]
    for s in range(nsteps):
        a, b, p = h[s % 3], h[(s + 1) % 3], h[(s + 2) % 3]
        if s > 0:
            p.zero_()
        sadj.sadj_adjoint_wave3d(radius, c, a, b, p)
    torch.cuda.synchronize()
    for k in (nsteps % 3, (nsteps + 1) % 3):
        assert np.array_equal(to_host(g[k]), to_host(h[k]))


def test_steps_argument_errors(sadj):
    import torch
    t = [torch.zeros(16, 16, 16, dtype=torch.float64, device="cuda") for _ in range(4)]
    with pytest.raises(sadj.SadjError) as e:
        sadj.sadj_adjoint_wave3d_steps(1, 2, t[0], t[1], t[1], t[3])
    assert e.value.status == 3
    with pytest.raises(sadj.SadjError) as e:
        sadj.sadj_adjoint_wave3d_steps(1, -1, *t)
    assert e.value.status == 2
    with pytest.raises(sadj.SadjError) as e:
        sadj.sadj_adjoint_wave3d_steps(5, 1, *t)
    assert e.value.status == 4


# ----------------------------------------------------------- Burgers time loop (stored states)
BC, BD = 0.1, 0.05


def _burgers_states(n, nsteps, seed, dtype):
    st = np.empty((nsteps + 1, n), dtype=dtype)
    st[0] = inputs.burgers_inputs(n, seed=seed, dtype=dtype)["u"]
    for t in range(1, nsteps + 1):
        st[t] = inputs.uniform(seed + t, "u_prev", (n,), -0.5, 0.5).astype(dtype)
    return st


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n,nsteps", [(3, 2), (64, 1), (257, 5), (1000, 4), (100003, 6)])
def test_burgers_forward_and_reverse_sweeps(sadj, n, nsteps, dtype):
    import torch
    Cd, Dd = (float(np.float32(BC)), float(np.float32(BD))) if dtype == np.float32 else (BC, BD)
    st0 = _burgers_states(n, nsteps, n, dtype)
    stg = to_gpu(st0)
    sadj.sadj_primal_burgers1d_steps(BC, BD, nsteps, stg)
    torch.cuda.synchronize()
    got_st = to_host(stg)
    want_st = oracle.burgers_primal_steps(st0, nsteps, Cd, Dd)
    assert np.array_equal(got_st[:, 0], st0[:, 0]) and np.array_equal(got_st[:, -1], st0[:, -1])
    assert_close(got_st, want_st, np.abs(want_st) + 1.0, dtype, "burgers forward sweep n=%d steps=%d" % (n, nsteps))
    # reverse sweep over the GPU's own stored states (what a solver would do); the oracle
    # sweeps over the same states, so differences are those of the adjoint steps alone
    lam0 = inputs.uniform(n, "r_bar", (n,), -1, 1).astype(dtype)
    lam1 = inputs.uniform(n, "u_bar", (n,), -1, 1).astype(dtype)
    lam0_p = lam0.copy(); lam0_p[0] = lam0_p[-1] = np.nan            # outside I: never used
    g0, g1 = to_gpu(lam0_p), to_gpu(lam1)
    sadj.sadj_adjoint_burgers1d_steps(BC, BD, nsteps, nsteps, stg, g0, g1)
    torch.cuda.synchronize()
    w0, w1 = oracle.burgers_adjoint_steps(got_st, nsteps, nsteps, lam0, lam1, Cd, Dd)
    got = to_host((g0, g1)[nsteps % 2])
    want = (w0, w1)[nsteps % 2]
    scale = np.abs(want) + np.abs(lam0.astype(np.float64)).max() * (1.5 ** nsteps)
    assert_close(got, want, scale, dtype, "burgers reverse sweep n=%d steps=%d" % (n, nsteps))


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
@pytest.mark.parametrize("n", [3, 17, 64, 239, 240, 241, 257, 495, 496, 497, 1000, 4099, 100003])
@pytest.mark.parametrize("nsteps", [6, 11, 17])
def test_fused_reverse_steps_equal_single_steps_bit_for_bit(sadj, n, nsteps, dtype):
    """Runs of five assigned steps go through one kernel that keeps a window of cells in
    registers (option burgers1d.fuse = 0, the default); the step-by-step sweep is the reference.
    Sizes around the window widths (240 / 496 finished cells per wave) and the clamped ends."""
    import torch
    st = to_gpu(_burgers_states(n, nsteps, 3 * n + nsteps, dtype))
    lam0 = inputs.uniform(n, "r_bar", (n,), -1, 1).astype(dtype)
    lam1 = inputs.uniform(n, "u_bar", (n,), -1, 1).astype(dtype)
    lam0[0] = lam0[-1] = np.nan                                        # outside I: never used
    out = []
    for fuse in (1, 0):
        sadj.set_option("burgers1d.fuse", fuse)
        g0, g1 = to_gpu(lam0), to_gpu(lam1)
        sadj.sadj_adjoint_burgers1d_steps(BC, BD, nsteps, nsteps, st, g0, g1)
        torch.cuda.synchronize()
        out.append(to_host((g0, g1)[nsteps % 2]))
    sadj.set_option("burgers1d.fuse", 0)
    assert np.isfinite(out[0]).all()
    assert np.array_equal(out[0], out[1])


def test_fused_reverse_steps_with_unaligned_rows_fall_back(sadj):
    """Rows of an odd length start at addresses that are not 16-byte aligned: those steps run
    one by one; the result is unchanged."""
    import torch
    n, nsteps = 1001, 12
    st = to_gpu(_burgers_states(n, nsteps, 5, np.float64))
    lam0 = inputs.uniform(n, "r_bar", (n,), -1, 1)
    lam1 = inputs.uniform(n, "u_bar", (n,), -1, 1)
    out = []
    for fuse in (1, 0):
        sadj.set_option("burgers1d.fuse", fuse)
        g0, g1 = to_gpu(lam0), to_gpu(lam1)
        sadj.sadj_adjoint_burgers1d_steps(BC, BD, nsteps, nsteps, st, g0, g1)
        torch.cuda.synchronize()
        out.append(to_host((g0, g1)[nsteps % 2]))
    sadj.set_option("burgers1d.fuse", 0)
    assert np.array_equal(out[0], out[1])


def test_burgers_sweep_argument_checks(sadj):
    import paper_1907_02818_amd as lib
    st = to_gpu(np.zeros((4, 100)))
    a, b = to_gpu(np.zeros(100)), to_gpu(np.zeros(100))
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_steps(BC, BD, 3, 4, st, a, b)      # more steps than states
    assert e.value.status == 2
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_steps(BC, BD, 3, 2, st, a, a)      # lam0 and lam1 overlap
    assert e.value.status == 3
    with pytest.raises(lib.SadjError) as e:
        sadj.sadj_adjoint_burgers1d_steps(BC, BD, 3, 2, st, st[1], b)  # lam0 inside the rows read
    assert e.value.status == 3
