"""ctypes front end of the CPU oracle (sadj_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.

Every function takes and returns NumPy float64 arrays in C order with the slowest
axis first (shape (nz,ny,nx), (ny,nx) or (n,)); float32 inputs are widened to
double first, which is how the fp32 workloads are checked: same rounded inputs,
fp64 arithmetic.  See sadj_oracle.c for what each routine computes and which
passage of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sadj_oracle.c")
_LIB = os.path.join(_HERE, "libsadj_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no fast-math, no OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


_P = ctypes.c_void_p
_L = ctypes.c_long
_I = ctypes.c_int
_D = ctypes.c_double


def _f64(a, writable=False):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if writable and not a.flags.writeable:
        a = a.copy()
    return a


def _ptr(a):
    return _P(a.ctypes.data) if a is not None else _P(0)


def _dims(shape):
    shape = tuple(int(s) for s in shape)
    ndim = len(shape)
    if ndim == 1:
        return ndim, shape[0], 1, 1
    if ndim == 2:
        return ndim, shape[1], shape[0], 1
    if ndim == 3:
        return ndim, shape[2], shape[1], shape[0]
    raise ValueError("1-, 2- or 3-D grids only")


def _check(rc, what):
    if rc != 0:
        raise ValueError("oracle %s: bad argument (rc=%d)" % (what, rc))


def star_weights(radius: int) -> np.ndarray:
    w = np.zeros(5)
    _check(_load().oracle_star_weights(_I(radius), _ptr(w)), "star_weights")
    return w[: radius + 1].copy()


def wave_primal(u, u_prev, c, radius: int, r_init=None) -> np.ndarray:
    """r = 2u - u_prev + c*Lap_w(u) on the primal interior; elsewhere r keeps r_init
    (zeros if not given)."""
    u, u_prev, c = _f64(u), _f64(u_prev), _f64(c)
    ndim, nx, ny, nz = _dims(u.shape)
    r = np.zeros_like(u) if r_init is None else _f64(r_init).copy()
    fn = _load().oracle_wave_primal
    _check(fn(_I(ndim), _I(radius), _L(nx), _L(ny), _L(nz), _ptr(u), _ptr(u_prev), _ptr(c), _ptr(r)),
           "wave_primal")
    return r


def wave_tangent(c, u_dot, u_prev_dot, radius: int) -> np.ndarray:
    c, u_dot, u_prev_dot = _f64(c), _f64(u_dot), _f64(u_prev_dot)
    ndim, nx, ny, nz = _dims(c.shape)
    r_dot = np.zeros_like(c)
    fn = _load().oracle_wave_tangent
    _check(fn(_I(ndim), _I(radius), _L(nx), _L(ny), _L(nz), _ptr(c), _ptr(u_dot), _ptr(u_prev_dot),
              _ptr(r_dot)), "wave_tangent")
    return r_dot


def wave_adjoint(c, r_bar, u_bar, radius: int, u_prev_bar=None, want_scale: bool = False):
    """Returns (u_bar_out, u_prev_bar_out or None, scale or None).  The inputs are
    not modified.  scale[j] = sum of |contribution| that reached index j."""
    c, r_bar = _f64(c), _f64(r_bar)
    ndim, nx, ny, nz = _dims(c.shape)
    ub = _f64(u_bar).copy()
    upb = _f64(u_prev_bar).copy() if u_prev_bar is not None else None
    scale = np.zeros_like(ub) if want_scale else None
    fn = _load().oracle_wave_adjoint
    _check(fn(_I(ndim), _I(radius), _L(nx), _L(ny), _L(nz), _ptr(c), _ptr(r_bar), _ptr(ub),
              _ptr(upb), _ptr(scale)), "wave_adjoint")
    return ub, upb, scale


def wave_adjoint_steps(c, lam0, lam1, lam2, radius: int, nsteps: int):
    """Reverse sweep of `nsteps` wave steps with three rotating buffers; returns the three
    buffers (copies) after the sweep, in the caller's order."""
    c = _f64(c)
    ndim, nx, ny, nz = _dims(c.shape)
    bufs = [_f64(x).copy() for x in (lam0, lam1, lam2)]
    fn = _load().oracle_wave_adjoint_steps
    _check(fn(_I(ndim), _I(radius), _L(nx), _L(ny), _L(nz), _L(nsteps), _ptr(c), _ptr(bufs[0]), _ptr(bufs[1]),
              _ptr(bufs[2])), "wave_adjoint_steps")
    return bufs


def _box_weights(w, ndim):
    """Weights as an array of shape (3,)*ndim indexed [oz+1][oy+1][ox+1] -> flat table of 27
    entries indexed (ox+1) + 3(oy+1) + 9(oz+1), zero where an axis is unused."""
    w = np.asarray(w, dtype=np.float64)
    assert w.shape == (3,) * ndim
    full = np.zeros((3, 3, 3))
    if ndim == 1:
        full[1, 1, :] = w
    elif ndim == 2:
        full[1, :, :] = w
    else:
        full[:] = w
    return np.ascontiguousarray(full.ravel())


def box_primal(w, u, c, r_init=None) -> np.ndarray:
    u, c = _f64(u), _f64(c)
    ndim, nx, ny, nz = _dims(u.shape)
    wt = _box_weights(w, ndim)
    r = np.zeros_like(u) if r_init is None else _f64(r_init).copy()
    _check(_load().oracle_box_primal(_I(ndim), _L(nx), _L(ny), _L(nz), _ptr(wt), _ptr(u), _ptr(c), _ptr(r)),
           "box_primal")
    return r


def box_adjoint(w, c, r_bar, u_bar, want_scale: bool = False):
    c, r_bar = _f64(c), _f64(r_bar)
    ndim, nx, ny, nz = _dims(c.shape)
    wt = _box_weights(w, ndim)
    ub = _f64(u_bar).copy()
    scale = np.zeros_like(ub) if want_scale else None
    _check(_load().oracle_box_adjoint(_I(ndim), _L(nx), _L(ny), _L(nz), _ptr(wt), _ptr(c), _ptr(r_bar), _ptr(ub),
                                      _ptr(scale)), "box_adjoint")
    return ub, scale


def star3d_primal(w, u, c, radius: int, r_init=None) -> np.ndarray:
    """w: 1 + 6*radius values: centre, then per axis x, y, z the offsets -R..-1, +1..+R."""
    u, c = _f64(u), _f64(c)
    w = _f64(np.asarray(w, dtype=np.float64).ravel())
    assert u.ndim == 3 and w.size == 1 + 6 * radius
    nz, ny, nx = u.shape
    r = np.zeros_like(u) if r_init is None else _f64(r_init).copy()
    _check(_load().oracle_star3d_primal(_I(radius), _L(nx), _L(ny), _L(nz), _ptr(w), _ptr(u), _ptr(c), _ptr(r)),
           "star3d_primal")
    return r


def star3d_adjoint(w, c, r_bar, u_bar, radius: int, want_scale: bool = False):
    """Returns (u_bar_out, scale or None)."""
    c, r_bar = _f64(c), _f64(r_bar)
    w = _f64(np.asarray(w, dtype=np.float64).ravel())
    assert c.ndim == 3 and w.size == 1 + 6 * radius
    nz, ny, nx = c.shape
    ub = _f64(u_bar).copy()
    scale = np.zeros_like(ub) if want_scale else None
    _check(_load().oracle_star3d_adjoint(_I(radius), _L(nx), _L(ny), _L(nz), _ptr(w), _ptr(c), _ptr(r_bar), _ptr(ub),
                                         _ptr(scale)), "star3d_adjoint")
    return ub, scale


def burgers_primal(u, C: float, D: float, r_init=None) -> np.ndarray:
    u = _f64(u)
    r = np.zeros_like(u) if r_init is None else _f64(r_init).copy()
    _check(_load().oracle_burgers_primal(_L(u.size), _D(C), _D(D), _ptr(u), _ptr(r)), "burgers_primal")
    return r


def burgers_tangent(u, u_dot, C: float, D: float) -> np.ndarray:
    u, u_dot = _f64(u), _f64(u_dot)
    r_dot = np.zeros_like(u)
    _check(_load().oracle_burgers_tangent(_L(u.size), _D(C), _D(D), _ptr(u), _ptr(u_dot), _ptr(r_dot)),
           "burgers_tangent")
    return r_dot


def burgers_adjoint(u, r_bar, u_bar, C: float, D: float, want_scale: bool = False):
    """Returns (u_bar_out, scale or None)."""
    u, r_bar = _f64(u), _f64(r_bar)
    ub = _f64(u_bar).copy()
    scale = np.zeros_like(ub) if want_scale else None
    _check(_load().oracle_burgers_adjoint(_L(u.size), _D(C), _D(D), _ptr(u), _ptr(r_bar), _ptr(ub),
                                          _ptr(scale)), "burgers_adjoint")
    return ub, scale


def burgers_primal_steps(states, nsteps: int, C: float, D: float) -> np.ndarray:
    """states: (rows >= nsteps+1, n); row 0 = initial state, boundary elements of all rows are
    inputs.  Returns a copy with rows 1..nsteps assigned on the interior."""
    st = _f64(states).copy()
    assert st.ndim == 2 and st.shape[0] >= nsteps + 1
    _check(_load().oracle_burgers_primal_steps(_L(st.shape[1]), _L(nsteps), _D(C), _D(D), _ptr(st)),
           "burgers_primal_steps")
    return st


def burgers_adjoint_steps(states, last: int, nsteps: int, lam0, lam1, C: float, D: float):
    """Reverse sweep over steps last-1 .. last-nsteps; returns the two buffers after the sweep."""
    st = _f64(states)
    assert st.ndim == 2 and st.shape[0] >= last
    a, b = _f64(lam0).copy(), _f64(lam1).copy()
    _check(_load().oracle_burgers_adjoint_steps(_L(st.shape[1]), _L(last), _L(nsteps), _D(C), _D(D), _ptr(st),
                                                _ptr(a), _ptr(b)), "burgers_adjoint_steps")
    return a, b


def lin3_primal(c, u, lo: int, hi: int, wm: float, w0: float, wp: float) -> np.ndarray:
    c, u = _f64(c), _f64(u)
    r = np.zeros_like(u)
    _check(_load().oracle_lin3_primal(_L(u.size), _L(lo), _L(hi), _D(wm), _D(w0), _D(wp), _ptr(c),
                                      _ptr(u), _ptr(r)), "lin3_primal")
    return r


def lin3_adjoint(c, r_bar, u_bar, lo: int, hi: int, wm: float, w0: float, wp: float) -> np.ndarray:
    c, r_bar = _f64(c), _f64(r_bar)
    ub = _f64(u_bar).copy()
    _check(_load().oracle_lin3_adjoint(_L(ub.size), _L(lo), _L(hi), _D(wm), _D(w0), _D(wp), _ptr(c),
                                       _ptr(r_bar), _ptr(ub)), "lin3_adjoint")
    return ub


_BODY = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double)
_PARTIALS = ctypes.CFUNCTYPE(None, ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                             ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                             ctypes.POINTER(ctypes.c_double))


def stencil1d_primal(f, u, p=None, r_init=None) -> np.ndarray:
    """r[i] = f(u[i-1], u[i], u[i+1], p[i]) on [1, n-2]; f is a Python callable of four floats.
    Slow (one callback per cell): for small n."""
    u = _f64(u)
    p = _f64(p) if p is not None else None
    r = _f64(r_init).copy() if r_init is not None else np.zeros_like(u)
    cb = _BODY(lambda um, u0, up, pp: float(f(um, u0, up, pp)))
    _check(_load().oracle_stencil1d_primal(_L(u.size), cb, _ptr(u), _ptr(p), _ptr(r)), "stencil1d_primal")
    return r


def stencil1d_adjoint(df, u, p, r_bar, u_bar, want_scale: bool = False):
    """Scatter adjoint of the loop above; df(um, u0, up, p) returns the three partials."""
    u, r_bar = _f64(u), _f64(r_bar)
    p = _f64(p) if p is not None else None
    ub = _f64(u_bar).copy()
    scale = np.zeros_like(ub) if want_scale else None

    def partials(um, u0, up, pp, dm, d0, dp):
        a, b, c = df(um, u0, up, pp)
        dm[0], d0[0], dp[0] = float(a), float(b), float(c)

    cb = _PARTIALS(partials)
    _check(_load().oracle_stencil1d_adjoint(_L(u.size), cb, _ptr(u), _ptr(p), _ptr(r_bar), _ptr(ub), _ptr(scale)),
           "stencil1d_adjoint")
    return (ub, scale) if want_scale else ub


_STAR_BODY = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(ctypes.c_double), ctypes.c_double)
_STAR_PARTIALS = ctypes.CFUNCTYPE(None, ctypes.POINTER(ctypes.c_double), ctypes.c_double,
                                  ctypes.POINTER(ctypes.c_double))


def starfn_reads(ndim: int, radius: int) -> int:
    """Number of reads of a star-shaped body: the centre and 2*radius per axis."""
    return 1 + 2 * radius * ndim


def starfn_primal(f, u, p, radius: int, r_init=None) -> np.ndarray:
    """r[i] = f(v, p[i]) on I for a star-shaped body in u.ndim dimensions; f takes a list of the
    reads (centre, then per axis x, y, z the offsets -R..-1, +1..+R) and p[i].  One Python
    callback per cell: for small grids."""
    u = _f64(u)
    p = _f64(p) if p is not None else None
    r = _f64(r_init).copy() if r_init is not None else np.zeros_like(u)
    nread = starfn_reads(u.ndim, radius)
    cb = _STAR_BODY(lambda v, pp: float(f([v[k] for k in range(nread)], pp)))
    ndim, nx, ny, nz = _dims(u.shape)
    _check(_load().oracle_starfn_primal(_I(ndim), _I(int(radius)), _L(nx), _L(ny), _L(nz), cb, _ptr(u), _ptr(p), _ptr(r)),
           "starfn_primal")
    return r


def starfn_adjoint(df, u, p, r_bar, u_bar, radius: int, want_scale: bool = False):
    """Scatter adjoint of the loop above; df(v, p) returns the partials with respect to the reads."""
    u, r_bar = _f64(u), _f64(r_bar)
    p = _f64(p) if p is not None else None
    ub = _f64(u_bar).copy()
    scale = np.zeros_like(ub) if want_scale else None
    nread = starfn_reads(u.ndim, radius)

    def partials(v, pp, d):
        out = df([v[k] for k in range(nread)], pp)
        for k in range(nread):
            d[k] = float(out[k])

    cb = _STAR_PARTIALS(partials)
    ndim, nx, ny, nz = _dims(u.shape)
    _check(_load().oracle_starfn_adjoint(_I(ndim), _I(int(radius)), _L(nx), _L(ny), _L(nz), cb, _ptr(u), _ptr(p),
                                         _ptr(r_bar), _ptr(ub), _ptr(scale)), "starfn_adjoint")
    return (ub, scale) if want_scale else ub
