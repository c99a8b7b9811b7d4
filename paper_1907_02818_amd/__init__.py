"""Python binding of libsadj (include/sadj.h): argument marshalling only.

Every function has the name of the C entry point it calls and takes torch tensors
that live on the GPU; torch is used for device memory and streams, nothing else.
All arithmetic happens in the HIP kernels of libsadj.so.  There is no CPU path: if
the shared library has not been built, importing a symbol raises.

Tensor layout: C-contiguous, slowest axis first, x last -- shape (n,), (ny, nx) or
(nz, ny, nx) -- which is the "x fastest" layout of the C ABI.
"""
from __future__ import annotations

import ctypes
import os

__all__ = [
    "SadjError", "lib_path", "load", "set_option", "get_option", "version",
    "sadj_primal_wave1d", "sadj_adjoint_wave1d", "sadj_primal_wave2d", "sadj_adjoint_wave2d",
    "sadj_primal_wave3d", "sadj_adjoint_wave3d", "sadj_primal_burgers1d", "sadj_adjoint_burgers1d",
    "sadj_adjoint_wave3d_steps", "sadj_primal_box", "sadj_adjoint_box",
    "sadj_primal_star3d", "sadj_adjoint_star3d", "sadj_primal_burgers1d_steps", "sadj_adjoint_burgers1d_steps",
    "sadj_adjoint_wave3d_atomic_scatter", "sadj_describe_wave3d_plan", "sadj_check_array",
    "sadj_stream_probe", "sadj_primal_burgers1d_ckpt", "sadj_adjoint_burgers1d_ckpt",
    "sadj_adjoint_burgers1d_ckpt_static", "sadj_static_scratch_bytes",
    "sadj_adjoint_wave3d_steps_fused", "sadj_describe_wave3d_sweep",
]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsadj.so")
_lib = None

SADJ_F32, SADJ_F64 = 0, 1


class SadjError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("libsadj status %d: %s" % (status, message))
        self.status = status


def lib_path() -> str:
    return _LIB_PATH


def load() -> ctypes.CDLL:
    """Load libsadj.so (built by `python -m paper_1907_02818_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime under the same soname as the system one; it
    # must be in the process first so that libsadj binds to the runtime that owns
    # torch's streams and allocations (two runtimes in one process cannot share them).
    import torch  # noqa: F401
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libsadj.so is not built: run `python -m paper_1907_02818_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    P, L, I, D = ctypes.c_void_p, ctypes.c_long, ctypes.c_int, ctypes.c_double
    lib.sadj_status_string.restype = ctypes.c_char_p
    lib.sadj_status_string.argtypes = [I]
    lib.sadj_version.restype = ctypes.c_char_p
    lib.sadj_version.argtypes = []
    lib.sadj_last_device_error.restype = ctypes.c_char_p
    lib.sadj_last_device_error.argtypes = []
    lib.sadj_set_option.argtypes = [ctypes.c_char_p, L]
    lib.sadj_get_option.argtypes = [ctypes.c_char_p, ctypes.POINTER(L)]
    lib.sadj_primal_wave1d.argtypes = [I, L, P, P, P, P, P]
    lib.sadj_adjoint_wave1d.argtypes = [I, L, P, P, P, P, P]
    lib.sadj_primal_wave2d.argtypes = [I, L, L, P, P, P, P, P]
    lib.sadj_adjoint_wave2d.argtypes = [I, L, L, P, P, P, P, P]
    lib.sadj_primal_wave3d.argtypes = [I, I, L, L, L, P, P, P, P, P]
    lib.sadj_adjoint_wave3d.argtypes = [I, I, L, L, L, P, P, P, P, P]
    lib.sadj_describe_wave3d_plan.argtypes = [I, I, L, L, L, I, ctypes.POINTER(L), ctypes.POINTER(ctypes.c_int), L]
    lib.sadj_adjoint_wave3d_atomic_scatter.argtypes = [I, I, L, L, L, P, P, P, P]
    lib.sadj_adjoint_wave3d_steps.argtypes = [I, I, L, L, L, L, P, P, P, P, P]
    lib.sadj_primal_star3d.argtypes = [I, I, L, L, L, ctypes.POINTER(D), P, P, P, P]
    lib.sadj_adjoint_star3d.argtypes = [I, I, L, L, L, ctypes.POINTER(D), P, P, P, P]
    lib.sadj_primal_box.argtypes = [I, I, L, L, L, ctypes.POINTER(D), P, P, P, P]
    lib.sadj_adjoint_box.argtypes = [I, I, L, L, L, ctypes.POINTER(D), P, P, P, P]
    lib.sadj_primal_burgers1d.argtypes = [I, L, D, D, P, P, P]
    lib.sadj_adjoint_burgers1d.argtypes = [I, L, D, D, P, P, P, P]
    lib.sadj_primal_burgers1d_steps.argtypes = [I, L, L, D, D, P, P]
    lib.sadj_adjoint_burgers1d_steps.argtypes = [I, L, L, L, D, D, P, P, P, P]
    lib.sadj_check_array.argtypes = [P, ctypes.c_size_t]
    lib.sadj_stream_probe.argtypes = [I, I, L, P, P, P, P]
    lib.sadj_primal_burgers1d_ckpt.argtypes = [I, L, L, L, D, D, P, P, P, P]
    lib.sadj_adjoint_burgers1d_ckpt.argtypes = [I, L, L, L, D, D, P, P, ctypes.c_size_t, P, P, P]
    lib.sadj_adjoint_burgers1d_ckpt_static.argtypes = [I, L, L, L, D, D, P, P, P, P]
    lib.sadj_adjoint_wave3d_steps_fused.argtypes = [I, I, L, L, L, L, P, P, P, P, P, P]
    lib.sadj_describe_wave3d_sweep.argtypes = [L, ctypes.POINTER(L), ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.sadj_static_scratch_bytes.argtypes = []
    lib.sadj_static_scratch_bytes.restype = ctypes.c_size_t
    for name in ("sadj_set_option", "sadj_get_option", "sadj_primal_wave1d", "sadj_adjoint_wave1d",
                 "sadj_primal_wave2d", "sadj_adjoint_wave2d", "sadj_primal_wave3d", "sadj_adjoint_wave3d",
                 "sadj_primal_burgers1d", "sadj_adjoint_burgers1d", "sadj_adjoint_wave3d_steps",
                 "sadj_primal_box", "sadj_adjoint_box", "sadj_adjoint_wave3d_atomic_scatter", "sadj_describe_wave3d_plan",
                 "sadj_primal_star3d", "sadj_adjoint_star3d",
                 "sadj_primal_burgers1d_steps", "sadj_adjoint_burgers1d_steps", "sadj_check_array",
                 "sadj_stream_probe", "sadj_primal_burgers1d_ckpt", "sadj_adjoint_burgers1d_ckpt",
                 "sadj_adjoint_burgers1d_ckpt_static", "sadj_adjoint_wave3d_steps_fused",
                 "sadj_describe_wave3d_sweep"):
        getattr(lib, name).restype = I
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        msg = load().sadj_status_string(status).decode()
        if status == 5:
            msg += " (" + load().sadj_last_device_error().decode() + ")"
        raise SadjError(status, msg)


def version() -> str:
    return load().sadj_version().decode()


def set_option(name: str, value: int) -> None:
    _check(load().sadj_set_option(name.encode(), int(value)))


def get_option(name: str) -> int:
    v = ctypes.c_long(0)
    _check(load().sadj_get_option(name.encode(), ctypes.byref(v)))
    return v.value


def _marshal(tensors, ndim, optional=()):
    """Common checks: same device/dtype/shape, contiguous, on the GPU.  Returns
    (dtype code, shape, pointers, stream handle)."""
    import torch

    ref = next(t for t in tensors if t is not None)
    if ref.dim() != ndim:
        raise ValueError("expected %d-D tensors" % ndim)
    if ref.dtype == torch.float64:
        code = SADJ_F64
    elif ref.dtype == torch.float32:
        code = SADJ_F32
    else:
        raise TypeError("float32 or float64 tensors only")
    ptrs = []
    for i, t in enumerate(tensors):
        if t is None:
            if i not in optional:
                raise ValueError("tensor %d is required" % i)
            ptrs.append(None)
            continue
        if not t.is_cuda:
            raise ValueError("libsadj works on GPU memory only (no CPU path)")
        if t.dtype != ref.dtype or t.shape != ref.shape or t.device != ref.device:
            raise ValueError("all tensors of a call share dtype, shape and device")
        if not t.is_contiguous():
            raise ValueError("tensors must be C-contiguous (x fastest)")
        ptrs.append(ctypes.c_void_p(t.data_ptr()))
    stream = ctypes.c_void_p(torch.cuda.current_stream(ref.device).cuda_stream)
    return code, tuple(ref.shape), ptrs, stream


def sadj_primal_wave1d(u, u_prev, c, r) -> None:
    code, (n,), p, s = _marshal([u, u_prev, c, r], 1)
    _check(load().sadj_primal_wave1d(code, n, *p, s))


def sadj_adjoint_wave1d(c, r_bar, u_bar, u_prev_bar=None) -> None:
    code, (n,), p, s = _marshal([c, r_bar, u_bar, u_prev_bar], 1, optional=(3,))
    _check(load().sadj_adjoint_wave1d(code, n, *p, s))


def sadj_primal_wave2d(u, u_prev, c, r) -> None:
    code, (ny, nx), p, s = _marshal([u, u_prev, c, r], 2)
    _check(load().sadj_primal_wave2d(code, nx, ny, *p, s))


def sadj_adjoint_wave2d(c, r_bar, u_bar, u_prev_bar=None) -> None:
    code, (ny, nx), p, s = _marshal([c, r_bar, u_bar, u_prev_bar], 2, optional=(3,))
    _check(load().sadj_adjoint_wave2d(code, nx, ny, *p, s))


def sadj_primal_wave3d(radius: int, u, u_prev, c, r) -> None:
    code, (nz, ny, nx), p, s = _marshal([u, u_prev, c, r], 3)
    _check(load().sadj_primal_wave3d(code, int(radius), nx, ny, nz, *p, s))


def sadj_adjoint_wave3d(radius: int, c, r_bar, u_bar, u_prev_bar=None) -> None:
    code, (nz, ny, nx), p, s = _marshal([c, r_bar, u_bar, u_prev_bar], 3, optional=(3,))
    _check(load().sadj_adjoint_wave3d(code, int(radius), nx, ny, nz, *p, s))


def sadj_check_array(address: int, nbytes: int) -> int:
    """Status (0 = ok) of the library's pointer check for the byte range at `address`."""
    return int(load().sadj_check_array(ctypes.c_void_p(int(address)), int(nbytes)))


def sadj_stream_probe(shape: int, a, b, out) -> None:
    """out += a * b over flat tensors (the streaming yardstick of the header)."""
    code, (n,), p, s = _marshal([a, b, out], 1)
    _check(load().sadj_stream_probe(code, int(shape), n, *p, s))


def sadj_describe_wave3d_plan(dtype_code: int, radius: int, nx: int, ny: int, nz: int, with_tiles: bool = True,
                              with_u_prev_bar: bool = False):
    """Host-only: (plan dict, list of (tile x, tile y, first plane, end plane) per workgroup id)."""
    plan = (ctypes.c_long * 8)()
    prev = int(bool(with_u_prev_bar))
    _check(load().sadj_describe_wave3d_plan(dtype_code, int(radius), nx, ny, nz, prev, plan, None, 0))
    ntx, nty, tw, th, total, tiles_a, ntz_a, ntz = (int(v) for v in plan)
    info = dict(ntx=ntx, nty=nty, tile_w=tw, tile_h=th, workgroups=total, tiles_a=tiles_a, ntz_a=ntz_a, ntz=ntz)
    if not with_tiles:
        return info, None
    buf = (ctypes.c_int * (4 * total))()
    _check(load().sadj_describe_wave3d_plan(dtype_code, int(radius), nx, ny, nz, prev, plan, buf, total))
    return info, [tuple(buf[4 * b:4 * b + 4]) for b in range(total)]


def sadj_adjoint_wave3d_atomic_scatter(radius: int, c, r_bar, u_bar) -> None:
    code, (nz, ny, nx), p, s = _marshal([c, r_bar, u_bar], 3)
    _check(load().sadj_adjoint_wave3d_atomic_scatter(code, int(radius), nx, ny, nz, *p, s))


def sadj_adjoint_wave3d_steps(radius: int, nsteps: int, c, lam0, lam1, lam2) -> None:
    code, (nz, ny, nx), p, s = _marshal([c, lam0, lam1, lam2], 3)
    _check(load().sadj_adjoint_wave3d_steps(code, int(radius), nx, ny, nz, int(nsteps), *p, s))


def sadj_adjoint_wave3d_steps_fused(radius: int, nsteps: int, c, lam0, lam1, lam2, work) -> None:
    code, (nz, ny, nx), p, s = _marshal([c, lam0, lam1, lam2, work], 3)
    _check(load().sadj_adjoint_wave3d_steps_fused(code, int(radius), nx, ny, nz, int(nsteps), *p, s))


def sadj_describe_wave3d_sweep(nsteps: int):
    """(body_pairs, [(pair, a, b, o0, o1), ...]) of the launches after step 0; body_pairs = -1: single
    steps over the caller's three buffers only."""
    body = ctypes.c_long(0)
    n = ctypes.c_int(0)
    tail = (ctypes.c_int * 60)()
    _check(load().sadj_describe_wave3d_sweep(int(nsteps), ctypes.byref(body), ctypes.byref(n), tail))
    return body.value, [tuple(tail[5 * i:5 * i + 5]) for i in range(n.value)]


def _box(fn_name, weights, tensors):
    ndim = tensors[0].dim()
    code, shape, p, s = _marshal(tensors, ndim)
    dims = list(shape[::-1]) + [1] * (3 - ndim)            # nx, ny, nz
    flat = [float(v) for v in _flatten(weights)]
    if len(flat) != 3 ** ndim:
        raise ValueError("weights must have 3**ndim entries, slowest axis first (shape (3,)*ndim)")
    w = (ctypes.c_double * len(flat))(*flat)
    _check(getattr(load(), fn_name)(code, ndim, dims[0], dims[1], dims[2], w, *p, s))


def _star(fn_name, radius, weights, tensors):
    code, (nz, ny, nx), p, s = _marshal(tensors, 3)
    flat = [float(v) for v in _flatten(weights)]
    if len(flat) != 1 + 6 * int(radius):
        raise ValueError("weights: centre, then 2*radius values per axis x, y, z (offsets -R..-1, +1..+R)")
    w = (ctypes.c_double * len(flat))(*flat)
    _check(getattr(load(), fn_name)(code, int(radius), nx, ny, nz, w, *p, s))


def sadj_primal_star3d(radius: int, weights, u, c, r) -> None:
    _star("sadj_primal_star3d", radius, weights, [u, c, r])


def sadj_adjoint_star3d(radius: int, weights, c, r_bar, u_bar) -> None:
    _star("sadj_adjoint_star3d", radius, weights, [c, r_bar, u_bar])


def _flatten(w):
    try:
        for x in w:
            yield from _flatten(x)
    except TypeError:
        yield w


def sadj_primal_box(weights, u, c, r) -> None:
    """weights: nested sequence / array of shape (3,)*ndim indexed [oz+1][oy+1][ox+1]."""
    _box("sadj_primal_box", weights, [u, c, r])


def sadj_adjoint_box(weights, c, r_bar, u_bar) -> None:
    _box("sadj_adjoint_box", weights, [c, r_bar, u_bar])


def sadj_primal_burgers1d(C: float, D: float, u, r) -> None:
    code, (n,), p, s = _marshal([u, r], 1)
    _check(load().sadj_primal_burgers1d(code, n, float(C), float(D), *p, s))


def sadj_adjoint_burgers1d(C: float, D: float, u, r_bar, u_bar) -> None:
    code, (n,), p, s = _marshal([u, r_bar, u_bar], 1)
    _check(load().sadj_adjoint_burgers1d(code, n, float(C), float(D), *p, s))


def sadj_primal_burgers1d_steps(C: float, D: float, nsteps: int, states) -> None:
    """states: (rows, n) tensor with rows >= nsteps + 1; row 0 is the initial state."""
    code, (rows, n), p, s = _marshal([states], 2)
    if rows < int(nsteps) + 1:
        raise ValueError("states needs nsteps + 1 rows")
    _check(load().sadj_primal_burgers1d_steps(code, n, int(nsteps), float(C), float(D), *p, s))


def sadj_adjoint_burgers1d_steps(C: float, D: float, last: int, nsteps: int, states, lam0, lam1) -> None:
    """states: (rows, n) tensor with rows >= last; lam0, lam1: (n,) tensors."""
    code, (rows, n), ps, s = _marshal([states], 2)
    code2, (n2,), pl, _ = _marshal([lam0, lam1], 1)
    if code2 != code or n2 != n or lam0.device != states.device:
        raise ValueError("states and lam buffers share dtype, row length and device")
    if rows < int(last):
        raise ValueError("states needs at least `last` rows")
    _check(load().sadj_adjoint_burgers1d_steps(code, n, int(last), int(nsteps), float(C), float(D), *ps, *pl, s))


def sadj_primal_burgers1d_ckpt(C: float, D: float, nsteps: int, every: int, ckpt, work, u_final=None) -> None:
    """ckpt: (rows, n) tensor with rows >= nsteps // every + 1, row 0 = initial state; work: (2, n)."""
    code, (rows, n), pc, s = _marshal([ckpt], 2)
    if rows < int(nsteps) // int(every) + 1:
        raise ValueError("ckpt needs nsteps // every + 1 rows")
    _, (wr, wn), pw, _ = _marshal([work], 2)
    if wr < 2 or wn != n or work.dtype != ckpt.dtype:
        raise ValueError("work needs two rows of n elements of the same dtype")
    pf = [None]
    if u_final is not None:
        _, (nf,), pf, _ = _marshal([u_final], 1)
        if nf != n or u_final.dtype != ckpt.dtype:
            raise ValueError("u_final: n elements of the same dtype")
    _check(load().sadj_primal_burgers1d_ckpt(code, n, int(nsteps), int(every), float(C), float(D), *pc, *pw, *pf, s))


def sadj_adjoint_burgers1d_ckpt(C: float, D: float, nsteps: int, every: int, ckpt, work, lam0, lam1) -> None:
    """ckpt as written by sadj_primal_burgers1d_ckpt; work: a tensor of at least (every-1)*n elements
    (None when every == 1); lam0, lam1: (n,) tensors."""
    code, (rows, n), pc, s = _marshal([ckpt], 2)
    code2, (n2,), pl, _ = _marshal([lam0, lam1], 1)
    if code2 != code or n2 != n:
        raise ValueError("ckpt and lam buffers share dtype and row length")
    if work is not None:
        if not work.is_cuda or work.dtype != ckpt.dtype or not work.is_contiguous():
            raise ValueError("work: contiguous GPU tensor of the same dtype")
        pw, wbytes = ctypes.c_void_p(work.data_ptr()), work.numel() * work.element_size()
    else:
        pw, wbytes = None, 0
    _check(load().sadj_adjoint_burgers1d_ckpt(code, n, int(nsteps), int(every), float(C), float(D), *pc, pw, wbytes, *pl, s))


def sadj_static_scratch_bytes() -> int:
    return int(load().sadj_static_scratch_bytes())


def sadj_adjoint_burgers1d_ckpt_static(C: float, D: float, nsteps: int, every: int, ckpt, lam0, lam1) -> None:
    """sadj_adjoint_burgers1d_ckpt with the library's fixed scratch array (no allocation)."""
    code, (rows, n), pc, s = _marshal([ckpt], 2)
    code2, (n2,), pl, _ = _marshal([lam0, lam1], 1)
    if code2 != code or n2 != n:
        raise ValueError("ckpt and lam buffers share dtype and row length")
    _check(load().sadj_adjoint_burgers1d_ckpt_static(code, n, int(nsteps), int(every), float(C), float(D), *pc, *pl, s))
