"""Seeded synthetic inputs for the adjoint-stencil workloads.

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests/benchmark.  It holds no stencil arithmetic: it only draws reproducible
fields (uniform noise, layered coefficient fields, a sine-plus-noise profile)
from a counter-based generator, so any element can be produced independently of
any other and the result does not depend on the platform, the chunking or the
NumPy version.

Generator: ``unit(seed, stream, k) = (mix(key + k*GOLDEN) >> 11) * 2**-53`` with
``key = mix(seed*GOLDEN + mix(stream))`` and ``mix`` the splitmix64 finaliser.

The workloads stand in for the paper's two test cases (Section 4.1: one step of
a 3-D seismic-wave solver with spatially varying speed; Section 4.2: one step of
a 1-D upwinded Burgers solver); the paper does not describe its field values.
"""
from __future__ import annotations

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# one stream id per array name, so that arrays are mutually independent
STREAMS = {
    "u": 1, "u_prev": 2, "c": 3, "r_bar": 4, "u_bar": 5, "u_prev_bar": 6,
    "u_dot": 7, "u_prev_dot": 8, "layers": 9, "aux": 10,
}


def _mix(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        s = _mix(np.array([stream], dtype=np.uint64))[0]
        k = _mix(np.array([np.uint64(seed) * _GOLDEN + s], dtype=np.uint64))[0]
    return k


def _unit_chunk(out, key, start, lo, hi):
    with np.errstate(over="ignore"):
        k = np.arange(start + lo, start + hi, dtype=np.uint64)
        k *= _GOLDEN
        k += key
        k ^= k >> np.uint64(30)
        k *= _M1
        k ^= k >> np.uint64(27)
        k *= _M2
        k ^= k >> np.uint64(31)
        k >>= np.uint64(11)
        np.multiply(k, 2.0 ** -53, out=out[lo:hi])


def unit(seed: int, stream: int, count: int, start: int = 0) -> np.ndarray:
    """`count` doubles in [0,1) for counters start..start+count-1 of (seed, stream).
    Large requests are filled chunk by chunk on a few threads; the values do not
    depend on the chunking."""
    out = np.empty(count, dtype=np.float64)
    key = _key(seed, stream)
    chunk = 1 << 20
    spans = [(lo, min(count, lo + chunk)) for lo in range(0, count, chunk)]
    if len(spans) <= 4:
        for lo, hi in spans:
            _unit_chunk(out, key, start, lo, hi)
    else:
        from concurrent.futures import ThreadPoolExecutor
        import os
        workers = max(1, min(8, (os.cpu_count() or 1)))
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(lambda s: _unit_chunk(out, key, start, s[0], s[1]), spans))
    return out


def uniform(seed: int, name: str, shape, lo: float, hi: float) -> np.ndarray:
    """iid U(lo,hi) array of the given shape, C order (last axis = x, unit stride)."""
    n = int(np.prod(shape))
    a = unit(seed, STREAMS[name], n)
    a *= (hi - lo)
    a += lo
    return a.reshape(shape)


def uniform_planes(seed: int, name: str, shape, lo: float, hi: float, z0: int, nplanes: int) -> np.ndarray:
    """Planes z0 .. z0+nplanes-1 (slowest axis) of the array uniform(seed, name, shape, lo, hi)
    would return, without generating the rest: the generator is counter-based."""
    per = int(np.prod(shape[1:]))
    a = unit(seed, STREAMS[name], nplanes * per, start=z0 * per)
    a *= (hi - lo)
    a += lo
    return a.reshape((nplanes,) + tuple(shape[1:]))


def layered_profile(seed: int, n_axis: int, nlayers: int, blend: int,
                    lo: float, hi: float) -> np.ndarray:
    """1-D piecewise-constant profile with linear blends across layer interfaces.

    `nlayers` layers of thickness ceil(n_axis/nlayers); each layer value ~U(lo,hi);
    the first `blend` cells of a layer ramp linearly from the previous layer's value.
    Every value is a convex combination of layer values, so it stays in [lo,hi].
    """
    thick = max(1, -(-n_axis // nlayers))
    vals = lo + (hi - lo) * unit(seed, STREAMS["layers"], n_axis // thick + 2)
    p = np.arange(n_axis)
    layer = p // thick
    t = p % thick
    prof = vals[layer].copy()
    b = min(blend, thick)
    ramp = (layer > 0) & (t < b)
    w = (t[ramp] + 0.5) / b
    prof[ramp] = vals[layer[ramp] - 1] * (1.0 - w) + vals[layer[ramp]] * w
    return prof


def _round_dtype(arrs: dict, dtype) -> dict:
    """fp32 workloads: every field is the fp64 draw rounded once to nearest float,
    returned as float32 arrays (the oracle widens them back to double)."""
    dtype = np.dtype(dtype)
    if dtype == np.float64:
        return arrs
    return {k: v.astype(dtype) for k, v in arrs.items()}


WAVE_FIELDS = ("u", "u_prev", "r_bar", "u_bar", "u_prev_bar", "c")


def wave_inputs(shape, c_lo: float, c_hi: float, seed: int = 0, dtype=np.float64,
                c_mode: str = "iid", nlayers: int = 16, blend: int = 4,
                fields=WAVE_FIELDS) -> dict:
    """Fields of a linear variable-coefficient wave workload on a grid `shape`
    (slowest axis first, x last).  u, u_prev, r_bar, u_bar, u_prev_bar ~ U(-1,1) iid.
    c_mode "iid": c ~ U(c_lo,c_hi) iid.  c_mode "layered": c depends only on the
    slowest axis through `layered_profile` (layered in z for 3-D, in y for 2-D).
    `fields` selects which arrays are produced (each array's values do not depend on
    which others are requested)."""
    shape = tuple(int(s) for s in shape)
    out = {name: uniform(seed, name, shape, -1.0, 1.0)
           for name in ("u", "u_prev", "r_bar", "u_bar", "u_prev_bar") if name in fields}
    if "c" not in fields:
        pass
    elif c_mode == "iid":
        out["c"] = uniform(seed, "c", shape, c_lo, c_hi)
    elif c_mode == "layered":
        prof = layered_profile(seed, shape[0], nlayers, blend, c_lo, c_hi)
        out["c"] = np.ascontiguousarray(
            np.broadcast_to(prof.reshape((-1,) + (1,) * (len(shape) - 1)), shape))
    else:
        raise ValueError(c_mode)
    return _round_dtype(out, dtype)


def burgers_inputs(n: int, seed: int = 0, dtype=np.float64, waves: int = 8) -> dict:
    """1-D Burgers workload: u = 0.75 sin(2 pi waves i/n) + 0.25 U(-1,1), which stays
    in (-1,1) and changes sign, so both upwind branches are exercised;
    r_bar, u_bar ~ U(-1,1)."""
    i = np.arange(n, dtype=np.float64)
    u = 0.75 * np.sin(2.0 * np.pi * waves * i / n) + 0.25 * uniform(seed, "u", (n,), -1.0, 1.0)
    out = {"u": u,
           "r_bar": uniform(seed, "r_bar", (n,), -1.0, 1.0),
           "u_bar": uniform(seed, "u_bar", (n,), -1.0, 1.0)}
    return _round_dtype(out, dtype)


# The five benchmark workloads.  `shape` is slowest axis first.
CONFIGS = {
    "wave1d": dict(kind="wave", shape=(4096,), radius=1, c=(0.01, 0.25), c_mode="iid"),
    "burgers1d": dict(kind="burgers", shape=(1 << 24,), C=0.1, D=0.05),
    "wave2d": dict(kind="wave", shape=(8192, 8192), radius=1, c=(0.01, 0.2),
                   c_mode="layered", nlayers=64, blend=8),
    "wave3d_r1": dict(kind="wave", shape=(512, 512, 512), radius=1, c=(0.01, 0.15),
                      c_mode="layered", nlayers=16, blend=4),
    "wave3d_r4": dict(kind="wave", shape=(512, 512, 512), radius=4, c=(0.01, 0.1),
                      c_mode="layered", nlayers=16, blend=4),
}


def config_inputs(name: str, shape=None, seed: int = 0, dtype=np.float64,
                  c_mode: str | None = None, fields=WAVE_FIELDS) -> dict:
    """Inputs of benchmark workload `name`, optionally on a smaller `shape`."""
    cfg = CONFIGS[name]
    shape = tuple(shape) if shape is not None else cfg["shape"]
    if cfg["kind"] == "burgers":
        return burgers_inputs(shape[0], seed=seed, dtype=dtype)
    return wave_inputs(shape, cfg["c"][0], cfg["c"][1], seed=seed, dtype=dtype,
                       c_mode=c_mode or cfg["c_mode"],
                       nlayers=cfg.get("nlayers", 16), blend=cfg.get("blend", 4), fields=fields)
