"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_1907_02818_amd as sadj

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sadj.h")

pytestmark = pytest.mark.skipif(not os.path.exists(sadj.lib_path()),
                                reason="libsadj.so not built (python -m paper_1907_02818_amd.build)")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sadj_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = _declared_functions()
    for n in ("sadj_primal_wave1d", "sadj_adjoint_wave1d", "sadj_primal_wave2d", "sadj_adjoint_wave2d",
              "sadj_primal_wave3d", "sadj_adjoint_wave3d", "sadj_primal_burgers1d",
              "sadj_adjoint_burgers1d", "sadj_adjoint_wave3d_steps", "sadj_adjoint_wave3d_atomic_scatter", "sadj_primal_burgers1d_steps", "sadj_adjoint_burgers1d_steps", "sadj_primal_star3d", "sadj_adjoint_star3d", "sadj_primal_box", "sadj_adjoint_box", "sadj_status_string", "sadj_version", "sadj_set_option",
              "sadj_get_option", "sadj_last_device_error"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = sadj.load()
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_binding_has_the_same_names():
    for name in _declared_functions():
        if name in ("sadj_status_string", "sadj_version", "sadj_set_option", "sadj_get_option",
                    "sadj_last_device_error"):
            continue
        assert callable(getattr(sadj, name))


def test_status_strings_and_version():
    lib = sadj.load()
    assert lib.sadj_status_string(0) == b"ok"
    seen = {lib.sadj_status_string(i) for i in range(6)}
    assert len(seen) == 6 and all(seen)
    assert lib.sadj_status_string(99)
    assert re.match(r"^\d+\.\d+\.\d+$", sadj.version())


def test_options_roundtrip_and_reject_unknown():
    old = sadj.get_option("wave3d.zchunk")
    sadj.set_option("wave3d.zchunk", 32)
    assert sadj.get_option("wave3d.zchunk") == 32
    sadj.set_option("wave3d.zchunk", old)
    for v in (1, 2, 0):
        sadj.set_option("wave3d.remainder", v)
        assert sadj.get_option("wave3d.remainder") == v
    with pytest.raises(sadj.SadjError):
        sadj.set_option("wave3d.remainder", 3)
    for v in (1, 0):
        sadj.set_option("wave3d.order", v)
        assert sadj.get_option("wave3d.order") == v
    with pytest.raises(sadj.SadjError):
        sadj.set_option("wave3d.order", 2)
    for name, vals in (("wave3d.xcdmap", (3, 2, 1, 0)), ("wave3d.band", (8, 0))):
        for v in vals:
            sadj.set_option(name, v)
            assert sadj.get_option(name) == v
    for v in (1, 0):
        sadj.set_option("stencil1d.functor", v)
        assert sadj.get_option("stencil1d.functor") == v
    with pytest.raises(sadj.SadjError) as e:
        sadj.set_option("no.such.option", 1)
    assert e.value.status == 4
    with pytest.raises(sadj.SadjError):
        sadj.set_option("wave3d.variant", -1)


P = ctypes.c_void_p
A, B, C_, D_ = (P(0x10000000), P(0x20000000), P(0x30000000), P(0x40000000))  # never dereferenced


def test_argument_errors_are_reported_before_any_launch():
    lib = sadj.load()
    F64 = 1
    # null pointers
    assert lib.sadj_adjoint_wave3d(F64, 4, 32, 32, 32, None, B, C_, None, None) == 1
    assert lib.sadj_adjoint_wave3d(F64, 4, 32, 32, 32, A, B, None, None, None) == 1
    assert lib.sadj_primal_wave3d(F64, 4, 32, 32, 32, A, B, C_, None, None) == 1
    assert lib.sadj_adjoint_burgers1d(F64, 100, 0.1, 0.05, A, None, C_, None) == 1
    # sizes: every extent must be at least 2R+1
    assert lib.sadj_adjoint_wave3d(F64, 4, 8, 32, 32, A, B, C_, None, None) == 2
    assert lib.sadj_adjoint_wave3d(F64, 1, 32, 2, 32, A, B, C_, None, None) == 2
    assert lib.sadj_adjoint_wave2d(F64, 2, 32, A, B, C_, None, None) == 2
    assert lib.sadj_adjoint_wave1d(F64, 2, A, B, C_, None, None) == 2
    assert lib.sadj_primal_burgers1d(F64, 2, 0.1, 0.05, A, B, None) == 2
    assert lib.sadj_adjoint_wave2d(F64, 1 << 20, 1 << 20, A, B, C_, None, None) == 2
    # aliasing: an output overlapping an input, or two outputs overlapping
    assert lib.sadj_adjoint_wave3d(F64, 1, 16, 16, 16, A, B, A, None, None) == 3
    assert lib.sadj_adjoint_wave3d(F64, 1, 16, 16, 16, A, B, P(0x20000000 + 8), None, None) == 3
    assert lib.sadj_adjoint_wave3d(F64, 1, 16, 16, 16, A, B, C_, C_, None) == 3
    assert lib.sadj_primal_wave1d(F64, 64, A, B, C_, B, None) == 3
    assert lib.sadj_adjoint_burgers1d(F64, 64, 0.1, 0.05, A, B, A, None) == 3
    # the multi-step sweep: null, negative step count, aliasing among the rotating buffers
    assert lib.sadj_adjoint_wave3d_steps(F64, 4, 32, 32, 32, 3, A, B, None, D_, None) == 1
    assert lib.sadj_adjoint_wave3d_steps(F64, 4, 32, 32, 32, -1, A, B, C_, D_, None) == 2
    assert lib.sadj_adjoint_wave3d_steps(F64, 4, 32, 32, 32, 3, A, B, C_, B, None) == 3
    assert lib.sadj_adjoint_wave3d_steps(F64, 4, 32, 32, 32, 3, A, A, C_, D_, None) == 3
    assert lib.sadj_adjoint_wave3d_steps(F64, 5, 32, 32, 32, 3, A, B, C_, D_, None) == 4
    # box stencils: host weight table required, ndim in 1..3
    W9 = (ctypes.c_double * 27)(*([1.0] * 27))
    assert lib.sadj_adjoint_box(F64, 2, 32, 32, 1, None, A, B, C_, None) == 1
    assert lib.sadj_adjoint_box(F64, 4, 32, 32, 32, W9, A, B, C_, None) == 4
    assert lib.sadj_adjoint_box(F64, 3, 32, 2, 32, W9, A, B, C_, None) == 2
    assert lib.sadj_primal_box(F64, 1, 64, 1, 1, W9, A, B, A, None) == 3
    # Burgers time loop: null, more steps than stored states, overlap of the two buffers /
    # of a buffer with the rows that are read (row = 100 doubles = 800 bytes)
    assert lib.sadj_primal_burgers1d_steps(F64, 100, 3, 0.1, 0.05, None, None) == 1
    assert lib.sadj_primal_burgers1d_steps(F64, 2, 3, 0.1, 0.05, A, None) == 2
    assert lib.sadj_primal_burgers1d_steps(F64, 100, -1, 0.1, 0.05, A, None) == 2
    assert lib.sadj_adjoint_burgers1d_steps(F64, 100, 5, 3, 0.1, 0.05, A, B, None, None) == 1
    assert lib.sadj_adjoint_burgers1d_steps(F64, 100, 2, 3, 0.1, 0.05, A, B, C_, None) == 2
    assert lib.sadj_adjoint_burgers1d_steps(F64, 100, 5, 3, 0.1, 0.05, A, B, B, None) == 3
    assert lib.sadj_adjoint_burgers1d_steps(F64, 100, 5, 3, 0.1, 0.05, A, P(0x10000000 + 3 * 800), C_, None) == 3
    # the atomic-scatter contrast call validates like the gather call
    assert lib.sadj_adjoint_wave3d_atomic_scatter(F64, 4, 32, 32, 32, A, None, C_, None) == 1
    assert lib.sadj_adjoint_wave3d_atomic_scatter(F64, 4, 32, 8, 32, A, B, C_, None) == 2
    assert lib.sadj_adjoint_wave3d_atomic_scatter(F64, 1, 16, 16, 16, A, B, B, None) == 3
    assert lib.sadj_adjoint_wave3d_atomic_scatter(F64, 0, 32, 32, 32, A, B, C_, None) == 4
    # general star: host table required, radius 1..4, extents, aliasing
    W25 = (ctypes.c_double * 25)(*([0.5] * 25))
    assert lib.sadj_adjoint_star3d(F64, 4, 32, 32, 32, None, A, B, C_, None) == 1
    assert lib.sadj_adjoint_star3d(F64, 0, 32, 32, 32, W25, A, B, C_, None) == 4
    assert lib.sadj_primal_star3d(F64, 4, 32, 8, 32, W25, A, B, C_, None) == 2
    assert lib.sadj_primal_star3d(F64, 4, 32, 32, 32, W25, A, B, B, None) == 3
    # unsupported radius / dtype
    assert lib.sadj_adjoint_wave3d(F64, 5, 32, 32, 32, A, B, C_, None, None) == 4
    assert lib.sadj_primal_wave3d(F64, 0, 32, 32, 32, A, B, C_, D_, None) == 4
    assert lib.sadj_adjoint_wave3d(7, 4, 32, 32, 32, A, B, C_, None, None) == 4
    assert lib.sadj_primal_wave2d(-1, 32, 32, A, B, C_, D_, None) == 4


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros(16, dtype=torch.float64)
    with pytest.raises(ValueError):
        sadj.sadj_adjoint_wave1d(t, t.clone(), t.clone())


def test_functor_header_example_is_built_and_exports_its_entry_points():
    """include/sadj_stencil1d.hpp is a header-only template API; the user-side example
    compiled against it alone (tests/functor_example) must load and export its two calls."""
    path = os.path.join(ROOT, "tests", "functor_example", "libsine_flux.so")
    if not os.path.exists(path):
        pytest.skip("tests/functor_example/libsine_flux.so not built (__graft_entry__.build())")
    sadj.load()                                    # torch's HIP runtime first
    lib = ctypes.CDLL(path)
    assert hasattr(lib, "sine_flux_primal") and hasattr(lib, "sine_flux_adjoint")


def test_every_option_the_library_knows_is_documented_in_the_header():
    """Option names are plain strings; the header's list and the library's must agree."""
    header = open(HEADER).read()
    documented = set(re.findall(r'"((?:wave[23]d|stencil1d|check)\.[a-z0-9]+)"', header))
    src = open(os.path.join(ROOT, "paper_1907_02818_amd", "csrc", "api.hip")).read()
    known = set(re.findall(r'"((?:wave[23]d|stencil1d|check)\.[a-z0-9]+)"', src))
    assert documented == known
    for name in sorted(known):
        assert isinstance(sadj.get_option(name), int)


@pytest.mark.parametrize("xcdmap,band,zchunk,split", [(0, 0, 0, 0), (1, 0, 7, 0), (2, 0, 0, 0), (3, 0, 16, 1), (1, 3, 0, 0),
                                                      (2, 8, 5, 0), (1, 2, 33, 0), (0, 0, 0, 1), (3, 4, 0, 0)])
@pytest.mark.parametrize("dtype_code,radius,shape", [(1, 4, (512, 512, 512)), (1, 4, (300, 500, 700)), (0, 4, (512, 512, 512)),
                                                     (1, 1, (1000, 1000, 1000)), (1, 2, (9, 9, 9)), (0, 3, (100, 33, 65)),
                                                     (1, 4, (768, 768, 768)), (1, 1, (3, 3, 3)), (1, 4, (400, 400, 400)),
                                                     (0, 1, (896, 896, 896)), (1, 4, (640, 640, 640)), (1, 4, (1 << 17, 9, 70)), (1, 4, (40, 300, 2100))])
def test_workgroups_tile_the_grid_exactly_once(dtype_code, radius, shape, xcdmap, band, zchunk, split):
    """Disjoint cover (Section 3.3.4): under every mapping option the workgroups' (tile,
    range of planes) pairs are disjoint and cover the grid: every tile of the x-y tiling
    appears, and the plane ranges of each tile partition 0 .. nz."""
    nz, ny, nx = shape
    try:
        sadj.set_option("wave3d.xcdmap", xcdmap)
        sadj.set_option("wave3d.band", band)
        sadj.set_option("wave3d.zchunk", zchunk)
        sadj.set_option("wave3d.split", split)
        info, tiles = sadj.sadj_describe_wave3d_plan(dtype_code, radius, nx, ny, nz)
    finally:
        sadj.set_option("wave3d.xcdmap", 0)
        sadj.set_option("wave3d.band", 0)
        sadj.set_option("wave3d.zchunk", 0)
        sadj.set_option("wave3d.split", 0)
    assert info["ntx"] * info["tile_w"] >= nx > (info["ntx"] - 1) * info["tile_w"]
    assert info["nty"] * info["tile_h"] >= ny > (info["nty"] - 1) * info["tile_h"]
    assert len(tiles) == info["workgroups"]
    ntiles = info["ntx"] * info["nty"]
    assert info["workgroups"] == info["tiles_a"] * info["ntz_a"] + (ntiles - info["tiles_a"]) * info["ntz"]
    if split == 1 or zchunk:
        assert info["tiles_a"] == 0
    ranges = {}
    for x, y, zs, ze in tiles:
        assert 0 <= x < info["ntx"] and 0 <= y < info["nty"] and 0 <= zs < ze <= nz
        ranges.setdefault((x, y), []).append((zs, ze))
    assert len(ranges) == ntiles
    for key, rs in ranges.items():
        rs.sort()
        assert rs[0][0] == 0 and rs[-1][1] == nz, key
        assert all(a[1] == b[0] for a, b in zip(rs, rs[1:])), key


def test_left_over_tiles_are_cut_finer_where_that_fills_the_chip():
    """768^3 in 64 x 32 tiles on 256 compute units (the count the planner assumes without a
    GPU): 288 tiles = one full round marching all planes + 32 tiles that are cut so that
    they fill a round too."""
    info, tiles = sadj.sadj_describe_wave3d_plan(1, 4, 768, 768, 768)
    assert (info["ntx"], info["nty"]) == (12, 24)
    assert (info["tiles_a"], info["ntz_a"], info["ntz"]) == (256, 1, 8)
    assert info["workgroups"] == 512
    # a column of two tiles: cut into as many chunks as it takes to give every compute unit one
    info, _ = sadj.sadj_describe_wave3d_plan(1, 4, 70, 9, 1 << 17, with_tiles=False)
    assert (info["ntx"], info["nty"], info["tiles_a"], info["workgroups"]) == (2, 1, 0, 256)
    # 512^3: two chunks of every tile fill the chip exactly; nothing is left over
    info, _ = sadj.sadj_describe_wave3d_plan(1, 4, 512, 512, 512, with_tiles=False)
    assert (info["tiles_a"], info["ntz"], info["workgroups"]) == (0, 2, 256)


def test_pointer_check_rejects_memory_the_device_cannot_use():
    """sadj_check_array on pageable host memory, and an entry point with "check.pointers"
    on: a status comes back and nothing is launched (holds with or without a GPU)."""
    import numpy as np
    a = np.zeros(1024)
    assert sadj.sadj_check_array(a.ctypes.data, a.nbytes) == 5
    assert sadj.sadj_check_array(0, 8) == 1
    bufs = [np.zeros(4096) for _ in range(3)]
    lib = sadj.load()
    sadj.set_option("check.pointers", 1)
    try:
        st = lib.sadj_adjoint_wave1d(1, 4096, bufs[0].ctypes.data, bufs[1].ctypes.data, bufs[2].ctypes.data, None, None)
    finally:
        sadj.set_option("check.pointers", 0)
    assert st == 5


def test_gather_kernels_use_no_atomics():
    """The method's point (Sections 1, 3.2): every u_bar element has exactly one writer, so
    no kernel of the method may contain an atomic; only the contrast kernel does."""
    import glob
    offenders = []
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_1907_02818_amd", "csrc", "*.h*")) +
                       [os.path.join(ROOT, "include", "sadj_stencil1d.hpp")]):
        code = re.sub(r"//.*|/\*.*?\*/", "", open(path).read(), flags=re.S)
        if re.search(r"atomic(?!<long>)", code, flags=re.I) and not path.endswith("wave3d_scatter_atomic.hip"):
            if os.path.basename(path) == "api.hip" and not re.search(r"atomicAdd|unsafeAtomic|__atomic|atomic_fetch", code):
                continue                               # std::atomic<long> option variables on the host
            offenders.append(os.path.basename(path))
    assert offenders == []


def test_a_row_chunk_option_that_needs_too_many_chunks_is_refused_before_any_launch():
    lib = sadj.load()
    sadj.set_option("wave2d.variant", 1)          # the strip march is the form that cuts y into chunks
    sadj.set_option("wave2d.ychunk", 1)
    try:
        rc = lib.sadj_adjoint_wave2d(1, 64, 70000, A, B, C_, None, None)
        assert rc == 4
        rc = lib.sadj_primal_wave2d(1, 64, 70000, A, B, C_, D_, None)
        assert rc == 4
    finally:
        sadj.set_option("wave2d.ychunk", 0)
        sadj.set_option("wave2d.variant", 0)


def test_plan_description_follows_the_shape_the_launch_takes():
    # fp64: 64 x 32 tiles with and without u_prev_bar; an odd nx takes the one-cell shape (64 x 32);
    # rows that are not cache-line multiples take 16-row tiles of 1 KB (radius 4) or 256 cells (radius 1)
    for prev in (False, True):
        info, _ = sadj.sadj_describe_wave3d_plan(1, 4, 512, 512, 512, with_tiles=False, with_u_prev_bar=prev)
        assert (info["tile_w"], info["tile_h"]) == (64, 32)
    info, _ = sadj.sadj_describe_wave3d_plan(0, 4, 512, 512, 512, with_tiles=False)
    assert (info["tile_w"], info["tile_h"]) == (128, 32)
    info, _ = sadj.sadj_describe_wave3d_plan(1, 4, 1000, 1000, 100, with_tiles=False)
    assert (info["tile_w"], info["tile_h"]) == (128, 16)
    info, _ = sadj.sadj_describe_wave3d_plan(1, 1, 1000, 1000, 100, with_tiles=False)
    assert (info["tile_w"], info["tile_h"]) == (256, 16)
    info, _ = sadj.sadj_describe_wave3d_plan(1, 4, 1001, 1000, 100, with_tiles=False)
    assert (info["tile_w"], info["tile_h"]) == (64, 32)


def test_wave_sweep_plan_ends_in_the_documented_buffers():
    """Host logic of sadj_adjoint_wave3d_steps_fused: whatever mix of fused pairs and single steps
    the plan holds, every launch writes to buffers it does not read, the steps add up, and the
    sweep ends with lam^{K+1-n} in buffer n%3 and lam^{K-n} in buffer (n+1)%3."""
    import paper_1907_02818_amd as lib
    lib.load()
    for n in list(range(0, 80)) + [1000, 1001, 1002, 1003, 1004, 1005, 12345678]:
        body, tail = lib.sadj_describe_wave3d_sweep(n)
        if n < 3:
            assert body == -1 and tail == []
            continue
        assert body >= 0
        a, b = (1, 2) if body % 2 == 0 else (0, 3)         # the body alternates (1,2) -> (0,3) -> (1,2)
        steps = 1 + 2 * body
        for pair, la, lb, o0, o1 in tail:
            assert (la, lb) == (a, b)
            if pair:
                assert len({la, lb, o0, o1}) == 4
                a, b = o0, o1
                steps += 2
            else:
                assert o0 not in (la, lb) and 0 <= o0 <= 3
                a, b = lb, o0
                steps += 1
        assert steps == n
        assert (a, b) == (n % 3, (n + 1) % 3)
        assert n - 1 - 2 * (body + sum(t[0] for t in tail)) <= 3      # at most three unfused steps after the first
