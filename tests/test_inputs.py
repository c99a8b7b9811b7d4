"""The seeded input generator: reproducible, chunk-independent, in range."""
import numpy as np
import pytest

import inputs

MASK = (1 << 64) - 1


def _mix_int(z):
    z &= MASK
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & MASK
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & MASK
    z ^= z >> 31
    return z


def _unit_int(seed, stream, k):
    """Python big-integer twin of inputs.unit for one counter."""
    golden = 0x9E3779B97F4A7C15
    key = _mix_int(seed * golden + _mix_int(stream))
    return (_mix_int(key + k * golden) >> 11) * 2.0 ** -53


@pytest.mark.parametrize("seed,stream", [(0, 1), (7, 3), (123456789, 10)])
def test_unit_matches_bigint_twin(seed, stream):
    got = inputs.unit(seed, stream, 50)
    want = np.array([_unit_int(seed, stream, k) for k in range(50)])
    assert np.array_equal(got, want)


def test_unit_is_counter_based():
    a = inputs.unit(3, 2, (1 << 22) + 1000)
    b = inputs.unit(3, 2, 1000, start=(1 << 22))
    assert np.array_equal(a[1 << 22:], b)
    assert 0.0 <= a.min() and a.max() < 1.0
    assert abs(a.mean() - 0.5) < 2e-3


def test_streams_differ_and_seeds_differ():
    a = inputs.uniform(0, "u", (1000,), -1, 1)
    assert not np.array_equal(a, inputs.uniform(0, "r_bar", (1000,), -1, 1))
    assert not np.array_equal(a, inputs.uniform(1, "u", (1000,), -1, 1))
    assert np.array_equal(a, inputs.uniform(0, "u", (1000,), -1, 1))


def test_wave_fields_ranges_and_layering():
    d = inputs.config_inputs("wave3d_r4", shape=(64, 12, 10))
    for k in ("u", "u_prev", "r_bar", "u_bar", "u_prev_bar"):
        assert d[k].shape == (64, 12, 10) and d[k].min() >= -1 and d[k].max() < 1
    c = d["c"]
    assert c.min() >= 0.01 and c.max() <= 0.1
    # layered in z: constant within a plane, several distinct layers
    assert np.all(c == c[:, :1, :1])
    assert len(np.unique(c[:, 0, 0])) > 4
    d2 = inputs.config_inputs("wave2d", shape=(256, 16))
    assert np.all(d2["c"] == d2["c"][:, :1])
    assert d2["c"].min() >= 0.01 and d2["c"].max() <= 0.2


def test_fp32_is_rounded_fp64():
    d64 = inputs.config_inputs("wave3d_r4", shape=(9, 9, 9), c_mode="iid")
    d32 = inputs.config_inputs("wave3d_r4", shape=(9, 9, 9), c_mode="iid", dtype=np.float32)
    for k in d64:
        assert d32[k].dtype == np.float32
        assert np.array_equal(d32[k], d64[k].astype(np.float32))


def test_burgers_profile_changes_sign_and_is_bounded():
    d = inputs.burgers_inputs(4096)
    u = d["u"]
    assert u.min() > -1 and u.max() < 1
    assert (u > 0.2).sum() > 500 and (u < -0.2).sum() > 500
    assert set(d) == {"u", "r_bar", "u_bar"}


def test_planes_of_a_field_can_be_generated_on_their_own():
    shape = (9, 6, 5)
    full = inputs.uniform(11, "r_bar", shape, -1.0, 1.0)
    for z0, k in ((0, 1), (3, 4), (8, 1)):
        assert np.array_equal(inputs.uniform_planes(11, "r_bar", shape, -1.0, 1.0, z0, k), full[z0:z0 + k])
