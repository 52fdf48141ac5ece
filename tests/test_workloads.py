"""Checks of the seeded input generators (no GPU)."""
import numpy as np

import workloads


def test_uniform_fill_is_reproducible_in_range_and_position_addressable():
    a = workloads.uniform_f32(1, 100, 37)
    b = workloads.uniform_f32(1, 100, 37)
    assert np.array_equal(a, b) and a.min() >= -1.0 and a.max() < 1.0
    assert abs(float(a.mean())) < 0.05
    L = workloads.lib()
    for e in (0, 1, 36, 37, 3699):
        assert a.ravel()[e] == np.float32(L.wl_uniform_f32_at(1, e))
    assert not np.array_equal(a, workloads.uniform_f32(2, 100, 37))
    # a wider view of the same stream shares its prefix
    c = workloads.uniform_f32(1, 10, 370)
    assert np.array_equal(c.ravel(), a.ravel())


def test_normal_fp16_fill_matches_numpy_rounding_statistics():
    h = workloads.normal_f16(5, 2000, 602)
    f = h.astype(np.float32)
    assert abs(float(f.mean())) < 0.01 and abs(float(f.std()) - 1.0) < 0.01
    assert np.isfinite(f).all()
    L = workloads.lib()
    assert h.ravel()[12345].view(np.uint16) == L.wl_normal_f16_at(5, 12345)


def test_fp32_to_fp16_rounding_matches_numpy():
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(50000) * 10.0 ** rng.integers(-9, 6, 50000)).astype(np.float32)
    x = np.concatenate([x, np.array([0.0, -0.0, 65504.0, 65519.99, 65520.0, 2.0**-24, 2.0**-25,
                                     2.0**-25 * 1.0001, 6.1e-5, np.inf, -np.inf], dtype=np.float32)])
    L = workloads.lib()
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([L.wl_f32_to_f16_rne(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_uniform_indices_cover_the_range():
    for dt in (np.int64, np.int32):
        i = workloads.indices_uniform(0, 100000, 1000, dt)
        assert i.dtype == dt and i.min() == 0 and i.max() == 999
        counts = np.bincount(i, minlength=1000)
        assert counts.min() > 50 and counts.max() < 160
