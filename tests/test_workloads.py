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


def test_power_law_graph_and_csr_sampler():
    N = 100_000
    offsets, ids = workloads.zipf_graph_csr(N, 50, 25, 0.6, 9)
    assert offsets.dtype == np.int64 and ids.dtype == np.int64 and offsets[0] == 0
    deg = np.diff(offsets)
    assert deg.min() == 25 and abs(deg.mean() - 50) < 0.05 and deg.max() > 10_000       # floor, mean, heavy head
    assert ids.min() >= 0 and ids.max() < N and ids.size == offsets[-1]
    # degree follows popularity rank: the most popular node has the largest degree
    hot = workloads.hottest_nodes(N, 100, 9)
    assert len(set(hot.tolist())) == 100 and deg[hot[0]] == deg.max()
    assert (np.diff(deg[hot]) <= 0).all()
    # popular nodes are named more often as neighbours
    counts = np.bincount(ids, minlength=N)
    assert counts[hot[:10]].mean() > 50 * counts.mean()
    a = workloads.sample_csr(offsets, ids, 64, (25, 10), 5, 0)
    b = workloads.sample_csr(offsets, ids, 64, (25, 10), 5, 0)
    c = workloads.sample_csr(offsets, ids, 64, (25, 10), 5, 1)
    assert np.array_equal(a, b) and not np.array_equal(a[:64], c[:64])                 # deterministic per (seed, batch)
    assert len(np.unique(a)) == a.size and a.size <= workloads.slot_bound(64, (25, 10))
    assert a.min() >= 0 and a.max() < N and a.size > 5_000
    # every ID after the seeds is a neighbour of an earlier ID (first-occurrence order, seeds first)
    nbrs = set()
    for v in a[:64]:
        nbrs.update(ids[offsets[v]:offsets[v + 1]].tolist())
    assert set(a[64:64 + 200].tolist()) <= nbrs | set(a[:64].tolist())


def test_procedural_sampler():
    N = 5_000_000
    a = workloads.sample_procedural(N, 30, 0.8, 4, 128, (15, 10, 5), 44, 0)
    b = workloads.sample_procedural(N, 30, 0.8, 4, 128, (15, 10, 5), 44, 0)
    assert np.array_equal(a, b) and len(np.unique(a)) == a.size
    assert a.min() >= 0 and a.max() < N and 20_000 < a.size <= workloads.slot_bound(128, (15, 10, 5))
    # the skew shows: the hottest 1 % of nodes take far more than 1 % of the batch
    hot = set(workloads.hottest_nodes(N, N // 100, 4).tolist())
    share = sum(int(v in hot) for v in a.tolist()) / a.size
    assert share > 0.10
