"""The seeded input generators: deterministic, prefix-stable, and of the stated distributions."""
import numpy as np

import workloads


def test_deterministic_and_prefix_stable():
    a = workloads.normal(64, 256, seed=11)
    b = workloads.normal(64, 256, seed=11)
    c = workloads.normal(16, 256, seed=11)
    d = workloads.normal(64, 256, seed=12)
    assert np.array_equal(a, b)
    assert np.array_equal(a[:16], c)
    assert not np.array_equal(a, d)


def test_distributions_have_the_stated_moments():
    x = workloads.normal(2000, 256, seed=1)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    u = workloads.uniform(2000, 256, seed=2)
    assert u.min() >= -1.0 and u.max() <= 1.0 and abs(u.mean()) < 0.01 and abs(u.var() - 1 / 3) < 0.01
    l = workloads.laplace(2000, 256, seed=4)
    assert abs(l.mean()) < 0.02 and abs(l.var() - 2.0) < 0.05
    s = workloads.normal(4000, 256, seed=1, row_scale=(0.5, 2.0))
    row_std = s.std(axis=1)
    assert 0.4 < row_std.min() < 0.6 and 1.8 < row_std.max() < 2.3


def test_ties_variant_snaps_the_stated_fraction_to_shared_levels():
    t = workloads.normal_ties(2000, 256, seed=3)
    levels = (-3.0 + 0.4 * np.arange(16)).astype(np.float32)
    frac = np.isin(t, levels).mean()
    assert 0.045 < frac < 0.055
    # ties do occur inside rows
    assert np.mean([len(np.unique(r)) < r.size for r in t]) > 0.5


def test_named_configs_have_the_stated_shapes():
    for name, cfg in workloads.CONFIGS.items():
        x = workloads.make(name, N=8)
        assert x.shape == (8, cfg["M"]) and x.dtype == np.float32 and np.isfinite(x).all()
