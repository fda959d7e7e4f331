"""Host-only checks of the seeded input generators (no GEMM arithmetic involved)."""
import numpy as np

from paper_1904_03383_amd import inputgen as ig


def test_uniform_grid_range_and_determinism():
    u = ig.uniform(11, (257, 129))
    assert u.dtype == np.float32 and u.shape == (257, 129)
    assert u.min() >= -1.0 and u.max() < 1.0
    # every value sits on the 2^-23 grid, hence is an exact fp32
    scaled = u.astype(np.float64) * 2.0 ** 23
    assert np.array_equal(scaled, np.round(scaled))
    assert np.array_equal(u, ig.uniform(11, (257, 129)))
    assert not np.array_equal(u, ig.uniform(12, (257, 129)))
    assert abs(float(u.mean())) < 0.02 and abs(float(u.std()) - 1 / np.sqrt(3)) < 0.02


def test_counter_based_subranges():
    full = ig.uniform(5, (1000,))
    assert np.array_equal(full[123:456], ig.uniform(5, (333,), start=123))
    fulln = ig.normal(5, (1000,))
    assert np.array_equal(fulln[900:], ig.normal(5, (100,), start=900))


def test_small_int_values():
    v = ig.small_int(3, (90000,))
    assert v.dtype == np.float32
    assert set(np.unique(v).tolist()) == {float(x) for x in range(-4, 5)}
    counts = np.bincount((v + 4).astype(np.int64), minlength=9)
    assert counts.min() > 9000 and counts.max() < 11000


def test_normal_moments():
    z = ig.normal(7, (400, 500)).astype(np.float64)
    assert np.isfinite(z).all()
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1.0) < 0.01
    assert abs(((z - z.mean()) ** 3).mean()) < 0.03           # skewness
    assert abs((z ** 4).mean() - 3.0) < 0.1                    # kurtosis


def test_named_configs():
    assert list(ig.CONFIGS) == ["c1_256x256x32", "c2_1024", "c3_batched_512x32x32x64",
                                "c4_4096x4096x128", "c5_4096"]
    a, b = ig.make_config("c1_256x256x32")
    assert a.shape == (1, 256, 32) and b.shape == (1, 32, 256)
    ai, bi = ig.make_config("c1_256x256x32", dist="int")
    assert np.abs(ai).max() <= 4 and np.array_equal(ai, np.round(ai))
    a3, b3 = ig.make_config("c3_batched_512x32x32x64")
    assert a3.shape == (512, 32, 64) and b3.shape == (512, 64, 32)
    assert a3.flags.c_contiguous and b3.flags.c_contiguous
    assert ig.config_seeds("c5_4096") == (1005, 2005)
