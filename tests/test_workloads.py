import math

import numpy as np

import workloads


def test_streams_are_windowable_and_normal():
    z = workloads.normal(5, 0, 10001)
    np.testing.assert_array_equal(z[37:137], workloads.normal(5, 37, 100))
    np.testing.assert_array_equal(z[38:41], workloads.normal(5, 38, 3))
    assert abs(z.mean()) < 0.05 and abs(z.std() - 1) < 0.05
    assert not np.array_equal(z[:100], workloads.normal(6, 0, 100))


def test_gaussian_matrix_blocks_agree():
    a = workloads.gaussian_matrix(9, 33, 70, col_block=16)
    b = workloads.gaussian_matrix(9, 33, 70, col_block=512)
    np.testing.assert_array_equal(a, b)
    assert a.flags.f_contiguous


def test_haar_is_orthogonal():
    q = workloads.haar_orthogonal(3, 50)
    assert np.abs(q.T @ q - np.eye(50)).max() < 1e-13


def test_spectra_shapes():
    for kind in ["geometric", "uniform", "arithmetic", "quartercircle", "clustered"]:
        s = workloads.spectrum(kind, 64, 1, smin=1e-3)
        assert s.shape == (64,) and np.all(np.diff(s) <= 0) and s[0] <= 1.0 + 2e-4 and s[-1] >= 0
    s = workloads.spectrum("geometric", 1024, 1, smin=1e-3)
    assert s[0] == 1.0 and abs(s[-1] - 1e-3) < 1e-15
    s = workloads.spectrum("clustered", 8192, 1)
    for k in range(8):
        blk = s[k * 1024:(k + 1) * 1024]
        assert np.all(np.abs(blk / 10 ** (-k / 2) - 1) <= 1e-4 * (1 + 1e-12))


def test_make_small_variants_and_fingerprint():
    a, info = workloads.make("c4", n=128)
    assert a.dtype == np.float32 and a.shape == (128, 128) and info["sigma"].size == 128
    f1 = workloads.fingerprint(a)
    assert workloads.fingerprint_matches(f1, workloads.fingerprint(a.copy()))
    b = a.copy()
    b[:, 3] *= 1.01
    assert not workloads.fingerprint_matches(f1, workloads.fingerprint(b))
    a1, info1 = workloads.make("c1")
    assert a1.dtype == np.float64 and info1["nb"] == 32
    assert abs(np.sum(a1.astype(np.float64) ** 2) / 256 ** 2 - 1) < 0.02
