"""Pins for the CPU oracle: every check compares it with something the paper
or the mathematics fixes, never with itself."""
import math
import os
import sys

import numpy as np
import pytest

import oracle
import workloads

EPS = 2.0 ** -52


# ---------------------------------------------------------------- reflector
@pytest.mark.parametrize("n", [2, 3, 17, 64])
@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_householder_matches_algorithm3_closed_form(n, sign):
    # Algorithm 3 (GEQRT): x = alpha + sign(alpha)*sqrt(alpha^2+|tail|^2),
    # tau_hat = 2 x^2 / (x^2 + |tail|^2), v = (1, tail/x), H a = -sign(alpha)|a| e1.
    a = workloads.normal(7 + n, 0, n)
    a[0] = sign * abs(a[0])
    beta, v, tau = oracle.householder(a)
    t2 = float(np.dot(a[1:], a[1:]))
    x = a[0] + math.copysign(math.sqrt(a[0] ** 2 + t2), a[0])
    tau_hat = 2 * x * x / (x * x + t2)
    assert abs(tau - tau_hat) <= 8 * EPS * tau_hat
    assert 1.0 <= tau <= 2.0
    np.testing.assert_allclose(v[1:], a[1:] / x, rtol=16 * EPS, atol=0)
    assert abs(beta - (-math.copysign(np.linalg.norm(a), a[0]))) <= 8 * EPS * abs(beta)
    h = np.eye(n) - tau * np.outer(v, v)
    np.testing.assert_allclose(h @ h.T, np.eye(n), atol=32 * EPS)
    ha = h @ a
    assert abs(ha[0] - beta) <= 16 * EPS * abs(beta)
    assert np.abs(ha[1:]).max() <= 16 * EPS * abs(beta)


def test_householder_zero_tail_is_identity():
    beta, v, tau = oracle.householder(np.array([3.0, 0.0, 0.0]))
    assert tau == 0.0 and beta == 3.0


# --------------------------------------------------------- bidiagonal solver
@pytest.mark.parametrize("n", [1, 2, 3, 10, 257, 1000])
def test_bdsvals_ones_bidiagonal_closed_form(n):
    # B^T B = tridiag(1, [1,2,...,2], 1) has eigenvalues 4 cos^2(k pi/(2n+1)).
    s = oracle.bdsvals(np.ones(n), np.ones(n - 1))
    k = np.arange(1, n + 1)
    ref = 2.0 * np.cos(k * np.pi / (2 * n + 1))
    np.testing.assert_allclose(s, ref, rtol=0, atol=8 * EPS * 2.0)


def test_bdsvals_2x2_closed_form():
    for (d0, d1, e0) in [(3.0, 4.0, 1.0), (1e-3, 2.0, 5.0), (-2.0, 0.5, -7.0), (1.0, 1.0, 0.0)]:
        s = oracle.bdsvals([d0, d1], [e0])
        f2 = d0 * d0 + d1 * d1 + e0 * e0
        det = abs(d0 * d1)
        big = math.sqrt((f2 + math.sqrt(max(f2 * f2 - 4 * det * det, 0.0))) / 2)
        small = det / big
        assert abs(s[0] - big) <= 8 * EPS * big
        assert abs(s[1] - small) <= 8 * EPS * big


def test_bdsvals_diagonal_and_signs():
    d = np.array([0.5, -3.0, 2.0, 0.0, -1e-8])
    s = oracle.bdsvals(d, np.zeros(4))
    np.testing.assert_allclose(s, np.sort(np.abs(d))[::-1], rtol=4 * EPS, atol=1e-30)
    # flipping signs of d and e never changes singular values
    dd = workloads.normal(3, 0, 50)
    ee = workloads.normal(4, 0, 49)
    s1 = oracle.bdsvals(dd, ee)
    s2 = oracle.bdsvals(-dd, np.abs(ee))
    np.testing.assert_allclose(s1, s2, rtol=0, atol=8 * EPS * s1[0])


def test_bdsvals_transposed_order_and_scaling():
    # sigma(B) = sigma(B^T): reversing d and e gives the lower bidiagonal's transpose.
    dd = workloads.normal(5, 0, 40)
    ee = workloads.normal(6, 0, 39)
    s1 = oracle.bdsvals(dd, ee)
    s2 = oracle.bdsvals(dd[::-1].copy(), ee[::-1].copy())
    np.testing.assert_allclose(s1, s2, rtol=0, atol=8 * EPS * s1[0])
    s3 = oracle.bdsvals(1e150 * dd, 1e150 * ee)
    np.testing.assert_allclose(s3 / 1e150, s1, rtol=0, atol=8 * EPS * s1[0])
    b = np.diag(dd) + np.diag(ee, 1)
    np.testing.assert_allclose(s1, np.linalg.svd(b, compute_uv=False), rtol=0, atol=32 * EPS * s1[0])


def test_bdsvals_empty_and_zero():
    assert oracle.bdsvals([], []).size == 0
    np.testing.assert_array_equal(oracle.bdsvals([0.0, 0.0], [0.0]), [0.0, 0.0])


# ------------------------------------------------------- bidiagonalisation
def _rebuild(f, tq, tp):
    m, n = f.shape
    u = np.eye(m)
    for k in range(n):
        v = np.zeros(m)
        v[k] = 1.0
        v[k + 1:] = f[k + 1:, k]
        u = u - tq[k] * np.outer(u @ v, v)
    vm = np.eye(n)
    for k in range(n - 1):
        w = np.zeros(n)
        if k + 1 < n:
            w[k + 1] = 1.0
            w[k + 2:] = f[k, k + 2:]
        vm = vm - tp[k] * np.outer(vm @ w, w)
    return u, vm


@pytest.mark.parametrize("m,n", [(1, 1), (2, 2), (3, 3), (12, 12), (33, 33), (40, 17)])
def test_bidiagonalize_factorisation(m, n):
    a = workloads.gaussian_matrix(11 + m + n, m, n)
    d, e, f, tq, tp = oracle.bidiagonalize(a)
    u, v = _rebuild(f, tq, tp)
    b = np.zeros((m, n))
    b[np.arange(n), np.arange(n)] = d
    if n > 1:
        b[np.arange(n - 1), np.arange(1, n)] = e
    nrm = np.linalg.norm(a)
    assert np.linalg.norm(u.T @ u - np.eye(m)) <= 50 * m * EPS
    assert np.linalg.norm(v.T @ v - np.eye(n)) <= 50 * n * EPS
    assert np.linalg.norm(a - u @ b @ v.T) <= 50 * m * EPS * nrm
    assert abs(np.sum(d * d) + np.sum(e * e) - nrm ** 2) <= 50 * m * EPS * nrm ** 2


# ----------------------------------------------------------------- whole
def test_svdvals_diagonal_matrix():
    dd = np.array([3.0, -7.0, 0.25, 0.0, 1e-5, -2.0])
    s = oracle.svdvals(np.diag(dd))
    np.testing.assert_allclose(s, np.sort(np.abs(dd))[::-1], rtol=0, atol=8 * EPS * 7.0)


@pytest.mark.parametrize("kind", ["arithmetic", "geometric", "quartercircle", "clustered"])
@pytest.mark.parametrize("n", [16, 96])
def test_svdvals_prescribed_spectrum(kind, n):
    # the paper's accuracy protocol: A = U Sigma V^T with Haar U, V and known Sigma
    sig = workloads.spectrum(kind, n, 99, smin=1e-3)
    a = workloads.haar_matrix(1234 + n, n, sig)
    s = oracle.svdvals(a)
    assert np.abs(s - sig).max() <= 20 * n * EPS * sig[0]


def test_svdvals_rank_one():
    u = workloads.normal(21, 0, 30)
    v = workloads.normal(22, 0, 30)
    s = oracle.svdvals(np.outer(u, v))
    s1 = np.linalg.norm(u) * np.linalg.norm(v)
    assert abs(s[0] - s1) <= 30 * EPS * s1
    assert s[1:].max() <= 30 * 30 * EPS * s1


@pytest.mark.parametrize("n", [2, 5, 16])
def test_svdvals_frobenius_and_determinant(n):
    a = workloads.gaussian_matrix(31 + n, n, n)
    s = oracle.svdvals(a)
    assert abs(np.sum(s * s) - np.sum(a * a)) <= 20 * n * EPS * np.sum(a * a)
    det = abs(np.linalg.det(a))          # LU route, independent of the oracle
    assert abs(np.prod(s) - det) <= 1e3 * n * EPS * max(det, 1e-300) * (s[0] / s[-1])


def _jacobi_eigs(sym):
    """Cyclic Jacobi eigenvalues of a small symmetric matrix (brute force)."""
    s = sym.copy()
    n = s.shape[0]
    for _ in range(60):
        off = math.sqrt(max(np.sum(s * s) - np.sum(np.diag(s) ** 2), 0.0))
        if off <= 1e-18 * np.linalg.norm(s):
            break
        for p in range(n - 1):
            for q in range(p + 1, n):
                if s[p, q] == 0.0:
                    continue
                theta = (s[q, q] - s[p, p]) / (2 * s[p, q])
                t = math.copysign(1.0, theta) / (abs(theta) + math.sqrt(theta * theta + 1))
                c = 1 / math.sqrt(t * t + 1)
                sn = t * c
                g = np.eye(n)
                g[p, p] = c
                g[q, q] = c
                g[p, q] = sn
                g[q, p] = -sn
                s = g.T @ s @ g
    return np.sort(np.diag(s))[::-1]


@pytest.mark.parametrize("n", [1, 2, 3, 6, 8])
def test_svdvals_vs_jacobi_on_gram_matrix(n):
    a = workloads.gaussian_matrix(41 + n, n, n)
    lam = _jacobi_eigs(a.T @ a)
    s = oracle.svdvals(a)
    np.testing.assert_allclose(s * s, np.maximum(lam, 0), rtol=0, atol=200 * n * EPS * lam[0])


def _one_sided_jacobi(a):
    """Hestenes one-sided Jacobi: column norms of A after orthogonalising columns."""
    g = a.copy()
    n = g.shape[1]
    for _ in range(40):
        rot = 0
        for p in range(n - 1):
            for q in range(p + 1, n):
                apq = g[:, p] @ g[:, q]
                app = g[:, p] @ g[:, p]
                aqq = g[:, q] @ g[:, q]
                if abs(apq) <= 1e-17 * math.sqrt(app * aqq):
                    continue
                rot += 1
                zeta = (aqq - app) / (2 * apq)
                t = math.copysign(1.0, zeta) / (abs(zeta) + math.sqrt(1 + zeta * zeta))
                c = 1 / math.sqrt(1 + t * t)
                sn = c * t
                gp = c * g[:, p] - sn * g[:, q]
                gq = sn * g[:, p] + c * g[:, q]
                g[:, p], g[:, q] = gp, gq
        if rot == 0:
            break
    return np.sort(np.linalg.norm(g, axis=0))[::-1]


@pytest.mark.parametrize("n", [12, 48])
def test_svdvals_vs_one_sided_jacobi(n):
    a = workloads.gaussian_matrix(51 + n, n, n)
    ref = _one_sided_jacobi(a)
    s = oracle.svdvals(a)
    np.testing.assert_allclose(s, ref, rtol=0, atol=50 * n * EPS * ref[0])


def test_svdvals_invariances():
    n = 40
    a = workloads.gaussian_matrix(61, n, n)
    s = oracle.svdvals(a)
    np.testing.assert_allclose(oracle.svdvals(a.T), s, rtol=0, atol=20 * n * EPS * s[0])
    np.testing.assert_allclose(oracle.svdvals(-2.5 * a), 2.5 * s, rtol=0, atol=50 * n * EPS * s[0])
    q1 = workloads.haar_orthogonal(62, n)
    q2 = workloads.haar_orthogonal(63, n)
    np.testing.assert_allclose(oracle.svdvals(q1 @ a @ q2), s, rtol=0, atol=50 * n * EPS * s[0])


@pytest.mark.parametrize("m,n", [(300, 300), (257, 129), (64, 1)])
def test_svdvals_vs_library(m, n):
    # a special case that reduces to a library routine (LAPACK through numpy)
    a = workloads.gaussian_matrix(71 + m, m, n)
    s = oracle.svdvals(a)
    ref = np.linalg.svd(a, compute_uv=False)
    np.testing.assert_allclose(s, ref, rtol=0, atol=10 * m * EPS * ref[0])


def test_svdvals_iid_statistics():
    # iid N(0,1/n): sum sigma^2 ~ n, sigma_max -> 2, spectrum follows the
    # quarter-circle law on [0,2] (the paper's third test distribution)
    n = 400
    a = workloads.gaussian_matrix(81, n, n, scale=1 / math.sqrt(n))
    s = oracle.svdvals(a)
    assert abs(np.sum(s * s) / n - 1.0) < 0.02
    assert 1.85 < s[0] < 2.1
    x = np.sort(s) / 2.0
    cdf = (2 / np.pi) * (x * np.sqrt(np.clip(1 - x * x, 0, 1)) + np.arcsin(np.clip(x, 0, 1)))
    emp = (np.arange(n) + 0.5) / n
    assert np.abs(cdf - emp).max() < 0.03


def test_svdvals_config1_matches_library_and_golden():
    a, info = workloads.make("c1")
    s = oracle.svdvals(a)
    ref = np.linalg.svd(np.asarray(a, dtype=np.float64), compute_uv=False)
    assert np.abs(s - ref).max() <= 10 * info["n"] * EPS * ref[0]
    _against_stored("c1", a, s)


def _against_stored(name, a, s):
    # the stored oracle result of the same workload (tests/golden, written by make_oracle_sigma.py):
    # the generator still produces the matrix the file was written for, and the oracle the same values
    sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden"))
    import make_oracle_sigma as golden
    stored = golden.load(name)
    assert stored is not None
    sig, meta = stored
    assert workloads.fingerprint_matches(meta["fingerprint"], workloads.fingerprint(a))
    assert np.abs(s - sig).max() <= 1e-12 * sig[0]


def test_svdvals_config2_matches_prescription_and_golden():
    a, info = workloads.make("c2")
    s = oracle.svdvals(a)
    assert np.abs(s - info["sigma"]).max() <= 10 * info["n"] * 2.0 ** -23 * info["sigma"][0]
    _against_stored("c2", a, s)
