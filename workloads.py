"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module holds no arithmetic of the singular value method itself: it only
synthesises matrices (and the spectra they are built from) with the shapes and
value distributions of the paper's workloads (square matrices, either i.i.d.
Gaussian entries or U diag(sigma) V^T with Haar-distributed orthogonal factors
and a prescribed spectrum; accuracy protocol of the paper's "Accuracy"
paragraph, Section 3.2).  Both the CPU oracle's tests and the HIP path's tests
draw their inputs from here; neither of the two implementations imports the
other.

Random numbers come from a counter-based generator (a SplitMix64 finaliser
applied to seed and element index, followed by a Box-Muller transform), so
any block of any matrix can be produced independently and the same numbers
are produced on every machine up to the last-bit behaviour of log/sin/cos.
"""
from __future__ import annotations

import numpy as np

SEED0 = 250806339

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

# name -> recipe.  "dtype" is the storage type handed to the library.
CONFIGS = {
    # 256x256 fp64, iid N(0,1), nb=32
    "c1": dict(n=256, dtype="f64", nb=32, kind="iid", var=1.0, seed_id=1),
    # 1024x1024 fp32, Haar U,V, sigma geometric 1 .. 1e-3, nb=32
    "c2": dict(n=1024, dtype="f32", nb=32, kind="haar", spectrum="geometric",
               smin=1e-3, seed_id=2),
    # 4096x4096 fp64, iid N(0,1/n), nb=64
    "c3a": dict(n=4096, dtype="f64", nb=64, kind="iid", var="1/n", seed_id=31),
    # 4096x4096 fp16 storage, Haar U,V, sigma uniform in [1e-2,1], nb=64
    "c3b": dict(n=4096, dtype="f16", nb=64, kind="haar", spectrum="uniform",
                smin=1e-2, seed_id=32),
    # 8192x8192 fp32, Haar U,V, 8 clusters of 1024, centres 10^(-k/2), nb=64
    "c4": dict(n=8192, dtype="f32", nb=64, kind="haar", spectrum="clustered",
               seed_id=4),
    # 32768x32768 fp32 iid N(0,1/n), nb=128
    "c5a": dict(n=32768, dtype="f32", nb=128, kind="iid", var="1/n", seed_id=51),
    # 16384x16384 fp64 iid N(0,1/n), nb=128
    "c5b": dict(n=16384, dtype="f64", nb=128, kind="iid", var="1/n", seed_id=52),
}

NP_DTYPE = {"f64": np.float64, "f32": np.float32, "f16": np.float16}
EPS = {"f64": 2.0 ** -52, "f32": 2.0 ** -23, "f16": 2.0 ** -10}


def config_seed(seed_id: int) -> int:
    return SEED0 + 1000 * int(seed_id)


def _mix(x: np.ndarray) -> np.ndarray:
    x = (x ^ (x >> np.uint64(30))) * _M1
    x = (x ^ (x >> np.uint64(27))) * _M2
    return x ^ (x >> np.uint64(31))


def uniform01(seed: int, start: int, count: int) -> np.ndarray:
    """count uniforms in [0,1) for stream positions start .. start+count-1."""
    with np.errstate(over="ignore"):
        idx = np.arange(start, start + count, dtype=np.uint64)
        key = _mix(np.uint64(seed) * _GOLDEN + np.uint64(0x632BE59BD9B4E019))
        bits = _mix(_mix(idx * _GOLDEN + key) ^ key)
    return (bits >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def normal(seed: int, start: int, count: int) -> np.ndarray:
    """count standard normals for stream positions start .. start+count-1.

    Position p uses the Box-Muller pair p//2, so any window of the stream can
    be generated on its own.
    """
    p0 = start // 2
    p1 = (start + count + 1) // 2
    u = uniform01(seed, 2 * p0, 2 * (p1 - p0))
    r = np.sqrt(-2.0 * np.log1p(-u[0::2]))
    ang = (2.0 * np.pi) * u[1::2]
    z = np.empty(2 * (p1 - p0), dtype=np.float64)
    z[0::2] = r * np.cos(ang)
    z[1::2] = r * np.sin(ang)
    off = start - 2 * p0
    return z[off:off + count]


def _pool_size(work_items: int) -> int:
    """Threads for the block-parallel loops below (numpy releases the interpreter lock
    inside its array kernels): one for small matrices, up to 16 for large ones."""
    import os
    if work_items < (1 << 24):
        return 1
    limit = int(os.environ.get("SVB_GEN_THREADS", "16"))   # 1: no thread pool (e.g. under a profiler)
    return max(1, min(limit, os.cpu_count() or 1))


def gaussian_matrix(seed: int, m: int, n: int, scale: float = 1.0,
                    out_dtype=np.float64, col_block: int = 512) -> np.ndarray:
    """m x n matrix, column-major (Fortran order), entry (i,j) = scale * z[i + j*m].

    Every entry depends on (seed, i + j*m) only, so the column blocks are produced
    independently (by a few threads for large matrices) with identical results."""
    a = np.empty((m, n), dtype=out_dtype, order="F")
    nthr = _pool_size(m * n)
    if nthr > 1:
        col_block = max(1, min(col_block, (1 << 22) // max(m, 1)))   # bounds the temporaries per thread

    def fill(j0):
        j1 = min(n, j0 + col_block)
        z = normal(seed, j0 * m, (j1 - j0) * m)
        a[:, j0:j1] = (scale * z).reshape((m, j1 - j0), order="F").astype(out_dtype)

    starts = range(0, n, col_block)
    if nthr == 1:
        for j0 in starts:
            fill(j0)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(nthr) as ex:
            list(ex.map(fill, starts))
    return a


def haar_orthogonal(seed: int, n: int) -> np.ndarray:
    """Haar-distributed orthogonal matrix: Q of the QR of a Gaussian matrix with
    the signs fixed so that R has a positive diagonal."""
    g = gaussian_matrix(seed, n, n)
    q, r = np.linalg.qr(g)
    s = np.sign(np.diag(r))
    s[s == 0] = 1.0
    return q * s[None, :]


def spectrum(kind: str, n: int, seed: int, smin: float = 0.0) -> np.ndarray:
    """Prescribed singular values, returned in descending order."""
    if kind == "geometric":          # 1 down to smin, constant ratio
        s = smin ** (np.arange(n) / max(n - 1, 1))
    elif kind == "uniform":          # iid uniform in [smin, 1]
        s = smin + (1.0 - smin) * uniform01(seed, 0, n)
    elif kind == "arithmetic":       # evenly spaced over (0,1]
        s = (np.arange(n, 0, -1)) / n
    elif kind == "quartercircle":    # quantiles of the quarter-circle law on [0,1]
        # density (4/pi) sqrt(1-x^2); invert the CDF by bisection on a grid
        p = (np.arange(n) + 0.5) / n
        lo = np.zeros(n)
        hi = np.ones(n)
        for _ in range(60):
            mid = 0.5 * (lo + hi)
            cdf = (2.0 / np.pi) * (mid * np.sqrt(1 - mid * mid) + np.arcsin(mid))
            lo = np.where(cdf < p, mid, lo)
            hi = np.where(cdf < p, hi, mid)
        s = 0.5 * (lo + hi)
    elif kind == "clustered":        # 8 equal clusters, centres 10^(-k/2), rel. spread 1e-4
        ncl = 8
        per = n // ncl
        u = 2.0 * uniform01(seed, 0, n) - 1.0
        centres = np.repeat(10.0 ** (-0.5 * np.arange(ncl)), per)
        if centres.size < n:
            centres = np.concatenate([centres, np.full(n - centres.size, centres[-1])])
        s = centres * (1.0 + 1e-4 * u)
    else:
        raise ValueError(f"unknown spectrum {kind!r}")
    return np.sort(np.asarray(s, dtype=np.float64))[::-1].copy()


def haar_matrix(seed: int, n: int, sigma: np.ndarray) -> np.ndarray:
    """A = U diag(sigma) V^T in fp64, column-major; U, V from streams seed, seed+1."""
    u = haar_orthogonal(seed, n)
    v = haar_orthogonal(seed + 1, n)
    a = (u * sigma[None, :]) @ v.T
    return np.asfortranarray(a)


def make(name: str, n: int | None = None, nb: int | None = None):
    """Build a workload.  Returns (A, info): A is column-major in the storage
    dtype of the config; info carries n, nb, dtype, seed and, for the
    prescribed-spectrum constructions, sigma (descending, fp64).

    n / nb override the config's size (same recipe, smaller matrix) so the
    parity tests can run the same distribution at sizes the oracle finishes
    in seconds."""
    cfg = dict(CONFIGS[name])
    if n is not None:
        cfg["n"] = int(n)
    if nb is not None:
        cfg["nb"] = int(nb)
    n = cfg["n"]
    seed = config_seed(cfg["seed_id"])
    dt = NP_DTYPE[cfg["dtype"]]
    info = dict(name=name, n=n, nb=cfg["nb"], dtype=cfg["dtype"], seed=seed, sigma=None)
    if cfg["kind"] == "iid":
        scale = 1.0 if cfg["var"] == 1.0 else 1.0 / np.sqrt(n)
        a = gaussian_matrix(seed, n, n, scale=scale, out_dtype=dt)
    else:
        sig = spectrum(cfg["spectrum"], n, seed + 2, cfg.get("smin", 0.0))
        a = np.asfortranarray(haar_matrix(seed, n, sig).astype(dt))
        info["sigma"] = sig
    return a, info


def fingerprint(a: np.ndarray) -> dict:
    """A tolerance-comparable summary of a matrix (sum, sum of squares and a
    few fixed entries) used to decide whether a stored oracle result belongs
    to the matrix at hand."""
    n0, n1 = a.shape
    rs = np.random.RandomState(12345)
    ii = rs.randint(0, n0, size=16)
    jj = rs.randint(0, n1, size=16)
    def part(j0):
        blk = a[:, j0:j0 + 1024].astype(np.float64)
        return float(blk.sum()), float((blk * blk).sum())

    nthr = _pool_size(n0 * n1)
    if nthr == 1:
        parts = [part(j0) for j0 in range(0, n1, 1024)]
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(nthr) as ex:
            parts = list(ex.map(part, range(0, n1, 1024)))
    s = float(sum(p[0] for p in parts))
    s2 = float(sum(p[1] for p in parts))
    return dict(shape=[int(n0), int(n1)], sum=s, sumsq=s2,
                samples=[float(a[i, j]) for i, j in zip(ii, jj)])


def fingerprint_matches(fa: dict, fb: dict, rtol: float = 1e-6) -> bool:
    if fa["shape"] != fb["shape"]:
        return False
    scale = np.sqrt(fa["sumsq"] / (fa["shape"][0] * fa["shape"][1]))
    ok = abs(fa["sumsq"] - fb["sumsq"]) <= rtol * abs(fa["sumsq"])
    ok = ok and abs(fa["sum"] - fb["sum"]) <= rtol * scale * fa["shape"][0] * fa["shape"][1]
    sa = np.array(fa["samples"])
    sb = np.array(fb["samples"])
    return bool(ok and np.all(np.abs(sa - sb) <= rtol * scale * 10))
