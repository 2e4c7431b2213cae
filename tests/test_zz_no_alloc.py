"""The entry point that allocates nothing (svb_gb2bd_noalloc: stage 2 with its sweep counters in a
fixed array inside the library's device image) against svb_gb2bd with a caller-supplied workspace:
same band in, same bidiagonal out, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest

import workloads

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
svb = pytest.importorskip("paper_2508_06339_amd")

TORCH_DT = {"f64": torch.float64, "f32": torch.float32}


def _band(dtype, n, nb, seed):
    npdt = workloads.NP_DTYPE[dtype]
    ldab = 3 * nb
    g = workloads.gaussian_matrix(seed, nb + 1, n)            # row r of g: super-diagonal nb - r
    bh = np.zeros((n, ldab), dtype=npdt)
    for j in range(n):
        for i in range(max(0, j - nb), j + 1):
            bh[j, i - j + 2 * nb - 1] = g[i - j + nb, j]
    return bh, ldab


def _run(dtype, n, nb, bh, ldab, noalloc):
    code = svb.SVB_F64 if dtype == "f64" else svb.SVB_F32
    band = torch.from_numpy(bh).cuda()
    d = torch.zeros(n, dtype=TORCH_DT[dtype], device="cuda")
    e = torch.zeros(n, dtype=TORCH_DT[dtype], device="cuda")
    if noalloc:
        rc = svb.svb_gb2bd_noalloc(code, n, nb, band, ldab, d, e)
    else:
        rc, wb = svb.svb_gb2bd_workspace_bytes(n, nb)
        assert rc == 0
        work = torch.empty(max(wb, 1), dtype=torch.uint8, device="cuda")
        rc = svb.svb_gb2bd(code, n, nb, band, ldab, d, e, work, wb)
    assert rc == 0, svb.svb_status_string(rc)
    torch.cuda.synchronize()
    return d.cpu().numpy(), e.cpu().numpy()


@pytest.mark.parametrize("dtype", ["f32", "f64"])
def test_noalloc_matches_workspace_entry_point(dtype):
    for n, nb, seed in [(1500, 64, 501), (700, 32, 502)]:      # the second call is the smaller one
        print(f"[case] gb2bd_noalloc {dtype} n={n} nb={nb}", flush=True)
        bh, ldab = _band(dtype, n, nb, seed)
        d0, e0 = _run(dtype, n, nb, bh, ldab, noalloc=False)
        d1, e1 = _run(dtype, n, nb, bh, ldab, noalloc=True)
        assert np.all(np.isfinite(d1)) and np.all(np.isfinite(e1))
        # same kernels, same order of operations: the two bidiagonals are identical
        np.testing.assert_array_equal(d1, d0)
        np.testing.assert_array_equal(e1, e0)
        fro2 = float(np.sum(bh.astype(np.float64) ** 2))
        eps = workloads.EPS[dtype]
        assert abs(np.sum(d1.astype(np.float64) ** 2) + np.sum(e1[: n - 1].astype(np.float64) ** 2) - fro2) <= 20 * n * eps * fro2


def test_noalloc_rejects_sizes_beyond_its_array():
    n, nb = 200000, 32
    t = torch.zeros(8, device="cuda")
    assert svb.svb_gb2bd_noalloc(svb.SVB_F32, n, nb, t, 3 * nb, t, t) == 3
