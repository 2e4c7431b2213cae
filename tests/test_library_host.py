"""CPU-side checks of the HIP library: it loads, exports every declared entry
point, validates arguments, and its host stage 3 agrees with closed forms.
No compute call touches a GPU here."""
import os
import re

import numpy as np
import pytest

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
svb = pytest.importorskip("paper_2508_06339_amd")

if not os.path.exists(svb.library_path()):
    pytest.skip("libsvb.so not built (run __graft_entry__.build())", allow_module_level=True)

EPS = 2.0 ** -52


def test_every_declared_symbol_is_exported():
    hdr = open(os.path.join(ROOT, "include", "svb.h")).read()
    names = set(re.findall(r"\b(svb_[a-z0-9_]+)\s*\(", hdr))
    assert {"svb_svdvals", "svb_ge2gb", "svb_gb2bd", "svb_bdsvals", "svb_workspace_bytes"} <= names
    lib = svb.load_library()
    for name in names:
        assert hasattr(lib, name), name


def test_product_path_does_not_reach_the_oracle():
    pkg = os.path.join(ROOT, "paper_2508_06339_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f


def test_argument_validation():
    ok, dev, host = svb.svb_workspace_bytes(svb.SVB_F32, 1024, 1024, 32)
    assert ok == 0 and dev > 0 and host == 0
    # general shapes are accepted (and add room for the padded copy); nb = 0 picks a tile size
    ok2, dev2, _ = svb.svb_workspace_bytes(svb.SVB_F32, 1000, 1000, 32)
    assert ok2 == 0 and dev2 >= dev + 3 * 1024 * 1024
    assert svb.svb_workspace_bytes(svb.SVB_F32, 1024, 512, 32)[0] == 0
    assert svb.svb_workspace_bytes(svb.SVB_F32, 512, 1024, 32)[0] == 0
    assert svb.svb_workspace_bytes(svb.SVB_BF16, 1024, 1024, 32)[0] == 0
    assert svb.svb_workspace_bytes(svb.SVB_F32, 1024, 1024, 0)[0] == 0
    assert svb.svb_workspace_bytes(svb.SVB_F32, 0, 7, 32)[0] == 0
    assert svb.svb_workspace_bytes(svb.SVB_F32, 1024, 1024, 48)[0] == 2      # nb
    assert svb.svb_workspace_bytes(7, 1024, 1024, 32)[0] == 2                # dtype
    assert svb.svb_workspace_bytes(svb.SVB_F64, -1, -1, 32)[0] == 1
    out = np.zeros(64, dtype=np.float32)
    # null device pointers are rejected before anything is launched
    assert svb.svb_svdvals(svb.SVB_F32, 64, 64, None, 64, out, 32, None, 0, stream=0) == 1
    assert svb.svb_svdvals(svb.SVB_F32, 0, 64, None, 64, out, 32, None, 0, stream=0) == 0   # nothing to do
    assert svb.svb_ge2gb(svb.SVB_F32, 64, 64, None, 64, 32, None, 96, None, 0, stream=0) == 1
    assert svb.svb_ge2gb(svb.SVB_F32, 60, 64, None, 64, 32, None, 96, None, 0, stream=0) == 2   # in place: whole tiles only
    assert svb.svb_gb2bd(svb.SVB_F16, 64, 32, None, 96, None, None, None, 0, stream=0) == 2
    assert svb.svb_gb2bd(svb.SVB_F32, 64, 32, None, 96, None, None, None, 0, stream=0) == 1
    assert svb.svb_gb2bd_noalloc(svb.SVB_F32, 64, 32, None, 96, None, None, stream=0) == 1
    assert svb.svb_gb2bd_noalloc(svb.SVB_F32, 1 << 20, 32, None, 96, None, None, stream=0) == 1  # null pointers first
    rc, wb = svb.svb_gb2bd_workspace_bytes(1000, 64)
    assert rc == 0 and wb >= 4 * 1000
    assert "workspace" in svb.svb_status_string(3)


def test_workspace_is_a_fraction_of_the_matrix():
    # in-place problems need panels, factors, the band and counters only: a few per cent of the matrix
    for dt, n, nb, size in [(svb.SVB_F32, 32768, 128, 4), (svb.SVB_F64, 16384, 128, 8), (svb.SVB_F32, 8192, 64, 4)]:
        rc, dev, _ = svb.svb_workspace_bytes(dt, n, n, nb)
        assert rc == 0
        assert dev <= 0.1 * n * n * size, (n, dev)
    rc, dev, _ = svb.svb_workspace_bytes(svb.SVB_F32, 32768, 32768, 128)
    assert dev <= 1 << 30


def test_tile_size_choice():
    assert svb.svb_choose_nb(svb.SVB_F32, 256, 256) == 32
    assert svb.svb_choose_nb(svb.SVB_F32, 8192, 8192) == 64
    assert svb.svb_choose_nb(svb.SVB_F16, 16384, 16384) == 64
    assert svb.svb_choose_nb(svb.SVB_F32, 32768, 40000) == 128
    assert svb.svb_choose_nb(svb.SVB_F64, 2048, 2048) == 32
    assert svb.svb_choose_nb(svb.SVB_F64, 4096, 4096) == 64
    assert svb.svb_choose_nb(svb.SVB_F32, 24576, 24576) == 64
    assert svb.svb_choose_nb(svb.SVB_F64, 32768, 32768) == 64
    assert svb.svb_choose_nb(svb.SVB_F32, 100000, 500) == 32     # the smaller dimension decides
    assert svb.svb_choose_nb(svb.SVB_F32, -1, 5) == 0


@pytest.mark.parametrize("n", [1, 2, 5, 16, 17, 100, 1000])
def test_bdsvals_closed_form(n):
    s = np.zeros(n)
    assert svb.svb_bdsvals(n, np.ones(n), np.ones(max(n - 1, 1)), s) == 0
    k = np.arange(1, n + 1)
    np.testing.assert_allclose(s, 2 * np.cos(k * np.pi / (2 * n + 1)), rtol=0, atol=16 * EPS)


def test_bdsvals_random_vs_library_and_edge_cases():
    n = 300
    d = workloads.normal(1, 0, n)
    e = workloads.normal(2, 0, n - 1)
    s = np.zeros(n)
    assert svb.svb_bdsvals(n, d, e, s) == 0
    ref = np.linalg.svd(np.diag(d) + np.diag(e, 1), compute_uv=False)
    np.testing.assert_allclose(s, ref, rtol=0, atol=64 * EPS * ref[0])
    z = np.zeros(4)
    assert svb.svb_bdsvals(4, np.zeros(4), np.zeros(3), z) == 0 and not z.any()
    assert svb.svb_bdsvals(0, np.zeros(0), np.zeros(0), np.zeros(0)) == 0
    bad = d.copy()
    bad[3] = np.nan
    assert svb.svb_bdsvals(n, bad, e, s) == 6
    dd = np.array([3.0, -1.0, 0.0, 2.0])
    assert svb.svb_bdsvals(4, dd, np.zeros(3), z) == 0
    np.testing.assert_allclose(z, [3.0, 2.0, 1.0, 0.0], atol=1e-15)


def test_bench_refuses_more_than_one_gpu():
    # one GPU only: the bench says so and exits before touching a device
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr
