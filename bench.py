#!/usr/bin/env python
"""Benchmark of the svdvals hot path on one MI355X.

A step is one complete pass dense -> band -> bidiagonal -> singular values
(svb_svdvals: all three stages on the GPU) on a seeded synthetic matrix that is
already resident in HBM.  W warm-up steps, K timed steps without per-kernel
instrumentation (-> value), then the same K steps again with the library's
per-kernel HIP events (-> roofline).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c4] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3, "f16": 157.3}   # MFMA peak of the arithmetic type used
PEAK_HBM_GBS = 8000.0


def device_matrix(name, torch, gaussian=False):
    """The workload matrix in HBM (column-major n x n in the storage dtype).

    iid workloads come from the shared CPU generator; the prescribed-spectrum
    workloads build U diag(sigma) V^T on the GPU with torch (QR of Gaussian
    matrices), which is input synthesis only."""
    import workloads
    cfg = workloads.CONFIGS[name]
    n = cfg["n"]
    tdt = {"f64": torch.float64, "f32": torch.float32, "f16": torch.float16}[cfg["dtype"]]
    if gaussian:
        # counter-collection runs only: same shape and dtype, iid N(0,1/n) drawn on the device
        gen = torch.Generator(device="cuda")
        gen.manual_seed(workloads.config_seed(cfg["seed_id"]))
        a = torch.randn(n, n, dtype=torch.float32, device="cuda", generator=gen) / float(np.sqrt(n))
        return a.to(tdt), dict(name=name, n=n, nb=cfg["nb"], dtype=cfg["dtype"], seed=0, sigma=None)
    if cfg["kind"] == "iid":
        a, info = workloads.make(name)
        return torch.from_numpy(np.ascontiguousarray(a.T)).cuda(), info
    seed = workloads.config_seed(cfg["seed_id"])
    sig = workloads.spectrum(cfg["spectrum"], n, seed + 2, cfg.get("smin", 0.0))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)

    def haar():
        g = torch.randn(n, n, dtype=torch.float64, device="cuda", generator=gen)
        q, r = torch.linalg.qr(g)
        return q * torch.sign(torch.diagonal(r))[None, :]

    u = haar()
    v = haar()
    a = (u * torch.from_numpy(sig).cuda()[None, :]) @ v.T
    del u, v
    info = dict(name=name, n=n, nb=cfg["nb"], dtype=cfg["dtype"], seed=seed, sigma=sig)
    return a.to(tdt).contiguous(), info


def cpu_baseline(name, sample_n):
    """The CPU oracle, as it stands, on the leading sample_n x sample_n block of
    the workload's recipe (same distribution, smaller matrix)."""
    import oracle
    import workloads
    a, info = workloads.make(name, n=sample_n)
    t0 = time.perf_counter()
    s = oracle.svdvals(a)
    dt = time.perf_counter() - t0
    flops = 8.0 / 3.0 * sample_n ** 3
    return dict(value=flops / dt / 1e12, unit="TFLOP/s", cores=oracle.num_threads(), kind="oracle",
                sample=f"same recipe at n={sample_n} ({dt:.1f} s, unblocked Householder bidiagonalisation + bisection, fp64)"), s


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="c4", help="workload name from workloads.CONFIGS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-n", type=int, default=4096)
    ap.add_argument("--lda-pad", type=int, default=0,
                    help="leading dimension of the matrix handed to the library = n + this many elements")
    ap.add_argument("--gaussian-input", action="store_true",
                    help="profiling aid: replace the workload's values by iid Gaussians of the same shape "
                         "(no QR-based synthesis on the device); the result line is marked accordingly")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads
    import paper_2508_06339_amd as svb

    svb.load_library()  # raises when the HIP library is missing: there is no fallback
    torch.cuda.set_device(0)
    a0, info = device_matrix(args.config, torch, args.gaussian_input)
    n, nb, dtype = info["n"], info["nb"], info["dtype"]
    dt_code = svb.dtype_code(a0.dtype)
    rc, wbytes, _ = svb.svb_workspace_bytes(dt_code, n, n, nb)
    assert rc == 0, svb.svb_status_string(rc)
    work = torch.empty(wbytes, dtype=torch.uint8, device="cuda")
    lda = n + args.lda_pad
    abuf = torch.empty((n, lda), dtype=a0.dtype, device="cuda")   # row j of this tensor = column j of the matrix
    a = abuf[:, :n]
    out = np.empty(n, dtype=np.float64 if dtype == "f64" else np.float32)
    stream = torch.cuda.current_stream().cuda_stream

    def one_step():
        a.copy_(a0)                      # stage 1 destroys its input; the refresh is not timed
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rc = svb.svb_svdvals(dt_code, n, n, abuf, lda, out, nb, work, wbytes, stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        assert rc == 0, svb.svb_status_string(rc)
        return t1 - t0, svb.svb_last_timings()

    for _ in range(args.warmup):
        one_step()
    # timed region: exactly K steps, no per-kernel instrumentation
    times, stages = [], []
    for _ in range(args.steps):
        t, st = one_step()
        times.append(t)
        stages.append(st)
    # the same K steps once more with the library's per-kernel HIP events (the kernels' own start and
    # stop time stamps on the streams they run on): the roofline figures come from this pass.  It is
    # kept out of the timed region because event handling lengthens the dependency chain of stage 1
    # (by about 4 % of a step on the default workload); its own time per step is reported beside it.
    svb.svb_profile_enable(True)
    ptimes = [one_step()[0] for _ in range(args.steps)]
    prof = {k: svb.svb_profile_get(i) for i, k in enumerate(["panel", "k1", "k2", "chase", "fused"])}
    svb.svb_profile_enable(False)

    total = float(np.sum(times))
    ms_per_step = total / args.steps * 1e3
    flops = 8.0 / 3.0 * n ** 3
    value = flops / (total / args.steps) / 1e12
    st = np.mean(np.array(stages), axis=0)

    # sanity of the result (not timed): prescribed spectrum or Frobenius invariant
    s = np.asarray(out, dtype=np.float64)
    check = {}
    if info.get("sigma") is not None:
        check["max_abs_err_vs_prescribed"] = float(np.abs(s - info["sigma"]).max())
        check["tolerance"] = float(10 * n * workloads.EPS[dtype] * info["sigma"][0])
    fro2 = float((a0.double() ** 2).sum().item())
    check["rel_frobenius_defect"] = abs(float(np.sum(s * s)) - fro2) / fro2

    # roofline of the dominant kernel (the one with the largest summed duration)
    dom = max(("k1", "k2", "fused"), key=lambda k: prof[k]["seconds"])
    pk = prof[dom]
    ach = pk["flops"] / pk["seconds"] / 1e12 if pk["seconds"] > 0 else 0.0
    peak = PEAK_TFLOPS[dtype]
    roofline = dict(kernel=dom, bound="mfma", achieved=ach, peak=peak, unit="TFLOP/s", frac=ach / peak,
                    traffic=None, launches=pk["launches"],
                    avg_launch_ms=pk["seconds"] / max(pk["launches"], 1) * 1e3)
    # HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one
    # (first-tree-level launches of the dominant kernel: the ones whose flops and bytes are credited)
    tfile = os.path.join(ROOT, "profiles", f"hbm_traffic_{args.config}_{n}_{dtype}_nb{nb}.json")
    roofline_stage2_traffic = None
    if os.path.exists(tfile):
        tr = json.load(open(tfile))
        kname = {"k1": "k1_mfma", "k2": "k2_mfma", "fused": "update_fused_kernel"}[dom]

        def first_level(k):
            # update_fused_kernel<T, C, NB, HT, LQ, TRI, MODE>: TRI marks the tree levels above the first
            if dom != "fused":
                return True
            targs = [a.strip() for a in k[k.index("<") + 1:k.rindex(">")].split(",")]
            return len(targs) < 6 or targs[5] != "true"

        lvl0 = {k: v for k, v in tr.items() if k.startswith(kname) and first_level(k)}
        rd = sum(v["read_GB"] for v in lvl0.values())
        wr = sum(v["write_GB"] for v in lvl0.values())
        if lvl0:
            halfsweeps = 2 * (n // nb - 1)                    # half-sweeps with a trailing matrix, one call
            roofline["traffic"] = (rd + wr) * 1e9 / halfsweeps
            roofline["traffic_unit"] = ("HBM bytes per half-sweep, first tree level, all its launches "
                                        "(FETCH_SIZE + WRITE_SIZE, calibrated)")
            roofline["algorithmic_bytes_per_halfsweep"] = pk["bytes"] / (halfsweeps * args.steps)
        chk = [v for k, v in tr.items() if k.startswith(("band_reduce_kernel", "chase_narrow_kernel", "chase_persistent"))]
        if chk:
            roofline_stage2_traffic = sum(v["read_GB"] + v["write_GB"] for v in chk) * 1e9
    upd_s = prof["k1"]["seconds"] + prof["k2"]["seconds"] + prof["fused"]["seconds"]
    ch = prof["chase"]
    ch_gbs = ch["bytes"] / ch["seconds"] / 1e9 if ch["seconds"] > 0 else 0.0
    roofline_stage2 = dict(kernel="chase", bound="hbm", achieved=ch_gbs, peak=PEAK_HBM_GBS, unit="GB/s",
                           frac=ch_gbs / PEAK_HBM_GBS, traffic=roofline_stage2_traffic)

    res = {
        "metric": "svdvals effective TFLOP/s (8/3 n^3 / time-to-singular-values)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"lda": lda, "workload": f"{args.config}: {n}x{n} {dtype}, nb={nb}, "
                               f"{'gaussian stand-in' if args.gaussian_input else workloads.CONFIGS[args.config]['kind']}"},
        "time_to_singular_values_ms": ms_per_step,
        "instrumented_pass_ms_per_step": float(np.mean(ptimes)) * 1e3,
        "stage_ms": {"stage1": st[0] * 1e3, "stage2": st[1] * 1e3, "stage3": st[2] * 1e3,
                     "panel": prof["panel"]["seconds"] / args.steps * 1e3,
                     "update": upd_s / args.steps * 1e3},
        "stage1_effective_tflops": flops / st[0] / 1e12 if st[0] > 0 else None,
        "stage1_frac_of_mfma_peak": flops / st[0] / 1e12 / peak if st[0] > 0 else None,
        "roofline": roofline,
        "roofline_stage2": roofline_stage2,
        "check": check,
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"], _ = cpu_baseline(args.config, args.cpu_sample_n)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
