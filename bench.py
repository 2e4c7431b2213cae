#!/usr/bin/env python
"""Benchmark of the svdvals hot path on one MI355X.

A step is one complete pass dense -> band -> bidiagonal -> singular values
(svb_svdvals: all three stages on the GPU) on a seeded synthetic matrix that is
already resident in HBM.  W warm-up steps, K timed steps without per-kernel
instrumentation (-> value), then the same K steps again with the library's
per-kernel HIP events (-> roofline).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c5a] [--also c4] [--no-cpu-baseline]
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

# dense MFMA peak of the operand type the trailing update multiplies in (f16 / bf16 storage: the
# 16-bit matrix instructions, f32 accumulate)
PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3, "f16": 2500.0, "bf16": 2500.0}
PEAK_HBM_GBS = 8000.0


def device_matrix(name, torch, gaussian=False, n_override=None):
    """The workload matrix in HBM (column-major n x n in the storage dtype).

    iid workloads come from the shared CPU generator; the prescribed-spectrum
    workloads build U diag(sigma) V^T on the GPU with torch (QR of Gaussian
    matrices), which is input synthesis only."""
    import workloads
    cfg = dict(workloads.CONFIGS[name])
    if n_override:
        cfg["n"] = int(n_override)
    n = cfg["n"]
    tdt = {"f64": torch.float64, "f32": torch.float32, "f16": torch.float16}[cfg["dtype"]]
    if gaussian:
        # counter-collection runs only: same shape and dtype, iid N(0,1/n) drawn on the device
        gen = torch.Generator(device="cuda")
        gen.manual_seed(workloads.config_seed(cfg["seed_id"]))
        # (a view of a slightly larger allocation: counter collection has crashed on allocations of
        # exactly 4 GiB)
        a = torch.empty(n, n + 16, dtype=tdt, device="cuda")[:, :n]
        for j0 in range(0, n, 4096):   # in blocks: no single launch touches more than 1 GiB
            blk = torch.randn(min(4096, n - j0), n, dtype=torch.float32, device="cuda", generator=gen)
            a[j0:j0 + 4096] = (blk / float(np.sqrt(n))).to(tdt)
        return a, dict(name=name, n=n, nb=cfg["nb"], dtype=cfg["dtype"], seed=0, sigma=None)
    if cfg["kind"] == "iid":
        a, info = workloads.make(name, n=n)
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
    res = dict(value=flops / dt / 1e12, unit="TFLOP/s", cores=oracle.num_threads(), kind="oracle",
               sample=f"same recipe at n={sample_n} ({dt:.1f} s, unblocked Householder bidiagonalisation + bisection, fp64)")
    # the oracle's one run on the whole workload, where its result is stored for the parity tests
    # (tests/golden, written by make_oracle_sigma.py on the build machine): its own time, as recorded there
    gfile = os.path.join(ROOT, "tests", "golden", f"sigma_{name}.txt")
    if os.path.exists(gfile):
        with open(gfile) as f:
            meta = json.loads(f.readline()[2:])
        if meta.get("oracle_seconds"):
            res["full_workload_run"] = dict(seconds=meta["oracle_seconds"], threads=meta.get("oracle_threads"),
                                            tflops=8.0 / 3.0 * meta["n"] ** 3 / meta["oracle_seconds"] / 1e12,
                                            where="build container (recorded in tests/golden)")
    return res, s


def run_workload(args, svb, torch, workloads, config, steps, warmup):
    """W warm-up steps, K timed steps, then K steps with the library's per-kernel events.
    Returns the measurements of one workload as a dict."""
    a0, info = device_matrix(config, torch, args.gaussian_input, args.n if config == args.config else None)
    n, nb, dtype = info["n"], info["nb"], info["dtype"]
    if args.nb >= 0 and config == args.config:
        nb = args.nb if args.nb > 0 else svb.svb_choose_nb(svb.dtype_code(a0.dtype), n, n)
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
        for j0 in range(0, n, 8192):     # stage 1 destroys its input; the refresh (in blocks) is not timed
            a[j0:j0 + 8192].copy_(a0[j0:j0 + 8192])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rc = svb.svb_svdvals(dt_code, n, n, abuf, lda, out, nb, work, wbytes, stream)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        assert rc == 0, svb.svb_status_string(rc)
        tp, tu, t2, t3 = svb.svb_last_timings()
        return t1 - t0, (max(tp, 0.0) + tu, t2, t3, tp)

    for _ in range(warmup):
        one_step()
    # timed region: exactly K steps, no per-kernel instrumentation
    times, stages = [], []
    for _ in range(steps):
        t, st = one_step()
        times.append(t)
        stages.append(st)
    # the same K steps once more with the library's per-kernel HIP events (the kernels' own start and
    # stop time stamps on the streams they run on): the roofline figures come from this pass.  It is
    # kept out of the timed region because event handling lengthens the dependency chain of stage 1
    # (a few per cent of a step on the small workloads); its own time per step is reported beside it.
    svb.svb_profile_enable(True)
    pruns = [one_step() for _ in range(steps)]
    prof = {k: svb.svb_profile_get(i) for i, k in enumerate(svb.SVB_PROF_NAMES)}
    svb.svb_profile_enable(False)
    exposed_panel = float(np.mean([r[1][3] for r in pruns]))

    total = float(np.sum(times))
    ms_per_step = total / steps * 1e3
    flops = 8.0 / 3.0 * n ** 3
    value = flops / (total / steps) / 1e12
    st = np.mean(np.array(stages), axis=0)

    # sanity of the result (not timed): prescribed spectrum or Frobenius invariant
    s = np.asarray(out, dtype=np.float64)
    check = {}
    if info.get("sigma") is not None:
        check["max_abs_err_vs_prescribed"] = float(np.abs(s - info["sigma"]).max())
        check["tolerance"] = float(10 * n * workloads.EPS[dtype] * info["sigma"][0])
    fro2 = 0.0
    for j0 in range(0, n, 4096):
        fro2 += float((a0[j0:j0 + 4096].double() ** 2).sum().item())
    check["rel_frobenius_defect"] = abs(float(np.sum(s * s)) - fro2) / fro2

    peak = PEAK_TFLOPS[dtype]
    cs = 8 if dtype == "f64" else 4
    kernels = {}
    for k, v in prof.items():
        kernels[k] = dict(ms_per_step=v["seconds"] / steps * 1e3, launches_per_step=v["launches"] / steps,
                          avg_launch_us=v["seconds"] / max(v["launches"], 1) * 1e6)
    # HBM bytes from the committed rocprofv3 --pmc summary of this workload, if there is one.  Where the
    # counters could only be collected on the workload's recipe at another order (the file name says
    # so), the measured ratio of counter bytes to algorithmic bytes is applied to this run's
    # algorithmic bytes.
    import glob
    tfile = os.path.join(ROOT, "profiles", f"hbm_traffic_{config}_{n}_{dtype}_nb{nb}.json")
    traffic, traffic_src = None, None
    if os.path.exists(tfile):
        traffic, traffic_src = json.load(open(tfile)), "counters on this workload"
    else:
        alt = sorted(glob.glob(os.path.join(ROOT, "profiles", f"hbm_traffic_{config}-recipe_*_{dtype}_nb{nb}.json")))
        if alt:
            traffic = json.load(open(alt[-1]))
            traffic_src = ("counter-to-algorithmic byte ratio measured on " + traffic["_meta"]["workload"] +
                           ", applied to this run's algorithmic bytes")
    exact_traffic = traffic is not None and traffic_src.startswith("counters")

    def counter_bytes(prefix, want_tri=None):
        """(bytes, launches) per svb_svdvals call of the kernels whose name starts with prefix."""
        if traffic is None:
            return None
        tot, cnt = 0.0, 0
        for name, v in traffic.items():
            if not name.startswith(prefix):
                continue
            if want_tri is not None:
                # update_fused_kernel<T, C, NB, HT, LQ, TRI, USET> / update_fused32_kernel<T, LQ, TRI>:
                # TRI marks the tree levels above the first
                targs = [x.strip() for x in name[name.index("<") + 1:name.rindex(">")].split(",")]
                tri = targs[2] if name.startswith("update_fused32") else targs[5]
                if (tri == "true") != want_tri:
                    continue
            tot += (v["read_GB"] + v["write_GB"]) * 1e9
            cnt += v["launches"]
        return (tot, cnt) if cnt else None

    # The kernel class that costs the most wall time.  Panel kernels run on their own stream beside
    # the updates and wait for compute units behind them, so their summed durations overlap the
    # updates'; what they add to a step is the part of stage 1 that no update kernel covers.
    cost = {k: v["ms_per_step"] for k, v in kernels.items()}
    cost["panel"] = min(cost["panel"], exposed_panel * 1e3)
    dom = max(cost, key=cost.get)
    upd = prof["update"]
    if dom in ("update", "update_upper"):
        # MFMA-bound contraction: credited flops of its first-level launches (both products,
        # 4 rows nb cols per launch; 8/3 n^3 over a run) / their summed duration
        ach = upd["flops"] / upd["seconds"] / 1e12 if upd["seconds"] > 0 else 0.0
        kname = ("update_fused16_kernel" if dtype in ("f16", "bf16") else
                 "update_fused32_kernel" if (dtype == "f32" and nb == 128) else "update_fused_kernel")
        roofline = dict(kernel=kname + " (first tree level: the launches with TRI = false)", bound="mfma", achieved=ach,
                        peak=peak,
                        unit="TFLOP/s", frac=ach / peak, traffic=None,
                        launches_per_step=upd["launches"] / steps,
                        avg_launch_ms=upd["seconds"] / max(upd["launches"], 1) * 1e3,
                        algorithmic_bytes_per_launch=upd["bytes"] / max(upd["launches"], 1),
                        algorithmic_flops_per_launch=upd["flops"] / max(upd["launches"], 1))
        cb = counter_bytes("update_fused", want_tri=False)
        if cb and exact_traffic:
            roofline["traffic"] = cb[0] / cb[1]
        elif cb and "update_first_level_algorithmic_GB" in traffic["_meta"]:
            ratio = cb[0] / (traffic["_meta"]["update_first_level_algorithmic_GB"] * 1e9)
            roofline["traffic"] = ratio * roofline["algorithmic_bytes_per_launch"]
            roofline["traffic_to_algorithmic_ratio"] = ratio
        if cb:
            roofline["traffic_unit"] = "HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, calibrated), first tree level"
            roofline["traffic_source"] = traffic_src
        allsec = upd["seconds"] + prof["update_upper"]["seconds"]
        roofline["frac_all_tree_levels"] = upd["flops"] / allsec / 1e12 / peak if allsec > 0 else None
    else:
        # a dependency chain (panel tree, band reduction, narrow chase, bisection): reported against
        # the HBM roofline by its algorithmic bytes, which it is nowhere near
        pk = prof[dom]
        ach = pk["bytes"] / pk["seconds"] / 1e9 if pk["seconds"] > 0 else 0.0
        roofline = dict(kernel=dom, bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=ach / PEAK_HBM_GBS, traffic=None, launches_per_step=pk["launches"] / steps,
                        avg_launch_ms=pk["seconds"] / max(pk["launches"], 1) * 1e3,
                        note="latency-bound dependency chain; the update kernel's MFMA figure is under roofline_update")
    roofline_update = dict(bound="mfma", achieved=upd["flops"] / upd["seconds"] / 1e12 if upd["seconds"] > 0 else 0.0,
                           peak=peak, unit="TFLOP/s")
    roofline_update["frac"] = roofline_update["achieved"] / peak
    # the same launches against the HBM roofline by their algorithmic bytes (the block read once and
    # written once): the bound that matters where the operands are 16 bits wide
    roofline_update["algorithmic_gbs"] = upd["bytes"] / upd["seconds"] / 1e9 if upd["seconds"] > 0 else 0.0
    roofline_update["hbm_frac"] = roofline_update["algorithmic_gbs"] / PEAK_HBM_GBS
    # stage 2: algorithmic bytes of the two kernels as built (every band block read once and written
    # once per block sweep; the narrow band once per bundle) over the stage's duration.  Both kernels
    # are dependency chains: the HBM roofline is not what limits them.
    s2_bytes = (prof["band_reduce"]["bytes"] + prof["narrow_chase"]["bytes"]) / steps
    s2_gbs = s2_bytes / st[1] / 1e9 if st[1] > 0 else 0.0
    roofline_stage2 = dict(kernels="band_reduce_kernel + chase_narrow_kernel", bound="hbm", achieved=s2_gbs,
                           peak=PEAK_HBM_GBS, unit="GB/s", frac=s2_gbs / PEAK_HBM_GBS, traffic=None,
                           algorithmic_bytes=s2_bytes, limited_by="latency of the sweep-to-sweep dependency chain",
                           one_phase_chase_model_bytes=3.0 * n * n * nb * cs)
    cb1, cb2 = counter_bytes("band_reduce_kernel"), counter_bytes("chase_narrow_kernel")
    if cb1 and cb2:
        t2 = cb1[0] + cb2[0]
        if not exact_traffic:
            t2 = t2 / (traffic["_meta"]["stage2_algorithmic_GB"] * 1e9) * s2_bytes
        roofline_stage2["traffic"] = t2
        roofline_stage2["traffic_gbs"] = t2 / st[1] / 1e9 if st[1] > 0 else None
        roofline_stage2["traffic_source"] = traffic_src
    kind = "gaussian stand-in" if args.gaussian_input else workloads.CONFIGS[config]["kind"]
    return {
        "value": value, "ms_per_step": ms_per_step, "dtype": dtype,
        "config": {"lda": lda, "workload": f"{config}: {n}x{n} {dtype}, nb={nb}, {kind}"},
        "time_to_singular_values_ms": ms_per_step,
        "instrumented_pass_ms_per_step": float(np.mean([r[0] for r in pruns])) * 1e3,
        "stage_ms": {"stage1": st[0] * 1e3, "stage2": st[1] * 1e3, "stage3": st[2] * 1e3,
                     "stage1_exposed_panel": exposed_panel * 1e3},
        "kernel_ms": kernels,
        "wall_time_share_ms": cost,
        "stage1_effective_tflops": flops / st[0] / 1e12 if st[0] > 0 else None,
        "stage1_frac_of_mfma_peak": flops / st[0] / 1e12 / peak if st[0] > 0 else None,
        "roofline": roofline,
        "roofline_update": roofline_update,
        "roofline_stage2": roofline_stage2,
        "check": check,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="c5a", help="workload name from workloads.CONFIGS (default: the largest "
                    "single-GPU configuration, 32768x32768 f32, nb=128)")
    ap.add_argument("--also", default="c4", help="comma-separated further workloads measured the same way and "
                    "reported under extra_workloads ('none' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-n", type=int, default=4096)
    ap.add_argument("--n", type=int, default=0,
                    help="profiling aid: the workload's recipe at another order n (a multiple of its nb); "
                         "the workload line shows the order used")
    ap.add_argument("--nb", type=int, default=-1,
                    help="profiling aid: tile size instead of the workload's (0: the library chooses)")
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
    main_res = run_workload(args, svb, torch, workloads, args.config, args.steps, args.warmup)
    res = {
        "metric": "svdvals effective TFLOP/s (8/3 n^3 / time-to-singular-values)",
        "value": main_res.pop("value"), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": main_res.pop("dtype"), "data": "synthetic",
    }
    res.update(main_res)
    extra = {}
    for name in [x for x in args.also.split(",") if x and x != "none" and x != args.config]:
        torch.cuda.empty_cache()
        extra[name] = run_workload(args, svb, torch, workloads, name, args.steps, args.warmup)
    if extra:
        res["extra_workloads"] = extra
    if not args.no_cpu_baseline:
        res["cpu_baseline"], _ = cpu_baseline(args.config, args.cpu_sample_n)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
