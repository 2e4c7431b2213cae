"""Time svb_svdvals over matrix orders and tile sizes on the current GPU.

The table this prints is what svb_choose_nb (nb = 0) was derived from on MI355X
(the paper tunes its TILESIZE per size and device the same way, Section 4, Table 3);
run it again on other hardware to re-derive the thresholds.

    python -m paper_2508_06339_amd.tune_nb [--out file.json] [--orders 1024,2048,...]
"""
from __future__ import annotations

import argparse
import json
import time

import numpy as np


def main():
    import torch
    from . import binding as svb

    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="")
    ap.add_argument("--orders", default="1024,2048,3072,4096,6144,8192,12288,16384,24576")
    args = ap.parse_args()
    svb.load_library()
    res = {}
    for dtype, tdt in (("f32", torch.float32), ("f64", torch.float64)):
        for n in [int(x) for x in args.orders.split(",")]:
            gen = torch.Generator(device="cuda")
            gen.manual_seed(n)
            a0 = (torch.randn(n, n, dtype=torch.float32, device="cuda", generator=gen) / np.sqrt(n)).to(tdt)
            for nb in (32, 64, 128):
                if n % nb or (nb == 32 and n > 8192):
                    continue
                code = svb.dtype_code(tdt)
                rc, wb, _ = svb.svb_workspace_bytes(code, n, n, nb)
                work = torch.empty(wb, dtype=torch.uint8, device="cuda")
                out = np.empty(n, dtype=np.float64 if dtype == "f64" else np.float32)
                a = torch.empty_like(a0)
                ts = []
                for _ in range(3):
                    a.copy_(a0)
                    torch.cuda.synchronize()
                    t0 = time.perf_counter()
                    rc = svb.svb_svdvals(code, n, n, a, n, out, nb, work, wb)
                    torch.cuda.synchronize()
                    ts.append(time.perf_counter() - t0)
                    assert rc == 0, svb.svb_status_string(rc)
                st = svb.svb_last_timings()
                res[f"{dtype} n={n} nb={nb}"] = dict(ms=min(ts) * 1e3, s1=st[1] * 1e3, s2=st[2] * 1e3, s3=st[3] * 1e3)
                print(f"{dtype} n={n:6d} nb={nb:4d}: {min(ts) * 1e3:9.2f} ms  (stage1 {st[1] * 1e3:8.2f}  "
                      f"stage2 {st[2] * 1e3:8.2f}  stage3 {st[3] * 1e3:6.2f})", flush=True)
            del a0
    if args.out:
        json.dump(res, open(args.out, "w"), indent=1)


if __name__ == "__main__":
    main()
