"""Write tests/golden/sigma_<config>.txt: the oracle's singular values for one
of the named workloads, with a fingerprint of the input matrix.

Calls only the generators (workloads.py) and the CPU oracle (oracle/); nothing
from the HIP path.  Usage:  python tests/golden/make_oracle_sigma.py c4 [c5b ...]
"""
import json
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle      # noqa: E402
import workloads   # noqa: E402


def main(names):
    for name in names:
        t0 = time.time()
        a, info = workloads.make(name)
        fp = workloads.fingerprint(a)
        t1 = time.time()
        s = oracle.svdvals(a)
        t2 = time.time()
        meta = dict(config=name, n=info["n"], dtype=info["dtype"], seed=info["seed"],
                    fingerprint=fp, oracle_seconds=round(t2 - t1, 2),
                    oracle_threads=oracle.num_threads())
        path = os.path.join(HERE, f"sigma_{name}.txt")
        with open(path, "w") as f:
            f.write("# " + json.dumps(meta) + "\n")
            for v in s:
                f.write(repr(float(v)) + "\n")
        print(f"{name}: generated in {t1 - t0:.1f}s, oracle {t2 - t1:.1f}s -> {path}", flush=True)


def load(name):
    """Returns (sigma, meta) or None when no stored result exists."""
    path = os.path.join(HERE, f"sigma_{name}.txt")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        meta = json.loads(f.readline()[2:])
        s = np.array([float(x) for x in f if x.strip()])
    return s, meta


if __name__ == "__main__":
    main(sys.argv[1:])
