"""Writes tests/golden/c1_oracle_f64.json from the CPU oracle alone (never from the HIP path).

The paper prints no worked example that can be recomputed without its trained weights, so the
stored values are the float64 oracle's own results on the smallest seeded workload.  They guard
the oracle against accidental changes of its arithmetic; the pins in tests/test_oracle_*.py are
what tie the oracle to the paper.  Run:  python tests/golden/make_golden.py
"""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as wl          # noqa: E402
from oracle import Oracle       # noqa: E402

PROBES = [(0, 0, 0), (0, 1, 0), (0, 48, 15), (1, 24, 7), (2, 0, 3), (3, 48, 0), (3, 30, 9)]


def compute():
    cfg = wl.CONFIGS["C1"]
    blob = wl.make_weights(cfg)
    z = wl.make_latent(cfg)
    orc = Oracle("f64")
    out = {"workload": "C1, weights seed 20250524+j, latent seed 7, tau 1e-3, mean-abs criterion, x0 = 0"}
    for name, mask in (("selective", ~1), ("sequential", 0), ("all_jacobi", ~0)):
        x, iters, deltas = orc.sample(cfg, blob, z, mask, cfg.tau)
        out[name] = {
            "iters": iters.tolist(),
            "last_delta": [[float(v) for v in row] for row in deltas],
            "probes": [[b, t, d, float(x[b, t, d])] for (b, t, d) in PROBES],
            "sum": float(x.sum()), "abs_sum": float(np.abs(x).sum()),
        }
    return out


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c1_oracle_f64.json")
    with open(path, "w") as f:
        json.dump(compute(), f, indent=1)
    print("wrote", path)
