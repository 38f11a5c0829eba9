"""The float64 oracle reproduces its stored results on the smallest workload (regression guard;
the file is written by tests/golden/make_golden.py from the oracle alone)."""
import json
import os

import numpy as np

import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


def test_oracle_reproduces_stored_config1_results(orc64, orc32):
    with open(os.path.join(HERE, "golden", "c1_oracle_f64.json")) as f:
        gold = json.load(f)
    cfg = wl.CONFIGS["C1"]
    blob = wl.make_weights(cfg); z = wl.make_latent(cfg)
    for name, mask in (("selective", ~1), ("sequential", 0), ("all_jacobi", ~0)):
        g = gold[name]
        x, iters, deltas = orc64.sample(cfg, blob, z, mask, cfg.tau)
        assert iters.tolist() == g["iters"]
        np.testing.assert_allclose(deltas, np.array(g["last_delta"]), rtol=1e-9, atol=1e-15)
        for b, t, d, v in g["probes"]:
            np.testing.assert_allclose(x[b, t, d], v, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(x.sum(), g["sum"], rtol=1e-10)
        # the float32 oracle takes the same number of passes and lands within 1e-4
        x32, it32, _ = orc32.sample(cfg, blob, z, mask, cfg.tau)
        assert it32.tolist() == g["iters"]
        assert np.abs(x32 - x).max() < 1e-4
