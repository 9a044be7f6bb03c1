#!/usr/bin/env python3
"""Writes the stored expected values of the full-size configurations from the CPU oracle ALONE.

    python tests/golden/make_oracle_goldens.py [2 3 5]

For each configuration the oracle (oracle/ols_oracle.py, fp32 state, double arithmetic, unrounded
operands) runs the whole job on the seeded synthetic inputs and the script stores, as JSON text:
the per-iteration mean loss, the per-worker losses of the last iteration, and a fixed sample of
parameter entries of the first and last replica and of the anchor together with their L2 norms.
Nothing here touches the HIP path.  Runtime on 8 cores: a few minutes (2), ~20 minutes (3, 5).
"""
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import ols_inputs as I                      # noqa: E402
from ols_inputs import generate as G        # noqa: E402
from oracle import workloads as OW          # noqa: E402

N_SAMPLE = 512


def sample_indices(d, seed):
    rng = np.random.default_rng(seed)
    return np.unique(np.concatenate([rng.integers(0, d, N_SAMPLE), [0, d - 1]]))


def main(which):
    for idx in which:
        cfg = I.get(idx)
        t0 = time.time()
        X, labels = G.mlp_data(cfg)
        x0 = G.mlp_init(cfg)

        def progress(k, s):
            if (k + 1) % 20 == 0:
                print("cfg%d iteration %d/%d  %.0f s" % (idx, k + 1, cfg.K, time.time() - t0), flush=True)

        st = OW.run_config(cfg, x0, OW.mlp_grad_fn(cfg.dims, X, labels), on_step=progress)
        cols = sample_indices(cfg.d, 1000 + idx)
        out = {
            "config": cfg.name, "m": cfg.m, "K": cfg.K, "d": cfg.d, "seed": cfg.seed,
            "oracle": "oracle/ols_oracle.py run(), store=float32, unrounded operands",
            "mean_loss": [float(v) for v in st["losses"].mean(axis=1)],
            "last_losses": [float(v) for v in st["losses"][-1]],
            "first_losses": [float(v) for v in st["losses"][0]],
            "cols": [int(c) for c in cols],
            "x_first": [float(v) for v in st["x"][0][cols]],
            "x_last": [float(v) for v in st["x"][-1][cols]],
            "z": [float(v) for v in st["z"][cols]],
            "norm_x": [float(np.linalg.norm(st["x"][i].astype(np.float64))) for i in range(cfg.m)],
            "norm_z": float(np.linalg.norm(st["z"].astype(np.float64))),
            "norm_x_minus_z": [float(np.linalg.norm(st["x"][i].astype(np.float64) - st["z"])) for i in range(cfg.m)],
        }
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_%s.json" % cfg.name)
        with open(path, "w") as f:
            json.dump(out, f)
        print("wrote %s in %.0f s" % (path, time.time() - t0), flush=True)


if __name__ == "__main__":
    main([int(a) for a in sys.argv[1:]] or [2, 3, 5])
