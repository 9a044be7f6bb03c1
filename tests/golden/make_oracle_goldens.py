#!/usr/bin/env python3
"""Writes the stored expected values of the full-size configurations from the CPU oracle ALONE.

    python tests/golden/make_oracle_goldens.py [2 3 5]

For each configuration the oracle (oracle/ols_oracle.py, fp32 state, double arithmetic, unrounded
operands) runs the whole job on the seeded synthetic inputs and the script stores, as JSON text:
the per-iteration mean loss, the per-worker losses of the first and last iteration, and a fixed sample of
entries (random positions, positions inside every layer's weight matrix and bias, the first and the last
entry) of EVERY replica's parameters and momentum buffer and of the anchor, together with L2 norms.
Nothing here touches the HIP path.  Runtime on 8 cores: a few minutes (2), 40-60 minutes (3, 5).
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

N_SAMPLE = 192        # positions drawn over the whole vector
N_PER_WEIGHT = 8      # plus this many inside every layer's weight matrix
N_PER_BIAS = 4        # and inside every layer's bias


def sample_indices(dims, seed):
    d = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
    rng = np.random.default_rng(seed)
    picks = [rng.integers(0, d, N_SAMPLE), [0, d - 1]]
    off = 0
    for l in range(len(dims) - 1):
        nw, nb = dims[l] * dims[l + 1], dims[l + 1]
        picks.append(off + rng.integers(0, nw, N_PER_WEIGHT))
        picks.append(off + nw + rng.integers(0, nb, N_PER_BIAS))
        off += nw + nb
    return np.unique(np.concatenate(picks))


def f32_text(a):
    """fp32 values as shortest text that reads back to the same fp32 (9 significant digits)."""
    return [float("%.9g" % v) for v in np.asarray(a, np.float32).ravel()]


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
        cols = sample_indices(cfg.dims, 1000 + idx)
        out = {
            "config": cfg.name, "m": cfg.m, "K": cfg.K, "d": cfg.d, "seed": cfg.seed,
            "oracle": "oracle/ols_oracle.py run(), store=float32, unrounded operands",
            "mean_loss": [float(v) for v in st["losses"].mean(axis=1)],
            "last_losses": [float(v) for v in st["losses"][-1]],
            "first_losses": [float(v) for v in st["losses"][0]],
            "cols": [int(c) for c in cols],
            "x": [f32_text(st["x"][i][cols]) for i in range(cfg.m)],        # [m][len(cols)]
            "buf": [f32_text(st["buf"][i][cols]) for i in range(cfg.m)],    # [m][len(cols)]
            "z": f32_text(st["z"][cols]),
            "norm_buf": [float(np.linalg.norm(st["buf"][i].astype(np.float64))) for i in range(cfg.m)],
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
