"""Full-size runs of the MLP configurations (2, 3, 5) in the launch configuration the benchmark
times, compared with expected values the CPU oracle alone produced beforehand
(tests/golden/make_oracle_goldens.py -> tests/golden/oracle_<config>.json): sampled entries of EVERY
replica's parameters and momentum buffer and of the anchor, the mean loss at every iteration and every
worker's loss at the last one."""
import json
import os

import numpy as np
import pytest

import ols_inputs as I
from ols_inputs import generate as G
from tests.helpers import l2_ratio

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

# The benchmark specification's bars: fp32 end-to-end parameters <= 1e-3 relative; bf16-GEMM runs <= 2e-2
# relative on the loss.  For the bf16 run's PARAMETERS the specification states nothing; 5e-2 (L2, per replica, over
# the sampled entries) is this test's own bar: operands carry 2^-9 relative rounding and 200 iterations compound it.
TOL = {2: dict(loss=1e-3, params=1e-3), 5: dict(loss=1e-3, params=1e-3), 3: dict(loss=2e-2, params=5e-2)}


@pytest.mark.parametrize("idx", [2, 5, 3])
def test_full_config_matches_stored_oracle_run(idx):
    from paper_2002_09539_amd.session import Session
    cfg = I.get(idx)
    path = os.path.join(GOLDEN, "oracle_%s.json" % cfg.name)
    gold = json.load(open(path))
    assert gold["K"] == cfg.K and gold["m"] == cfg.m and gold["d"] == cfg.d and gold["seed"] == cfg.seed
    cols = np.array(gold["cols"])
    X, labels = G.mlp_data(cfg)
    x0 = G.mlp_init(cfg)
    runs = []
    for library_loop in (False, True):     # one call per step (losses at every iteration), then ols_run_steps
        with Session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
            s.attach_mlp(cfg.dims, cfg.batch, cfg.gemm_dtype)
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            losses = []
            if library_loop:
                s.run_resident(cfg.K, Xd, yd)
                losses.append(s.losses())
            else:
                s.run(cfg.K, lambda k: s.set_batch(Xd[:, k % cfg.nb], yd[:, k % cfg.nb]), losses=losses)
            s.sync()
            full = s.all_params()
            runs.append(dict(x=full[:, cols], z=s.params(-1)[cols], buf=s.momentum()[:, cols],
                             norm_x=np.linalg.norm(full.astype(np.float64), axis=1), losses=np.array(losses)))
            del full
    a, b = runs
    # the loop inside the library issues the same launches as one call per step: identical bits
    for name in ("x", "z", "buf"):
        assert np.array_equal(a[name], b[name]), name
    assert np.array_equal(a["losses"][-1], b["losses"][-1])
    tol = TOL[idx]
    losses = a["losses"]
    mean_loss = losses.mean(axis=1)
    rel = np.abs(mean_loss - np.array(gold["mean_loss"])) / np.abs(gold["mean_loss"])
    assert rel.max() <= tol["loss"], "mean loss deviates by %.3e at iteration %d" % (rel.max(), rel.argmax())
    rel_last = np.abs(losses[-1] - np.array(gold["last_losses"])) / np.abs(gold["last_losses"])
    assert rel_last.max() <= tol["loss"], "worker %d's last loss deviates by %.3e" % (rel_last.argmax(), rel_last.max())
    gx, gb = np.array(gold["x"]), np.array(gold["buf"])
    assert gx.shape == (cfg.m, len(cols)) and gb.shape == gx.shape
    for i in range(cfg.m):                                      # every replica, element by element on the sample
        assert l2_ratio(a["x"][i], gx[i]) <= tol["params"], "replica %d" % i
        assert l2_ratio(a["buf"][i], gb[i]) <= max(tol["params"], 2e-3), "momentum of replica %d" % i
    assert l2_ratio(a["z"], gold["z"]) <= tol["params"]
    assert np.abs(a["norm_x"] / np.array(gold["norm_x"]) - 1).max() <= tol["params"]
    # the run really trains: the loss falls well below its starting value
    assert mean_loss[-10:].mean() < 0.7 * mean_loss[:2].mean()
