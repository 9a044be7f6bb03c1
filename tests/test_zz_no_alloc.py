"""The entry point for callers that cannot allocate (ols_run_steps_static: the attached model's workspace lives in a
static device array of the library) against the entry point it is a variant of (ols_run_steps with a caller-provided
workspace), through the C boundary: two calls in a row on one GPU, the second with a smaller input, both compared with
the existing entry point (identical launches, so identical bits) and with the CPU oracle at the end-to-end tolerance."""
import numpy as np
import pytest

import ols_inputs as I
from ols_inputs import generate as G
from oracle import workloads as OW
from tests.helpers import l2_ratio

from paper_2002_09539_amd import binding as B

pytestmark = pytest.mark.gpu

E2E_TOL = 1e-3


def _case(m, dims, batch, nb, seed):
    cfg = I.get(2).scaled(m=m, dims=tuple(dims), batch=batch, nb=nb, seed=seed, n_classes=dims[-1])
    X, labels = G.mlp_data(cfg)
    return cfg, X, labels, G.mlp_init(cfg)


def _run(cfg, X, labels, x0, K, static):
    from paper_2002_09539_amd.session import Session
    with Session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_mlp(cfg.dims, cfg.batch, "f32", workspace=not static)
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        if static:
            s.run_resident_static(K, Xd, yd)
        else:
            s.run_resident(K, Xd, yd)
        losses = s.losses()
        out = dict(x=s.all_params(), z=s.params(-1), buf=s.momentum(), losses=losses)
    return out


# first a case whose forward GEMM splits K (partial sums in the workspace) and spans several tiles, then a smaller,
# ragged one that reuses the same static array with stale contents from the first
CASES = [   # (m, dims, batch, nb, seed, K)
    (2, (3072, 512, 10), 128, 2, 71, 6),
    (3, (100, 72, 10), 36, 2, 72, 5),
]


def test_static_workspace_matches_bound_workspace_two_calls_in_a_row():
    assert B.ols_static_workspace_bytes() == 64 << 20
    for case in CASES:
        cfg, X, labels, x0 = _case(*case[:5])
        K = case[5]
        got = _run(cfg, X, labels, x0, K, static=True)
        ref = _run(cfg, X, labels, x0, K, static=False)
        for name in ("x", "z", "buf", "losses"):
            assert np.array_equal(got[name], ref[name]), "%s differs (case %r)" % (name, case)
        want = OW.run_config(cfg, x0, OW.mlp_grad_fn(cfg.dims, X, labels), K=K)
        for i in range(cfg.m):
            assert l2_ratio(got["x"][i], want["x"][i]) <= E2E_TOL
        assert l2_ratio(got["z"], want["z"]) <= E2E_TOL


def test_static_workspace_rejects_what_it_cannot_hold():
    from paper_2002_09539_amd.session import Session
    # 16 workers x batch 128 x 2048 hidden units x two hidden layers: more than 64 MiB of activations and deltas
    cfg = I.get(2).scaled(m=16, dims=(64, 2048, 2048, 10), batch=256)
    with Session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_mlp(cfg.dims, cfg.batch, "f32", workspace=False)
        assert B.ols_workspace_bytes(s.h) > B.ols_static_workspace_bytes()
        s.init_params(G.mlp_init(cfg))
        dummy = s.upload(np.zeros((cfg.m, 1, cfg.batch, 64), np.float32))
        labels = s.upload(np.zeros((cfg.m, 1, cfg.batch), np.int32))
        with pytest.raises(B.OlsError) as e:
            s.run_resident_static(1, dummy, labels)
        assert e.value.code == B.OLS_ENOMEM
    cfg = I.get(2).scaled(m=2, dims=(64, 64, 10), batch=16)
    with Session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_mlp(cfg.dims, cfg.batch, "bf16", workspace=True)
        s.init_params(G.mlp_init(cfg))
        dummy = s.upload(np.zeros((cfg.m, 1, cfg.batch, 64), np.float32))
        labels = s.upload(np.zeros((cfg.m, 1, cfg.batch), np.int32))
        with pytest.raises(B.OlsError) as e:
            s.run_resident_static(1, dummy, labels)
        assert e.value.code == B.OLS_EINVAL
