"""GPU parity of the general mixing step X <- X W (one pass over the m + 1 rows [x^(1..m), z]) against
the CPU oracle's definition X @ W, through the C boundary.

Tolerance: every output element is an fp32 fma chain of m + 1 terms over inputs of comparable size; each
fma rounds once (2^-24 relative to the running sum), so the error against the double result is bounded by
(m + 1) 2^-24 times the largest partial sum.  For the column-stochastic matrices used here (non-negative
weights summing to one) partial sums stay below the row maximum, which gives the bar written below;
for m <= 16 it is the benchmark specification's 1e-6 for fp32 averaging kernels."""
import numpy as np
import pytest
import torch

import ols_inputs as I
from ols_inputs import generate as G
from oracle import ols_oracle as O
from oracle import workloads as OW
from tests.helpers import max_norm_ratio

from paper_2002_09539_amd import binding as B

pytestmark = pytest.mark.gpu


def tol_for(m):
    return max(1e-6, (m + 1) * 2.0 ** -24)


def make_session(*a, **kw):
    from paper_2002_09539_amd.session import Session
    return Session(*a, **kw)


def column_stochastic(n, seed):
    rng = np.random.default_rng(seed)
    W = rng.random((n, n)) + 0.05
    return (W / W.sum(axis=0, keepdims=True)).astype(np.float32)


def stream_inputs(m, d, n_grads, seed):
    cfg = I.get(4).scaled(m=m, d_flat=d, seed=seed)
    return G.stream_x0(cfg), [G.stream_gradient(cfg, j) for j in range(n_grads)]


def run_gpu(sess, x0, grads, K, W):
    dev = [torch.zeros(sess.m, sess.ld, dtype=torch.float32, device=sess.device) for _ in grads]
    for t, g in zip(dev, grads):
        t[:, : sess.d] = torch.from_numpy(g).to(sess.device)
    torch.cuda.synchronize()
    sess.bind(dev[0])
    sess.init_params(x0)
    sess.set_mixing(W)
    sess.run(K, lambda k: sess.set_gradient(dev[k % len(dev)]))
    return sess.all_params(), sess.params(-1), sess.momentum()


@pytest.mark.parametrize("m,d", [(1, 100), (4, 1000), (8, 4099), (16, 70001), (17, 5000), (32, 3001),
                                 (40, 2050), (64, 1023), (100, 777)])
def test_one_mixing_step_matches_definition(m, d):
    """tau = 1, one iteration: local step, then X W with a random column-stochastic W, every register
    width and row-count variant of the kernel, ragged d."""
    x0, grads = stream_inputs(m, d, 1, seed=11 + m)
    W = column_stochastic(m + 1, 100 + m)
    st = O.run_general_mixing(x0, m, 1, 0.1, 1, OW.stream_grad_fn(grads), W.astype(np.float64), mu=0.9)
    with make_session(m, d, 1, 0.5, 0.1, 0.9) as s:
        x, z, buf = run_gpu(s, x0, grads, 1, W)
    tol = tol_for(m)
    for i in range(m):
        assert max_norm_ratio(x[i], st["x"][i]) <= tol, "replica %d" % i
    assert max_norm_ratio(z, st["z"]) <= tol
    assert max(max_norm_ratio(buf[i], st["buf"][i]) for i in range(m)) <= 1e-6


@pytest.mark.parametrize("kind", ["paper", "averaging", "elastic"])
def test_named_matrices_over_several_rounds(kind):
    m, d, tau, K, gamma, alpha = 8, 20011, 3, 12, 0.05, 0.6
    x0, grads = stream_inputs(m, d, 4, seed=21)
    W = {"paper": O.mixing_matrix(m, alpha), "averaging": O.periodic_averaging_matrix(m),
         "elastic": O.elastic_symmetric_matrix(m, 0.05)}[kind].astype(np.float32)
    st = O.run_general_mixing(x0, m, tau, gamma, K, OW.stream_grad_fn(grads), W.astype(np.float64), mu=0.9)
    with make_session(m, d, tau, alpha, gamma, 0.9) as s:
        x, z, _ = run_gpu(s, x0, grads, K, W)
    assert max(max_norm_ratio(x[i], st["x"][i]) for i in range(m)) <= 5e-6     # K / tau = 4 mixing steps
    assert max_norm_ratio(z, st["z"]) <= 5e-6
    if kind == "averaging":     # every replica and the anchor hold the same bits after a synchronisation
        assert all(np.array_equal(x[0], x[i]) for i in range(1, m)) and np.array_equal(x[0], z)


def test_paper_matrix_agrees_with_pull_and_average_kernels():
    """The same run through the pull-back + anchor-mean kernels and through the mixing kernel with the
    paper's W: two different fp32 evaluation orders of the same rule, equal within rounding."""
    m, d, tau, K, gamma, alpha = 16, 50021, 2, 8, 0.1, 0.6
    x0, grads = stream_inputs(m, d, 2, seed=31)
    with make_session(m, d, tau, alpha, gamma, 0.9) as s:
        xa, za, _ = run_gpu(s, x0, grads, K, None)
    with make_session(m, d, tau, alpha, gamma, 0.9) as s:
        xb, zb, _ = run_gpu(s, x0, grads, K, O.mixing_matrix(m, alpha).astype(np.float32))
    assert max(max_norm_ratio(xb[i], xa[i]) for i in range(m)) <= 5e-6
    assert max_norm_ratio(zb, za) <= 5e-6


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_mixing_with_an_attached_mlp(dtype):
    """Periodic averaging of MLP replicas (gradient kernels apply the local step, the synchronisation is
    the mixing kernel; with bf16 GEMMs it also refreshes the bf16 weight copy)."""
    m, dims, batch, tau, K = 4, (64, 48, 32, 10), 16, 2, 6
    cfg = I.get(2).scaled(m=m, dims=dims, batch=batch, nb=3, seed=41, n_classes=10)
    X, labels = G.mlp_data(cfg)
    x0 = G.mlp_init(cfg)
    W = O.periodic_averaging_matrix(m).astype(np.float32)
    st = O.run_general_mixing(x0, m, tau, 0.05, K, OW.mlp_grad_fn(dims, X, labels), W.astype(np.float64), mu=0.9)
    with make_session(m, cfg.d, tau, 0.5, 0.05, 0.9) as s:
        s.attach_mlp(dims, batch, dtype)
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.set_mixing(W)
        losses = []
        s.run(K, lambda k: s.set_batch(Xd[:, k % 3], yd[:, k % 3]), losses=losses)
        x, z = s.all_params(), s.params(-1)
    rel = np.abs(np.array(losses) - st["losses"]) / np.abs(st["losses"])
    if dtype == "f32":
        assert rel.max() <= 1e-3
        assert max(np.linalg.norm(x[i] - st["x"][i]) / np.linalg.norm(st["x"][i]) for i in range(m)) <= 1e-3
    else:
        assert rel.max() <= 2e-2      # the bar for bf16-GEMM runs, on the loss
    assert all(np.array_equal(x[0], x[i]) for i in range(1, m)) and np.array_equal(x[0], z)
