"""Pins of the oracle's stale-average synchronisation ("Related Works": the local updates of a round are
applied to the average of the models as they stood tau iterations before, so that averaging and local
computation can overlap).  No GPU.

What fixes it other than itself: with constant gradients the iterates have a closed form in which a
worker's own gradient counts at once and the others' one round late; with gradients linear in x the
replica mean follows plain gradient descent on the averaged objective, whatever the synchronisation
does to the spread; identical workers never notice the synchronisation; one worker is plain SGD; a
scalar two-worker run is recomputed with explicit Python floats.  The last test plants mistakes in the
oracle (on the CPU) and checks that these pins notice them."""
import numpy as np
import pytest

from oracle import ols_oracle as O

F64 = np.float64


def const_grad_fn(G):
    return lambda i, k, x: (0.0, G[i])


def quad_grad_fn(centers, a=1.0):
    return lambda i, k, x: (0.5 * a * float(np.sum((np.asarray(x, F64) - centers[i]) ** 2)),
                            a * (np.asarray(x, F64) - centers[i]))


@pytest.mark.parametrize("m,tau,rounds,extra", [(3, 2, 1, 0), (3, 2, 4, 1), (5, 3, 3, 2), (2, 1, 5, 0)])
def test_constant_gradients_closed_form(m, tau, rounds, extra):
    """After R >= 1 synchronisations and j further local steps:
    x_i = x0 - gamma tau [(R - 1) gbar + g_i] - gamma j g_i."""
    rng = np.random.default_rng(3)
    d, gamma = 6, 0.05
    G = rng.normal(size=(m, d))
    x0 = rng.normal(size=d)
    out = O.run_stale_average(x0, m, tau, gamma, rounds * tau + extra, const_grad_fn(G), store=F64)
    gbar = G.mean(axis=0)
    for i in range(m):
        want = x0 - gamma * tau * ((rounds - 1) * gbar + G[i]) - gamma * extra * G[i]
        np.testing.assert_allclose(out["x"][i], want, rtol=0, atol=1e-13)
    if extra == 0:
        np.testing.assert_allclose(out["z"], x0 - gamma * tau * rounds * gbar, rtol=0, atol=1e-13)
        np.testing.assert_array_equal(out["snap"], out["x"])


@pytest.mark.parametrize("mu", [0.0, 0.9])
def test_replica_mean_follows_gradient_descent_on_the_average(mu):
    """Linear gradients a (x - c_i): the synchronisation leaves the replica mean where it was, so the mean
    obeys the single-model (momentum) recursion on 0.5 a ||x - cbar||^2."""
    rng = np.random.default_rng(4)
    m, d, tau, K, gamma, a = 4, 5, 3, 14, 0.1, 0.7
    centers = rng.normal(size=(m, d))
    x0 = rng.normal(size=d)
    out = O.run_stale_average(x0, m, tau, gamma, K, quad_grad_fn(centers, a), mu=mu, store=F64)
    cbar = centers.mean(axis=0)
    x, b = x0.astype(F64).copy(), np.zeros(d)
    for _ in range(K):           # PyTorch-style Nesterov written out
        g = a * (x - cbar)
        b = mu * b + g
        x = x - gamma * (g + mu * b if mu else g)
    np.testing.assert_allclose(out["x"].mean(axis=0), x, rtol=0, atol=1e-12)


def test_sync_preserves_the_mean_and_the_progress():
    rng = np.random.default_rng(5)
    m, d = 6, 9
    snap = rng.normal(size=(m, d))
    x = snap + 0.1 * rng.normal(size=(m, d))
    z = snap.mean(axis=0)
    new = O.stale_average_sync(x, snap, z)
    np.testing.assert_allclose(new.mean(axis=0), x.mean(axis=0), rtol=0, atol=1e-14)
    # every worker keeps exactly its own progress, measured from the common point
    np.testing.assert_allclose(new - z[None, :], x - snap, rtol=0, atol=1e-14)


@pytest.mark.parametrize("mu,nesterov", [(0.0, True), (0.9, True), (0.9, False)])
def test_identical_workers_and_single_worker_are_plain_sgd(mu, nesterov):
    rng = np.random.default_rng(6)
    d, tau, K, gamma = 5, 2, 9, 0.08
    c = rng.normal(size=d)
    x0 = rng.normal(size=d)
    one = O.run(x0, 1, tau, 0.0, gamma, K, quad_grad_fn(c[None, :], 1.1), mu=mu, nesterov=nesterov, store=F64)
    for m in (1, 4):
        centers = np.repeat(c[None, :], m, axis=0)
        out = O.run_stale_average(x0, m, tau, gamma, K, quad_grad_fn(centers, 1.1), mu=mu, nesterov=nesterov,
                                  store=F64)
        for i in range(m):
            np.testing.assert_allclose(out["x"][i], one["x"][0], rtol=0, atol=1e-13)


def test_scalar_two_workers_brute_force():
    """f_1 = 0.5 (x - 1)^2, f_2 = (x + 2)^2, tau = 2, plain floats and explicit bookkeeping."""
    gamma, tau, K, x0 = 0.1, 2, 7, 0.5
    xa = xb = sa = sb = x0
    avg = x0
    for k in range(K):
        xa = xa - gamma * (xa - 1.0)
        xb = xb - gamma * 2.0 * (xb + 2.0)
        if (k + 1) % tau == 0:
            xa, xb = avg + (xa - sa), avg + (xb - sb)
            sa, sb = xa, xb
            avg = 0.5 * (sa + sb)
    fn = lambda i, k, x: (0.0, (x - 1.0) if i == 0 else 2.0 * (x + 2.0))
    out = O.run_stale_average(np.array([x0]), 2, tau, gamma, K, fn, store=F64)
    np.testing.assert_allclose(out["x"][:, 0], [xa, xb], rtol=0, atol=1e-14)
    np.testing.assert_allclose(out["z"][0], avg, rtol=0, atol=1e-14)


def test_float32_store_rounds_once_per_write():
    rng = np.random.default_rng(7)
    m, d, tau, K, gamma = 3, 40, 2, 6, 0.05
    centers = rng.normal(size=(m, d))
    x0 = rng.normal(size=d)
    a = O.run_stale_average(x0, m, tau, gamma, K, quad_grad_fn(centers), mu=0.9, store=np.float32)
    b = O.run_stale_average(x0.astype(np.float32), m, tau, gamma, K, quad_grad_fn(centers), mu=0.9, store=F64)
    assert a["x"].dtype == np.float32 and a["snap"].dtype == np.float32
    np.testing.assert_allclose(a["x"], b["x"], rtol=2e-6, atol=2e-6)


# ---- planted mistakes -------------------------------------------------------------------------------------
def _pins():
    return [lambda: test_constant_gradients_closed_form(3, 2, 4, 1),
            lambda: test_replica_mean_follows_gradient_descent_on_the_average(0.9),
            test_sync_preserves_the_mean_and_the_progress,
            lambda: test_identical_workers_and_single_worker_are_plain_sgd(0.9, True),
            test_scalar_two_workers_brute_force]


def _some_pin_fails():
    for pin in _pins():
        try:
            pin()
        except AssertionError:
            return True
    return False


def _sync_forgets_progress(x, snap, z):
    return np.repeat(np.asarray(z, F64)[None, :], np.asarray(x).shape[0], axis=0)


def _sync_wrong_sign(x, snap, z):
    return np.asarray(z, F64)[None, :] - (np.asarray(x, F64) - np.asarray(snap, F64))


def _sync_progress_from_average(x, snap, z):   # subtracts the average instead of the worker's own snapshot
    return np.asarray(z, F64)[None, :] + (np.asarray(x, F64) - np.asarray(snap, F64).mean(axis=0)[None, :])


def _average_is_sum(xs):
    return np.asarray(xs, F64).sum(axis=0)


@pytest.mark.parametrize("name,wrong", [("stale_average_sync", _sync_forgets_progress),
                                        ("stale_average_sync", _sync_wrong_sign),
                                        ("stale_average_sync", _sync_progress_from_average),
                                        ("anchor_average", _average_is_sum)])
def test_planted_mistakes_are_noticed(monkeypatch, name, wrong):
    assert not _some_pin_fails()
    monkeypatch.setattr(O, name, wrong)
    assert _some_pin_fails()
