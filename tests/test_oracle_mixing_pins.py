"""Pins of the oracle's general mixing step X <- X W (Section 2, "Matrix-Form Update Rule", with the
remark that other column-stochastic W can take the printed one's place).  No GPU.

What fixes it other than itself: the paper's own W must reproduce the vector-form iteration (pull-back,
then anchor average of the post-pull models); the periodic-averaging W must reproduce Local SGD's rule
as printed in the first display of Section 2, written out here as explicit loops; consensus is a fixed
point of every column-stochastic W; two mixing steps compose to the matrix product; the symmetric
elastic W preserves the plain sum of all m + 1 columns (it is doubly stochastic)."""
import numpy as np
import pytest

from oracle import ols_oracle as O

F64 = np.float64


def quad_grad_fn(centers, a=1.0):
    """Worker i minimises 0.5 a ||x - c_i||^2: exact gradient a (x - c_i)."""
    return lambda i, k, x: (0.5 * a * float(np.sum((np.asarray(x, F64) - centers[i]) ** 2)),
                            a * (np.asarray(x, F64) - centers[i]))


def random_column_stochastic(n, rng):
    W = rng.random((n, n)) + 0.05
    return W / W.sum(axis=0, keepdims=True)


@pytest.mark.parametrize("m,tau,mu", [(3, 2, 0.0), (5, 3, 0.9), (1, 1, 0.0)])
def test_paper_matrix_reproduces_vector_form(m, tau, mu):
    rng = np.random.default_rng(1)
    d, K, alpha, gamma = 7, 11, 0.6, 0.07
    centers = rng.normal(size=(m, d))
    x0 = rng.normal(size=d)
    fn = quad_grad_fn(centers)
    want = O.run(x0, m, tau, alpha, gamma, K, fn, mu=mu, store=F64)
    got = O.run_general_mixing(x0, m, tau, gamma, K, fn, O.mixing_matrix(m, alpha), mu=mu, store=F64)
    np.testing.assert_allclose(got["x"], want["x"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(got["z"], want["z"], rtol=0, atol=1e-13)
    if mu:
        np.testing.assert_allclose(got["buf"], want["buf"], rtol=0, atol=1e-13)


def test_periodic_averaging_is_local_sgd_as_printed():
    """x_{k+1}^{(i)} = (1/m) sum_j [x_k^{(j)} - gamma g_j] when (k+1) mod tau == 0, else the local step."""
    rng = np.random.default_rng(2)
    m, d, tau, K, gamma = 4, 6, 3, 10, 0.05
    centers = rng.normal(size=(m, d))
    x0 = rng.normal(size=d)
    fn = quad_grad_fn(centers, a=1.3)
    x = [x0.astype(F64).copy() for _ in range(m)]
    for k in range(K):
        half = []
        for j in range(m):
            _, g = fn(j, k, x[j])
            half.append(x[j] - gamma * g)
        if (k + 1) % tau == 0:
            mean = np.zeros(d)
            for j in range(m):
                mean += half[j]
            mean /= m
            x = [mean.copy() for _ in range(m)]
        else:
            x = half
    got = O.run_general_mixing(x0, m, tau, gamma, K, fn, O.periodic_averaging_matrix(m), store=F64)
    np.testing.assert_allclose(got["x"], np.stack(x), rtol=0, atol=1e-13)


@pytest.mark.parametrize("n", [2, 5, 17])
def test_consensus_is_a_fixed_point_of_column_stochastic_mixing(n):
    rng = np.random.default_rng(n)
    W = random_column_stochastic(n, rng)
    c = rng.normal(size=9)
    X = np.repeat(c[:, None], n, axis=1)
    np.testing.assert_allclose(O.mix(X, W), X, rtol=0, atol=1e-14)
    # and only then: a matrix whose columns do not sum to one moves the consensus
    W_bad = W.copy()
    W_bad[0, 0] += 0.1
    assert np.abs(O.mix(X, W_bad) - X).max() > 1e-3


def test_mixing_steps_compose_and_use_columns_as_output_weights():
    rng = np.random.default_rng(4)
    n, d = 6, 5
    X = rng.normal(size=(d, n))
    W1, W2 = random_column_stochastic(n, rng), random_column_stochastic(n, rng)
    np.testing.assert_allclose(O.mix(O.mix(X, W1), W2), O.mix(X, W1 @ W2), rtol=0, atol=1e-13)
    # output column j is the combination of the input columns with the weights W[:, j], written out
    j = 2
    want = np.zeros(d)
    for i in range(n):
        want += W1[i, j] * X[:, i]
    np.testing.assert_allclose(O.mix(X, W1)[:, j], want, rtol=0, atol=1e-14)
    # a transposed operand is a different result
    assert np.abs(O.mix(X, W1) - np.asarray(X) @ W1.T).max() > 1e-3


def test_named_matrices_have_the_stated_structure():
    m, alpha = 5, 0.1
    P = O.periodic_averaging_matrix(m)
    E = O.elastic_symmetric_matrix(m, alpha)
    W = O.mixing_matrix(m, 0.6)
    one = np.ones(m + 1)
    for M in (P, E, W):
        np.testing.assert_allclose(one @ M, one, atol=1e-15)          # column-stochastic
    np.testing.assert_allclose(E, E.T, atol=0)                        # symmetric ...
    np.testing.assert_allclose(E @ one, one, atol=1e-15)              # ... hence doubly stochastic
    assert np.abs(W @ one - one).max() > 0.1                          # the paper's W is NOT row-stochastic
    rng = np.random.default_rng(5)
    X = rng.normal(size=(4, m + 1))
    np.testing.assert_allclose(O.mix(X, E).sum(axis=1), X.sum(axis=1), atol=1e-13)   # plain sum preserved
    # elastic step written out: x_i - alpha (x_i - z), z + alpha sum_i (x_i - z)
    got = O.mix(X, E)
    for i in range(m):
        np.testing.assert_allclose(got[:, i], X[:, i] - alpha * (X[:, i] - X[:, m]), atol=1e-14)
    np.testing.assert_allclose(got[:, m], X[:, m] + alpha * (X[:, :m] - X[:, [m]]).sum(axis=1), atol=1e-14)


def test_fp32_store_rounds_once_per_mixing_step():
    rng = np.random.default_rng(6)
    m, d = 3, 50
    x0 = rng.normal(size=d).astype(np.float32)
    centers = rng.normal(size=(m, d))
    W = random_column_stochastic(m + 1, rng)
    st = O.run_general_mixing(x0, m, 1, 0.1, 1, quad_grad_fn(centers), W, store=np.float32)
    half = np.stack([(x0.astype(F64) - 0.1 * (x0.astype(F64) - centers[i])).astype(np.float32) for i in range(m)])
    X = np.concatenate([half.astype(F64), x0.astype(F64)[None, :]], axis=0).T
    want = (X @ W).astype(np.float32)
    assert np.array_equal(st["x"], want[:, :m].T) and np.array_equal(st["z"], want[:, m])
