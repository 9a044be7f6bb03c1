"""Pins for the CPU oracle: what the paper and plain mathematics fix, checked
without any GPU.  Each test names the passage of arXiv 2002.09539 it rests on.
"""
import numpy as np
import pytest
import torch

from oracle import ols_oracle as O

F64 = np.float64


def quad_grad(a, centers):
    """g_i(x) = a (x - c_i): gradient of F_i = 0.5 a ||x - c_i||^2 (deterministic)."""
    return lambda i, k, x: (0.0, a * (np.asarray(x, F64) - centers[i]))


def rand(shape, seed):
    return np.random.default_rng(seed).standard_normal(shape)


# ---------------------------------------------------------------------------
# closed forms on quadratics (derived from the three update rules of Section 2)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("tau,alpha", [(1, 0.5), (2, 0.6), (4, 0.5), (8, 0.25)])
def test_closed_form_identical_quadratic(tau, alpha):
    m, d, a, gamma, rounds = 5, 7, 0.7, 0.3, 6
    x0 = rand(d, 1)
    st = O.run(x0, m, tau, alpha, gamma, rounds * tau, quad_grad(a, np.zeros((m, d))), store=F64)
    rho = 1.0 - gamma * a
    factor = ((1.0 - alpha) * rho ** tau + alpha) ** rounds
    np.testing.assert_allclose(st["x"], np.tile(factor * x0, (m, 1)), rtol=1e-13)
    np.testing.assert_allclose(st["z"], factor * x0, rtol=1e-13)


def test_closed_form_identical_quadratic_with_a_learning_rate_schedule():
    """gamma_k varies (Section 4: warm-up, then step decays): round r multiplies x by
    (1 - alpha) prod_{k in r} (1 - gamma_k a) + alpha; a constant schedule is the plain run."""
    m, d, a, tau, alpha, rounds = 3, 5, 0.7, 3, 0.6, 4
    x0 = rand(d, 11)
    gammas = [0.02 * (k + 1) for k in range(5)] + [0.3] * 4 + [0.03] * 3        # warm-up, plateau, decay
    st = O.run(x0, m, tau, alpha, lambda k: gammas[k], rounds * tau, quad_grad(a, np.zeros((m, d))), store=F64)
    factor = 1.0
    for r in range(rounds):
        rho = np.prod([1.0 - gammas[k] * a for k in range(r * tau, (r + 1) * tau)])
        factor *= (1.0 - alpha) * rho + alpha
    np.testing.assert_allclose(st["x"], np.tile(factor * x0, (m, 1)), rtol=1e-13)
    np.testing.assert_allclose(st["z"], factor * x0, rtol=1e-13)
    const = O.run(x0, m, tau, alpha, lambda k: 0.3, rounds * tau, quad_grad(a, rand((m, d), 12)), mu=0.9, store=F64)
    plain = O.run(x0, m, tau, alpha, 0.3, rounds * tau, quad_grad(a, rand((m, d), 12)), mu=0.9, store=F64)
    np.testing.assert_array_equal(const["x"], plain["x"])


def test_closed_form_heterogeneous_quadratic():
    """Mean and deviations of the replicas after each round, F_i = 0.5 a ||x - c_i||^2."""
    m, d, a, gamma, tau, alpha = 4, 6, 0.9, 0.2, 3, 0.6
    c = rand((m, d), 2)
    x0 = rand(d, 3)
    rho_t = (1.0 - gamma * a) ** tau
    cbar = c.mean(axis=0)
    mean, dev = x0.copy(), np.zeros((m, d))
    for rounds in range(1, 5):
        mean = ((1 - alpha) * rho_t + alpha) * mean + (1 - alpha) * (1 - rho_t) * cbar
        dev = (1 - alpha) * (rho_t * dev + (1 - rho_t) * (c - cbar))
        st = O.run(x0, m, tau, alpha, gamma, rounds * tau, quad_grad(a, c), store=F64)
        np.testing.assert_allclose(st["x"].mean(axis=0), mean, rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(st["x"] - st["x"].mean(axis=0), dev, rtol=1e-11, atol=1e-14)
        np.testing.assert_allclose(st["z"], mean, rtol=1e-12, atol=1e-14)


def test_momentum_quadratic_matrix_power():
    """Local Nesterov momentum (Momentum Variant paragraph) on a 1-d quadratic: the state
    [x_1..x_m, buf_1..buf_m, z, 1] evolves by one constant affine map per round."""
    m, a, gamma, mu, tau, alpha = 3, 0.8, 0.15, 0.9, 2, 0.6
    c = np.array([0.5, -1.0, 2.0])
    n = 2 * m + 2
    step = np.eye(n)
    for i in range(m):
        # buf' = mu buf + a (x - c);  x' = x - gamma (a (x - c) + mu buf')
        step[m + i, :] = 0
        step[m + i, m + i] = mu
        step[m + i, i] = a
        step[m + i, n - 1] = -a * c[i]
        step[i, :] = 0
        step[i, i] = 1 - gamma * a * (1 + mu)
        step[i, m + i] = -gamma * mu * mu
        step[i, n - 1] = gamma * a * (1 + mu) * c[i]
    pull = np.eye(n)
    for i in range(m):
        pull[i, i] = 1 - alpha
        pull[i, 2 * m] = alpha
    avg = np.eye(n)
    avg[2 * m, :] = 0
    avg[2 * m, :m] = 1.0 / m
    round_map = avg @ pull @ np.linalg.matrix_power(step, tau)
    x0 = 1.7
    s0 = np.concatenate([np.full(m, x0), np.zeros(m), [x0, 1.0]])
    rounds = 5
    want = np.linalg.matrix_power(round_map, rounds) @ s0
    st = O.run(np.array([x0]), m, tau, alpha, gamma, rounds * tau,
               quad_grad(a, c[:, None]), mu=mu, nesterov=True, store=F64)
    got = np.concatenate([st["x"][:, 0], st["buf"][:, 0], st["z"], [1.0]])
    np.testing.assert_allclose(got, want, rtol=1e-12)


# ---------------------------------------------------------------------------
# Appendix A: mixing matrix identities, matrix form, virtual sequence
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("m,alpha", [(1, 0.3), (4, 0.6), (16, 0.5)])
def test_mixing_matrix_identities(m, alpha):
    W = O.mixing_matrix(m, alpha)
    one = np.ones(m + 1)
    v = np.concatenate([np.full(m, (1 - alpha) / m), [alpha]])
    np.testing.assert_allclose(one @ W, one, atol=1e-15)          # column-stochastic
    np.testing.assert_allclose(W @ v, v, atol=1e-15)              # W v = v
    assert abs(v @ one - 1.0) < 1e-15
    # spectral bound of Appendix A: ||P - v 1^T||_2 ... every non-unit eigenvalue has modulus <= 1 - alpha
    eig = np.sort(np.abs(np.linalg.eigvals(W)))
    assert abs(eig[-1] - 1.0) < 1e-12 and np.all(eig[:-1] <= 1 - alpha + 1e-12)


def lsq_problem(m, nb, B, d, seed):
    A = rand((m, nb, B, d), seed)
    y = rand((m, nb, B), seed + 1)
    return A, y, (lambda i, k, x: O.lsq_loss_grad(x, A[i, k % nb], y[i, k % nb]))


@pytest.mark.parametrize("tau", [1, 2, 3])
def test_vector_form_equals_matrix_form(tau):
    m, d, alpha, gamma, K = 4, 9, 0.6, 0.05, 7          # K not a multiple of tau on purpose
    _, _, gf = lsq_problem(m, 3, 5, d, 10)
    x0 = rand(d, 12)
    st = O.run(x0, m, tau, alpha, gamma, K, gf, store=F64)
    X = O.run_matrix_form(x0, m, tau, alpha, gamma, K, gf)
    np.testing.assert_allclose(st["x"].T, X[:, :m], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(st["z"], X[:, m], rtol=1e-12, atol=1e-14)


def test_matrix_form_on_mlp_gradients():
    dims = (6, 5, 4)
    m, tau, alpha, gamma, K = 3, 2, 0.5, 0.1, 6
    Xd = rand((m, 2, 4, dims[0]), 20)
    lab = np.random.default_rng(21).integers(0, dims[-1], (m, 2, 4))
    gf = lambda i, k, x: O.mlp_loss_grad(x, dims, Xd[i, k % 2], lab[i, k % 2])
    d = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(2))
    x0 = 0.3 * rand(d, 22)
    st = O.run(x0, m, tau, alpha, gamma, K, gf, store=F64)
    X = O.run_matrix_form(x0, m, tau, alpha, gamma, K, gf)
    np.testing.assert_allclose(st["x"].T, X[:, :m], rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(st["z"], X[:, m], rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("tau", [1, 2, 5])
def test_virtual_sequence_recursion_every_step(tau):
    """y_{k+1} = y_k - (1 - alpha) gamma mean_i g_i(x_k^{(i)}) at every k (Appendix A)."""
    m, d, alpha, gamma, K = 5, 8, 0.6, 0.03, 11
    _, _, gf = lsq_problem(m, 4, 6, d, 30)
    x0 = rand(d, 31)
    grads = {}

    def recording(i, k, x):
        loss, g = gf(i, k, x)
        grads.setdefault(k, []).append(g)
        return loss, g

    ys = [O.virtual_sequence(np.tile(x0, (m, 1)), x0, alpha)]
    O.run(x0, m, tau, alpha, gamma, K, recording, store=F64,
          on_step=lambda k, s: ys.append(O.virtual_sequence(s["x"], s["z"], alpha)))
    for k in range(K):
        want = ys[k] - (1 - alpha) * gamma * np.mean(grads[k], axis=0)
        np.testing.assert_allclose(ys[k + 1], want, rtol=1e-12, atol=1e-14)


def test_mean_identity_and_consensus_contraction():
    """Last column of W: mean(x after pull) = (1-alpha) mean(x_half) + alpha z_old = new z;
    deviations from the mean contract by exactly (1 - alpha) at a pull."""
    m, d, alpha = 6, 10, 0.6
    x_half = rand((m, d), 40)
    z_old = rand(d, 41)
    pulled = np.stack([O.pull_back(x_half[i], z_old, alpha) for i in range(m)])
    z_new = O.anchor_average(pulled)
    np.testing.assert_allclose(pulled.mean(axis=0), (1 - alpha) * x_half.mean(axis=0) + alpha * z_old,
                               rtol=1e-13)
    np.testing.assert_allclose(z_new, pulled.mean(axis=0), rtol=1e-15)
    np.testing.assert_allclose(pulled - pulled.mean(axis=0),
                               (1 - alpha) * (x_half - x_half.mean(axis=0)), rtol=1e-12, atol=1e-15)
    # the same through the matrix form
    Xh = np.concatenate([x_half.T, z_old[:, None]], axis=1)
    Xn = O.matrix_form_step(Xh, np.zeros_like(Xh), 0.0, O.mixing_matrix(m, alpha))
    np.testing.assert_allclose(Xn[:, :m], pulled.T, rtol=1e-13)
    np.testing.assert_allclose(Xn[:, m], z_new, rtol=1e-13)


# ---------------------------------------------------------------------------
# degenerate cases
# ---------------------------------------------------------------------------
def test_identical_data_keeps_replicas_identical():
    m, d, tau = 4, 16, 2
    A = rand((1, 3, 5, d), 50)
    y = rand((1, 3, 5), 51)
    gf = lambda i, k, x: O.lsq_loss_grad(x, A[0, k % 3], y[0, k % 3])

    def check(k, s):
        assert all(np.array_equal(s["x"][0], s["x"][i]) for i in range(1, m))
        if (k + 1) % tau == 0:
            np.testing.assert_array_equal(s["z"], s["x"][0])

    O.run(rand(d, 52), m, tau, 0.6, 0.02, 10, gf, mu=0.9, store=np.float32, on_step=check)


def torch_sgd_reference(x0, A, y, lr, mu, nesterov, K):
    """Independent run with the CPU library's optimizer and autograd (fp64)."""
    w = torch.tensor(x0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([w], lr=lr, momentum=mu, nesterov=nesterov and mu > 0)
    nb = A.shape[0]
    for k in range(K):
        opt.zero_grad()
        r = torch.tensor(A[k % nb]) @ w - torch.tensor(y[k % nb])
        (0.5 * (r * r).mean()).backward()
        opt.step()
    return w.detach().numpy()


@pytest.mark.parametrize("mu,nesterov", [(0.0, True), (0.9, True), (0.9, False)])
def test_alpha_zero_is_independent_momentum_sgd(mu, nesterov):
    """alpha = 0 switches the pull-back off: m independent local runs, equal to the
    library's (PyTorch, as in Section 4) SGD with Nesterov / heavy-ball momentum."""
    m, d, K = 3, 12, 9
    A, y, gf = lsq_problem(m, 4, 6, d, 60)
    x0 = rand(d, 61)
    st = O.run(x0, m, 2, 0.0, 0.02, K, gf, mu=mu, nesterov=nesterov, store=F64)
    for i in range(m):
        np.testing.assert_allclose(st["x"][i], torch_sgd_reference(x0, A[i], y[i], 0.02, mu, nesterov, K),
                                   rtol=1e-11, atol=1e-13)


def test_alpha_one_resets_to_anchor():
    m, d, tau = 4, 8, 3
    _, _, gf = lsq_problem(m, 2, 5, d, 70)
    x0 = rand(d, 71)

    def check(k, s):
        # x_half - 1 (x_half - z) equals z up to rounding of the difference
        np.testing.assert_allclose(s["z"], x0, rtol=1e-14, atol=1e-15)
        if (k + 1) % tau == 0:
            np.testing.assert_allclose(s["x"], np.tile(x0, (m, 1)), rtol=1e-14, atol=1e-15)

    O.run(x0, m, tau, 1.0, 0.05, 9, gf, store=F64, on_step=check)


def test_tau_one_identical_workers_is_sgd_with_effective_lr():
    """tau = 1, same data everywhere: plain SGD with step (1 - alpha) gamma (Appendix A,
    effective learning rate)."""
    m, d, alpha, gamma, K = 3, 10, 0.5, 0.04, 12
    A = rand((3, 6, d), 80)
    y = rand((3, 6), 81)
    gf = lambda i, k, x: O.lsq_loss_grad(x, A[k % 3], y[k % 3])
    x0 = rand(d, 82)
    st = O.run(x0, m, 1, alpha, gamma, K, gf, store=F64)
    want = torch_sgd_reference(x0, A, y, (1 - alpha) * gamma, 0.0, False, K)
    for i in range(m):
        np.testing.assert_allclose(st["x"][i], want, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(st["z"], want, rtol=1e-11, atol=1e-13)


def test_single_worker():
    """m = 1: the anchor equals the model after each pull, and the pull mixes the round's
    end point with its start point."""
    d, tau, alpha, gamma = 6, 3, 0.6, 0.05
    A, y, gf = lsq_problem(1, 2, 4, d, 90)
    x0 = rand(d, 91)
    start = x0.copy()
    trace = []
    O.run(x0, 1, tau, alpha, gamma, 2 * tau, gf, store=F64,
          on_step=lambda k, s: trace.append((s["x"][0].copy(), s["z"].copy())))
    for r in range(2):
        w = start.copy()
        for k in range(r * tau, (r + 1) * tau):       # tau plain steps from the round start
            _, g = gf(0, k, w)
            w = w - gamma * g
        xr, zr = trace[(r + 1) * tau - 1]
        np.testing.assert_allclose(xr, (1 - alpha) * w + alpha * start, rtol=1e-12)
        np.testing.assert_array_equal(zr, xr)
        start = xr


def test_pull_leaves_momentum_buffer_untouched():
    """The local buffer is fed by local gradients only: it must not depend on alpha."""
    m, d, tau, K = 3, 8, 2, 2
    _, _, gf = lsq_problem(m, 2, 4, d, 100)
    x0 = rand(d, 101)
    a = O.run(x0, m, tau, 0.0, 0.05, K, gf, mu=0.9, store=F64)
    b = O.run(x0, m, tau, 0.7, 0.05, K, gf, mu=0.9, store=F64)
    np.testing.assert_array_equal(a["buf"], b["buf"])         # same up to the first pull
    assert not np.allclose(a["x"], b["x"])


def test_trailing_steps_when_K_not_multiple_of_tau():
    m, d, tau = 2, 5, 4
    _, _, gf = lsq_problem(m, 2, 4, d, 110)
    x0 = rand(d, 111)
    st = O.run(x0, m, tau, 0.6, 0.05, 3, gf, store=F64)       # fewer than tau steps: no pull at all
    np.testing.assert_array_equal(st["z"], x0)
    ref = O.run(x0, m, tau, 0.0, 0.05, 3, gf, store=F64)
    np.testing.assert_array_equal(st["x"], ref["x"])


# ---------------------------------------------------------------------------
# anchor momentum (Momentum Variant paragraph)
# ---------------------------------------------------------------------------
def test_anchor_momentum_beta_zero_reduces_to_mean():
    xs, z = rand((5, 7), 120), rand(7, 121)
    z_new, v_new = O.anchor_momentum_update(z, np.zeros(7), xs, 0.0)
    np.testing.assert_allclose(z_new, O.anchor_average(xs), rtol=1e-14)
    np.testing.assert_allclose(v_new, O.anchor_average(xs) - z, rtol=1e-14)


def test_anchor_momentum_matrix_power():
    """Identical workers, tau = 1, 1-d quadratic: [x, z, v] follows a constant linear map."""
    a, gamma, alpha, beta = 0.5, 0.2, 0.6, 0.7
    rho = 1 - gamma * a
    # x' = (1-alpha) rho x + alpha z ; v' = beta v + (x' - z) ; z' = z + v'
    Mx = np.array([(1 - alpha) * rho, alpha, 0.0])
    Mv = np.array([0.0, 0.0, beta]) + Mx - np.array([0.0, 1.0, 0.0])
    Mz = np.array([0.0, 1.0, 0.0]) + Mv
    M = np.stack([Mx, Mz, Mv])
    want = np.linalg.matrix_power(M, 6) @ np.array([1.3, 1.3, 0.0])
    st = O.run(np.array([1.3]), 4, 1, alpha, gamma, 6, quad_grad(a, np.zeros((4, 1))),
               beta_z=beta, store=F64)
    np.testing.assert_allclose([st["x"][0, 0], st["z"][0], st["v"][0]], want, rtol=1e-12)


def test_anchor_momentum_alpha_one_freezes_anchor():
    m, d = 3, 5
    _, _, gf = lsq_problem(m, 2, 4, d, 130)
    x0 = rand(d, 131)
    st = O.run(x0, m, 2, 1.0, 0.05, 6, gf, beta_z=0.7, store=F64)
    np.testing.assert_allclose(st["z"], x0, rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(st["v"], np.zeros(d), atol=1e-15)


# ---------------------------------------------------------------------------
# gradients: finite differences and the CPU library's autograd
# ---------------------------------------------------------------------------
def finite_difference(f, x, h=1e-6):
    g = np.zeros_like(x)
    for j in range(x.size):
        e = np.zeros_like(x)
        e[j] = h
        g[j] = (f(x + e) - f(x - e)) / (2 * h)
    return g


def test_lsq_gradient():
    A, y, x = rand((7, 5), 140), rand(7, 141), rand(5, 142)
    loss, g = O.lsq_loss_grad(x, A, y)
    np.testing.assert_allclose(g, finite_difference(lambda w: O.lsq_loss_grad(w, A, y)[0], x), rtol=1e-6,
                               atol=1e-8)
    w_ls = np.linalg.lstsq(A, y, rcond=None)[0]               # stationary point of the loss
    np.testing.assert_allclose(O.lsq_loss_grad(w_ls, A, y)[1], 0, atol=1e-13)
    assert abs(loss - 0.5 * np.mean((A @ x - y) ** 2)) < 1e-14
    # brute force, element by element
    brute = sum(0.5 * (sum(A[s, j] * x[j] for j in range(5)) - y[s]) ** 2 for s in range(7)) / 7
    assert abs(loss - brute) < 1e-13


@pytest.mark.parametrize("dims", [(5, 4, 3), (6, 5, 4, 3), (4, 6, 5, 4, 3)])
def test_mlp_gradient_finite_differences(dims):
    B = 5
    d = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
    x = 0.5 * rand(d, 150)
    X = rand((B, dims[0]), 151)
    lab = np.random.default_rng(152).integers(0, dims[-1], B)
    _, g = O.mlp_loss_grad(x, dims, X, lab)
    fd = finite_difference(lambda w: O.mlp_loss_grad(w, dims, X, lab)[0], x)
    np.testing.assert_allclose(g, fd, rtol=2e-6, atol=1e-8)


@pytest.mark.parametrize("dims", [(7, 6, 3), (9, 8, 7, 6, 10)])
def test_mlp_against_library_autograd(dims):
    """Forward loss and gradient against torch's CPU Linear/ReLU/cross_entropy in fp64,
    including the flat [in][out]-then-bias layout."""
    B = 6
    d = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(len(dims) - 1))
    x = 0.4 * rand(d, 160)
    X = rand((B, dims[0]), 161)
    lab = np.random.default_rng(162).integers(0, dims[-1], B)
    loss, g = O.mlp_loss_grad(x, dims, X, lab)

    params, off = [], 0
    for l in range(len(dims) - 1):
        W = torch.tensor(x[off:off + dims[l] * dims[l + 1]].reshape(dims[l], dims[l + 1]),
                         requires_grad=True)
        off += dims[l] * dims[l + 1]
        b = torch.tensor(x[off:off + dims[l + 1]], requires_grad=True)
        off += dims[l + 1]
        params += [W, b]
    h = torch.tensor(X)
    for l in range(len(dims) - 1):
        h = h @ params[2 * l] + params[2 * l + 1]
        if l < len(dims) - 2:
            h = torch.relu(h)
    tl = torch.nn.functional.cross_entropy(h, torch.tensor(lab, dtype=torch.long))
    tl.backward()
    tg = np.concatenate([p.grad.numpy().ravel() for p in params])
    assert abs(loss - tl.item()) < 1e-12
    np.testing.assert_allclose(g, tg, rtol=1e-10, atol=1e-13)


def test_mlp_loss_brute_force():
    dims = (3, 2, 2)
    x = np.array([0.1, -0.2, 0.3, 0.4, -0.5, 0.6, 0.05, -0.05, 0.7, -0.8, 0.9, 1.0, 0.0, 0.1])
    X = np.array([[1.0, 2.0, -1.0], [0.5, -0.5, 0.25]])
    lab = np.array([1, 0])
    import math
    total = 0.0
    for s in range(2):
        hid = [max(0.0, sum(X[s, k] * x[k * 2 + n] for k in range(3)) + x[6 + n]) for n in range(2)]
        lg = [sum(hid[k] * x[8 + k * 2 + n] for k in range(2)) + x[12 + n] for n in range(2)]
        total += math.log(sum(math.exp(v) for v in lg)) - lg[lab[s]]
    assert abs(O.mlp_loss_grad(x, dims, X, lab)[0] - total / 2) < 1e-14


def test_relu_derivative_at_zero_is_zero():
    dims = (2, 2, 2)
    # first layer maps the sample exactly onto pre-activation 0 for unit 0
    x = np.array([1.0, 0.5, -1.0, 0.5, 0.0, 0.0, 1.0, -1.0, 0.5, 2.0, 0.0, 0.0])
    X = np.array([[1.0, 1.0]])
    _, g = O.mlp_loss_grad(x, dims, X, np.array([0]))
    gW1 = g[:4].reshape(2, 2)
    assert np.all(gW1[:, 0] == 0.0) and np.any(gW1[:, 1] != 0.0)


def test_bf16_rounding_matches_library():
    a = (rand(4096, 170) * 3).astype(np.float32)
    a[:4] = [1.0, 1.00390625, 1.01171875, -0.0]               # exact, tie-to-even (down), tie-to-even (up)
    want = torch.tensor(a).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(a), want)


def test_fp32_store_rounds_once_per_update():
    """float32 state: each stored value is the double-precision update of the stored
    inputs rounded once."""
    m, d = 2, 64
    x0 = rand(d, 180).astype(np.float32)
    g = rand((m, d), 181).astype(np.float32)
    st = O.run(x0, m, 1, 0.6, 0.1, 1, lambda i, k, x: (0.0, g[i]), mu=0.9, store=np.float32)
    x64 = x0.astype(F64)
    for i in range(m):
        buf = g[i].astype(F64)
        half = x64 - 0.1 * (g[i] + 0.9 * buf)
        np.testing.assert_array_equal(st["x"][i], (half - 0.6 * (half - x64)).astype(np.float32))
        np.testing.assert_array_equal(st["buf"][i], buf.astype(np.float32))
    assert st["x"].dtype == np.float32 and st["z"].dtype == np.float32


def test_bf16_diagnostic_mode():
    """The bf16-operand mode rounds only what enters hidden-layer products: with no hidden layer
    and bf16-representable inputs it changes nothing; on a small MLP it stays within bf16
    rounding of the exact gradient."""
    dims = (8, 5)
    x = rand(8 * 5 + 5, 190)
    X = O.round_to_bf16(rand((6, 8), 191).astype(np.float32))
    lab = np.random.default_rng(192).integers(0, 5, 6)
    a = O.mlp_loss_grad(x, dims, X, lab)
    b = O.mlp_loss_grad(x, dims, X, lab, bf16_operands=True)
    assert a[0] == b[0] and np.array_equal(a[1], b[1])
    dims = (16, 12, 10, 4)
    d = sum(dims[l] * dims[l + 1] + dims[l + 1] for l in range(3))
    x = 0.4 * rand(d, 193)
    X = rand((8, 16), 194)
    lab = np.random.default_rng(195).integers(0, 4, 8)
    a = O.mlp_loss_grad(x, dims, X, lab)
    b = O.mlp_loss_grad(x, dims, X, lab, bf16_operands=True)
    assert abs(a[0] - b[0]) < 2e-2 * abs(a[0]) and a[0] != b[0]
    assert np.abs(a[1] - b[1]).max() < 3e-2 * np.abs(a[1]).max()
