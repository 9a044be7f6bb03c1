"""CPU oracle for Overlap Local-SGD (arXiv 2002.09539).  TEST INFRASTRUCTURE ONLY.

A plain, slow, step-by-step numpy implementation of the paper's update rules,
written from the paper and sharing no code with the HIP path.  Only the tests,
the smoke check and the benchmark's CPU-baseline leg may call it; the product
path never does.

The method is an iteration, so the oracle is the algorithm itself, taken in the
paper's order (Section 2, "Proposed Algorithm"):

    local step   x_{k+1/2}^{(i)} = x_k^{(i)} - gamma * g_i(x_k^{(i)}; xi_k^{(i)})
    pull-back    x_{k+1}^{(i)}   = x_{k+1/2}^{(i)} - alpha (x_{k+1/2}^{(i)} - z_k)   iff (k+1) mod tau == 0
    anchor       z_{k+1}         = (1/m) sum_i x_{k+1}^{(i)}                         iff (k+1) mod tau == 0

plus the momentum variant of the same section (local Nesterov momentum whose
buffer sees local gradients only; anchor momentum v, beta) and, as a second and
independent formulation, the matrix form X_{k+1} = (X_k - gamma G_k) W_k.

Precision: all arithmetic is IEEE double.  The state (x, buf, z, v) is kept in a
`store` dtype: float64 for the pure reference, or float32 to mirror the fp32
master copies a device holds, in which case every update is evaluated in double
from the stored values and rounded exactly once when written back.

Readings of points the paper leaves open (each also listed in the design
notes): k counts from 0 and the first pull happens after tau local steps using
z_0 = x_0; the local momentum is PyTorch-style Nesterov (buf <- mu buf + g,
step direction g + mu buf), heavy-ball as an option, buffer initially zero and
untouched by the pull-back; mini-batch losses are means over the batch; the
ReLU derivative at 0 is 0; the anchor averages the post-pull models.

The stale-average synchronisation of "Related Works" (`stale_average_sync`,
`run_stale_average`) is pinned by tests/test_oracle_stale_average_pins.py.

Pinned by tests/test_oracle_pins.py (closed forms on quadratics, the mixing
matrix identities and virtual-sequence recursion of Appendix A, degenerate
cases alpha in {0,1}, tau = 1, m = 1, finite differences, and CPU library
routines for the gradient, the cross-entropy and the Nesterov step).
"""
import numpy as np

F64 = np.float64


# ----------------------------------------------------------------------------
# update rules (Section 2, eqs. "local update", "pull-back", "anchor update")
# ----------------------------------------------------------------------------
def local_momentum_step(x, buf, g, gamma, mu=0.0, nesterov=True):
    """One local step of a single worker; returns (x_half, buf_new) in double.

    mu == 0: x_half = x - gamma g (first update rule of Section 2).
    mu > 0 ("Momentum Variant" paragraph; the buffer is fed by the local
    gradient only): buf <- mu buf + g, then the step direction is g + mu buf
    (Nesterov) or buf (heavy ball).
    """
    x = np.asarray(x, F64)
    g = np.asarray(g, F64)
    if mu == 0.0:
        return x - gamma * g, (None if buf is None else np.asarray(buf, F64))
    buf_new = mu * np.asarray(buf, F64) + g
    direction = g + mu * buf_new if nesterov else buf_new
    return x - gamma * direction, buf_new


def pull_back(x_half, z, alpha):
    """Second update rule of Section 2: x_half - alpha (x_half - z), in double."""
    x_half = np.asarray(x_half, F64)
    return x_half - alpha * (x_half - np.asarray(z, F64))


def anchor_average(xs):
    """Anchor update rule of Section 2: the mean of the m post-pull models."""
    xs = np.asarray(xs, F64)
    return xs.sum(axis=0) / xs.shape[0]


def anchor_momentum_update(z, v, xs, beta_z):
    """Momentum form of the anchor ("Momentum Variant" paragraph):
    v <- beta v + (mean_i x^{(i)} - z);  z <- z + v.  beta = 0 gives the plain mean."""
    z = np.asarray(z, F64)
    v_new = beta_z * np.asarray(v, F64) + (anchor_average(xs) - z)
    return z + v_new, v_new


def virtual_sequence(xs, z, alpha):
    """y = (1 - alpha) mean_i x^{(i)} + alpha z (Appendix A)."""
    return (1.0 - alpha) * anchor_average(xs) + alpha * np.asarray(z, F64)


# ----------------------------------------------------------------------------
# matrix form (Section 2, "Matrix-Form Update Rule"; Appendix A)
# ----------------------------------------------------------------------------
def mixing_matrix(m, alpha):
    """The (m+1)x(m+1) column-stochastic W of a synchronisation step.

    Blocks: upper-left (1-alpha) I, upper-right column (1-alpha) 1/m,
    lower-left row alpha 1^T, lower-right alpha.
    """
    W = np.zeros((m + 1, m + 1), F64)
    W[:m, :m] = (1.0 - alpha) * np.eye(m)
    W[:m, m] = (1.0 - alpha) / m
    W[m, :m] = alpha
    W[m, m] = alpha
    return W


def periodic_averaging_matrix(m):
    """W of Local SGD's synchronisation (first display of Section 2): every model becomes the
    mean of the m half-step models; the extra (anchor) column takes the same mean and row m,
    the old anchor, contributes nothing.  Column-stochastic."""
    W = np.zeros((m + 1, m + 1), F64)
    W[:m, :] = 1.0 / m
    return W


def elastic_symmetric_matrix(m, alpha):
    """A symmetric, doubly stochastic W of the kind Section 3 ascribes to elastic averaging:
    x_i <- x_i - alpha (x_i - z) and z <- z + alpha sum_i (x_i - z)."""
    W = np.zeros((m + 1, m + 1), F64)
    W[:m, :m] = (1.0 - alpha) * np.eye(m)
    W[m, :m] = alpha
    W[:m, m] = alpha
    W[m, m] = 1.0 - m * alpha
    return W


def mix(X, W):
    """X W for X = [x^(1..m), z] of shape d x (m+1): output column j is sum_i W[i][j] X[:, i]."""
    return np.asarray(X, F64) @ np.asarray(W, F64)


def matrix_form_step(X, G, gamma, W):
    """X_{k+1} = (X_k - gamma G_k) W_k with X = [x^(1..m), z] of shape d x (m+1)."""
    return (np.asarray(X, F64) - gamma * np.asarray(G, F64)) @ W


# ----------------------------------------------------------------------------
# per-worker stochastic gradients g_i (mean loss over the worker's mini-batch)
# ----------------------------------------------------------------------------
def lsq_loss_grad(w, A, y):
    """Least squares: loss = (1/B) sum_s 0.5 (a_s.w - y_s)^2, g = (1/B) A^T (A w - y)."""
    w, A, y = np.asarray(w, F64), np.asarray(A, F64), np.asarray(y, F64)
    r = A @ w - y
    B = A.shape[0]
    return 0.5 * float(r @ r) / B, (A.T @ r) / B


def round_to_bf16(a):
    """Round-to-nearest-even of fp32 values to bfloat16, returned as float64."""
    u = np.asarray(a, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(F64)


def mlp_unpack(x, dims):
    """Views (W_l [in][out], b_l [out]) of the flat parameter vector, in layer order."""
    out, off = [], 0
    for l in range(len(dims) - 1):
        n_in, n_out = dims[l], dims[l + 1]
        W = x[off:off + n_in * n_out].reshape(n_in, n_out)
        off += n_in * n_out
        b = x[off:off + n_out]
        off += n_out
        out.append((W, b))
    assert off == x.shape[0]
    return out


def mlp_loss_grad(x, dims, X, labels, bf16_operands=False):
    """ReLU MLP with softmax cross-entropy, mean over the batch.

    Returns (loss, flat gradient in the layout of `x`).

    bf16_operands is a DIAGNOSTIC mode for a device path that feeds its hidden-layer matrix
    products with bfloat16 operands: the stored activations and back-propagated deltas of the
    hidden layers, and the weights of the hidden layers, are rounded to bfloat16 wherever they
    enter a product (or a bias-gradient sum, which reads the stored delta); products and sums
    stay in double, and the output layer keeps its weights and its delta unrounded.  The gate for
    such a path is still the unrounded computation (bf16_operands=False).
    """
    q = round_to_bf16 if bf16_operands else (lambda a: np.asarray(a, F64))
    x = np.asarray(x, F64)
    layers = mlp_unpack(x, dims)
    L = len(layers)
    B = X.shape[0]
    acts = [np.asarray(X, F64)]
    for l, (W, b) in enumerate(layers):
        hidden = l < L - 1
        pre = q(acts[-1]) @ (q(W) if hidden else W) + b
        acts.append(np.maximum(pre, 0.0) if hidden else pre)
    logits = acts[-1]
    shifted = logits - logits.max(axis=1, keepdims=True)
    logsumexp = np.log(np.exp(shifted).sum(axis=1))
    rows = np.arange(B)
    loss = float((logsumexp - shifted[rows, labels]).mean())
    delta = np.exp(shifted - logsumexp[:, None])          # softmax probabilities
    delta[rows, labels] -= 1.0
    delta /= B
    g = np.empty_like(x)
    g_layers = mlp_unpack(g, dims)
    for l in range(L - 1, -1, -1):
        hidden = l < L - 1
        W, _ = layers[l]
        gW, gb = g_layers[l]
        d_in = q(delta) if hidden else delta
        gW[...] = q(acts[l]).T @ d_in
        gb[...] = d_in.sum(axis=0)
        if l > 0:
            delta = (d_in @ (q(W) if hidden else W).T) * (acts[l] > 0.0)
    return loss, g


# ----------------------------------------------------------------------------
# the whole iteration
# ----------------------------------------------------------------------------
def run(x0, m, tau, alpha, gamma, K, grad_fn, mu=0.0, nesterov=True, beta_z=0.0,
        store=np.float32, on_step=None):
    """K iterations of Overlap Local-SGD for m workers from the common point x0.

    grad_fn(i, k, x_i) -> (loss, g): worker i's mini-batch loss and gradient at
    iteration k, evaluated at its own current model.  on_step(k, state), if
    given, is called after iteration k with the live state dict.  gamma is a
    number, or a function k -> learning rate of iteration k (Section 4 trains
    with a warm-up and step decays: the rate then changes between iterations,
    the update rules stay as they are).

    Returns dict(x [m][d], buf [m][d] or None, z [d], v [d] or None,
    losses [K][m]) with the state in the `store` dtype.
    """
    x0 = np.asarray(x0)
    d = x0.shape[0]
    x = np.repeat(x0.astype(store)[None, :], m, axis=0)       # x_0^{(i)} = z_0 (Theorem 1)
    z = x0.astype(store).copy()
    buf = np.zeros((m, d), store) if mu != 0.0 else None
    v = np.zeros(d, store) if beta_z != 0.0 else None
    losses = np.zeros((K, m), F64)
    state = dict(x=x, buf=buf, z=z, v=v, losses=losses)
    for k in range(K):
        sync = (k + 1) % tau == 0
        gamma_k = gamma(k) if callable(gamma) else gamma
        for i in range(m):
            loss, g = grad_fn(i, k, x[i])
            losses[k, i] = loss
            x_half, b_new = local_momentum_step(x[i], None if buf is None else buf[i],
                                                g, gamma_k, mu, nesterov)
            if buf is not None:
                buf[i] = b_new.astype(store)
            # the pull uses the anchor as it stood before this step's refresh
            x[i] = (pull_back(x_half, z, alpha) if sync else x_half).astype(store)
        if sync:
            if v is None:
                z[...] = anchor_average(x).astype(store)
            else:
                z_new, v_new = anchor_momentum_update(z, v, x, beta_z)
                z[...] = z_new.astype(store)
                v[...] = v_new.astype(store)
        if on_step is not None:
            on_step(k, state)
    return state


def run_general_mixing(x0, m, tau, gamma, K, grad_fn, W, mu=0.0, nesterov=True, store=np.float32):
    """The iteration X_{k+1} = (X_k - gamma G_k) W_k of Section 2 with an arbitrary matrix W at the
    synchronisation steps ((k+1) mod tau == 0; identity otherwise), local momentum as in `run`.
    W is given in double; a device applies it in fp32, so callers comparing against one pass
    W.astype(float32).  Returns the same dict as `run` (v is None)."""
    x0 = np.asarray(x0)
    d = x0.shape[0]
    W = np.asarray(W, F64)
    assert W.shape == (m + 1, m + 1)
    x = np.repeat(x0.astype(store)[None, :], m, axis=0)
    z = x0.astype(store).copy()
    buf = np.zeros((m, d), store) if mu != 0.0 else None
    losses = np.zeros((K, m), F64)
    for k in range(K):
        for i in range(m):
            loss, g = grad_fn(i, k, x[i])
            losses[k, i] = loss
            x_half, b_new = local_momentum_step(x[i], None if buf is None else buf[i], g, gamma, mu, nesterov)
            if buf is not None:
                buf[i] = b_new.astype(store)
            x[i] = x_half.astype(store)
        if (k + 1) % tau == 0:
            X = np.concatenate([x.astype(F64), z.astype(F64)[None, :]], axis=0).T      # d x (m+1)
            Xn = mix(X, W)
            x[...] = Xn[:, :m].T.astype(store)
            z[...] = Xn[:, m].astype(store)
    return dict(x=x, buf=buf, z=z, v=None, losses=losses)


def stale_average_sync(x, snap, z):
    """The synchronisation of the stale-average alternative described in "Related Works" (the local
    updates of the last tau iterations are applied to the average of the models as they stood tau
    iterations before): x^(i) <- z + (x^(i) - s^(i)), where s^(i) is worker i's model right after the
    previous synchronisation and z the average of those.  Returns the new models (double)."""
    x = np.asarray(x, F64)
    snap = np.asarray(snap, F64)
    return np.asarray(z, F64)[None, :] + (x - snap)


def run_stale_average(x0, m, tau, gamma, K, grad_fn, mu=0.0, nesterov=True, store=np.float32):
    """K iterations of local SGD whose synchronisation is `stale_average_sync`: local steps as in `run`,
    and after every tau-th one each model becomes (average of the previous synchronisation's models) +
    (its own progress since then); the new models are then remembered and averaged for the next
    synchronisation.  Initially every model and the average equal x0.  Returns the dict of `run`
    plus snap [m][d]; z is the average of the models after the last synchronisation."""
    x0 = np.asarray(x0)
    d = x0.shape[0]
    x = np.repeat(x0.astype(store)[None, :], m, axis=0)
    snap = x.copy()
    z = x0.astype(store).copy()
    buf = np.zeros((m, d), store) if mu != 0.0 else None
    losses = np.zeros((K, m), F64)
    for k in range(K):
        for i in range(m):
            loss, g = grad_fn(i, k, x[i])
            losses[k, i] = loss
            x_half, b_new = local_momentum_step(x[i], None if buf is None else buf[i], g, gamma, mu, nesterov)
            if buf is not None:
                buf[i] = b_new.astype(store)
            x[i] = x_half.astype(store)
        if (k + 1) % tau == 0:
            x[...] = stale_average_sync(x, snap, z).astype(store)
            snap[...] = x
            z[...] = anchor_average(x).astype(store)
    return dict(x=x, buf=buf, z=z, v=None, snap=snap, losses=losses)


def run_matrix_form(x0, m, tau, alpha, gamma, K, grad_fn):
    """The same iteration through X_{k+1} = (X_k - gamma G_k) W_k (no momentum), in double.

    Returns X_K of shape d x (m+1): columns x^(1..m), then z.
    """
    x0 = np.asarray(x0, F64)
    d = x0.shape[0]
    X = np.repeat(x0[:, None], m + 1, axis=1)
    P = mixing_matrix(m, alpha)
    eye = np.eye(m + 1)
    for k in range(K):
        G = np.zeros((d, m + 1), F64)
        for i in range(m):
            _, G[:, i] = grad_fn(i, k, X[:, i])
        X = matrix_form_step(X, G, gamma, P if (k + 1) % tau == 0 else eye)
    return X
