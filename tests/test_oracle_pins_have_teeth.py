"""Plants plausible mistakes in the CPU oracle (on the CPU, in the oracle only) and checks that the
pins of tests/test_oracle_pins.py notice each of them.  A pin that a wrong oracle still passes would
pin nothing."""
import numpy as np
import pytest

from oracle import ols_oracle as O
from tests import test_oracle_pins as P

F64 = np.float64


def pins():
    """A representative subset of the pins, each as a zero-argument callable."""
    return [
        lambda: P.test_closed_form_identical_quadratic(2, 0.6),
        P.test_closed_form_heterogeneous_quadratic,
        P.test_momentum_quadratic_matrix_power,
        lambda: P.test_mixing_matrix_identities(4, 0.6),
        lambda: P.test_vector_form_equals_matrix_form(2),
        lambda: P.test_virtual_sequence_recursion_every_step(2),
        P.test_mean_identity_and_consensus_contraction,
        lambda: P.test_alpha_zero_is_independent_momentum_sgd(0.9, True),
        lambda: P.test_alpha_zero_is_independent_momentum_sgd(0.9, False),
        P.test_alpha_one_resets_to_anchor,
        P.test_tau_one_identical_workers_is_sgd_with_effective_lr,
        P.test_single_worker,
        P.test_pull_leaves_momentum_buffer_untouched,
        P.test_anchor_momentum_matrix_power,
        P.test_lsq_gradient,
        lambda: P.test_mlp_gradient_finite_differences((6, 5, 4, 3)),
        lambda: P.test_mlp_against_library_autograd((9, 8, 7, 6, 10)),
        P.test_mlp_loss_brute_force,
        P.test_relu_derivative_at_zero_is_zero,
        P.test_bf16_rounding_matches_library,
    ]


def some_pin_fails():
    for pin in pins():
        try:
            pin()
        except AssertionError:
            return True
    return False


def test_unmodified_oracle_passes_every_pin():
    assert not some_pin_fails()


def wrong_pull_sign(x_half, z, alpha):
    x_half = np.asarray(x_half, F64)
    return x_half + alpha * (x_half - np.asarray(z, F64))


def wrong_pull_toward_itself(x_half, z, alpha):            # forgets the anchor
    return (1.0 - alpha) * np.asarray(x_half, F64)


def wrong_mean_is_sum(xs):
    return np.asarray(xs, F64).sum(axis=0)


def wrong_heavy_ball_always(x, buf, g, gamma, mu=0.0, nesterov=True):
    return ORIG["local_momentum_step"](x, buf, g, gamma, mu, False)


def wrong_momentum_dampened(x, buf, g, gamma, mu=0.0, nesterov=True):
    x, g = np.asarray(x, F64), np.asarray(g, F64)
    if mu == 0.0:
        return x - gamma * g, buf
    b = mu * np.asarray(buf, F64) + (1.0 - mu) * g
    return x - gamma * (g + mu * b if nesterov else b), b


def wrong_anchor_momentum(z, v, xs, beta_z):               # momentum also scales the fresh increment
    z = np.asarray(z, F64)
    v_new = beta_z * (np.asarray(v, F64) + (ORIG["anchor_average"](xs) - z))
    return z + v_new, v_new


def wrong_mixing_matrix(m, alpha):                         # transposed: row- instead of column-stochastic
    return ORIG["mixing_matrix"](m, alpha).T


def wrong_lsq(w, A, y):                                    # transposed operand / missing 1/B
    loss, g = ORIG["lsq_loss_grad"](w, A, y)
    return loss, g * A.shape[0]


def wrong_mlp_no_relu_mask(x, dims, X, labels, bf16_operands=False):
    loss, g = ORIG["mlp_loss_grad"](x, dims, X, labels, bf16_operands)
    layers = O.mlp_unpack(g, dims)
    layers[0][0][...] *= 1.01                              # a first-layer gradient that is slightly off
    return loss, g


def wrong_mlp_loss_sum(x, dims, X, labels, bf16_operands=False):
    loss, g = ORIG["mlp_loss_grad"](x, dims, X, labels, bf16_operands)
    return loss * X.shape[0], g * X.shape[0]               # sum instead of mean over the batch


def wrong_bf16_truncation(a):
    u = np.asarray(a, np.float32).view(np.uint32) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(F64)


ORIG = {n: getattr(O, n) for n in ("pull_back", "anchor_average", "local_momentum_step", "anchor_momentum_update",
                                   "mixing_matrix", "lsq_loss_grad", "mlp_loss_grad", "round_to_bf16")}

MUTANTS = [
    ("pull_back", wrong_pull_sign),
    ("pull_back", wrong_pull_toward_itself),
    ("anchor_average", wrong_mean_is_sum),
    ("local_momentum_step", wrong_heavy_ball_always),
    ("local_momentum_step", wrong_momentum_dampened),
    ("anchor_momentum_update", wrong_anchor_momentum),
    ("mixing_matrix", wrong_mixing_matrix),
    ("lsq_loss_grad", wrong_lsq),
    ("mlp_loss_grad", wrong_mlp_no_relu_mask),
    ("mlp_loss_grad", wrong_mlp_loss_sum),
    ("round_to_bf16", wrong_bf16_truncation),
]


@pytest.mark.parametrize("name,mutant", MUTANTS, ids=[m[1].__name__ for m in MUTANTS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    monkeypatch.setattr(O, name, mutant)
    assert some_pin_fails(), "no pin noticed %s" % mutant.__name__


def test_stale_anchor_ordering_mistakes_are_caught(monkeypatch):
    """Using the refreshed anchor in the same step's pull, or averaging the pre-pull models, must fail."""
    real_run = O.run

    def run_refresh_before_pull(x0, m, tau, alpha, gamma, K, grad_fn, mu=0.0, nesterov=True, beta_z=0.0,
                                store=np.float32, on_step=None):
        x0 = np.asarray(x0)
        x = np.repeat(x0.astype(store)[None, :], m, axis=0)
        z = x0.astype(store).copy()
        losses = np.zeros((K, m))
        state = dict(x=x, buf=None, z=z, v=None, losses=losses)
        for k in range(K):
            half = np.stack([O.local_momentum_step(x[i], None, grad_fn(i, k, x[i])[1], gamma)[0] for i in range(m)])
            if (k + 1) % tau == 0:
                z[...] = O.anchor_average(half).astype(store)          # WRONG: pre-pull models, and before the pull
                x[...] = np.stack([O.pull_back(half[i], z, alpha) for i in range(m)]).astype(store)
            else:
                x[...] = half.astype(store)
            if on_step is not None:
                on_step(k, state)
        return state

    monkeypatch.setattr(O, "run", run_refresh_before_pull)
    caught = False
    for pin in (P.test_closed_form_heterogeneous_quadratic, lambda: P.test_vector_form_equals_matrix_form(2),
                lambda: P.test_virtual_sequence_recursion_every_step(2)):
        try:
            pin()
        except AssertionError:
            caught = True
    assert caught
    monkeypatch.setattr(O, "run", real_run)
