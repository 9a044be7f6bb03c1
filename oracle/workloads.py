"""Glue between the seeded workload tensors and the oracle's iteration.

TEST INFRASTRUCTURE ONLY (see ols_oracle.py).  Builds the grad_fn callbacks the
oracle's `run` expects.  Mini-batches are visited cyclically and in order
(Section 4: the data is partitioned per node and never shuffled): worker i at
iteration k uses its batch number k mod nb.
"""
import numpy as np

from . import conv_oracle as CO
from . import ols_oracle as O


def lsq_grad_fn(A, y):
    """A [m][nb][B][d], y [m][nb][B]."""
    nb = A.shape[1]
    return lambda i, k, x: O.lsq_loss_grad(x, A[i, k % nb], y[i, k % nb])


def mlp_grad_fn(dims, X, labels, bf16_operands=False):
    """X [m][nb][B][in], labels [m][nb][B]."""
    nb = X.shape[1]
    return lambda i, k, x: O.mlp_loss_grad(x, dims, X[i, k % nb], labels[i, k % nb],
                                           bf16_operands=bf16_operands)


def conv_grad_fn(dims, X, labels, batch_norm=False, bf16_operands=False):
    """dims = (channels, height, width, classes); X [m][nb][B][H][W][C], labels [m][nb][B]."""
    nb = X.shape[1]
    if batch_norm:
        return lambda i, k, x: CO.convblock_bn_loss_grad(x, dims[0], dims[3], X[i, k % nb], labels[i, k % nb],
                                                         bf16_operands=bf16_operands)
    return lambda i, k, x: CO.convblock_loss_grad(x, dims[0], dims[3], X[i, k % nb], labels[i, k % nb],
                                                  bf16_operands=bf16_operands)


def stream_grad_fn(grads):
    """grads: list of [m][d] gradient tensors, tensor (k mod len) used at iteration k."""
    n = len(grads)
    return lambda i, k, x: (0.0, grads[k % n][i])


def run_config(cfg, x0, grad_fn, K=None, store=np.float32, on_step=None):
    return O.run(x0, cfg.m, cfg.tau, cfg.alpha, cfg.gamma, cfg.K if K is None else K, grad_fn,
                 mu=cfg.mu, nesterov=cfg.nesterov, beta_z=cfg.beta_z, store=store, on_step=on_step)
