"""Shared helpers of the GPU parity tests: error metrics and lock-step runs of the HIP path and the
CPU oracle on the same seeded inputs."""
import numpy as np


def max_norm_ratio(got, want):
    """||got - want||_inf / ||want||_inf (the gate for per-step fp32 parity)."""
    want = np.asarray(want, np.float64)
    denom = np.abs(want).max()
    err = np.abs(np.asarray(got, np.float64) - want).max()
    return err / denom if denom > 0 else err


def l2_ratio(got, want):
    want = np.asarray(want, np.float64)
    denom = np.linalg.norm(want)
    err = np.linalg.norm(np.asarray(got, np.float64) - want)
    return err / denom if denom > 0 else err


def oracle_states(O, x0, m, tau, alpha, gamma, K, grad_fn, **kw):
    """Runs the oracle and returns a list of per-iteration snapshots (x, buf, z, v)."""
    snaps = []

    def snap(k, s):
        snaps.append({n: (None if s[n] is None else s[n].copy()) for n in ("x", "buf", "z", "v")})

    st = O.run(x0, m, tau, alpha, gamma, K, grad_fn, on_step=snap, **kw)
    return snaps, st


def gpu_states(sess, K, before_step=None):
    """Runs the HIP path for K iterations and snapshots its state after each one."""
    from paper_2002_09539_amd import binding as B
    snaps = []
    for _ in range(K):
        k = B.ols_iteration(sess.h)
        if before_step is not None:
            before_step(k)
        sess.local_step()
        if (k + 1) % sess.tau == 0:
            sess.sync_pull()
            sess.anchor_update_async()
        snaps.append(dict(x=sess.all_params(), z=sess.params(-1), buf=sess.momentum(),
                          v=None if sess.v is None else sess.v[: sess.d].cpu().numpy()))
    return snaps
