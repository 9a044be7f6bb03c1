"""GPU parity of the batch-normalised residual block (convolutions without bias, training-mode normalisation per worker
over its own mini-batch, shortcut, pooling, classifier) against the CPU oracle (oracle/conv_oracle.py), through the C
boundary: loss and every gradient group of one step at ragged and tile-sized shapes, inputs whose channel means dwarf
their spread, whole Overlap Local-SGD runs, and the schedule variants."""
import numpy as np
import pytest

import ols_inputs as I
from ols_inputs import generate as G
from oracle import conv_oracle as CO
from oracle import workloads as OW
from tests.helpers import l2_ratio, max_norm_ratio

from paper_2002_09539_amd import binding as B

pytestmark = pytest.mark.gpu

# fp32 against the fp64 oracle, max-norm relative per parameter group.  The normalisation's backward subtracts the
# channel means of dy and dy xhat from every element and the kernel gradient is orthogonal to the kernel (the loss does
# not change when a kernel is scaled), so rounding does not average out as far as in the plain block.
GRAD_TOL = 1e-4
E2E_TOL = 1e-3      # the benchmark specification's bar for fp32 end-to-end parameters
# A ReLU input within single-precision rounding of zero may fall on the other side on the device, and one activation
# taken the other way moves the gradient by about 1 / sqrt(activations) of its norm (0.8 % at 16 384 activations): the
# loss is not differentiable there and neither side is wrong.  The multi-step cases therefore use seeds for which the
# oracle's own trajectory keeps every ReLU input at least this far from zero (inputs of order one, a few hundred
# single-precision accumulations each), and say so with an assertion.
RELU_MARGIN = 4e-6
GROUPS = ("Wa", "ga", "ba", "Wb", "gb", "bb", "Wh", "bh")


def make_session(*a, **kw):
    from paper_2002_09539_amd.session import Session
    return Session(*a, **kw)


def bn_case(m, dims, batch, nb, seed, **kw):
    cfg = I.get(7).scaled(m=m, dims=tuple(dims), batch=batch, nb=nb, seed=seed, **kw)
    X, labels = G.conv_data(cfg)
    return cfg, X, labels, G.conv_init(cfg)


def groups_of(C, classes):
    idx = np.arange(CO.convblock_bn_param_count(C, classes))
    return dict(zip(GROUPS, CO.convblock_bn_unpack(idx, C, classes)))


def one_step(cfg, dims, batch, X, labels, x0, eps=1e-5):
    with make_session(cfg.m, cfg.d, 2, 0.6, 0.05, 0.0) as s:
        s.attach_convblock(*dims, batch, batch_norm=True, eps=eps)
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.set_batch(Xd[:, 0], yd[:, 0])
        s.local_step()
        return s.gradient(), s.losses()


@pytest.mark.parametrize("m,dims,batch", [
    (2, (16, 5, 6, 4), 3),        # 90 pixels: one range, stripes with a tail
    (3, (32, 8, 8, 10), 5),       # 320 pixels
    (2, (48, 7, 9, 10), 4),       # 12 channel vectors: the workgroup's last threads idle
    (2, (80, 6, 6, 7), 3),        # more than 64 channels
    (2, (64, 32, 32, 10), 6),     # the benchmark's per-image shape: 6144 pixels in three ranges
    (2, (64, 32, 32, 10), 5),     # 5120 pixels: three ranges, the last one short
    (1, (16, 1, 1, 3), 2),        # two pixels per channel
    (2, (16, 40, 3, 5), 2),
    (1, (256, 4, 4, 6), 2),       # the widest block: one stripe per channel vector row of the workgroup
    (1, (112, 5, 3, 4), 3),       # 28 channel vectors: 9 stripes, four idle threads
])
def test_gradient_and_loss_match_oracle(m, dims, batch):
    cfg, X, labels, x0 = bn_case(m, dims, batch, 1, seed=141)
    x0 = x0 + G.generic_normal(7, 5, x0.shape, sigma=0.05)      # scales away from one, shifts away from zero
    g, losses = one_step(cfg, dims, batch, X, labels, x0)
    for i in range(m):
        loss, grad = CO.convblock_bn_loss_grad(x0, dims[0], dims[3], X[i, 0], labels[i, 0])
        assert abs(losses[i] - loss) <= 1e-5 * abs(loss)
        for name, sl in groups_of(dims[0], dims[3]).items():
            sl = sl.ravel()
            assert max_norm_ratio(g[i][sl], grad[sl]) <= GRAD_TOL, "worker %d %s" % (i, name)


def test_large_channel_means_do_not_cancel():
    """Inputs shifted by 30 standard deviations: the convolution outputs have channel means far above their spread, where
    a variance formed as mean of squares minus squared mean would lose its digits in single precision."""
    m, dims, batch = 2, (32, 16, 16, 10), 12            # 3072 pixels: two ranges
    cfg, X, labels, x0 = bn_case(m, dims, batch, 1, seed=142)
    X = (X + np.float32(30.0)).astype(np.float32)
    g, losses = one_step(cfg, dims, batch, X, labels, x0)
    for i in range(m):
        loss, grad = CO.convblock_bn_loss_grad(x0, dims[0], dims[3], X[i, 0], labels[i, 0])
        assert abs(losses[i] - loss) <= 1e-4 * abs(loss)
        for name, sl in groups_of(dims[0], dims[3]).items():
            sl = sl.ravel()
            assert max_norm_ratio(g[i][sl], grad[sl]) <= 2e-3, "worker %d %s" % (i, name)


def test_eps_is_the_callers():
    m, dims, batch = 2, (16, 6, 6, 4), 4
    cfg, X, labels, x0 = bn_case(m, dims, batch, 1, seed=143)
    C, n_w = dims[0], 9 * dims[0] * dims[0]
    x0 = x0.copy()                                      # small kernels: the variances fall below eps = 1e-3
    x0[:n_w] *= np.float32(0.01)
    x0[n_w + 2 * C:2 * n_w + 2 * C] *= np.float32(0.01)
    g, losses = one_step(cfg, dims, batch, X, labels, x0, eps=1e-3)
    for i in range(m):
        loss, grad = CO.convblock_bn_loss_grad(x0, dims[0], dims[3], X[i, 0], labels[i, 0], eps=1e-3)
        other, _ = CO.convblock_bn_loss_grad(x0, dims[0], dims[3], X[i, 0], labels[i, 0], eps=1e-5)
        assert abs(other - loss) > 1e-3 * abs(loss)      # the case does depend on eps
        assert abs(losses[i] - loss) <= 1e-5 * abs(loss)
        assert max_norm_ratio(g[i], grad) <= GRAD_TOL


@pytest.mark.parametrize("m,dims,batch,tau,K", [(3, (16, 6, 5, 4), 4, 2, 7), (2, (32, 8, 8, 10), 8, 3, 6)])
def test_small_runs_match_oracle(m, dims, batch, tau, K):
    cfg, X, labels, x0 = bn_case(m, dims, batch, 2, seed=244, tau=tau)
    grad_fn, margins = OW.conv_grad_fn(cfg.dims, X, labels, batch_norm=True), []

    def watched(i, k, x):
        margins.append(CO.convblock_relu_margin(x, dims[0], dims[3], X[i, k % 2], batch_norm=True))
        return grad_fn(i, k, x)
    st = OW.run_config(cfg, x0, watched, K=K)
    assert min(margins) >= RELU_MARGIN, "ill-conditioned case: pick another seed"
    with make_session(m, cfg.d, tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_convblock(*dims, batch, batch_norm=True)
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        losses = []
        s.run(K, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]), losses=losses)
        x, z, buf = s.all_params(), s.params(-1), s.momentum()
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(m)) <= E2E_TOL
    assert max(l2_ratio(buf[i], st["buf"][i]) for i in range(m)) <= E2E_TOL
    assert l2_ratio(z, st["z"]) <= E2E_TOL
    np.testing.assert_allclose(np.array(losses), st["losses"], rtol=1e-3)


def test_full_shape_short_run_matches_oracle():
    """The benchmark's per-worker shape (64 channels, 32 x 32, batch 128) on 2 of the 16 workers for one round, in the
    launch configuration the benchmark times (ols_run_steps over the resident data)."""
    cfg = I.get(7).scaled(m=2, nb=2, K=2)
    X, labels = G.conv_data(cfg)
    x0 = G.conv_init(cfg)
    st = OW.run_config(cfg, x0, OW.conv_grad_fn(cfg.dims, X, labels, batch_norm=True))
    with make_session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_convblock(*cfg.dims, cfg.batch, batch_norm=True)
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.run_resident(cfg.K, Xd, yd)
        x, z, losses = s.all_params(), s.params(-1), s.losses()
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(cfg.m)) <= E2E_TOL
    assert l2_ratio(z, st["z"]) <= E2E_TOL
    np.testing.assert_allclose(losses, st["losses"][-1], rtol=1e-3)


def test_schedule_variants_and_library_loop_are_bit_identical():
    m, dims, batch, tau, K = 3, (32, 6, 6, 5), 4, 2, 7
    cfg, X, labels, x0 = bn_case(m, dims, batch, 2, seed=343)
    outs = []
    for opts, library in (((), True), ((), False), (((B.OLS_OPT_SERIALIZE, 1),), True),
                          (((B.OLS_OPT_ANCHOR_DELAY_US, 2000),), True), (((B.OLS_OPT_FUSE_PULL, 0),), True)):
        with make_session(m, cfg.d, tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
            for key, val in opts:
                s.set_option(key, val)
            s.attach_convblock(*dims, batch, batch_norm=True)
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            if library:
                s.run_resident(K, Xd, yd)
            else:
                s.run(K, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]))
            outs.append((s.all_params(), s.params(-1), s.momentum(), s.losses()))
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert np.array_equal(a, b)
