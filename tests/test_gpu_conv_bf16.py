"""GPU parity of the residual block with bf16 convolution operands (fp32 accumulation; operand tensors stored with their
zero border) against the CPU oracle (oracle/conv_oracle.py), through the C boundary: one step against the oracle with
the same rounding points (tight) and against the unrounded oracle (the benchmark specification's bf16 gate: loss within
2e-2), whole Overlap Local-SGD runs, the schedule variants."""
import numpy as np
import pytest

import ols_inputs as I
from ols_inputs import generate as G
from oracle import conv_oracle as CO
from oracle import workloads as OW
from tests.helpers import l2_ratio, max_norm_ratio

from paper_2002_09539_amd import binding as B

pytestmark = pytest.mark.gpu

BF16_LOSS_TOL = 2e-2        # the benchmark specification's bar for bf16 runs, relative on the loss


def make_session(*a, **kw):
    from paper_2002_09539_amd.session import Session
    return Session(*a, **kw)


def conv_case(m, dims, batch, nb, seed, **kw):
    cfg = I.get(8).scaled(m=m, dims=tuple(dims), batch=batch, nb=nb, seed=seed, **kw)
    X, labels = G.conv_data(cfg)
    return cfg, X, labels, G.conv_init(cfg)


def groups_of(C, classes):
    idx = np.arange(CO.convblock_param_count(C, classes))
    return dict(zip(("Wa", "ba", "Wb", "bb", "Wh", "bh"), CO.convblock_unpack(idx, C, classes)))


@pytest.mark.parametrize("m,dims,batch", [
    (2, (64, 5, 6, 4), 3),         # 168 padded pixels: one ragged tile, one range of the kernel gradient
    (3, (64, 8, 8, 10), 5),        # 500 padded pixels: two tiles, the second ragged
    (1, (128, 6, 6, 7), 3),        # 128 channels: two contraction chunks, two output tiles, 2 x 2 blocks of the gradient
    (2, (64, 32, 32, 10), 6),      # the benchmark's per-image shape: 28 tiles, several pixel ranges
    (1, (64, 1, 1, 3), 2),         # a single position: every tap but the centre reads the border
    (2, (64, 40, 3, 5), 2),        # narrow images
    (1, (64, 3, 100, 4), 1),       # wide images: the long halo (the larger strip variant of the kernel gradient)
    (1, (64, 2, 128, 3), 1),       # the widest image the kernels take
    (2, (64, 7, 33, 5), 3),        # one column past the short-halo variants
    (1, (192, 4, 5, 3), 2),        # three contraction chunks, three output tiles, 3 x 3 blocks of the gradient
    (1, (128, 3, 40, 4), 2),       # the long-halo variants with two chunks / two output tiles, and the fused tail
    (2, (128, 8, 8, 5), 3),        # the fused tail on two output tiles; samples of 100 padded pixels straddle wavefronts
    (1, (256, 6, 8, 3), 2),        # the widest channel count the block takes: four chunks, four output tiles
])
def test_gradient_and_loss(m, dims, batch):
    cfg, X, labels, x0 = conv_case(m, dims, batch, 1, seed=515)
    x0 = x0 + G.generic_normal(7, 6, x0.shape, sigma=0.02)      # non-zero biases as well
    with make_session(m, cfg.d, 2, 0.6, 0.05, 0.0) as s:
        s.attach_convblock(*dims, batch, gemm_dtype="bf16")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.set_batch(Xd[:, 0], yd[:, 0])
        s.local_step()
        g, losses = s.gradient(), s.losses()
    for i in range(m):
        loss_q, grad_q = CO.convblock_loss_grad(x0, dims[0], dims[3], X[i, 0], labels[i, 0], bf16_operands=True)
        loss, grad = CO.convblock_loss_grad(x0, dims[0], dims[3], X[i, 0], labels[i, 0])
        assert abs(losses[i] - loss) <= BF16_LOSS_TOL * abs(loss)
        assert abs(losses[i] - loss_q) <= 1e-5 * abs(loss_q)
        for name, sl in groups_of(dims[0], dims[3]).items():
            sl = sl.ravel()
            # With the same rounding points the two sides agree to 1e-7 .. 1e-6 -- unless fp32 against double
            # accumulation moves a value across a bf16 rounding boundary (one bf16 ulp = 0.4 % of that value).  The
            # pooled delta of a (sample, channel) is ONE value copied to all positions, so one such event moves a whole
            # channel of a sample at once: seen at 2e-3 .. 5e-3 in L2 and 2e-2 in max-norm on the smallest cases.
            tight = name in ("Wh", "bh")       # the classifier's gradients do not pass through a rounded delta
            assert l2_ratio(g[i][sl], grad_q[sl]) <= (1e-4 if tight else 1e-2), "worker %d %s (rounded oracle)" % (i, name)
            assert max_norm_ratio(g[i][sl], grad_q[sl]) <= (1e-4 if tight else 3e-2), "worker %d %s (rounded oracle)" % (i, name)
            assert l2_ratio(g[i][sl], grad[sl]) <= 0.1, "worker %d %s" % (i, name)


def test_small_run_tracks_oracle():
    m, dims, batch, tau, K = 3, (64, 6, 5, 4), 4, 2, 8
    cfg, X, labels, x0 = conv_case(m, dims, batch, 2, seed=616, tau=tau)
    st = OW.run_config(cfg, x0, OW.conv_grad_fn(cfg.dims, X, labels), K=K)                       # the unrounded target
    sq = OW.run_config(cfg, x0, OW.conv_grad_fn(cfg.dims, X, labels, bf16_operands=True), K=K)   # same rounding points
    with make_session(m, cfg.d, tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_convblock(*dims, batch, gemm_dtype="bf16")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        losses = []
        s.run(K, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]), losses=losses)
        x, z = s.all_params(), s.params(-1)
    rel = np.abs(np.array(losses) - st["losses"]) / np.abs(st["losses"])
    assert rel.max() <= BF16_LOSS_TOL
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(m)) <= 2e-2
    assert max(l2_ratio(x[i], sq["x"][i]) for i in range(m)) <= 5e-3
    assert l2_ratio(z, sq["z"]) <= 5e-3


def test_full_shape_short_run_matches_oracle():
    """The benchmark's per-worker shape (64 channels, 32 x 32, batch 128) on 2 of the 16 workers for one round, in the
    launch configuration the benchmark times (ols_run_steps over the resident data)."""
    cfg = I.get(8).scaled(m=2, nb=2, K=2)
    X, labels = G.conv_data(cfg)
    x0 = G.conv_init(cfg)
    st = OW.run_config(cfg, x0, OW.conv_grad_fn(cfg.dims, X, labels))
    with make_session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_convblock(*cfg.dims, cfg.batch, gemm_dtype="bf16")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.run_resident(cfg.K, Xd, yd)
        x, z, losses = s.all_params(), s.params(-1), s.losses()
    np.testing.assert_allclose(losses, st["losses"][-1], rtol=BF16_LOSS_TOL)
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(cfg.m)) <= 2e-2
    assert l2_ratio(z, st["z"]) <= 2e-2


def test_schedule_variants_and_library_loop_are_bit_identical():
    m, dims, batch, tau, K = 3, (64, 6, 6, 5), 4, 2, 7
    cfg, X, labels, x0 = conv_case(m, dims, batch, 2, seed=717)
    outs = []
    for opts, library in (((), True), ((), False), (((B.OLS_OPT_SERIALIZE, 1),), True),
                          (((B.OLS_OPT_ANCHOR_DELAY_US, 2000),), True), (((B.OLS_OPT_FUSE_PULL, 0),), True)):
        with make_session(m, cfg.d, tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
            for key, val in opts:
                s.set_option(key, val)
            s.attach_convblock(*dims, batch, gemm_dtype="bf16")
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
