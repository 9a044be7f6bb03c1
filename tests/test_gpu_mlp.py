"""GPU parity of the per-worker MLP forward/backward (grouped MFMA GEMMs, output layer, bias
gradients) and of whole MLP runs against the CPU oracle, through the C boundary."""
import numpy as np
import pytest

import ols_inputs as I
from ols_inputs import generate as G
from oracle import ols_oracle as O
from oracle import workloads as OW
from tests.helpers import l2_ratio, max_norm_ratio

from paper_2002_09539_amd import binding as B

pytestmark = pytest.mark.gpu

GRAD_TOL = 2e-5     # fp32 MFMA accumulation over K <= 3072 terms against the fp64 oracle, max-norm relative
E2E_TOL = 1e-3


def make_session(*a, **kw):
    from paper_2002_09539_amd.session import Session
    return Session(*a, **kw)


def small_mlp_case(m, dims, batch, nb, seed, noniid=0):
    cfg = I.get(2).scaled(m=m, dims=tuple(dims), batch=batch, nb=nb, seed=seed, noniid_classes=noniid,
                          n_classes=dims[-1])
    X, labels = G.mlp_data(cfg)
    x0 = G.mlp_init(cfg)
    return cfg, X, labels, x0


def layer_slices(dims):
    out, off = [], 0
    for l in range(len(dims) - 1):
        w = slice(off, off + dims[l] * dims[l + 1])
        off = w.stop
        b = slice(off, off + dims[l + 1])
        off = b.stop
        out.append((w, b))
    return out


@pytest.mark.parametrize("m,dims,batch", [
    (3, (100, 72, 10), 36),            # ragged in every tile dimension
    (2, (64, 96, 40, 7), 20),          # two hidden layers: exercises the delta GEMM
    (2, (256, 192, 132, 10), 132),     # several tiles per dimension plus tails
    (5, (128, 64, 64, 64, 16), 64),    # exact tile multiples, three hidden layers
    (2, (40, 12), 8),                  # no hidden layer at all
    (4, (3072, 512, 10), 128),         # configuration 2's layer shapes
    (4, (3072, 1024, 10), 64),         # configuration 5's layer shapes
    (2, (64, 48, 24), 12),             # more than 16 classes: the 32-class variant of the output-layer kernels
    (2, (96, 1040, 32), 20),           # 32 classes, last hidden layer wider than two staging passes, ragged
    (2, (64, 1544, 10), 24),           # last hidden layer wider than one 1024-unit pass, ragged
])
def test_gradient_and_loss_match_oracle(m, dims, batch):
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 1, seed=101)
    x0 = x0 + G.generic_normal(3, 1, x0.shape, sigma=0.02)      # non-zero biases as well
    with make_session(m, cfg.d, 2, 0.6, 0.05, 0.0) as s:
        s.set_option(B.OLS_OPT_FUSE_GEMM_UPDATE, 0)     # keep the gradients in g so they can be read
        s.attach_mlp(dims, batch, "f32")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.set_batch(Xd[:, 0], yd[:, 0])
        s.local_step()
        g, losses = s.gradient(), s.losses()
    for i in range(m):
        loss, grad = O.mlp_loss_grad(x0, dims, X[i, 0], labels[i, 0])
        assert abs(losses[i] - loss) <= 1e-5 * abs(loss)
        for l, (w, b) in enumerate(layer_slices(dims)):
            assert max_norm_ratio(g[i][w], grad[w]) <= GRAD_TOL, "worker %d dW%d" % (i, l)
            assert max_norm_ratio(g[i][b], grad[b]) <= GRAD_TOL, "worker %d db%d" % (i, l)


@pytest.mark.parametrize("m,dims,batch,tau,K,noniid", [
    (4, (96, 64, 10), 32, 2, 12, 0),
    (6, (64, 48, 32, 10), 16, 3, 10, 2),
])
def test_small_mlp_runs_match_oracle(m, dims, batch, tau, K, noniid):
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 3, seed=202, noniid=noniid)
    st = O.run(x0, m, tau, 0.6, 0.05, K, OW.mlp_grad_fn(dims, X, labels), mu=0.9)
    with make_session(m, cfg.d, tau, 0.6, 0.05, 0.9) as s:
        s.attach_mlp(dims, batch, "f32")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        losses = []
        s.run(K, lambda k: s.set_batch(Xd[:, k % 3], yd[:, k % 3]), losses=losses)
        x, z = s.all_params(), s.params(-1)
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(m)) <= E2E_TOL
    assert l2_ratio(z, st["z"]) <= E2E_TOL
    np.testing.assert_allclose(np.array(losses), st["losses"], rtol=1e-3)


def test_config2_shapes_short_run():
    """Configuration 2's model, batch and hyper-parameters on 4 of the 16 workers for 3 rounds."""
    cfg = I.get(2).scaled(m=4, nb=3, K=6)
    X, labels = G.mlp_data(cfg)
    x0 = G.mlp_init(cfg)
    st = OW.run_config(cfg, x0, OW.mlp_grad_fn(cfg.dims, X, labels))
    with make_session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_mlp(cfg.dims, cfg.batch, "f32")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        losses = []
        s.run(cfg.K, lambda k: s.set_batch(Xd[:, k % cfg.nb], yd[:, k % cfg.nb]), losses=losses)
        x, z = s.all_params(), s.params(-1)
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(cfg.m)) <= E2E_TOL
    assert l2_ratio(z, st["z"]) <= E2E_TOL
    np.testing.assert_allclose(np.array(losses), st["losses"], rtol=1e-3)


def test_config5_shapes_short_run():
    """Configuration 5's model, batch, non-IID labels and hyper-parameters (tau = 8) on 4 of the 64 workers for 2
    rounds on the default route (update fused into the gradient kernels, loop inside the library): every replica,
    momentum buffer and the anchor element by element."""
    cfg = I.get(5).scaled(m=4, nb=3, K=16)
    X, labels = G.mlp_data(cfg)
    x0 = G.mlp_init(cfg)
    st = OW.run_config(cfg, x0, OW.mlp_grad_fn(cfg.dims, X, labels))
    with make_session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_mlp(cfg.dims, cfg.batch, "f32")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.run_resident(cfg.K, Xd, yd)
        x, z, buf, losses = s.all_params(), s.params(-1), s.momentum(), s.losses()
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(cfg.m)) <= E2E_TOL
    assert max(l2_ratio(buf[i], st["buf"][i]) for i in range(cfg.m)) <= E2E_TOL
    assert l2_ratio(z, st["z"]) <= E2E_TOL
    np.testing.assert_allclose(losses, st["losses"][-1], rtol=1e-3)


# ---------------------------------------------------------------------------------------------
# bf16 GEMM operands, fp32 accumulation (configuration 3's arithmetic)
# ---------------------------------------------------------------------------------------------
BF16_LOSS_TOL = 2e-2        # the benchmark specification's bar for bf16-GEMM runs, relative on the loss


@pytest.mark.parametrize("m,dims,batch", [
    (2, (72, 40, 10), 24),               # ragged tiles
    (2, (256, 136, 264, 10), 136),       # several tiles plus tails, two hidden layers
    (3, (128, 128, 128, 128, 16), 64),   # exact multiples, three hidden layers
    (2, (64, 8), 16),                    # no hidden layer
    (2, (3072, 2048, 2048, 10), 256),    # configuration 3's layer shapes
    (2, (64, 1544, 24), 24),             # 24 classes and a ragged last hidden layer wider than a staging pass
])
def test_bf16_gradient_and_loss(m, dims, batch):
    """Against the oracle with the same operand rounding (tight), and against the unrounded oracle
    (the gate: loss within 2e-2; gradients within bf16 rounding)."""
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 1, seed=303)
    x0 = x0 + G.generic_normal(5, 2, x0.shape, sigma=0.02)
    with make_session(m, cfg.d, 2, 0.6, 0.05, 0.0) as s:
        s.set_option(B.OLS_OPT_FUSE_GEMM_UPDATE, 0)     # keep the gradients in g so they can be read
        s.attach_mlp(dims, batch, "bf16")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        s.set_batch(Xd[:, 0], yd[:, 0])
        s.local_step()
        g, losses = s.gradient(), s.losses()
    for i in range(m):
        loss_q, grad_q = O.mlp_loss_grad(x0, dims, X[i, 0], labels[i, 0], bf16_operands=True)
        loss, grad = O.mlp_loss_grad(x0, dims, X[i, 0], labels[i, 0])
        assert abs(losses[i] - loss) <= BF16_LOSS_TOL * abs(loss)
        assert abs(losses[i] - loss_q) <= 1e-3 * abs(loss_q)
        for l, (w, b) in enumerate(layer_slices(dims)):
            # fp32 vs double accumulation can move a stored activation across a bf16 rounding
            # boundary (one bf16 ulp = 0.4 % of that element): rare, so tight in L2, looser in max-norm
            assert l2_ratio(g[i][w], grad_q[w]) <= 2e-3, "worker %d dW%d (rounded oracle)" % (i, l)
            assert max_norm_ratio(g[i][w], grad_q[w]) <= 1e-2, "worker %d dW%d (rounded oracle)" % (i, l)
            assert max_norm_ratio(g[i][b], grad_q[b]) <= 1e-2, "worker %d db%d (rounded oracle)" % (i, l)
            # against the unrounded gradient only a loose L2 bound holds: a ReLU unit whose
            # pre-activation is near zero can switch under bf16 rounding and change a whole row
            assert l2_ratio(g[i][w], grad[w]) <= 0.1, "worker %d dW%d" % (i, l)


def test_bf16_small_run_loss_tracks_oracle():
    m, dims, batch, tau, K = 4, (128, 96, 64, 10), 32, 4, 16
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 4, seed=404)
    st = O.run(x0, m, tau, 0.5, 0.05, K, OW.mlp_grad_fn(dims, X, labels), mu=0.9)
    with make_session(m, cfg.d, tau, 0.5, 0.05, 0.9) as s:
        s.attach_mlp(dims, batch, "bf16")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        losses = []
        s.run(K, lambda k: s.set_batch(Xd[:, k % 4], yd[:, k % 4]), losses=losses)
        x, z = s.all_params(), s.params(-1)
    rel = np.abs(np.array(losses) - st["losses"]) / np.abs(st["losses"])
    assert rel.max() <= BF16_LOSS_TOL
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(m)) <= 2e-2


def test_config3_shapes_short_run():
    """Configuration 3's model (3072-2048-2048-2048-10, bf16 operands), batch 256 and hyper-parameters (tau = 4) on 2 of
    the 16 workers for 2 rounds on the default route: the mean mini-batch loss within the benchmark specification's
    2e-2 of the UNROUNDED oracle at every iteration, and every replica and the anchor element by element (the
    specification states no bar for parameters of a bf16 run; 5e-2 in L2 is this test's own)."""
    cfg = I.get(3).scaled(m=2, nb=2, K=8)
    X, labels = G.mlp_data(cfg)
    x0 = G.mlp_init(cfg)
    st = OW.run_config(cfg, x0, OW.mlp_grad_fn(cfg.dims, X, labels))
    with make_session(cfg.m, cfg.d, cfg.tau, cfg.alpha, cfg.gamma, cfg.mu) as s:
        s.attach_mlp(cfg.dims, cfg.batch, "bf16")
        Xd, yd = s.upload(X), s.upload(labels)
        s.init_params(x0)
        losses = []
        s.run(cfg.K, lambda k: s.set_batch(Xd[:, k % cfg.nb], yd[:, k % cfg.nb]), losses=losses)
        x, z = s.all_params(), s.params(-1)
    rel = np.abs(np.array(losses).mean(axis=1) - st["losses"].mean(axis=1)) / np.abs(st["losses"].mean(axis=1))
    assert rel.max() <= BF16_LOSS_TOL, rel
    assert max(l2_ratio(x[i], st["x"][i]) for i in range(cfg.m)) <= 5e-2
    assert l2_ratio(z, st["z"]) <= 5e-2


@pytest.mark.parametrize("dtype,dims,batch", [("f32", (96, 64, 40, 10), 36), ("bf16", (128, 72, 64, 10), 40)])
@pytest.mark.parametrize("tau,second_buffer", [(1, True), (2, True), (3, False)])
def test_update_fused_into_gradient_kernels_is_bit_identical(dtype, dims, batch, tau, second_buffer):
    """The gradient kernels applying the step (+ pull-back) in their epilogues must leave exactly the
    state the separate streaming kernels leave (same fp32 operation sequence per element)."""
    m, K = 3, 7
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 2, seed=505)
    states = []
    for fused in (1, 0):
        with make_session(m, cfg.d, tau, 0.6, 0.05, 0.9, overlap_buffer=second_buffer) as s:
            s.set_option(B.OLS_OPT_FUSE_GEMM_UPDATE, fused)
            s.attach_mlp(dims, batch, dtype)
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            losses = []
            s.run(K, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]), losses=losses)
            states.append((s.all_params(), s.params(-1), s.momentum(), np.array(losses)))
    for a, b in zip(states[0], states[1]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("dtype,dims,batch", [("f32", (96, 72, 10), 36), ("f32", (64, 48, 100, 24), 132),
                                              ("bf16", (128, 72, 64, 10), 40), ("bf16", (64, 1040, 32), 72)])
@pytest.mark.parametrize("fused", [1, 0])
def test_output_layer_gradients_as_guest_workgroups_are_bit_identical(dtype, dims, batch, fused):
    """The output layer's weight / bias gradients computed by extra workgroups of the weight-gradient GEMM's launch
    (default) or by a kernel of their own: same per-lane summation order, so identical bits -- with the update
    fused into the gradient kernels and without, up to 16 and up to 32 classes, widths that are no multiple of
    the 32 hidden units a workgroup owns, batches that are no multiple of the samples staged per pass."""
    m, K = 3, 5
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 2, seed=707)
    states = []
    for guest in (1, 0):
        with make_session(m, cfg.d, 2, 0.6, 0.05, 0.9) as s:
            s.set_option(B.OLS_OPT_HEAD_DW_GUEST, guest)
            s.set_option(B.OLS_OPT_FUSE_GEMM_UPDATE, fused)
            s.set_option(B.OLS_OPT_KERNEL_TIMING, 1)
            s.attach_mlp(dims, batch, dtype)
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            losses = []
            s.run(K, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]), losses=losses)
            s.sync()
            assert ("head_bwd" in s.kernel_stats()) == (guest == 0)
            grads = s.gradient() if not fused else None
            states.append((s.all_params(), s.params(-1), s.momentum(), np.array(losses), grads))
    for a, b in zip(states[0], states[1]):
        assert (a is None and b is None) or np.array_equal(a, b)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_library_driven_loop_equals_one_call_per_step(dtype):
    m, dims, batch, K = 3, (64, 40, 10), 24, 9
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 4, seed=909)
    outs = []
    for library in (True, False):
        with make_session(m, cfg.d, 2, 0.6, 0.05, 0.9) as s:
            s.attach_mlp(dims, batch, dtype)
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            if library:
                s.run_resident(K, Xd, yd)
            else:
                s.run(K, lambda k: s.set_batch(Xd[:, k % 4], yd[:, k % 4]))
            outs.append((s.all_params(), s.params(-1), s.momentum(), s.losses()))
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("m,dims,batch", [(2, (3072, 512, 10), 128),          # configuration 2: split-K forward GEMM
                                          (3, (1024, 256, 128, 10), 64),    # delta GEMM, single tile row
                                          (2, (3072, 1024, 10), 64)])       # configuration 5
def test_f32_full_tile_kernels_match_bounds_checked_kernels_bit_for_bit(m, dims, batch):
    """Layer shapes that are whole numbers of tiles take the fp32 GEMM kernels without bounds checks (uniform base
    plus fixed lane offsets); forcing the bounds-checked kernels on the same shapes must give identical bits."""
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 2, seed=1010)
    states = []
    for force in (0, 1):
        with make_session(m, cfg.d, 2, 0.6, 0.05, 0.9) as s:
            s.set_option(B.OLS_OPT_GEMM_FORCE_GENERAL, force)
            s.attach_mlp(dims, batch, "f32")
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            losses = []
            s.run(5, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]), losses=losses)
            states.append((s.all_params(), s.params(-1), s.momentum(), np.array(losses)))
    for a, b in zip(states[0], states[1]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("m,dims,batch,tau", [(2, (3072, 512, 10), 128, 2),      # configuration 2: K = 128
                                              (3, (256, 192, 128, 10), 64, 3),   # K = 64, two hidden layers
                                              (2, (128, 64, 10), 256, 1),        # K = 256, one tile per worker
                                              (5, (1024, 1024, 10), 64, 2)])     # more tiles than workgroups walk at once
def test_pipelined_weight_gradient_kernel_is_bit_identical(m, dims, batch, tau):
    """The persistent weight-gradient kernel that spreads the update of one tile over the K loop of the next must
    leave exactly the state of the kernel that contracts and updates tile by tile (same MFMA order, same update
    arithmetic)."""
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 2, seed=1111)
    states = []
    for variant in (16, 11):
        with make_session(m, cfg.d, tau, 0.6, 0.05, 0.9) as s:
            s.set_option(B.OLS_OPT_TUNING, B.TUNE_DW + variant)
            s.attach_mlp(dims, batch, "f32")
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            losses = []
            s.run(2 * tau + 1, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]), losses=losses)
            states.append((s.all_params(), s.params(-1), s.momentum(), np.array(losses)))
    for a, b in zip(states[0], states[1]):
        assert np.array_equal(a, b)


def test_bf16_full_tile_kernel_matches_bounds_checked_kernel_bit_for_bit():
    """Configuration 3's layer shapes take the branch-free full-tile forward / delta kernels; forcing the
    bounds-checked kernel on the same shapes must give identical bits (same slices, same MFMA order)."""
    m, dims, batch, K = 2, (3072, 2048, 2048, 2048, 10), 256, 3
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 2, seed=606)
    states = []
    for force in (0, 1):
        with make_session(m, cfg.d, 2, 0.5, 0.05, 0.9) as s:
            s.set_option(B.OLS_OPT_GEMM_FORCE_GENERAL, force)
            s.attach_mlp(dims, batch, "bf16")
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            losses = []
            s.run(K, lambda k: s.set_batch(Xd[:, k % 2], yd[:, k % 2]), losses=losses)
            states.append((s.all_params(), s.params(-1), np.array(losses)))
    for a, b in zip(states[0], states[1]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("dtype,dims,batch", [("f32", (96, 64, 40, 10), 36), ("bf16", (128, 72, 64, 10), 40)])
@pytest.mark.parametrize("tau,second_buffer,guest", [(1, True, 1), (1, False, 1), (2, True, 1), (2, True, 0), (3, False, 0)])
def test_late_refresh_is_awaited_by_the_first_updating_launch(dtype, dims, batch, tau, second_buffer, guest):
    """The main stream waits for the anchor refresh only in front of the first launch of a step that pulls toward the
    anchor or overwrites what the refresh reads (not in front of that step's forward and delta kernels).  With the
    refresh held back by an emulated latency far longer than a step, any launch that needed the wait and did not get
    it would read a stale anchor or overwrite the models under the refresh: the overlapped schedule must still leave
    exactly the bits of the serialised one."""
    m, K = 3, 3 * tau + 1
    cfg, X, labels, x0 = small_mlp_case(m, dims, batch, 2, seed=1212)
    states = []
    for serialize, delay in ((0, 3000), (1, 0)):
        with make_session(m, cfg.d, tau, 0.6, 0.05, 0.9, overlap_buffer=second_buffer) as s:
            s.set_option(B.OLS_OPT_SERIALIZE, serialize)
            s.set_option(B.OLS_OPT_ANCHOR_DELAY_US, delay)
            s.set_option(B.OLS_OPT_HEAD_DW_GUEST, guest)
            s.attach_mlp(dims, batch, dtype)
            Xd, yd = s.upload(X), s.upload(labels)
            s.init_params(x0)
            s.run_resident(K, Xd, yd)
            states.append((s.all_params(), s.params(-1), s.momentum(), s.losses()))
    for a, b in zip(states[0], states[1]):
        assert np.array_equal(a, b)
