"""Pins of the convolutional oracle (oracle/conv_oracle.py) to things other than itself: torch's CPU conv2d and
autograd as library routines, a pure-Python brute-force convolution, single-tap kernels whose result is a shifted copy
of the input (tap orientation and zero padding), central finite differences of the whole loss, closed forms of the
classifier head, and planted mistakes that these pins must notice.  No GPU."""
import numpy as np
import pytest

from oracle import conv_oracle as CO


def rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def brute_force_conv(inp, W, b):
    """The definition as nested Python loops (tiny inputs only)."""
    n, H, Wd, cin = inp.shape
    cout = W.shape[3]
    out = np.zeros((n, H, Wd, cout))
    for i in range(n):
        for y in range(H):
            for x in range(Wd):
                for co in range(cout):
                    acc = b[co]
                    for kh in range(3):
                        for kw in range(3):
                            yy, xx = y + kh - 1, x + kw - 1
                            if 0 <= yy < H and 0 <= xx < Wd:
                                for ci in range(cin):
                                    acc += inp[i, yy, xx, ci] * W[kh, kw, ci, co]
                    out[i, y, x, co] = acc
    return out


def test_forward_equals_brute_force_loops():
    inp, W, b = rand((2, 4, 5, 3), 1), rand((3, 3, 3, 2), 2), rand((2,), 3)
    np.testing.assert_allclose(CO.conv3x3_forward(inp, W, b), brute_force_conv(inp, W, b), rtol=0, atol=1e-13)


@pytest.mark.parametrize("kh,kw", [(0, 0), (0, 1), (1, 2), (2, 0), (2, 2), (1, 1)])
def test_single_tap_kernel_is_a_shifted_copy_with_zero_border(kh, kw):
    """W = identity over channels at one tap: out[y][x] = in[y + kh - 1][x + kw - 1], zero where that leaves the image.
    A flipped kernel (true convolution), a transposed tap index or a wrong padding fails here."""
    C, H, Wd = 3, 5, 6
    inp = rand((2, H, Wd, C), 4)
    W = np.zeros((3, 3, C, C))
    W[kh, kw] = np.eye(C)
    out = CO.conv3x3_forward(inp, W, np.zeros(C))
    want = np.zeros_like(inp)
    for y in range(H):
        for x in range(Wd):
            yy, xx = y + kh - 1, x + kw - 1
            if 0 <= yy < H and 0 <= xx < Wd:
                want[:, y, x, :] = inp[:, yy, xx, :]
    np.testing.assert_array_equal(out, want)


def test_channel_mixing_direction():
    """Input channel ci feeds output channel co through W[.][.][ci][co] (a transposed operand fails)."""
    inp = np.zeros((1, 3, 3, 2))
    inp[0, 1, 1, 0] = 1.0                          # only input channel 0 is lit
    W = np.zeros((3, 3, 2, 3))
    W[1, 1, 0, 2] = 5.0                            # ... and feeds output channel 2
    W[1, 1, 1, 0] = 7.0
    out = CO.conv3x3_forward(inp, W, np.zeros(3))
    assert out[0, 1, 1, 2] == 5.0 and out[0, 1, 1, 0] == 0.0 and out[0, 1, 1, 1] == 0.0


def test_forward_and_backward_match_torch_conv2d():
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    inp, W, b, dout = rand((3, 6, 5, 4), 5), rand((3, 3, 4, 7), 6), rand((7,), 7), rand((3, 6, 5, 7), 8)
    ti = torch.tensor(inp).permute(0, 3, 1, 2).requires_grad_(True)        # NCHW
    tw = torch.tensor(W).permute(3, 2, 0, 1).contiguous().requires_grad_(True)   # [out][in][kh][kw]
    tb = torch.tensor(b, requires_grad=True)
    to = F.conv2d(ti, tw, tb, stride=1, padding=1)
    np.testing.assert_allclose(CO.conv3x3_forward(inp, W, b), to.detach().permute(0, 2, 3, 1).numpy(), atol=1e-12)
    to.backward(torch.tensor(dout).permute(0, 3, 1, 2))
    d_inp, dW, db = CO.conv3x3_backward(inp, W, dout)
    np.testing.assert_allclose(d_inp, ti.grad.permute(0, 2, 3, 1).numpy(), atol=1e-12)
    np.testing.assert_allclose(dW, tw.grad.permute(2, 3, 1, 0).numpy(), atol=1e-11)
    np.testing.assert_allclose(db, tb.grad.numpy(), atol=1e-12)


def block_case(seed, B=3, C=4, H=5, Wd=4, classes=3):
    d = CO.convblock_param_count(C, classes)
    x = rand((d,), seed, 0.3)
    X = rand((B, H, Wd, C), seed + 1)
    labels = np.random.default_rng(seed + 2).integers(0, classes, B)
    return x, C, classes, X, labels


def test_block_gradient_matches_central_finite_differences():
    x, C, classes, X, labels = block_case(10)
    loss, g = CO.convblock_loss_grad(x, C, classes, X, labels)
    rng = np.random.default_rng(0)
    # every parameter group is probed: both kernels, both conv biases, classifier weights and bias
    Wa, ba, Wb, bb, Wh, bh = CO.convblock_unpack(np.arange(x.size), C, classes)
    picks = np.concatenate([rng.choice(grp.ravel(), min(6, grp.size), replace=False) for grp in (Wa, ba, Wb, bb, Wh, bh)])
    eps = 1e-6
    for j in picks:
        e = np.zeros_like(x)
        e[j] = eps
        fd = (CO.convblock_loss_grad(x + e, C, classes, X, labels)[0] - CO.convblock_loss_grad(x - e, C, classes, X, labels)[0]) / (2 * eps)
        assert abs(fd - g[j]) <= 1e-7 * max(1.0, abs(g[j])), (j, fd, g[j])
    assert loss > 0


def test_block_matches_torch_autograd_including_the_flat_layout():
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    x, C, classes, X, labels = block_case(20, B=4, C=3, H=4, Wd=6, classes=5)
    loss, g = CO.convblock_loss_grad(x, C, classes, X, labels)
    tx = torch.tensor(x, requires_grad=True)
    off = 0

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        t = tx[off:off + n].reshape(shape)
        off += n
        return t
    Wa, ba, Wb, bb, Wh, bh = (take(s) for s in ((3, 3, C, C), (C,), (3, 3, C, C), (C,), (C, classes), (classes,)))
    tX = torch.tensor(X).permute(0, 3, 1, 2)
    a1 = F.relu(F.conv2d(tX, Wa.permute(3, 2, 0, 1), ba, padding=1))
    a2 = F.relu(F.conv2d(a1, Wb.permute(3, 2, 0, 1), bb, padding=1) + tX)
    logits = a2.mean(dim=(2, 3)) @ Wh + bh
    tl = F.cross_entropy(logits, torch.tensor(labels), reduction="mean")
    tl.backward()
    assert abs(loss - tl.item()) <= 1e-12 * abs(loss)
    np.testing.assert_allclose(g, tx.grad.numpy(), atol=1e-12)


def test_zero_kernels_reduce_the_block_to_the_shortcut():
    """Wa = Wb = 0, zero biases: a2 = relu(X), the classifier sees the mean of relu(X): a closed form for the loss."""
    C, classes, B, H, Wd = 3, 4, 2, 3, 3
    x = np.zeros(CO.convblock_param_count(C, classes))
    Wa, ba, Wb, bb, Wh, bh = CO.convblock_unpack(x, C, classes)
    Wh[...] = rand((C, classes), 30)
    bh[...] = rand((classes,), 31)
    X = rand((B, H, Wd, C), 32)
    labels = np.array([1, 3])
    loss, g = CO.convblock_loss_grad(x, C, classes, X, labels)
    logits = np.maximum(X, 0).mean(axis=(1, 2)) @ Wh + bh
    want = np.mean([np.log(np.exp(l).sum()) - l[y] for l, y in zip(logits, labels)])
    assert abs(loss - want) <= 1e-13
    # the first convolution feeds only the (zero) second kernel: its gradient vanishes, the second one's does not
    gWa, gba, gWb, gbb, _, _ = CO.convblock_unpack(g, C, classes)
    assert not gWa.any() and not gba.any() and np.abs(gbb).max() > 0


# ---- the pins have teeth: a plausible mistake planted in the oracle fails one of them ---------------------
def _flipped_forward(inp, W, b):
    return _ORIG_FWD(inp, W[::-1, ::-1], b)            # true convolution instead of cross-correlation


def _no_padding_shift(inp, W, b):
    return _ORIG_FWD(np.roll(inp, 1, axis=2), W, b)    # a wrong horizontal offset with wrap-around


def _transposed_channels(inp, W, b):
    return _ORIG_FWD(inp, np.swapaxes(W, 2, 3), b)


_ORIG_FWD = CO.conv3x3_forward


@pytest.mark.parametrize("broken", [_flipped_forward, _no_padding_shift, _transposed_channels])
def test_planted_forward_mistakes_are_noticed(monkeypatch, broken):
    monkeypatch.setattr(CO, "conv3x3_forward", broken)
    failures = 0
    for check in (lambda: test_single_tap_kernel_is_a_shifted_copy_with_zero_border(0, 1),
                  test_forward_and_backward_match_torch_conv2d, test_block_gradient_matches_central_finite_differences):
        try:
            check()
        except (AssertionError, ValueError):      # a shape that no longer fits is a noticed mistake as well
            failures += 1
    assert failures >= 1


def test_planted_backward_mistakes_are_noticed(monkeypatch):
    orig = CO.conv3x3_backward

    def no_relu_mask_equivalent(inp, W, dout):          # drops the bias gradient's sum over positions
        d_inp, dW, db = orig(inp, W, dout)
        return d_inp, dW, db / 2
    monkeypatch.setattr(CO, "conv3x3_backward", no_relu_mask_equivalent)
    with pytest.raises(AssertionError):
        test_block_gradient_matches_central_finite_differences()

    def swapped_taps(inp, W, dout):
        d_inp, dW, db = orig(inp, W, dout)
        return d_inp, dW[::-1, ::-1], db
    monkeypatch.setattr(CO, "conv3x3_backward", swapped_taps)
    with pytest.raises(AssertionError):
        test_block_matches_torch_autograd_including_the_flat_layout()


# ---- batch normalisation ------------------------------------------------------------------------------------
def test_batchnorm_output_has_the_prescribed_channel_statistics():
    z, g, b = rand((4, 3, 5, 6), 40, 2.0) + 3.0, rand((6,), 41), rand((6,), 42)
    out, xhat, inv_std = CO.batchnorm_forward(z, g, b)
    np.testing.assert_allclose(xhat.mean(axis=(0, 1, 2)), 0.0, atol=1e-13)
    np.testing.assert_allclose(out.mean(axis=(0, 1, 2)), b, atol=1e-12)
    # biased variance of the normalised values is var / (var + eps): just below one
    var = z.var(axis=(0, 1, 2))
    np.testing.assert_allclose(xhat.var(axis=(0, 1, 2)), var / (var + CO.BN_EPS), rtol=1e-12)
    np.testing.assert_allclose(inv_std, 1.0 / np.sqrt(var + CO.BN_EPS), rtol=1e-13)


def test_batchnorm_matches_torch_forward_and_backward():
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    z, g, b, dout = rand((3, 4, 5, 6), 50), rand((6,), 51), rand((6,), 52), rand((3, 4, 5, 6), 53)
    tz = torch.tensor(z).permute(0, 3, 1, 2).contiguous().requires_grad_(True)
    tg, tb = torch.tensor(g, requires_grad=True), torch.tensor(b, requires_grad=True)
    to = F.batch_norm(tz, None, None, tg, tb, training=True, eps=CO.BN_EPS)
    out, xhat, inv_std = CO.batchnorm_forward(z, g, b)
    np.testing.assert_allclose(out, to.detach().permute(0, 2, 3, 1).numpy(), atol=1e-12)
    to.backward(torch.tensor(dout).permute(0, 3, 1, 2))
    d_z, d_g, d_b = CO.batchnorm_backward(dout, xhat, inv_std, g)
    np.testing.assert_allclose(d_z, tz.grad.permute(0, 2, 3, 1).numpy(), atol=1e-12)
    np.testing.assert_allclose(d_g, tg.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(d_b, tb.grad.numpy(), atol=1e-12)


def bn_block_case(seed, B=3, C=4, H=5, Wd=4, classes=3):
    d = CO.convblock_bn_param_count(C, classes)
    x = rand((d,), seed, 0.3)
    Wa, ga, ba, Wb, gb, bb, Wh, bh = CO.convblock_bn_unpack(x, C, classes)
    ga += 1.0
    gb += 1.0                                         # scales around one, as at initialisation
    X = rand((B, H, Wd, C), seed + 1)
    labels = np.random.default_rng(seed + 2).integers(0, classes, B)
    return x, C, classes, X, labels


def test_bn_block_gradient_matches_central_finite_differences():
    x, C, classes, X, labels = bn_block_case(60)
    loss, g = CO.convblock_bn_loss_grad(x, C, classes, X, labels)
    rng = np.random.default_rng(1)
    groups = CO.convblock_bn_unpack(np.arange(x.size), C, classes)
    picks = np.concatenate([rng.choice(grp.ravel(), min(5, grp.size), replace=False) for grp in groups])
    eps = 1e-6
    for j in picks:
        e = np.zeros_like(x)
        e[j] = eps
        fd = (CO.convblock_bn_loss_grad(x + e, C, classes, X, labels)[0] - CO.convblock_bn_loss_grad(x - e, C, classes, X, labels)[0]) / (2 * eps)
        assert abs(fd - g[j]) <= 2e-7 * max(1.0, abs(g[j])), (j, fd, g[j])


def test_bn_block_matches_torch_autograd_including_the_flat_layout():
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    x, C, classes, X, labels = bn_block_case(70, B=4, C=3, H=4, Wd=6, classes=5)
    loss, g = CO.convblock_bn_loss_grad(x, C, classes, X, labels)
    tx = torch.tensor(x, requires_grad=True)
    off = 0

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        t = tx[off:off + n].reshape(shape)
        off += n
        return t
    Wa, ga, ba, Wb, gb, bb, Wh, bh = (take(s) for s in ((3, 3, C, C), (C,), (C,), (3, 3, C, C), (C,), (C,), (C, classes), (classes,)))
    tX = torch.tensor(X).permute(0, 3, 1, 2)
    bn = lambda z, g_, b_: F.batch_norm(z, None, None, g_, b_, training=True, eps=CO.BN_EPS)
    a1 = F.relu(bn(F.conv2d(tX, Wa.permute(3, 2, 0, 1), None, padding=1), ga, ba))
    a2 = F.relu(bn(F.conv2d(a1, Wb.permute(3, 2, 0, 1), None, padding=1), gb, bb) + tX)
    logits = a2.mean(dim=(2, 3)) @ Wh + bh
    tl = F.cross_entropy(logits, torch.tensor(labels), reduction="mean")
    tl.backward()
    assert abs(loss - tl.item()) <= 1e-12 * abs(loss)
    np.testing.assert_allclose(g, tx.grad.numpy(), atol=1e-11)


def test_bn_makes_the_loss_invariant_to_the_scale_of_a_kernel():
    """A convolution followed by batch normalisation: scaling the kernel leaves the output (up to eps) and hence the
    loss unchanged, and the kernel's gradient is orthogonal to the kernel."""
    x, C, classes, X, labels = bn_block_case(80)
    loss, g = CO.convblock_bn_loss_grad(x, C, classes, X, labels, eps=0.0)
    x2 = x.copy()
    Wa2 = CO.convblock_bn_unpack(x2, C, classes)[0]
    Wa2 *= 3.0
    loss2, _ = CO.convblock_bn_loss_grad(x2, C, classes, X, labels, eps=0.0)
    assert abs(loss - loss2) <= 1e-12
    Wa, gWa = CO.convblock_bn_unpack(x, C, classes)[0], CO.convblock_bn_unpack(g, C, classes)[0]
    assert abs((Wa * gWa).sum()) <= 1e-12 * np.abs(Wa * gWa).sum()


def test_planted_batchnorm_mistakes_are_noticed(monkeypatch):
    orig_f, orig_b = CO.batchnorm_forward, CO.batchnorm_backward

    def unbiased_variance(z, gamma, beta, eps=CO.BN_EPS):
        z = np.asarray(z, np.float64)
        axes = tuple(range(z.ndim - 1))
        mean, var = z.mean(axis=axes), z.var(axis=axes, ddof=1)
        inv = 1.0 / np.sqrt(var + eps)
        xhat = (z - mean) * inv
        return np.asarray(gamma) * xhat + np.asarray(beta), xhat, inv
    monkeypatch.setattr(CO, "batchnorm_forward", unbiased_variance)
    with pytest.raises(AssertionError):
        test_batchnorm_matches_torch_forward_and_backward()
    monkeypatch.setattr(CO, "batchnorm_forward", orig_f)

    def drops_the_projection(dout, xhat, inv_std, gamma):     # treats mean and variance as constants
        d_z, d_g, d_b = orig_b(dout, xhat, inv_std, gamma)
        return np.asarray(gamma) * inv_std * np.asarray(dout), d_g, d_b
    monkeypatch.setattr(CO, "batchnorm_backward", drops_the_projection)
    with pytest.raises(AssertionError):
        test_bn_block_gradient_matches_central_finite_differences()


@pytest.mark.parametrize("batch_norm", [False, True])
def test_relu_margin_is_the_smallest_relu_input(batch_norm):
    """Against torch's conv2d / batch_norm; and moving one bias (or shift) by the margin's own element puts a ReLU input
    on zero, which the helper must then report."""
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F
    x, C, classes, X, labels = (bn_block_case if batch_norm else block_case)(80, B=2, C=3, H=4, Wd=3, classes=2)
    tX = torch.tensor(X).permute(0, 3, 1, 2)
    if batch_norm:
        Wa, ga, ba, Wb, gb, bb, _, _ = (torch.tensor(np.array(v)) for v in CO.convblock_bn_unpack(x, C, classes))
        bn = lambda z, g_, b_: F.batch_norm(z, None, None, g_, b_, training=True, eps=CO.BN_EPS)
        n1 = bn(F.conv2d(tX, Wa.permute(3, 2, 0, 1), None, padding=1), ga, ba)
        n2 = bn(F.conv2d(F.relu(n1), Wb.permute(3, 2, 0, 1), None, padding=1), gb, bb) + tX
    else:
        Wa, ba, Wb, bb, _, _ = (torch.tensor(np.array(v)) for v in CO.convblock_unpack(x, C, classes))
        n1 = F.conv2d(tX, Wa.permute(3, 2, 0, 1), ba, padding=1)
        n2 = F.conv2d(F.relu(n1), Wb.permute(3, 2, 0, 1), bb, padding=1) + tX
    want = min(n1.abs().min().item(), n2.abs().min().item())
    got = CO.convblock_relu_margin(x, C, classes, X, batch_norm=batch_norm)
    assert got > 1e-4 and abs(got - want) <= 1e-12
    # the second ReLU's inputs move one to one with the second bias / shift: cancel the smallest of them
    flat = n2.permute(0, 2, 3, 1).reshape(-1, C).numpy()
    pos = np.unravel_index(np.abs(flat).argmin(), flat.shape)
    y = x.copy()
    views = CO.convblock_bn_unpack(y, C, classes) if batch_norm else CO.convblock_unpack(y, C, classes)
    views[5 if batch_norm else 3][pos[1]] -= flat[pos]
    assert CO.convblock_relu_margin(y, C, classes, X, batch_norm=batch_norm) <= 1e-12


# ---- the bf16-operand diagnostic mode of the plain block ------------------------------------------------------------
def _torch_bf16_block(x, C, classes, X, labels, round_d_z1=True):
    """The same rounding points in torch: values rounded through bfloat16 with the rounding passed through as the
    identity in the backward pass, and the deltas at both convolution outputs rounded by gradient hooks."""
    import torch
    import torch.nn.functional as F

    def rnd(t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    def ste(t):
        return t + (rnd(t) - t).detach()
    tx = torch.tensor(x, requires_grad=True)
    off = 0

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        t = tx[off:off + n].reshape(shape)
        off += n
        return t
    Wa, ba, Wb, bb, Wh, bh = (take(s) for s in ((3, 3, C, C), (C,), (3, 3, C, C), (C,), (C, classes), (classes,)))
    tX = torch.tensor(X).permute(0, 3, 1, 2)
    z1 = F.conv2d(rnd(tX), ste(Wa).permute(3, 2, 0, 1), ba, padding=1)
    if round_d_z1:
        z1.register_hook(rnd)
    a1 = ste(F.relu(z1))
    z2 = F.conv2d(a1, ste(Wb).permute(3, 2, 0, 1), bb, padding=1) + tX
    z2.register_hook(rnd)
    logits = F.relu(z2).mean(dim=(2, 3)) @ Wh + bh
    tl = F.cross_entropy(logits, torch.tensor(labels), reduction="mean")
    tl.backward()
    return tl.item(), tx.grad.numpy()


def test_bf16_operand_mode_matches_torch_with_the_same_rounding_points():
    pytest.importorskip("torch")
    x, C, classes, X, labels = block_case(90, B=4, C=3, H=4, Wd=6, classes=5)
    loss, g = CO.convblock_loss_grad(x, C, classes, X, labels, bf16_operands=True)
    tl, tg = _torch_bf16_block(x, C, classes, X, labels)
    assert abs(loss - tl) <= 1e-12 * abs(loss)
    np.testing.assert_allclose(g, tg, atol=1e-12)
    exact_loss, exact_g = CO.convblock_loss_grad(x, C, classes, X, labels)
    assert 1e-5 < abs(loss - exact_loss) / abs(exact_loss) < 2e-2          # the mode rounds, and stays within the gate
    assert 1e-4 < np.abs(g - exact_g).max() / np.abs(exact_g).max() < 5e-2
    # teeth: leaving one delta unrounded is a different computation
    _, tg_wrong = _torch_bf16_block(x, C, classes, X, labels, round_d_z1=False)
    assert np.abs(g - tg_wrong).max() > 1e-6 * np.abs(g).max()


def test_bf16_operand_mode_is_the_plain_block_on_bf16_exact_operands():
    """Kernels of +-1 on one tap, inputs that are small integers, zero biases: every operand and every intermediate
    sum is exactly representable, so the mode must not change the forward pass."""
    C, classes, B, H, Wd = 2, 3, 2, 3, 3
    x = np.zeros(CO.convblock_param_count(C, classes))
    Wa, ba, Wb, bb, Wh, bh = CO.convblock_unpack(x, C, classes)
    Wa[1, 1, 0, 1] = 1.0
    Wa[0, 2, 1, 0] = -1.0
    Wb[2, 0, 0, 0] = 1.0
    Wb[1, 1, 1, 1] = 2.0
    Wh[...] = np.array([[0.5, -0.25, 1.0], [1.0, 0.5, -0.5]])
    X = np.random.default_rng(5).integers(-3, 4, (B, H, Wd, C)).astype(np.float64)
    labels = np.array([0, 2])
    a, _ = CO.convblock_loss_grad(x, C, classes, X, labels, bf16_operands=True)
    b, _ = CO.convblock_loss_grad(x, C, classes, X, labels)
    assert a == b


# ---- the same mode of the batch-normalised block -----------------------------------------------------------------------
def _torch_bf16_bn_block(x, C, classes, X, labels, round_d_z2=True):
    """Rounding points of the normalised block in torch: the batch, the kernels and a1 rounded with the rounding passed
    through as the identity; the deltas at both convolution outputs rounded by gradient hooks (the hook on a
    convolution's output sees the normalisation's input gradient, which is what becomes the operand)."""
    import torch
    import torch.nn.functional as F

    def rnd(t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    def ste(t):
        return t + (rnd(t) - t).detach()
    tx = torch.tensor(x, requires_grad=True)
    off = 0

    def take(shape):
        nonlocal off
        n = int(np.prod(shape))
        t = tx[off:off + n].reshape(shape)
        off += n
        return t
    Wa, ga, ba, Wb, gb, bb, Wh, bh = (take(s) for s in ((3, 3, C, C), (C,), (C,), (3, 3, C, C), (C,), (C,), (C, classes), (classes,)))
    tX = torch.tensor(X).permute(0, 3, 1, 2)
    bn = lambda z, g_, b_: F.batch_norm(z, None, None, g_, b_, training=True, eps=CO.BN_EPS)
    z1 = F.conv2d(rnd(tX), ste(Wa).permute(3, 2, 0, 1), None, padding=1)
    z1.register_hook(rnd)
    a1 = ste(F.relu(bn(z1, ga, ba)))
    z2 = F.conv2d(a1, ste(Wb).permute(3, 2, 0, 1), None, padding=1)
    if round_d_z2:
        z2.register_hook(rnd)
    logits = F.relu(bn(z2, gb, bb) + tX).mean(dim=(2, 3)) @ Wh + bh
    tl = F.cross_entropy(logits, torch.tensor(labels), reduction="mean")
    tl.backward()
    return tl.item(), tx.grad.numpy()


def test_bf16_operand_mode_of_the_bn_block_matches_torch_with_the_same_rounding_points():
    pytest.importorskip("torch")
    x, C, classes, X, labels = bn_block_case(91, B=4, C=3, H=4, Wd=6, classes=5)
    loss, g = CO.convblock_bn_loss_grad(x, C, classes, X, labels, bf16_operands=True)
    tl, tg = _torch_bf16_bn_block(x, C, classes, X, labels)
    assert abs(loss - tl) <= 1e-12 * abs(loss)
    np.testing.assert_allclose(g, tg, atol=1e-11)
    exact_loss, exact_g = CO.convblock_bn_loss_grad(x, C, classes, X, labels)
    assert 1e-6 < abs(loss - exact_loss) / abs(exact_loss) < 2e-2          # the mode rounds, and stays within the gate
    assert 1e-4 < np.abs(g - exact_g).max() / np.abs(exact_g).max() < 1e-1
    # teeth: leaving one delta unrounded is a different computation
    _, tg_wrong = _torch_bf16_bn_block(x, C, classes, X, labels, round_d_z2=False)
    assert np.abs(g - tg_wrong).max() > 1e-6 * np.abs(g).max()


@pytest.mark.parametrize("batch_norm", [False, True])
def test_relu_margin_in_the_bf16_mode_matches_torch_with_the_same_rounding_points(batch_norm):
    torch = pytest.importorskip("torch")
    import torch.nn.functional as F

    def rnd(t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    x, C, classes, X, labels = (bn_block_case if batch_norm else block_case)(92, B=3, C=4, H=5, Wd=4, classes=3)
    tX = torch.tensor(X).permute(0, 3, 1, 2)
    if batch_norm:
        Wa, ga, ba, Wb, gb, bb, _, _ = (torch.tensor(np.array(v)) for v in CO.convblock_bn_unpack(x, C, classes))
        bn = lambda z, g_, b_: F.batch_norm(z, None, None, g_, b_, training=True, eps=CO.BN_EPS)
        n1 = bn(F.conv2d(rnd(tX), rnd(Wa).permute(3, 2, 0, 1), None, padding=1), ga, ba)
        n2 = bn(F.conv2d(rnd(F.relu(n1)), rnd(Wb).permute(3, 2, 0, 1), None, padding=1), gb, bb) + tX
    else:
        Wa, ba, Wb, bb, _, _ = (torch.tensor(np.array(v)) for v in CO.convblock_unpack(x, C, classes))
        n1 = F.conv2d(rnd(tX), rnd(Wa).permute(3, 2, 0, 1), ba, padding=1)
        n2 = F.conv2d(rnd(F.relu(n1)), rnd(Wb).permute(3, 2, 0, 1), bb, padding=1) + tX
    want = min(n1.abs().min().item(), n2.abs().min().item())
    got = CO.convblock_relu_margin(x, C, classes, X, batch_norm=batch_norm, bf16_operands=True)
    assert abs(got - want) <= 1e-12
    assert got != CO.convblock_relu_margin(x, C, classes, X, batch_norm=batch_norm)      # the mode does round
