"""CPU oracle for the convolutional workload of Overlap Local-SGD.  TEST INFRASTRUCTURE ONLY.

The paper's experiments (Section 4, "Experimental setting") train ResNet-18 on CIFAR-10 with a mini-batch of 128
per node; the update rules of Section 2 are model-agnostic and live in ols_oracle.py.  This module supplies the
per-worker stochastic gradient g_i for the first residual stage of that network at CIFAR resolution, written out
from the definition of the operations, in double, with no blocking or fusion:

    a1     = relu(conv3x3(X;  Wa) + ba)
    a2     = relu(conv3x3(a1; Wb) + bb + X)           the residual ("basic") block, identity shortcut
    pooled = mean over the H x W positions of a2
    logits = pooled Wh + bh;   loss = mean over the batch of softmax cross-entropy

With batch normalisation (the block as the residual network has it; `convblock_bn_loss_grad`) the convolutions carry
no bias and each is followed by a normalisation over the mini-batch and the positions, per channel, in training mode:

    z1 = conv3x3(X; Wa);   a1 = relu(bn(z1; ga, ba))
    z2 = conv3x3(a1; Wb);  a2 = relu(bn(z2; gb, bb) + X)
    bn(z; g, b)[n][y][x][c] = g[c] (z[n][y][x][c] - mean_c) / sqrt(var_c + eps) + b[c]

with mean_c and the (biased) variance var_c taken over all samples and positions of the worker's mini-batch.

Readings (the paper names the architecture and nothing more): the block is the two-convolution residual block with
identity shortcut, 3 x 3 kernels, stride 1, zero padding 1; without batch normalisation biases take its place; with
it, the statistics are those of the worker's own mini-batch (each worker normalises alone, as each node of the paper's
cluster does), the variance is the biased one, eps = 1e-5 (the common framework default), and no running averages are
kept (they play no part in training); "convolution" is the cross-correlation every
deep-learning framework computes: out[y][x] = sum_{kh,kw} in[y + kh - 1][x + kw - 1] W[kh][kw]; the ReLU derivative
at 0 is 0; the loss is the mean over the mini-batch (as for the other models).

Layouts (an interface shared with the device path; each side computes its own offsets): activations are
[batch][height][width][channel]; the flat parameter vector holds Wa [3][3][C][C] (kh, kw, input channel, output
channel), ba [C], Wb [3][3][C][C], bb [C], Wh [C][classes], bh [classes], in that order; with batch normalisation
Wa, ga [C], ba [C], Wb, gb [C], bb [C], Wh, bh (scale before shift).

`bf16_operands=True` is a DIAGNOSTIC mode of the plain block for a device path that feeds its convolutions bf16
operands (as `mlp_loss_grad` has one for the matrix products of the MLP): every tensor is rounded to bf16, to nearest
even, at the point where it becomes an operand of a convolution's products -- the input batch, both kernels, a1, and
the deltas d_z2 and d_z1 -- while sums, biases, the shortcut, pooling, classifier and the master parameters stay as they
are.  The gradient it returns is what back-propagation computes from those rounded tensors (the rounding itself is
passed through as the identity).  The target of the benchmark specification's bf16 gate is still the unrounded
computation.  The batch-normalised block has the same mode with the same rule: the input batch, both kernels, a1, and
the deltas at the two convolution outputs (which there are the normalisations' input gradients) are rounded; the
convolution outputs, the normalisations, their statistics and their parameters are not operands of a convolution.

Only tests/, the smoke check and the benchmark's CPU-baseline leg may import this module.
Pinned by tests/test_oracle_conv_pins.py: torch's CPU conv2d, batch_norm and autograd as library routines, a pure-Python
brute-force convolution, single-tap kernels that pin the tap orientation and the zero padding, the normalised output's
per-channel mean and variance, central finite differences of the whole loss, and planted mistakes that those pins must
notice.
"""
import numpy as np

from .ols_oracle import round_to_bf16

F64 = np.float64


def conv3x3_forward(inp, W, b):
    """out[n][y][x][co] = b[co] + sum_{kh,kw,ci} inp[n][y+kh-1][x+kw-1][ci] W[kh][kw][ci][co], zero outside the image."""
    inp, W, b = np.asarray(inp, F64), np.asarray(W, F64), np.asarray(b, F64)
    n, H, Wd, _ = inp.shape
    padded = np.zeros((n, H + 2, Wd + 2, inp.shape[3]), F64)
    padded[:, 1:H + 1, 1:Wd + 1, :] = inp
    out = np.zeros((n, H, Wd, W.shape[3]), F64) + b
    for kh in range(3):
        for kw in range(3):
            out += padded[:, kh:kh + H, kw:kw + Wd, :] @ W[kh, kw]
    return out


def conv3x3_backward(inp, W, dout):
    """Gradients of sum(out * dout) for out = conv3x3_forward(inp, W, b): (d_inp, d_W, d_b)."""
    inp, W, dout = np.asarray(inp, F64), np.asarray(W, F64), np.asarray(dout, F64)
    n, H, Wd, cin = inp.shape
    padded = np.zeros((n, H + 2, Wd + 2, cin), F64)
    padded[:, 1:H + 1, 1:Wd + 1, :] = inp
    d_padded = np.zeros_like(padded)
    dW = np.zeros_like(W)
    for kh in range(3):
        for kw in range(3):
            window = padded[:, kh:kh + H, kw:kw + Wd, :]
            dW[kh, kw] = window.reshape(-1, cin).T @ dout.reshape(-1, dout.shape[3])
            d_padded[:, kh:kh + H, kw:kw + Wd, :] += dout @ W[kh, kw].T
    return d_padded[:, 1:H + 1, 1:Wd + 1, :], dW, dout.sum(axis=(0, 1, 2))


def convblock_param_count(C, classes):
    return 2 * (9 * C * C + C) + C * classes + classes


def convblock_unpack(x, C, classes):
    """Views (Wa, ba, Wb, bb, Wh, bh) of the flat parameter vector."""
    out, off = [], 0
    for shape in ((3, 3, C, C), (C,), (3, 3, C, C), (C,), (C, classes), (classes,)):
        size = int(np.prod(shape))
        out.append(x[off:off + size].reshape(shape))
        off += size
    assert off == x.shape[0]
    return out


def convblock_loss_grad(x, C, classes, X, labels, bf16_operands=False):
    """Residual block + pooled linear classifier: (mean cross-entropy over the batch, flat gradient in x's layout).
    X [B][H][W][C], labels [B].  bf16_operands: the diagnostic mode of the module header."""
    q = round_to_bf16 if bf16_operands else (lambda a: np.asarray(a, F64))
    x = np.asarray(x, F64)
    X = np.asarray(X, F64)
    Wa, ba, Wb, bb, Wh, bh = convblock_unpack(x, C, classes)
    Xq, Wa, Wb = q(X), q(Wa), q(Wb)                                      # operands of the convolutions
    B = X.shape[0]
    a1 = q(np.maximum(conv3x3_forward(Xq, Wa, ba), 0.0))
    a2 = np.maximum(conv3x3_forward(a1, Wb, bb) + X, 0.0)                # the shortcut is not an operand
    pooled = a2.mean(axis=(1, 2))
    logits = pooled @ Wh + bh
    shifted = logits - logits.max(axis=1, keepdims=True)
    logsumexp = np.log(np.exp(shifted).sum(axis=1))
    rows = np.arange(B)
    loss = float((logsumexp - shifted[rows, labels]).mean())
    dlogits = np.exp(shifted - logsumexp[:, None])
    dlogits[rows, labels] -= 1.0
    dlogits /= B
    g = np.empty_like(x)
    gWa, gba, gWb, gbb, gWh, gbh = convblock_unpack(g, C, classes)
    gWh[...] = pooled.T @ dlogits
    gbh[...] = dlogits.sum(axis=0)
    d_pooled = dlogits @ Wh.T
    positions = X.shape[1] * X.shape[2]
    d_z2 = q((d_pooled[:, None, None, :] / positions) * (a2 > 0.0))    # through the mean and the second ReLU
    d_a1, dWb, dbb = conv3x3_backward(a1, Wb, d_z2)
    gWb[...] = dWb
    gbb[...] = dbb
    d_z1 = q(d_a1 * (a1 > 0.0))
    _, dWa, dba = conv3x3_backward(Xq, Wa, d_z1)                        # the input is data: its gradient is not needed
    gWa[...] = dWa
    gba[...] = dba
    return loss, g


BN_EPS = 1e-5


def batchnorm_forward(z, gamma, beta, eps=BN_EPS):
    """Training-mode batch normalisation per channel (last axis) over all other axes: returns (out, xhat, inv_std)."""
    z, gamma, beta = np.asarray(z, F64), np.asarray(gamma, F64), np.asarray(beta, F64)
    axes = tuple(range(z.ndim - 1))
    mean = z.mean(axis=axes)
    var = ((z - mean) ** 2).mean(axis=axes)            # biased variance
    inv_std = 1.0 / np.sqrt(var + eps)
    xhat = (z - mean) * inv_std
    return gamma * xhat + beta, xhat, inv_std


def batchnorm_backward(dout, xhat, inv_std, gamma):
    """Gradients of sum(out * dout) through batchnorm_forward: (d_z, d_gamma, d_beta).
    d_z = gamma inv_std (dout - mean(dout) - xhat mean(dout xhat)), the means per channel over samples and positions."""
    dout, xhat = np.asarray(dout, F64), np.asarray(xhat, F64)
    axes = tuple(range(dout.ndim - 1))
    d_beta = dout.sum(axis=axes)
    d_gamma = (dout * xhat).sum(axis=axes)
    count = dout.size // dout.shape[-1]
    d_z = np.asarray(gamma, F64) * inv_std * (dout - d_beta / count - xhat * (d_gamma / count))
    return d_z, d_gamma, d_beta


def convblock_bn_param_count(C, classes):
    return 2 * (9 * C * C + 2 * C) + C * classes + classes


def convblock_bn_unpack(x, C, classes):
    """Views (Wa, ga, ba, Wb, gb, bb, Wh, bh) of the flat parameter vector."""
    out, off = [], 0
    for shape in ((3, 3, C, C), (C,), (C,), (3, 3, C, C), (C,), (C,), (C, classes), (classes,)):
        size = int(np.prod(shape))
        out.append(x[off:off + size].reshape(shape))
        off += size
    assert off == x.shape[0]
    return out


def convblock_bn_loss_grad(x, C, classes, X, labels, eps=BN_EPS, bf16_operands=False):
    """The residual block with batch normalisation + pooled linear classifier: (mean cross-entropy over the batch,
    flat gradient in x's layout).  X [B][H][W][C], labels [B].  bf16_operands: the diagnostic mode of the module header."""
    q = round_to_bf16 if bf16_operands else (lambda a: np.asarray(a, F64))
    x = np.asarray(x, F64)
    X = np.asarray(X, F64)
    Wa, ga, ba, Wb, gb, bb, Wh, bh = convblock_bn_unpack(x, C, classes)
    Xq, Wa, Wb = q(X), q(Wa), q(Wb)                                      # operands of the convolutions
    B = X.shape[0]
    zero = np.zeros(C)
    z1 = conv3x3_forward(Xq, Wa, zero)
    n1, xhat1, istd1 = batchnorm_forward(z1, ga, ba, eps)
    a1 = q(np.maximum(n1, 0.0))
    z2 = conv3x3_forward(a1, Wb, zero)
    n2, xhat2, istd2 = batchnorm_forward(z2, gb, bb, eps)
    a2 = np.maximum(n2 + X, 0.0)
    pooled = a2.mean(axis=(1, 2))
    logits = pooled @ Wh + bh
    shifted = logits - logits.max(axis=1, keepdims=True)
    logsumexp = np.log(np.exp(shifted).sum(axis=1))
    rows = np.arange(B)
    loss = float((logsumexp - shifted[rows, labels]).mean())
    dlogits = np.exp(shifted - logsumexp[:, None])
    dlogits[rows, labels] -= 1.0
    dlogits /= B
    g = np.empty_like(x)
    gWa, gga, gba, gWb, ggb, gbb, gWh, gbh = convblock_bn_unpack(g, C, classes)
    gWh[...] = pooled.T @ dlogits
    gbh[...] = dlogits.sum(axis=0)
    d_pooled = dlogits @ Wh.T
    positions = X.shape[1] * X.shape[2]
    d_n2 = (d_pooled[:, None, None, :] / positions) * (a2 > 0.0)       # through the mean and the second ReLU
    d_z2, dgb, dbb = batchnorm_backward(d_n2, xhat2, istd2, gb)
    ggb[...] = dgb
    gbb[...] = dbb
    d_z2 = q(d_z2)
    d_a1, dWb, _ = conv3x3_backward(a1, Wb, d_z2)
    gWb[...] = dWb
    d_n1 = d_a1 * (a1 > 0.0)
    d_z1, dga, dba = batchnorm_backward(d_n1, xhat1, istd1, ga)
    gga[...] = dga
    gba[...] = dba
    _, dWa, _ = conv3x3_backward(Xq, Wa, q(d_z1))                       # the input is data: its gradient is not needed
    gWa[...] = dWa
    return loss, g


def convblock_relu_margin(x, C, classes, X, batch_norm=False, eps=BN_EPS, bf16_operands=False):
    """Smallest |input of a ReLU| in the block's forward pass.  The loss is not differentiable where such an input is
    zero: a device computing in single precision may take the other branch when the margin is within its rounding, and
    one activation taken the other way moves the gradient by about 1 / sqrt(number of activations) of its norm.  Parity
    cases use this to show that their inputs sit away from those points.  bf16_operands: the forward pass of the
    diagnostic mode of the module header."""
    q = round_to_bf16 if bf16_operands else (lambda a: np.asarray(a, F64))
    x = np.asarray(x, F64)
    X = np.asarray(X, F64)
    if batch_norm:
        Wa, ga, ba, Wb, gb, bb, _, _ = convblock_bn_unpack(x, C, classes)
        zero = np.zeros(C)
        n1 = batchnorm_forward(conv3x3_forward(q(X), q(Wa), zero), ga, ba, eps)[0]
        n2 = batchnorm_forward(conv3x3_forward(q(np.maximum(n1, 0.0)), q(Wb), zero), gb, bb, eps)[0] + X
    else:
        Wa, ba, Wb, bb, _, _ = convblock_unpack(x, C, classes)
        n1 = conv3x3_forward(q(X), q(Wa), ba)
        n2 = conv3x3_forward(q(np.maximum(n1, 0.0)), q(Wb), bb) + X
    return float(min(np.abs(n1).min(), np.abs(n2).min()))
